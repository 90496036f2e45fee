"""KVTC reference coder on the CPU -- TEST INFRASTRUCTURE, NOT A PRODUCT PATH.

A plain, slow NumPy implementation of the KV-cache transform coder of
"KV Cache Transform Coding for Compact Storage in LLM Inference"
(calibration, encode, decode, entropy stage), written step by step in the
paper's order and notation.  It exists so that the GPU library can be checked
against something that can be verified by eye.  Only the tests, the smoke
check and the CPU-baseline leg of the benchmark may import it; it shares no
code with the GPU path and imports nothing from it.

Arithmetic is float64 unless a step fixes another precision:
  * the basis V is stored in 16 bits (paper, appendix on PCA matrix sizes): bf16 here;
  * the projected coefficients are handed to the quantiser as float32, and the
    decision "which integer code" is taken in float32, the precision the GPU
    kernels take it in;
  * the shared per-group shift and scale are 16-bit (paper, Section
    "Quantization"): IEEE fp16 here, shift rounded down, scale rounded up.

Pins (see tests/test_oracle_*.py): PCA against the closed-form covariance of
the synthetic generator and against the Eckart-Young identity; the quantiser
against its closed-form error bound, the Frobenius identity of Section
"Quantization" (second display) and a worked byte example; the fp16 directed
roundings against an exhaustive table of all fp16 values; the bit allocation
against brute-force enumeration on tiny problems; pack/unpack against each
other and the worked example; the record size against the bit budget.
The *specific* allocation the dynamic programme returns on a large input has
no external fixture: parity unpinned for that (it never reaches the GPU as
anything but data).
"""
from __future__ import annotations

import zlib
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import numpy as np

# --------------------------------------------------------------------------
# number formats
# --------------------------------------------------------------------------

def bf16_bits(x) -> np.ndarray:
    """float -> bfloat16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    return ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)


def bf16_to_f32(bits) -> np.ndarray:
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(x) -> np.ndarray:
    """Values rounded to bfloat16, returned as float32."""
    return bf16_to_f32(bf16_bits(x))


FP16_MAX = np.float32(65504.0)


def fp16_floor(x) -> np.ndarray:
    """Largest finite fp16 value <= x (x float32); saturates at +-65504."""
    x = np.clip(np.asarray(x, dtype=np.float32), -FP16_MAX, FP16_MAX)
    with np.errstate(over="ignore"):
        h = x.astype(np.float16)
    too_big = h.astype(np.float32) > x
    with np.errstate(over="ignore"):
        h = np.where(too_big, np.nextafter(h, np.float16(-np.inf)), h).astype(np.float16)
    return h


def fp16_ceil(x) -> np.ndarray:
    """Smallest finite fp16 value >= x (x float32); saturates at +-65504."""
    x = np.clip(np.asarray(x, dtype=np.float32), -FP16_MAX, FP16_MAX)
    with np.errstate(over="ignore"):
        h = x.astype(np.float16)
    too_small = h.astype(np.float32) < x
    with np.errstate(over="ignore"):
        h = np.where(too_small, np.nextafter(h, np.float16(np.inf)), h).astype(np.float16)
    return h


# --------------------------------------------------------------------------
# calibration, part 1: PCA  (paper, Section "Feature decorrelation", eq. 2-3)
# --------------------------------------------------------------------------

def pca(C: np.ndarray) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """mu, V, S with C - mu = U diag(S) V^T, singular values descending.

    Sign convention (the paper leaves it open): each column of V has its
    largest-magnitude entry positive.
    """
    C = np.asarray(C, dtype=np.float64)
    mu = C.mean(axis=0)
    _, S, Vt = np.linalg.svd(C - mu[None, :], full_matrices=False)
    V = Vt.T.copy()
    idx = np.argmax(np.abs(V), axis=0)
    sgn = np.sign(V[idx, np.arange(V.shape[1])])
    sgn[sgn == 0] = 1.0
    V *= sgn[None, :]
    return mu, V, S


# --------------------------------------------------------------------------
# the quantiser of one group (paper, Section "Quantization": groups of
# subsequent PCA coordinates share a 16-bit shift and a 16-bit scale; uniform
# min-max quantisation as in KIVI, applied in the decorrelated domain)
# --------------------------------------------------------------------------

def quantise_group(d32: np.ndarray, bits: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Quantise one group of coefficients of every token.

    d32: [T, n] float32.  Returns (shift [T] fp16, scale [T] fp16, codes [T, n] uint32).
      lo = min_j d, hi = max_j d
      shift = fp16_floor(lo)
      scale = fp16_ceil((hi - shift) / (2^bits - 1))        float32 arithmetic
      code  = clip(rint((d - shift) * (1/scale)), 0, 2^bits - 1), 0 if scale == 0
    Every float operation above is a single float32 operation (subtract,
    divide, reciprocal, multiply), the precision the decision is taken in.
    """
    d32 = np.asarray(d32, dtype=np.float32)
    qmax = np.float32((1 << bits) - 1)
    lo = d32.min(axis=1)
    hi = d32.max(axis=1)
    shift = fp16_floor(lo)
    shift32 = shift.astype(np.float32)
    with np.errstate(over="ignore", invalid="ignore"):
        scale = fp16_ceil((hi - shift32) / qmax)
    scale32 = scale.astype(np.float32)
    with np.errstate(divide="ignore"):
        inv = np.where(scale32 > 0, np.float32(1.0) / scale32, np.float32(0.0)).astype(np.float32)
    q = (d32 - shift32[:, None]) * inv[:, None]            # float32 sub, float32 mul
    with np.errstate(invalid="ignore"):
        codes = np.clip(np.rint(q), np.float32(0.0), qmax)  # rint = round half to even
    codes = np.nan_to_num(codes, nan=0.0).astype(np.uint32)
    return shift, scale, codes


def dequantise_group(shift: np.ndarray, scale: np.ndarray, codes: np.ndarray) -> np.ndarray:
    """d_hat = shift + code * scale, float64 (exact for these operand sizes)."""
    return shift.astype(np.float64)[:, None] + codes.astype(np.float64) * scale.astype(np.float64)[:, None]


# --------------------------------------------------------------------------
# calibration, part 2: bit allocation by dynamic programming
# (paper, Section "Quantization" and appendix "Dynamic programming algorithm")
# --------------------------------------------------------------------------

def bit_budget(p: int, cr: float) -> int:
    """Per-token budget in bits for a target compression ratio of 16-bit features:
    whole 32-bit words, headers and padding included, so the achieved ratio is >= cr."""
    return 32 * int((16 * p) // (32 * cr))


@dataclass(frozen=True)
class Block:
    start: int     # first PCA coordinate
    n: int         # number of coordinates
    bits: int      # 0 = dropped ("None" type)


class BlockErrors:
    """error_change(start, n, bits) = ||blk - Q(blk)||^2 - ||blk||^2 on the calibration
    coefficients P (squared Frobenius norms, float64), cached."""

    def __init__(self, P32: np.ndarray):
        self.P32 = np.asarray(P32, dtype=np.float32)
        self.energy = (self.P32.astype(np.float64) ** 2).sum(axis=0)   # per coordinate
        self._cache = {}

    def change(self, start: int, n: int, bits: int) -> float:
        if bits == 0:
            return 0.0
        key = (start, n, bits)
        v = self._cache.get(key)
        if v is None:
            blk = self.P32[:, start:start + n]
            sh, sc, co = quantise_group(blk, bits)
            err = blk.astype(np.float64) - dequantise_group(sh, sc, co)
            v = float((err * err).sum() - self.energy[start:start + n].sum())
            self._cache[key] = v
        return v


def dp_allocate(errors: BlockErrors, n_features: int, budget_bits: int,
                block_sizes: Sequence[int] = (16, 64, 256, 1024),
                widths: Sequence[int] = (1, 2, 3, 4, 5, 6, 7, 8),
                header_bits: int = 32, unit: int = 16) -> Tuple[List[Block], float]:
    """Bit allocation under a per-token budget (paper, appendix "Dynamic programming
    algorithm": least error over the first i coordinates within b bits, plus the decision
    that reached it; optimal by induction on i and b).

    State: gain[i, b] = the least change of the squared error, relative to dropping
    everything, that the first i coordinates can reach with at most b bits.  The last
    block of such a prefix has one of the allowed sizes n and a type: "None" (zero bits,
    cost 0, change 0: the coordinates are dropped) or uniform min-max quantisation at a
    width w from `widths`, cost n*w + header_bits (the shared 16-bit shift and 16-bit
    scale), change errors.change(start, n, w).  So

        gain[i, b] = min(0, min over (n, type) with cost <= b of gain[i - n, b - cost] + change)

    where the 0 is the prefix left wholly at zero bits (the paper's tables start from that
    state for every i, which is also what makes a prefix of any length droppable).  A whole
    row is computed at once: for a fixed last block the candidates over all b are the
    earlier row shifted right by the block's cost.  "At most b" needs no separate carry
    from b - 1: the earlier rows are already non-increasing in b.

    `unit` is the granularity of block boundaries and of the budget axis.  unit=1 is the
    algorithm as stated (a block may end at any coordinate).  unit=16 adds one
    restriction: blocks start and end at multiples of 16 coordinates, so every cost is a
    multiple of 16 bits and the budget axis can be walked in 16-bit steps with the same
    result.  Ties: a candidate replaces the incumbent only when strictly better;
    candidates are tried with block sizes ascending and types in the listed order.
    Returns (blocks in coordinate order, zero-bit blocks included; best error).
    """
    assert n_features % unit == 0 and header_bits % unit == 0 and all(s % unit == 0 for s in block_sizes)
    nu = n_features // unit
    qb = budget_bits // unit
    types = [0] + list(widths)
    gain = np.zeros((nu + 1, qb + 1), dtype=np.float64)
    choice = np.full((nu + 1, qb + 1), -1, dtype=np.int32)       # index into `moves` of row i; -1 = prefix dropped
    moves_of_row: List[List[Tuple[int, int, int]]] = [[]]          # per row: (block units, width, cost units)
    for i in range(1, nu + 1):
        moves = [(size // unit, w, 0 if w == 0 else (size * w + header_bits) // unit)
                 for size in sorted(block_sizes) if size // unit <= i for w in types]
        moves_of_row.append(moves)
        row = gain[i]
        for k, (su, w, cost) in enumerate(moves):
            if cost > qb:
                continue
            cand = gain[i - su, :qb + 1 - cost] + errors.change((i - su) * unit, su * unit, w)
            better = cand < row[cost:]
            row[cost:][better] = cand[better]
            choice[i, cost:][better] = k
    blocks: List[Block] = []
    i, b = nu, qb
    while i > 0 and choice[i, b] >= 0:
        su, w, cost = moves_of_row[i][int(choice[i, b])]
        blocks.append(Block((i - su) * unit, su * unit, w))
        i, b = i - su, b - cost
    if i > 0:      # the rest of the prefix was never worth any bits
        blocks.append(Block(0, i * unit, 0))
    blocks.reverse()
    return blocks, float(errors.energy[:n_features].sum() + gain[nu, qb])


def allocation_error(errors: BlockErrors, n_features: int, blocks: Sequence[Block]) -> float:
    """Total squared error of an allocation, evaluated directly (not through the tables)."""
    e = float(errors.energy[:n_features].sum())
    for blk in blocks:
        e += errors.change(blk.start, blk.n, blk.bits)
    return e


def allocation_bits(blocks: Sequence[Block], header_bits: int = 32) -> int:
    return sum(b.n * b.bits + header_bits for b in blocks if b.bits > 0)


# --------------------------------------------------------------------------
# plan = what calibration hands to the coder (per layer, per K/V, per ratio)
# --------------------------------------------------------------------------

@dataclass
class Plan:
    p: int
    r: int
    kept: np.ndarray            # [r] indices of the kept PCA coordinates
    mu32: np.ndarray            # [p] float32
    v_bits: np.ndarray          # [p, r] uint16: kept columns of V as bf16
    v64: np.ndarray             # [p, r] float64: the same values
    c32: np.ndarray             # [r] float32: mu^T V_kept
    group_n: np.ndarray         # [G] coordinates per kept group
    group_bits: np.ndarray      # [G] width per kept group
    coef_bits: np.ndarray       # [r] width of each kept coordinate
    coef_off: np.ndarray        # [r] bit offset of each kept coordinate's code in the record
    coef_group: np.ndarray      # [r] group index of each kept coordinate
    record_bytes: int           # R

    @property
    def n_groups(self) -> int:
        return int(self.group_n.shape[0])


def compile_plan(mu: np.ndarray, V: np.ndarray, blocks: Sequence[Block]) -> Plan:
    """Drop zero-bit blocks, trim V to the kept coordinates (paper, end of Section
    "Quantization"), round it to bf16, and lay out the record:
    G header dwords, then the codes group by group, LSB first, padded to 32 bits."""
    p = V.shape[0]
    kept_blocks = [b for b in blocks if b.bits > 0]
    kept = np.concatenate([np.arange(b.start, b.start + b.n) for b in kept_blocks]) if kept_blocks \
        else np.zeros(0, dtype=np.int64)
    r = int(kept.shape[0])
    v_bits = bf16_bits(V[:, kept]) if r else np.zeros((p, 0), dtype=np.uint16)
    v64 = bf16_to_f32(v_bits).astype(np.float64)
    mu32 = np.asarray(mu, dtype=np.float32)
    c32 = (mu32.astype(np.float64) @ v64).astype(np.float32)
    group_n = np.array([b.n for b in kept_blocks], dtype=np.int64)
    group_bits = np.array([b.bits for b in kept_blocks], dtype=np.int64)
    G = len(kept_blocks)
    coef_bits = np.repeat(group_bits, group_n) if G else np.zeros(0, dtype=np.int64)
    coef_group = np.repeat(np.arange(G), group_n) if G else np.zeros(0, dtype=np.int64)
    coef_off = 32 * G + np.concatenate([[0], np.cumsum(coef_bits)[:-1]]) if r else np.zeros(0, dtype=np.int64)
    total_bits = 32 * G + int(coef_bits.sum())
    R = 4 * ((total_bits + 31) // 32)
    return Plan(p, r, kept, mu32, v_bits, v64, c32, group_n, group_bits,
                coef_bits.astype(np.int64), np.asarray(coef_off, dtype=np.int64), coef_group.astype(np.int64), R)


def calibrate(C: np.ndarray, cr: float, n_dp_tokens: int = 2048,
              block_sizes: Sequence[int] = (16, 64, 256, 1024),
              widths: Sequence[int] = (1, 2, 3, 4, 5, 6, 7, 8)) -> Tuple[Plan, dict]:
    """PCA + bit allocation + plan on a calibration matrix C [n, p] (values as the
    coder will see them, i.e. already in the cache's dtype)."""
    mu, V, S = pca(C)
    return calibrate_from_pca(C, mu, V, S, cr, n_dp_tokens, block_sizes, widths)


def calibrate_from_pca(C, mu, V, S, cr, n_dp_tokens=2048, block_sizes=(16, 64, 256, 1024),
                       widths=(1, 2, 3, 4, 5, 6, 7, 8), errors: Optional[BlockErrors] = None):
    p = V.shape[0]
    if errors is None:
        errors = dp_errors(C, mu, V, n_dp_tokens)
    sizes = [s for s in block_sizes if s <= p]
    B = bit_budget(p, cr)
    blocks, best = dp_allocate(errors, p, B, sizes, widths)
    plan = compile_plan(mu, V, blocks)
    info = dict(budget_bits=B, blocks=blocks, dp_error=best, singular_values=S, errors=errors)
    return plan, info


def dp_errors(C, mu, V, n_dp_tokens=2048) -> BlockErrors:
    """Coefficients P = (C - mu) V of the first n_dp_tokens calibration tokens, as the
    coder computes them (stored bf16 basis, float32 result), wrapped for the DP."""
    Cs = np.asarray(C[:n_dp_tokens], dtype=np.float64)
    Vb = bf16_round(V).astype(np.float64)
    mu32 = np.asarray(mu, dtype=np.float32).astype(np.float64)
    P32 = ((Cs - mu32[None, :]) @ Vb).astype(np.float32)
    return BlockErrors(P32)


# --------------------------------------------------------------------------
# encode  (paper, Section "Method": compression = project, quantise, pack)
# --------------------------------------------------------------------------

def project(plan: Plan, x: np.ndarray) -> np.ndarray:
    """d = (x - mu) V_kept in float64, handed on as float32.  x: [T, p] values of the
    cache dtype (any float array holding them exactly)."""
    x = np.asarray(x, dtype=np.float64)
    d = (x - plan.mu32.astype(np.float64)[None, :]) @ plan.v64
    return d.astype(np.float32)


def quantise(plan: Plan, d32: np.ndarray):
    """Per token and kept group: shift, scale (fp16) and the codes."""
    T = d32.shape[0]
    G = plan.n_groups
    shift = np.zeros((T, G), dtype=np.float16)
    scale = np.zeros((T, G), dtype=np.float16)
    codes = np.zeros((T, plan.r), dtype=np.uint32)
    j = 0
    for g in range(G):
        n, b = int(plan.group_n[g]), int(plan.group_bits[g])
        shift[:, g], scale[:, g], codes[:, j:j + n] = quantise_group(d32[:, j:j + n], b)
        j += n
    return shift, scale, codes


def pack(plan: Plan, shift: np.ndarray, scale: np.ndarray, codes: np.ndarray) -> np.ndarray:
    """Records [T, R] uint8.  A record is a little-endian bit string: G header dwords
    (shift's fp16 bits in bits 0-15, scale's in bits 16-31), then each kept coordinate's
    code in PCA order, least significant bit first, no gaps, zero-padded to 32 bits."""
    T = codes.shape[0]
    G = plan.n_groups
    bits = np.zeros((T, plan.record_bytes * 8), dtype=np.uint8)
    sh = np.ascontiguousarray(shift, dtype=np.float16).view(np.uint16).reshape(T, G)
    sc = np.ascontiguousarray(scale, dtype=np.float16).view(np.uint16).reshape(T, G)
    for g in range(G):
        for k in range(16):
            bits[:, 32 * g + k] = (sh[:, g] >> k) & 1
            bits[:, 32 * g + 16 + k] = (sc[:, g] >> k) & 1
    for j in range(plan.r):
        o = int(plan.coef_off[j])
        for k in range(int(plan.coef_bits[j])):
            bits[:, o + k] = (codes[:, j] >> k) & 1
    return np.packbits(bits, axis=1, bitorder="little")


def encode(plan: Plan, x: np.ndarray) -> np.ndarray:
    d32 = project(plan, x)
    shift, scale, codes = quantise(plan, d32)
    return pack(plan, shift, scale, codes)


# --------------------------------------------------------------------------
# decode  (paper, Section "Method": decompression reverses the steps; eq. 3)
# --------------------------------------------------------------------------

def unpack(plan: Plan, records: np.ndarray):
    records = np.ascontiguousarray(records, dtype=np.uint8).reshape(-1, plan.record_bytes)
    T = records.shape[0]
    G = plan.n_groups
    bits = np.unpackbits(records, axis=1, bitorder="little")
    sh = np.zeros((T, G), dtype=np.uint16)
    sc = np.zeros((T, G), dtype=np.uint16)
    for g in range(G):
        for k in range(16):
            sh[:, g] |= bits[:, 32 * g + k].astype(np.uint16) << k
            sc[:, g] |= bits[:, 32 * g + 16 + k].astype(np.uint16) << k
    codes = np.zeros((T, plan.r), dtype=np.uint32)
    for j in range(plan.r):
        o = int(plan.coef_off[j])
        for k in range(int(plan.coef_bits[j])):
            codes[:, j] |= bits[:, o + k].astype(np.uint32) << k
    return sh.view(np.float16), sc.view(np.float16), codes


def dequantise(plan: Plan, shift, scale, codes) -> np.ndarray:
    """d_hat [T, r] float64."""
    g = plan.coef_group
    return shift.astype(np.float64)[:, g] + codes.astype(np.float64) * scale.astype(np.float64)[:, g]


def back_project(plan: Plan, d_hat: np.ndarray) -> np.ndarray:
    """x_hat = d_hat V_kept^T + mu, float64."""
    return d_hat @ plan.v64.T + plan.mu32.astype(np.float64)[None, :]


def decode(plan: Plan, records: np.ndarray, out: str = "f64", operand_bf16: bool = False) -> np.ndarray:
    """Reconstruct [T, p].  out: "f64" (no final rounding), "bf16" or "f32" (values of
    that dtype, returned as float32).  operand_bf16=True additionally rounds d_hat to
    float32 and then to bf16 before the product, which is what a bf16 matrix unit is
    fed; it is a checking aid, not the definition."""
    shift, scale, codes = unpack(plan, records)
    d_hat = dequantise(plan, shift, scale, codes)
    if operand_bf16:
        d_hat = bf16_round(d_hat.astype(np.float32)).astype(np.float64)
    x_hat = back_project(plan, d_hat)
    if out == "f64":
        return x_hat
    if out == "f32":
        return x_hat.astype(np.float32)
    if out == "bf16":
        return bf16_round(x_hat.astype(np.float32))
    raise ValueError(out)


# --------------------------------------------------------------------------
# entropy stage (paper, Section "Entropy coding"): DEFLATE over the byte array
# --------------------------------------------------------------------------

def deflate(records: np.ndarray, level: int = 6) -> bytes:
    return zlib.compress(np.ascontiguousarray(records, dtype=np.uint8).tobytes(), level)


def inflate(blob: bytes, plan: Plan) -> np.ndarray:
    return np.frombuffer(zlib.decompress(blob), dtype=np.uint8).reshape(-1, plan.record_bytes)


def compression_ratios(plan: Plan, n_tokens: int, records: np.ndarray, level: int = 6):
    raw = 2 * plan.p * n_tokens
    return raw / records.size, raw / len(deflate(records, level))


# --------------------------------------------------------------------------
# plan bundles on disk (the calibration result is data for the coder)
# --------------------------------------------------------------------------

def plan_from_arrays(mu32: np.ndarray, v_bits: np.ndarray, group_n, group_bits) -> Plan:
    """Rebuild a Plan from what a bundle stores: mean, kept basis columns (bf16 bits) and
    the kept groups.  The kept coordinates are renumbered 0..r-1."""
    p, r = v_bits.shape
    blocks, s = [], 0
    for n, b in zip(group_n, group_bits):
        blocks.append(Block(s, int(n), int(b)))
        s += int(n)
    assert s == r
    plan = compile_plan(np.asarray(mu32, dtype=np.float32), bf16_to_f32(v_bits).astype(np.float64), blocks)
    assert np.array_equal(plan.v_bits, np.asarray(v_bits, dtype=np.uint16))
    return plan


def save_plan(path: str, plan: Plan, **meta) -> None:
    np.savez(path, mu32=plan.mu32, v_bits=plan.v_bits, group_n=plan.group_n.astype(np.int32),
             group_bits=plan.group_bits.astype(np.int32), kept=plan.kept.astype(np.int32),
             **{k: np.asarray(v) for k, v in meta.items()})
