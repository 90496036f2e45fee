"""Plans over the concatenated features of several layers -- TEST INFRASTRUCTURE, NOT A PRODUCT PATH.

Paper, Section "Feature decorrelation": for every sampled position the keys (or values) of l layers
and h heads are concatenated into one vector of p = l*h*d_head features and ONE basis is computed
for it; appendix "PCA matrix sizes": that basis is cut to its first few thousand components (8K or
10K for the tested models) before the bit allocation removes more; appendix "PCA feature concat size
vs performance": more layers under one basis give better accuracy at the same ratio.

Such a plan keeps more coordinates than the per-layer ones: thousands.  Nothing in the method
changes -- project, quantise group by group, pack -- but the byte layout (on which the paper is
silent) is cut into SECTIONS here: consecutive kept groups are gathered into sections of at most
1024 coordinates and 64 groups; section c is coded exactly like a plan made of those groups alone
(its own records: the groups' header dwords, then their codes, padded to 32 bits), and the stream
of a tensor of T tokens is the T records of section 0, then the T records of section 1, ..., each
section starting on a 16-byte boundary.  The codes and headers are those of the unsectioned plan
(a group's quantisation never looks outside the group); only their place in the byte array differs.

Only the tests may import this module; it shares no code with the GPU library.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple

import numpy as np

import kvtc_oracle as ko

MAX_SECTION_COORDS = 1024
MAX_SECTION_GROUPS = 64


def split_groups(group_n: Sequence[int], max_coords: int = MAX_SECTION_COORDS,
                 max_groups: int = MAX_SECTION_GROUPS) -> List[Tuple[int, int]]:
    """Consecutive groups -> sections [g0, g1), greedily: a section takes groups while it stays
    within max_coords coordinates and max_groups groups."""
    out = []
    g0, n, G = 0, 0, len(group_n)
    for g in range(G):
        gn = int(group_n[g])
        assert 0 < gn <= max_coords
        if g > g0 and (n + gn > max_coords or g - g0 >= max_groups):
            out.append((g0, g))
            g0, n = g, 0
        n += gn
    if G:
        out.append((g0, G))
    return out


def sections_of(plan: ko.Plan) -> List[ko.Plan]:
    """The plan of each section: the same mean, the section's columns of the basis, its groups."""
    starts = np.concatenate([[0], np.cumsum(plan.group_n)]).astype(np.int64)
    secs = []
    for g0, g1 in split_groups(plan.group_n):
        j0, j1 = int(starts[g0]), int(starts[g1])
        secs.append(ko.plan_from_arrays(plan.mu32, np.ascontiguousarray(plan.v_bits[:, j0:j1]),
                                        plan.group_n[g0:g1], plan.group_bits[g0:g1]))
    return secs


def record_bytes(plan: ko.Plan) -> int:
    """Bytes per token over all sections."""
    return sum(s.record_bytes for s in sections_of(plan))


def section_offsets(section_record_bytes: Sequence[int], n_tokens: int) -> List[int]:
    """Byte offset of each section's records in a tensor's stream, and the total length as the last
    entry: sections back to back, each start rounded up to 16 bytes."""
    offs, pos = [], 0
    for R in section_record_bytes:
        pos = (pos + 15) // 16 * 16
        offs.append(pos)
        pos += int(R) * int(n_tokens)
    offs.append(pos)
    return offs


def encode_wide(plan: ko.Plan, x: np.ndarray) -> np.ndarray:
    """Stream (uint8, one dimension) of a tensor x [T, p] under a sectioned plan."""
    secs = sections_of(plan)
    T = x.shape[0]
    offs = section_offsets([s.record_bytes for s in secs], T)
    out = np.zeros(offs[-1], dtype=np.uint8)
    for s, o in zip(secs, offs):
        out[o:o + T * s.record_bytes] = ko.encode(s, x).reshape(-1)
    return out


def unpack_wide(plan: ko.Plan, stream: np.ndarray, n_tokens: int):
    """Headers [T, G] and codes [T, r] of the whole plan, gathered from the sections."""
    secs = sections_of(plan)
    offs = section_offsets([s.record_bytes for s in secs], n_tokens)
    sh, sc, co = [], [], []
    for s, o in zip(secs, offs):
        a, b, c = ko.unpack(s, stream[o:o + n_tokens * s.record_bytes])
        sh.append(a); sc.append(b); co.append(c)
    return np.concatenate(sh, axis=1), np.concatenate(sc, axis=1), np.concatenate(co, axis=1)


def decode_wide(plan: ko.Plan, stream: np.ndarray, n_tokens: int, out: str = "f64", operand_bf16: bool = False) -> np.ndarray:
    """x_hat = d_hat V_kept^T + mu over ALL kept coordinates (eq. 3 of the paper), float64; `out` and
    `operand_bf16` as in kvtc_oracle.decode."""
    shift, scale, codes = unpack_wide(plan, stream, n_tokens)
    d_hat = ko.dequantise(plan, shift, scale, codes)
    if operand_bf16:
        d_hat = ko.bf16_round(d_hat.astype(np.float32)).astype(np.float64)
    x_hat = ko.back_project(plan, d_hat)
    if out == "f64":
        return x_hat
    if out == "f32":
        return x_hat.astype(np.float32)
    if out == "bf16":
        return ko.bf16_round(x_hat.astype(np.float32))
    raise ValueError(out)


def calibrate_wide(C: np.ndarray, cr: float, rank_cap: int, n_dp_tokens: int = 1024,
                   block_sizes: Sequence[int] = (16, 64, 256, 1024),
                   widths: Sequence[int] = (1, 2, 3, 4, 5, 6, 7, 8)):
    """PCA of the concatenated features, the basis cut to its first rank_cap components (appendix
    "PCA matrix sizes"), then the bit allocation over those components under the per-token budget of
    the ratio.  The budget counts what is stored per token: every section's record, its padding to
    32 bits included -- the allocation is re-run with 32 bits less until the records fit."""
    p = C.shape[1]
    assert rank_cap % 16 == 0 and 16 <= rank_cap <= p
    mu, V, S = ko.pca(C)
    Vc = V[:, :rank_cap]
    errors = ko.dp_errors(C, mu, Vc, n_dp_tokens)
    sizes = [s for s in block_sizes if s <= rank_cap]
    B = ko.bit_budget(p, cr)
    budget = B
    while True:
        blocks, best = ko.dp_allocate(errors, rank_cap, budget, sizes, widths)
        plan = ko.compile_plan(mu, Vc, blocks)
        if 8 * record_bytes(plan) <= B:
            break
        budget -= 32
    return plan, dict(budget_bits=B, dp_budget_bits=budget, blocks=blocks, dp_error=best, singular_values=S)
