"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on identical inputs.

Bars (written out here):
  * packed stream: the GPU stream must equal the oracle's packing of the GPU's own headers
    and codes bit for bit (canonical layout, zero padding);
  * codes: differ from the oracle's by at most 1 LSB on at most 1e-4 of the entries
    (rounding-boundary ties follow the fp32 projection, whose summation order differs);
    headers may differ by one fp16 ulp on a small fraction of (token, group) pairs for the
    same reason -- reported; above 1 % every differing header must lie inside the envelope the
    fp32 summation error bound of the projection allows (and the rate stay below 10 %);
  * reconstruction: within 1e-2 of the tensor's range (max - min) of the oracle's float64
    decode of the same stream, and within bf16-output rounding of the oracle's decode that
    feeds bf16 operands like the matrix cores do.
"""
import numpy as np
import pytest
import torch

import kvtc_oracle as ko
import kvtc_synth as ks
import paper_2511_01815_amd as kv

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _gpu_plan(oplan):
    groups = list(zip(oplan.group_n.tolist(), oplan.group_bits.tolist()))
    plan = kv.Plan(oplan.p, oplan.r, oplan.mu32, oplan.v_bits, groups)
    assert plan.record_bytes == oplan.record_bytes
    return plan


def _to_dev(x_host, dtype):
    """x_host: float32 values (already representable in the cache dtype)."""
    if dtype == kv.KVTC_BF16:
        bits = ks.f32_to_bf16_bits(x_host)
        return torch.from_numpy(bits.view(np.int16)).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(x_host, dtype=np.float32)).to(DEV)


def _from_dev(t):
    if t.dtype == torch.bfloat16:
        return ks.bf16_bits_to_f32(t.view(torch.int16).cpu().numpy().view(np.uint16))
    return t.cpu().numpy()


def _ulp_apart(a16, b16):
    """|difference| in fp16 ulps between two fp16 bit-pattern arrays (as ordered integers)."""
    def key(u):
        u = u.astype(np.int32)
        return np.where(u & 0x8000, -(u & 0x7fff), u & 0x7fff)
    return np.abs(key(a16) - key(b16))


def _headers_within_fp32_envelope(oplan, x_vals, d32, sh_g, sc_g, moved, label):
    """Every header that differs from the oracle's must be one the oracle itself produces for group extremes
    moved by no more than the fp32 summation error of the projection: a coordinate d_j = sum_i x_i v_ij - c_j
    accumulated in fp32 in any order is within (n - 1) * 2^-24 * (sum_i |x_i v_ij| + |c_j|), n = p + 1 terms, of the
    exact value.  The headers are monotone in the extremes (shift in lo; scale in hi - shift), so the reachable
    headers form an interval whose ends come from (lo - e, hi + e) and (lo + e, hi - e).  Weak coordinates
    (|d_j| far below the terms that cancel in it) make this envelope, and the mismatch rate, larger."""
    V = np.abs(oplan.v64)
    c = np.abs(oplan.mu32.astype(np.float64) @ oplan.v64)
    bound = (np.abs(np.asarray(x_vals, dtype=np.float64)) @ V + c[None, :]) * (oplan.p * 2.0 ** -24)
    j = 0
    for g in range(oplan.n_groups):
        n, b = int(oplan.group_n[g]), int(oplan.group_bits[g])
        rows = np.nonzero(moved[:, g])[0]
        if rows.size:
            d = d32[rows, j:j + n].astype(np.float64)
            e = bound[rows, j:j + n].max(axis=1)
            lo, hi = d.min(axis=1), d.max(axis=1)
            wide = np.stack([lo - e, hi + e], axis=1).astype(np.float32)
            tight = np.stack([lo + e, np.maximum(hi - e, lo + e)], axis=1).astype(np.float32)
            sh_lo, sc_hi, _ = ko.quantise_group(wide, b)
            sh_hi, sc_lo, _ = ko.quantise_group(tight, b)
            shg = sh_g[rows, g].astype(np.float64)
            scg = sc_g[rows, g].astype(np.float64)
            assert np.all((shg >= sh_lo.astype(np.float64)) & (shg <= sh_hi.astype(np.float64))), (label, g, "shift outside the envelope")
            # scale also moves with the shift it is measured from: widest range / tightest range bound it
            assert np.all((scg >= np.minimum(sc_lo, sc_hi).astype(np.float64)) & (scg <= np.maximum(sc_lo, sc_hi).astype(np.float64))), \
                (label, g, "scale outside the envelope")
        j += n


RATES = []        # one entry per checked stream; tests/conftest.py prints them in the terminal summary

# Header mismatches (always exactly one fp16 ulp, always inside the fp32 summation envelope).  Measured over this
# suite: 0 .. 3.5e-3 of (token, group) pairs on every stream but the 8x plans of the steep-spectrum layers, whose
# weakest kept groups reach 1.1e-2 (their coordinates are far smaller than the terms that cancel in them); those
# tests pass a bar of their own.
HDR_BAR = 1e-2


def check_stream(oplan, x_vals, rec_gpu, label="", hdr_bar=HDR_BAR):
    """Codes / headers / packing of a GPU stream against the oracle.  x_vals: the bf16-exact
    input values the kernel saw.  Returns stats (also appended to RATES).

    Plans with widths of at most 8 bits (everything calibration produces): the raw code
    mismatch rate must be <= 1e-4, no second look.  Headers: at most one fp16 ulp from the
    oracle's, every differing one inside the fp32 summation envelope, and their rate <= hdr_bar.
    Hand-built plans with widths above 8 bits get the arithmetic bar mean(2^b) * 2^-20 for the
    codes, and -- only they -- may have the codes of groups whose header moved re-decided with
    the GPU's header; that is printed, recorded as `redecided` and shows in the summary."""
    T = x_vals.shape[0]
    assert rec_gpu.shape == (T, oplan.record_bytes)
    d32 = ko.project(oplan, x_vals)
    sh_r, sc_r, co_r = ko.quantise(oplan, d32)
    sh_g, sc_g, co_g = ko.unpack(oplan, rec_gpu)
    # bit-exact packing of identical codes
    np.testing.assert_array_equal(ko.pack(oplan, sh_g, sc_g, co_g), rec_gpu, err_msg=f"{label}: stream not canonical")
    # headers
    sh_ne = sh_g.view(np.uint16) != sh_r.view(np.uint16)
    sc_ne = sc_g.view(np.uint16) != sc_r.view(np.uint16)
    hdr_rate = float((sh_ne | sc_ne).mean())
    assert _ulp_apart(sh_g.view(np.uint16), sh_r.view(np.uint16)).max() <= 1, label
    assert _ulp_apart(sc_g.view(np.uint16), sc_r.view(np.uint16)).max() <= 1, label
    # Any fp32 summation order is a valid projection, so a header may differ from the oracle's (fp64 sum, rounded
    # once) exactly when the group's extremes moved by no more than the fp32 summation error can move them: every
    # differing header is held to that envelope, whatever the rate; the rate has a bar of its own on top.
    n_moved = int((sh_ne | sc_ne).sum())
    envelope = n_moved > 0
    if envelope:
        _headers_within_fp32_envelope(oplan, x_vals, d32, sh_g, sc_g, sh_ne | sc_ne, label)
    # (a stream of a few tokens has too few headers for a rate: up to two single-ulp mismatches pass there)
    assert hdr_rate <= hdr_bar or n_moved <= 2, (label, "header mismatch rate", hdr_rate, hdr_bar)
    # codes
    diff = np.abs(co_g.astype(np.int64) - co_r.astype(np.int64))
    rate = float((diff != 0).mean())
    assert diff.max() <= 1, (label, int(diff.max()))
    # A code flips when the fp32 projection error (relative ~2^-22 of the group range after 64
    # accumulation steps) straddles a rounding boundary, i.e. with probability ~2^b * 2^-21 per entry:
    # far inside 1e-4 up to 8 bits; plans built by hand with wider codes get that arithmetic bound.
    wide = int(oplan.coef_bits.max()) > 8
    bar = max(1e-4, float(np.mean(2.0 ** oplan.coef_bits)) * 2.0 ** -20) if wide else 1e-4
    redecided, rate2 = False, None
    if rate > bar:
        assert wide, (label, "code mismatch rate", rate, bar)
        # a header that moved by one ulp shifts every code boundary of its group; compare
        # those groups against the oracle's decision taken with the GPU's header
        bad_g = (sh_ne | sc_ne)[:, oplan.coef_group]
        sh32 = sh_g.astype(np.float32)[:, oplan.coef_group]
        sc32 = sc_g.astype(np.float32)[:, oplan.coef_group]
        with np.errstate(divide="ignore"):
            inv = np.where(sc32 > 0, np.float32(1) / sc32, np.float32(0)).astype(np.float32)
        qmax = ((1 << oplan.coef_bits) - 1).astype(np.float32)[None, :]
        alt = np.clip(np.rint((d32 - sh32) * inv), 0, qmax).astype(np.int64)
        diff2 = np.where(bad_g, np.abs(co_g.astype(np.int64) - alt), diff)
        rate2 = float((diff2 != 0).mean())
        redecided = True
        print(f"[parity] {label}: raw code rate {rate:.3e} above {bar:.3e}; codes of moved-header groups re-decided "
              f"with the GPU's headers: {rate2:.3e}")
        assert diff2.max() <= 1 and rate2 <= bar, (label, rate, rate2)
    st = dict(label=label, code_rate=rate, code_bar=bar, hdr_rate=hdr_rate, hdr_bar=hdr_bar, envelope=envelope,
              redecided=redecided, code_rate_redecided=rate2, tokens=int(T), r=int(oplan.r),
              max_bits=int(oplan.coef_bits.max()))
    RATES.append(st)
    return st


def check_recon(oplan, rec_gpu, xh_gpu, x_vals, out_bf16, label=""):
    rng_x = float(x_vals.max() - x_vals.min())
    ref = ko.decode(oplan, rec_gpu)                         # definition, float64
    err = np.abs(xh_gpu.astype(np.float64) - ref).max()
    assert err <= 1e-2 * rng_x, (label, err, rng_x)
    mirror = ko.decode(oplan, rec_gpu, operand_bf16=True)   # bf16 operands, exact sums
    tol = 3e-5 * np.abs(mirror).max() + (2.0 ** -8 * np.abs(mirror) if out_bf16 else 0.0)
    assert np.all(np.abs(xh_gpu.astype(np.float64) - mirror) <= tol), (label, np.abs(xh_gpu - mirror).max())
    return err / rng_x


def roundtrip(oplan, plan, x_vals, dtype, ld_pad=0, label="", **bars):
    T, p = x_vals.shape
    ld = p + ld_pad
    xd = torch.zeros((T, ld), dtype=torch.bfloat16 if dtype == kv.KVTC_BF16 else torch.float32, device=DEV)
    xd[:, :p] = _to_dev(x_vals, dtype)
    R = plan.record_bytes
    guard = 64
    out = torch.full((T * R + guard,), 0xA5, dtype=torch.uint8, device=DEV)
    kv.kvtc_encode(plan.handle, xd, dtype, T, ld, out, T * R)
    xh = torch.full_like(xd, 7.0)
    kv.kvtc_decode(plan.handle, out, T * R, T, xh, dtype, ld)
    torch.cuda.synchronize()
    o = out.cpu().numpy()
    assert np.all(o[T * R:] == 0xA5), f"{label}: wrote past the stream"
    rec = o[:T * R].reshape(T, R)
    if ld_pad:
        assert torch.all(xh[:, p:] == 7.0), f"{label}: wrote into the row padding"
    xh_host = _from_dev(xh[:, :p].contiguous())
    seen = ko.bf16_round(x_vals)
    st = check_stream(oplan, seen, rec, label, **bars)
    st["recon"] = check_recon(oplan, rec, xh_host, seen, dtype == kv.KVTC_BF16, label)
    return st


# ---- fixtures: calibrated plans ---------------------------------------------------------------------

@pytest.fixture(scope="module")
def c1():
    wl = ks.WORKLOADS["c1"]
    L = ks.make_layer(ks.layer_spec("c1", 0, 0))
    C_ = ko.bf16_round(ks.draw_f32(L, wl.n_calib, ks.CALIB_DRAW))
    oplan, _ = ko.calibrate(C_, 4.0)
    return L, oplan, _gpu_plan(oplan)


@pytest.fixture(scope="module")
def c2():
    wl = ks.WORKLOADS["c2"]
    out = {}
    for kvi in (0, 1):
        L = ks.make_layer(ks.layer_spec("c2", 0, kvi))
        C_ = ks.bf16_bits_to_f32(ks.draw_bf16(L, wl.n_calib, ks.CALIB_DRAW))
        mu, V, S = ko.pca(C_)
        errs = ko.dp_errors(C_, mu, V)
        plans = {cr: ko.calibrate_from_pca(C_, mu, V, S, cr, errors=errs)[0] for cr in ((8.0, 16.0, 40.0) if kvi == 0 else (16.0,))}
        out[kvi] = (L, plans)
    return out


# ---- tests ------------------------------------------------------------------------------------------

def test_config1_fp32_whole_tensor(c1):
    L, oplan, plan = c1
    X = ks.draw_f32(L, ks.WORKLOADS["c1"].n_tokens, ks.TEST_DRAW)
    st = roundtrip(oplan, plan, X, kv.KVTC_F32, label="c1")
    print("c1", st)


@pytest.mark.parametrize("T", [1, 31, 33, 255, 257, 1000])
def test_ragged_tails(c1, T):
    L, oplan, plan = c1
    X = ks.draw_f32(L, T, 77 + T)
    roundtrip(oplan, plan, X, kv.KVTC_F32, label=f"tail{T}")
    roundtrip(oplan, plan, ko.bf16_round(X), kv.KVTC_BF16, ld_pad=24, label=f"tail{T}-bf16-strided")


def test_config2_single_layer_16x(c2):
    wl = ks.WORKLOADS["c2"]
    for kvi, T in ((0, wl.n_tokens), (1, 5000)):
        L, plans = c2[kvi]
        oplan = plans[16.0]
        plan = _gpu_plan(oplan)
        X = ks.bf16_bits_to_f32(ks.draw_bf16(L, T, ks.TEST_DRAW))
        st = roundtrip(oplan, plan, X, kv.KVTC_BF16, label=f"c2-kv{kvi}")
        print("c2", kvi, "r", oplan.r, "R", oplan.record_bytes, st)
        assert oplan.record_bytes <= 128


@pytest.mark.parametrize("cr", [8.0, 40.0])
def test_config2_other_ratios(c2, cr):
    L, plans = c2[0]
    oplan = plans[cr]
    plan = _gpu_plan(oplan)
    X = ks.bf16_bits_to_f32(ks.draw_bf16(L, 4099, ks.TEST_DRAW + 1))
    st = roundtrip(oplan, plan, X, kv.KVTC_BF16, label=f"c2@{cr}")
    print("c2", cr, "r", oplan.r, st)


def _manual(p, groups, seed):
    rng = np.random.default_rng(seed)
    V = np.linalg.qr(rng.standard_normal((p, p)))[0]
    mu = rng.standard_normal(p) * 0.1
    blocks, s = [], 0
    for n, b in groups:
        blocks.append(ko.Block(s, n, b))
        s += n
    return ko.compile_plan(mu, V, blocks)


@pytest.mark.parametrize("name,p,groups", [
    ("all-widths", 128, [(16, 16), (16, 12), (16, 9), (16, 7), (16, 5), (16, 3), (16, 2), (16, 1)]),
    ("full-rank-1024", 1024, [(16, 8), (16, 6), (64, 5), (64, 4), (96, 3), (256, 2), (512, 1)]),
    ("one-wide-group", 1024, [(1024, 2)]),
    ("mid-rank-640", 1024, [(64, 7), (256, 3), (320, 2)]),
    ("gap-in-middle", 256, [(16, 6), (0, 0), (32, 3)]),
    ("tiny", 64, [(16, 4)]),
])
def test_manual_plans(name, p, groups):
    if name == "gap-in-middle":          # a zero-width block between kept groups
        rng = np.random.default_rng(5)
        V = np.linalg.qr(rng.standard_normal((p, p)))[0]
        oplan = ko.compile_plan(rng.standard_normal(p) * 0.1, V,
                                [ko.Block(0, 16, 6), ko.Block(16, 48, 0), ko.Block(64, 32, 3), ko.Block(96, 160, 0)])
        assert oplan.r == 48
    else:
        oplan = _manual(p, groups, 11)
    plan = _gpu_plan(oplan)
    rng = np.random.default_rng(21)
    scale = np.arange(1, p + 1, dtype=np.float64) ** -0.7
    X = ko.bf16_round(((rng.standard_normal((777, p)) * scale) @ np.linalg.qr(rng.standard_normal((p, p)))[0]
                       + 0.05).astype(np.float32))
    st = roundtrip(oplan, plan, X, kv.KVTC_BF16, label=name)
    st2 = roundtrip(oplan, plan, X, kv.KVTC_F32, label=name + "-f32")
    print(name, st, st2)


# One plan per padded width the kernels are built for (32-coordinate tiles: 2, 4, 6, 8, 10, 12, 16, 18, 20, 24, 32;
# decode also has 7, 9 and 17 tiles), so that every encode and decode variant runs against the oracle in each of its forms.
VARIANT_RANKS = [64, 128, 192, 224, 256, 288, 320, 384, 512, 544, 576, 640, 768, 1024]


def _variant_plan(r):
    """r kept coordinates of a 1024-feature tensor: 16-coordinate groups of mixed widths in front, then
    64-coordinate groups, widths falling with the coordinate index."""
    groups, left = [(16, 8), (16, 7), (16, 5), (16, 6)], r - 64
    widths = [4, 3, 3, 2, 2, 2, 1, 1]
    k = 0
    while left > 0:
        n = min(64, left) if left % 64 == 0 or left > 64 else left
        groups.append((n, widths[min(k, len(widths) - 1)]))
        left -= n
        k += 1
    assert sum(n for n, _ in groups) == r
    return _manual(1024, groups, 100 + r)


def _variant_data(T, seed):
    p = 1024
    rng = np.random.default_rng(seed)
    scale = np.arange(1, p + 1, dtype=np.float64) ** -0.7
    Qx = np.linalg.qr(np.random.default_rng(77).standard_normal((p, p)))[0]
    return ko.bf16_round(((rng.standard_normal((T, p)) * scale) @ Qx + 0.05).astype(np.float32))


@pytest.mark.parametrize("r", VARIANT_RANKS)
def test_every_kernel_variant_in_every_form(r):
    """Each padded width has a bulk and a short-job encode kernel and a two-tile and a one-tile decode kernel, each
    with its own LDS ring, stage and wait-count constants.  Three forms reach them all:
      (a) a single call of 50 tokens: the short-job encode variant (where the width has one) and the one-tile decode;
      (b) a single call too long for the short-job path (more 64-token tiles than workgroup slots): bulk encode
          through the single-tensor arguments, checked on sampled rows and, whole, against form (c);
      (c) a batch with jobs of 300, 70 and 5 tokens: bulk encode and the short-job launch side by side, bulk decode."""
    oplan = _variant_plan(r)
    plan = _gpu_plan(oplan)
    p, R = 1024, oplan.record_bytes
    # (a) bf16 and fp32
    Xa = _variant_data(50, r)
    roundtrip(oplan, plan, Xa, kv.KVTC_BF16, label=f"variant{r}-short")
    roundtrip(oplan, plan, Xa, kv.KVTC_F32, label=f"variant{r}-short-f32")
    # (c) batch, bf16 and fp32
    lens = [300, 70, 5]
    row0 = [0, 300, 370]
    Xc = _variant_data(375, r + 1)
    batch = kv.Batch([plan])
    jobs_dev = torch.from_numpy(kv.make_jobs([0, 0, 0], lens, row0).view(np.uint8)).to(DEV)
    offs = torch.zeros(4, dtype=torch.int64, device=DEV)
    kv.kvtc_offsets(batch.handle, jobs_dev, 3, offs)
    for dtype in (kv.KVTC_BF16, kv.KVTC_F32):
        xd = _to_dev(Xc, dtype)
        out = torch.full((375 * R + 64,), 0x5A, dtype=torch.uint8, device=DEV)
        status = torch.zeros(2, dtype=torch.int32, device=DEV)
        kv.kvtc_encode_batch(batch.handle, jobs_dev, 3, xd, dtype, p, offs, out, 375 * R, status[0:1])
        xh = torch.zeros_like(xd)
        kv.kvtc_decode_batch(batch.handle, jobs_dev, 3, out, 375 * R, offs, xh, dtype, p, status[1:2])
        torch.cuda.synchronize()
        assert status.cpu().tolist() == [0, 0]
        o = out.cpu().numpy()
        assert np.all(o[375 * R:] == 0x5A)
        rec = o[:375 * R].reshape(375, R)
        tag = f"variant{r}-batch" + ("-f32" if dtype == kv.KVTC_F32 else "")
        check_stream(oplan, Xc, rec, tag)
        check_recon(oplan, rec, _from_dev(xh), Xc, dtype == kv.KVTC_BF16, tag)
    # (b) long single call, generated on the GPU; the same rows through a batch of one job must give the same bytes
    T = 50000
    g = torch.Generator(device=DEV)
    g.manual_seed(1000 + r)
    mix = torch.from_numpy((np.arange(1, p + 1, dtype=np.float64)[:, None] ** -0.7 *
                            np.linalg.qr(np.random.default_rng(77).standard_normal((p, p)))[0]).astype(np.float32)).to(DEV)
    xl = (torch.randn((T, p), generator=g, device=DEV) @ mix + 0.05).to(torch.bfloat16)
    out1 = torch.full((T * R + 64,), 0xA5, dtype=torch.uint8, device=DEV)
    kv.kvtc_encode(plan.handle, xl, kv.KVTC_BF16, T, p, out1, T * R)
    xh1 = torch.empty_like(xl)
    kv.kvtc_decode(plan.handle, out1, T * R, T, xh1, kv.KVTC_BF16, p)
    jobs1 = torch.from_numpy(kv.make_jobs([0], [T], [0]).view(np.uint8)).to(DEV)
    offs1 = torch.zeros(2, dtype=torch.int64, device=DEV)
    kv.kvtc_offsets(batch.handle, jobs1, 1, offs1)
    out2 = torch.full_like(out1, 0xA5)
    status = torch.zeros(2, dtype=torch.int32, device=DEV)
    kv.kvtc_encode_batch(batch.handle, jobs1, 1, xl, kv.KVTC_BF16, p, offs1, out2, T * R, status[0:1])
    xh2 = torch.empty_like(xl)
    kv.kvtc_decode_batch(batch.handle, jobs1, 1, out2, T * R, offs1, xh2, kv.KVTC_BF16, p, status[1:2])
    torch.cuda.synchronize()
    assert status.cpu().tolist() == [0, 0]
    assert torch.equal(out1, out2), "single call and batch of one job wrote different streams"
    assert torch.equal(xh1.view(torch.int16), xh2.view(torch.int16)), "single call and batch of one job decoded differently"
    rows = np.unique(np.concatenate([[0, 1, 63, 64, 127, 128, 191, 192, 255, 256, T - 2, T - 1],
                                     np.random.default_rng(r).integers(0, T, size=200)]))
    idx = torch.from_numpy(rows).to(DEV)
    xv = _from_dev(xl.index_select(0, idx))
    recs = out1[:T * R].view(T, R).index_select(0, idx).cpu().numpy()
    check_stream(oplan, xv, recs, f"variant{r}-long")
    check_recon(oplan, recs, _from_dev(xh1.index_select(0, idx)), xv, True, f"variant{r}-long")


def test_degenerate_inputs(c1):
    L, oplan, plan = c1
    p = oplan.p
    X = np.zeros((300, p), dtype=np.float32)                 # constant tokens: zero range in every group
    X[100:200] = oplan.mu32[None, :]
    X[200:] = 3.0
    roundtrip(oplan, plan, ko.bf16_round(X), kv.KVTC_BF16, label="constant")
    # n_tokens == 0 is a no-op; capacity errors come back as status codes
    buf = torch.zeros(64, dtype=torch.uint8, device=DEV)
    x = torch.zeros((4, p), dtype=torch.bfloat16, device=DEV)
    kv.kvtc_encode(plan.handle, x, kv.KVTC_BF16, 0, p, buf, 0)
    with pytest.raises(kv.KvtcError) as e:
        kv.kvtc_encode(plan.handle, x, kv.KVTC_BF16, 4, p, buf, 4 * plan.record_bytes - 1)
    assert e.value.status == 3
    with pytest.raises(kv.KvtcError) as e:
        kv.kvtc_decode(plan.handle, buf, 10, 4, x, kv.KVTC_BF16, p)
    assert e.value.status == 3
    with pytest.raises(kv.KvtcError) as e:
        kv.kvtc_encode(plan.handle, x, kv.KVTC_BF16, 4, p - 8, buf, 1 << 20)
    assert e.value.status == 1
    with pytest.raises(kv.KvtcError) as e:
        kv.kvtc_encode(plan.handle, x.view(torch.uint8).flatten()[2:].data_ptr(), kv.KVTC_BF16, 1, p, buf, 1 << 20)
    assert e.value.status == 1
    with pytest.raises(kv.KvtcError) as e:          # row pitch above the documented limit
        kv.kvtc_encode(plan.handle, x, kv.KVTC_BF16, 1, (1 << 21) + 8, buf, 1 << 20)
    assert e.value.status == 1
    with pytest.raises(kv.KvtcError) as e:
        kv.kvtc_decode(plan.handle, buf, 64, 1, x, kv.KVTC_BF16, (1 << 21) + 8)
    assert e.value.status == 1
    torch.cuda.synchronize()


def test_batched_ragged_jobs_with_gpu_offsets(c1, c2):
    """Several tensors, different plans and lengths, one launch per direction; offsets from the GPU
    prefix sum equal the host cumulative sum; an over-capacity job is skipped and reported."""
    _, plans2 = c2[0]
    oplans = [plans2[16.0], plans2[40.0], plans2[8.0]]
    gplans = [_gpu_plan(o) for o in oplans]
    batch = kv.Batch(gplans)
    L = c2[0][0]
    lens = [700, 0, 1, 513, 2049, 300]
    pidx = [0, 1, 2, 1, 0, 2]
    row0 = np.concatenate([[0], np.cumsum(lens)[:-1]]) + 3          # rows start at 3: base offset honoured
    total_rows = int(sum(lens)) + 3
    Xall = ks.bf16_bits_to_f32(ks.draw_bf16(L, total_rows, 4242))
    xd = _to_dev(Xall, kv.KVTC_BF16)
    jobs = kv.make_jobs(pidx, lens, row0)
    jobs_dev = torch.from_numpy(jobs.view(np.uint8)).to(DEV)
    offs = torch.zeros(len(lens) + 1, dtype=torch.int64, device=DEV)
    kv.kvtc_offsets(batch.handle, jobs_dev, len(lens), offs)
    want = np.concatenate([[0], np.cumsum([n * oplans[i].record_bytes for n, i in zip(lens, pidx)])])
    torch.cuda.synchronize()
    np.testing.assert_array_equal(offs.cpu().numpy(), want)
    cap = int(want[-1])
    out = torch.full((cap + 64,), 0x5A, dtype=torch.uint8, device=DEV)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    kv.kvtc_encode_batch(batch.handle, jobs_dev, len(lens), xd, kv.KVTC_BF16, 1024, offs, out, cap, status)
    xh = torch.zeros_like(xd)
    status2 = torch.zeros(1, dtype=torch.int32, device=DEV)
    kv.kvtc_decode_batch(batch.handle, jobs_dev, len(lens), out, cap, offs, xh, kv.KVTC_BF16, 1024, status2)
    torch.cuda.synchronize()
    assert int(status.item()) == 0 and int(status2.item()) == 0
    o = out.cpu().numpy()
    assert np.all(o[cap:] == 0x5A)
    xh_host = _from_dev(xh)
    assert np.all(xh_host[:3] == 0)
    for j, (n, i) in enumerate(zip(lens, pidx)):
        if n == 0:
            continue
        rec = o[want[j]:want[j + 1]].reshape(n, -1)
        xv = Xall[row0[j]:row0[j] + n]
        check_stream(oplans[i], xv, rec, f"ragged-job{j}")
        check_recon(oplans[i], rec, xh_host[row0[j]:row0[j] + n], xv, True, f"ragged-job{j}")
        # the batched stream equals what the single-tensor entry point writes
        single = torch.zeros(n * oplans[i].record_bytes, dtype=torch.uint8, device=DEV)
        kv.kvtc_encode(gplans[i].handle, xd[row0[j]:], kv.KVTC_BF16, n, 1024, single, single.numel())
        torch.cuda.synchronize()
        np.testing.assert_array_equal(single.cpu().numpy().reshape(n, -1), rec)
    # capacity: cut the buffer inside job 4 -> jobs 4 and 5 are skipped, status = 1 + 4
    out2 = torch.full((cap + 64,), 0x5A, dtype=torch.uint8, device=DEV)
    status.zero_()
    small = int(want[4]) + 100
    kv.kvtc_encode_batch(batch.handle, jobs_dev, len(lens), xd, kv.KVTC_BF16, 1024, offs, out2, small, status)
    torch.cuda.synchronize()
    assert int(status.item()) == 5
    o2 = out2.cpu().numpy()
    np.testing.assert_array_equal(o2[:want[4]], o[:want[4]])
    assert np.all(o2[want[4]:] == 0x5A)
    # a bad plan index is reported the same way
    jobs_bad = kv.make_jobs([0, 9], [10, 10], [0, 10])
    jb = torch.from_numpy(jobs_bad.view(np.uint8)).to(DEV)
    offs2 = torch.zeros(3, dtype=torch.int64, device=DEV)
    kv.kvtc_offsets(batch.handle, jb, 2, offs2)
    status.zero_()
    kv.kvtc_encode_batch(batch.handle, jb, 2, xd, kv.KVTC_BF16, 1024, offs2, out2, cap, status)
    torch.cuda.synchronize()
    assert offs2.cpu().numpy().tolist() == [0, 10 * oplans[0].record_bytes, 10 * oplans[0].record_bytes]
    assert int(status.item()) == 2


def test_batch_with_stream_starts_off_the_16_byte_grid():
    """A job of a plan with 8-byte records in front shifts the next job's stream start to 8 mod 16 although
    that job's records are whole 16-byte pieces: encode must fall back to dword stores for it and decode to
    the skewed record image; both must still give the single-tensor results."""
    p = 128
    small = _manual(p, [(16, 1)], 3)                        # 32 header bits + 16 code bits -> 8-byte records
    wide = _manual(p, [(16, 8), (32, 4), (64, 2)], 4)       # 96 + 128 + 128 + 128 bits -> 60 bytes ...
    wide16 = _manual(p, [(16, 8), (16, 8), (32, 4), (64, 2)], 5)   # 128 + 128 + 128 + 128 + 128 bits -> 80 bytes = 5 pieces
    assert small.record_bytes == 8 and wide.record_bytes == 60 and wide16.record_bytes == 80
    oplans = [small, wide16, wide]
    gplans = [_gpu_plan(o) for o in oplans]
    batch = kv.Batch(gplans)
    lens = [1, 700, 2, 650, 5]
    pidx = [0, 1, 0, 2, 1]
    row0 = np.concatenate([[0], np.cumsum(lens)[:-1]])
    rng = np.random.default_rng(8)
    scale = np.arange(1, p + 1, dtype=np.float64) ** -0.7
    Xall = ko.bf16_round(((rng.standard_normal((int(sum(lens)), p)) * scale) @ np.linalg.qr(rng.standard_normal((p, p)))[0]).astype(np.float32))
    xd = _to_dev(Xall, kv.KVTC_BF16)
    jobs_dev = torch.from_numpy(kv.make_jobs(pidx, lens, row0).view(np.uint8)).to(DEV)
    offs = torch.zeros(len(lens) + 1, dtype=torch.int64, device=DEV)
    kv.kvtc_offsets(batch.handle, jobs_dev, len(lens), offs)
    torch.cuda.synchronize()
    want = np.concatenate([[0], np.cumsum([n * oplans[i].record_bytes for n, i in zip(lens, pidx)])])
    np.testing.assert_array_equal(offs.cpu().numpy(), want)
    assert want[1] % 16 == 8 and want[3] % 16 != 0            # job 1 (whole pieces) and job 3 start off the grid
    cap = int(want[-1])
    out = torch.full((cap + 64,), 0x5A, dtype=torch.uint8, device=DEV)
    status = torch.zeros(2, dtype=torch.int32, device=DEV)
    kv.kvtc_encode_batch(batch.handle, jobs_dev, len(lens), xd, kv.KVTC_BF16, p, offs, out, cap, status[0:1])
    xh = torch.zeros_like(xd)
    kv.kvtc_decode_batch(batch.handle, jobs_dev, len(lens), out, cap, offs, xh, kv.KVTC_BF16, p, status[1:2])
    torch.cuda.synchronize()
    assert status.cpu().tolist() == [0, 0]
    o = out.cpu().numpy()
    assert np.all(o[cap:] == 0x5A)
    xh_host = _from_dev(xh)
    for j, (n, i) in enumerate(zip(lens, pidx)):
        rec = o[want[j]:want[j + 1]].reshape(n, -1)
        xv = Xall[row0[j]:row0[j] + n]
        check_stream(oplans[i], xv, rec, f"offgrid-job{j}")
        check_recon(oplans[i], rec, xh_host[row0[j]:row0[j] + n], xv, True, f"offgrid-job{j}")
        single = torch.zeros(n * oplans[i].record_bytes, dtype=torch.uint8, device=DEV)
        kv.kvtc_encode(gplans[i].handle, xd[row0[j]:], kv.KVTC_BF16, n, p, single, single.numel())
        torch.cuda.synchronize()
        np.testing.assert_array_equal(single.cpu().numpy().reshape(n, -1), rec)


def test_batch_mixes_short_and_long_jobs_and_plans_without_a_short_variant():
    """Jobs of at most 64 tokens run on narrow tiles when their plan has such a variant (a separate small
    launch), others do not; every job must come out as from the single-tensor call."""
    p = 1024
    full = _manual(p, [(16, 8), (16, 6), (64, 5), (64, 4), (96, 3), (256, 2), (512, 1)], 11)   # full rank: bulk tiles only
    mid = _manual(p, [(64, 7), (128, 3)], 12)                                                  # 192 coordinates
    oplans = [full, mid]
    gplans = [_gpu_plan(o) for o in oplans]
    batch = kv.Batch(gplans)
    lens = [5, 5, 300, 64, 65, 33, 1]
    pidx = [0, 1, 1, 1, 1, 0, 1]
    row0 = np.concatenate([[0], np.cumsum(lens)[:-1]])
    rng = np.random.default_rng(9)
    scale = np.arange(1, p + 1, dtype=np.float64) ** -0.7
    Xall = ko.bf16_round(((rng.standard_normal((int(sum(lens)), p)) * scale) @ np.linalg.qr(rng.standard_normal((p, p)))[0]).astype(np.float32))
    xd = _to_dev(Xall, kv.KVTC_BF16)
    jobs_dev = torch.from_numpy(kv.make_jobs(pidx, lens, row0).view(np.uint8)).to(DEV)
    offs = torch.zeros(len(lens) + 1, dtype=torch.int64, device=DEV)
    kv.kvtc_offsets(batch.handle, jobs_dev, len(lens), offs)
    torch.cuda.synchronize()
    want = offs.cpu().numpy()
    cap = int(want[-1])
    out = torch.full((cap + 64,), 0x5A, dtype=torch.uint8, device=DEV)
    status = torch.zeros(2, dtype=torch.int32, device=DEV)
    kv.kvtc_encode_batch(batch.handle, jobs_dev, len(lens), xd, kv.KVTC_BF16, p, offs, out, cap, status[0:1])
    xh = torch.zeros_like(xd)
    kv.kvtc_decode_batch(batch.handle, jobs_dev, len(lens), out, cap, offs, xh, kv.KVTC_BF16, p, status[1:2])
    torch.cuda.synchronize()
    assert status.cpu().tolist() == [0, 0]
    o = out.cpu().numpy()
    assert np.all(o[cap:] == 0x5A)
    xh_host = _from_dev(xh)
    for j, (n, i) in enumerate(zip(lens, pidx)):
        rec = o[want[j]:want[j + 1]].reshape(n, -1)
        xv = Xall[row0[j]:row0[j] + n]
        check_stream(oplans[i], xv, rec, f"mix-job{j}")
        check_recon(oplans[i], rec, xh_host[row0[j]:row0[j] + n], xv, True, f"mix-job{j}")
        single = torch.zeros(n * oplans[i].record_bytes, dtype=torch.uint8, device=DEV)
        kv.kvtc_encode(gplans[i].handle, xd[row0[j]:], kv.KVTC_BF16, n, p, single, single.numel())
        back = torch.zeros((n, p), dtype=torch.bfloat16, device=DEV)
        kv.kvtc_decode(gplans[i].handle, single, single.numel(), n, back, kv.KVTC_BF16, p)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(single.cpu().numpy().reshape(n, -1), rec)
        np.testing.assert_array_equal(_from_dev(back), xh_host[row0[j]:row0[j] + n])
