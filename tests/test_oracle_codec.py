"""Pins for the oracle's quantiser, record format, bit allocation and decode (CPU only)."""
import itertools
import os

import numpy as np
import pytest

import kvtc_oracle as ko
import kvtc_synth as ks

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "worked_record.txt")


def _golden():
    out = {}
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, *v = line.split()
            out[k] = v
    return out


def _manual_plan(p, groups, V=None, mu=None):
    """Plan with the given kept groups [(n, bits), ...] over the first sum(n) coordinates."""
    blocks, s = [], 0
    for n, b in groups:
        blocks.append(ko.Block(s, n, b))
        s += n
    if V is None:
        V = np.eye(p)
    if mu is None:
        mu = np.zeros(p)
    return ko.compile_plan(mu, V, blocks)


# ---- quantiser -------------------------------------------------------------

def test_worked_example_quantiser_and_record_bytes():
    g = _golden()
    d = np.array([[float(v) for v in g["d"]]], dtype=np.float32)
    bits = int(g["bits"][0])
    shift, scale, codes = ko.quantise_group(d, bits)
    assert shift.view(np.uint16)[0] == int(g["shift_fp16"][0], 16)
    assert scale.view(np.uint16)[0] == int(g["scale_fp16"][0], 16)
    assert codes[0].tolist() == [int(v) for v in g["codes"]]
    np.testing.assert_array_equal(ko.dequantise_group(shift, scale, codes)[0], [float(v) for v in g["d_hat"]])
    plan = _manual_plan(4, [(4, bits)])
    rec = ko.pack(plan, shift[:, None], scale[:, None], codes)
    assert plan.record_bytes == 8
    assert rec[0].tolist() == [int(v, 16) for v in g["record"]]
    # through the whole encoder as well (identity basis, zero mean)
    assert ko.encode(plan, d)[0].tolist() == [int(v, 16) for v in g["record"]]


def test_worked_example_two_groups_odd_widths():
    g = _golden()
    widths = [int(v) for v in g["record2_widths"]]
    sizes = [int(v) for v in g["record2_sizes"]]
    plan = _manual_plan(8, list(zip(sizes, widths)))
    hdr = [int(v, 16) for v in g["record2_headers"]]
    shift = np.array([[hdr[0], hdr[2]]], dtype=np.uint16).view(np.float16)
    scale = np.array([[hdr[1], hdr[3]]], dtype=np.uint16).view(np.float16)
    codes = np.array([[int(v) for v in g["record2_codes"]]], dtype=np.uint32)
    rec = ko.pack(plan, shift, scale, codes)
    assert rec[0].tolist() == [int(v, 16) for v in g["record2"]]
    sh2, sc2, co2 = ko.unpack(plan, rec)
    np.testing.assert_array_equal(sh2.view(np.uint16), shift.view(np.uint16))
    np.testing.assert_array_equal(sc2.view(np.uint16), scale.view(np.uint16))
    np.testing.assert_array_equal(co2, codes)


@pytest.mark.parametrize("bits", [1, 2, 3, 5, 8, 12, 16])
def test_quantiser_error_bound_and_nearest_code(bits):
    """Because shift rounds down and scale rounds up, the group range is covered and
    every entry is reconstructed to within scale/2; the chosen code is the nearest of
    all 2^b levels (checked by brute force over the levels)."""
    rng = np.random.default_rng(bits)
    d = (rng.standard_normal((300, 16)) * rng.uniform(0.01, 30, (300, 1))).astype(np.float32)
    shift, scale, codes = ko.quantise_group(d, bits)
    s64, c64 = shift.astype(np.float64), scale.astype(np.float64)
    assert np.all(s64 <= d.min(1)) and np.all(s64 + c64 * (2 ** bits - 1) >= d.max(1) * (1 - 1e-7) - 1e-12)
    assert codes.max() <= 2 ** bits - 1
    d_hat = ko.dequantise_group(shift, scale, codes)
    slack = 4 * np.finfo(np.float32).eps * np.abs(d).max(1, keepdims=True) * max(1, 2 ** bits / 64)
    assert np.all(np.abs(d_hat - d) <= c64[:, None] / 2 + slack)
    if bits <= 8:
        levels = s64[:, None, None] + np.arange(2 ** bits)[None, None, :] * c64[:, None, None]
        best = np.abs(levels - d[:, :, None].astype(np.float64)).min(axis=2)
        assert np.all(np.abs(d_hat - d) <= best + slack)


def test_quantiser_degenerate_groups():
    d = np.full((3, 16), 0.37109375, dtype=np.float32)      # exactly representable in fp16
    shift, scale, codes = ko.quantise_group(d, 4)
    assert np.all(scale == 0) and np.all(codes == 0) and np.all(shift.astype(np.float32) == d[:, 0])
    d = np.full((2, 16), 0.1, dtype=np.float32)             # not representable: tiny positive range
    shift, scale, codes = ko.quantise_group(d, 4)
    assert np.all(scale > 0) and np.all(codes <= 15)
    assert np.abs(ko.dequantise_group(shift, scale, codes) - 0.1).max() <= scale.astype(np.float64).max() / 2 + 1e-9
    big = np.array([[-1e6, 1e6] + [0.0] * 14], dtype=np.float32)      # saturating header
    shift, scale, codes = ko.quantise_group(big, 8)
    assert np.isfinite(shift.astype(np.float32)).all() and np.isfinite(scale.astype(np.float32)).all()
    assert codes.max() <= 255
    with np.errstate(all="ignore"):
        ko.quantise_group(np.array([[np.nan] + [1.0] * 15], dtype=np.float32), 3)   # must not raise


def test_frobenius_identity_in_decorrelated_domain():
    """||D V^T - D^q V^T||_F = ||D - D^q||_F for an orthonormal V (paper, Section
    "Quantization", second display)."""
    L = ks.make_layer(ks.LayerSpec(p=64, alpha=1.0, seed=31))
    C = ks.draw(L, 2000, 1)
    mu, V, _ = ko.pca(C)
    D = ((C - mu) @ V).astype(np.float32)
    sh, sc, co = ko.quantise_group(D[:, :32], 4)
    Dq = np.zeros_like(D, dtype=np.float64)
    Dq[:, :32] = ko.dequantise_group(sh, sc, co)
    lhs = np.linalg.norm(D.astype(np.float64) @ V.T - Dq @ V.T)
    rhs = np.linalg.norm(D.astype(np.float64) - Dq)
    assert lhs == pytest.approx(rhs, rel=1e-10)


def test_orthonormal_basis_reconstructs_at_16_bits():
    """Full rank, every width 16, un-rounded orthonormal basis: the only error is the
    quantiser's, ||x_hat - x||_inf <= ||d_hat - d||_2 <= sqrt(p) * max_g scale_g / 2."""
    p = 128
    L = ks.make_layer(ks.LayerSpec(p=p, alpha=1.2, seed=41))
    C = ks.draw(L, 1024, 1)
    X = ks.draw(L, 512, 2)
    mu, V, _ = ko.pca(C)
    mu32 = mu.astype(np.float32).astype(np.float64)
    D = ((X - mu32) @ V).astype(np.float32)
    d_hat = np.zeros((512, p))
    smax = np.zeros(512)
    for s in range(0, p, 16):
        sh, sc, co = ko.quantise_group(D[:, s:s + 16], 16)
        d_hat[:, s:s + 16] = ko.dequantise_group(sh, sc, co)
        smax = np.maximum(smax, sc.astype(np.float64))
    x_hat = d_hat @ V.T + mu32
    bound = np.sqrt(p) * smax / 2 + 1e-5
    assert np.all(np.abs(x_hat - X).max(axis=1) <= bound)
    assert np.abs(x_hat - X).max() <= 3e-4 * (X.max() - X.min())
    # the same through plan/encode/decode: the stored basis is bf16, which is orthonormal
    # only to ~1e-3, so the bar is looser there
    plan = ko.compile_plan(mu, V, [ko.Block(s, 16, 16) for s in range(0, p, 16)])
    Xb = ko.bf16_round(X.astype(np.float32))
    xh = ko.decode(plan, ko.encode(plan, Xb))
    assert np.abs(xh - Xb).max() <= 1e-2 * (Xb.max() - Xb.min())


# ---- record format ----------------------------------------------------------

def _bigint_pack(plan, sh_bits, sc_bits, codes):
    """Independent packer: one Python integer per record."""
    out = []
    for t in range(codes.shape[0]):
        v = 0
        for g in range(plan.n_groups):
            v |= int(sh_bits[t, g]) << (32 * g)
            v |= int(sc_bits[t, g]) << (32 * g + 16)
        pos = 32 * plan.n_groups
        j = 0
        for g in range(plan.n_groups):
            for _ in range(int(plan.group_n[g])):
                v |= int(codes[t, j]) << pos
                pos += int(plan.group_bits[g])
                j += 1
        out.append(list(v.to_bytes(plan.record_bytes, "little")))
    return np.array(out, dtype=np.uint8)


def test_pack_unpack_roundtrip_all_widths_and_bigint_packer():
    rng = np.random.default_rng(7)
    groups = [(int(rng.choice([1, 3, 16, 5])), int(b)) for b in rng.permutation(np.arange(1, 17))]
    r = sum(n for n, _ in groups)
    plan = _manual_plan(r + 3, groups)
    T = 37
    codes = np.stack([rng.integers(0, 2 ** int(b), T) for b in plan.coef_bits], axis=1).astype(np.uint32)
    sh = rng.integers(0, 65536, (T, plan.n_groups)).astype(np.uint16)
    sc = rng.integers(0, 65536, (T, plan.n_groups)).astype(np.uint16)
    rec = ko.pack(plan, sh.view(np.float16), sc.view(np.float16), codes)
    total_bits = 32 * plan.n_groups + sum(n * b for n, b in groups)
    assert rec.shape == (T, plan.record_bytes) and plan.record_bytes == 4 * ((total_bits + 31) // 32)
    np.testing.assert_array_equal(rec, _bigint_pack(plan, sh, sc, codes))
    sh2, sc2, co2 = ko.unpack(plan, rec)
    np.testing.assert_array_equal(sh2.view(np.uint16), sh)
    np.testing.assert_array_equal(sc2.view(np.uint16), sc)
    np.testing.assert_array_equal(co2, codes)
    # padding bits are zero
    allbits = np.unpackbits(rec, axis=1, bitorder="little")
    assert allbits[:, total_bits:].sum() == 0
    # entropy stage is lossless
    np.testing.assert_array_equal(ko.inflate(ko.deflate(rec), plan), rec)


def test_max_width_codes_use_every_bit():
    plan = _manual_plan(16, [(16, 16)])
    codes = np.full((2, 16), 0xFFFF, dtype=np.uint32)
    z = np.zeros((2, 1), dtype=np.float16)
    rec = ko.pack(plan, z, z, codes)
    assert plan.record_bytes == 4 + 32 and np.all(rec[:, 4:] == 0xFF) and np.all(rec[:, :4] == 0)


# ---- bit allocation ----------------------------------------------------------

def _brute_force(errors, p, budget, sizes, widths, header):
    best = [np.inf]

    def rec(i, used, err):
        if i == p:
            best[0] = min(best[0], err)
            return
        for s in sizes:
            if i + s > p:
                continue
            for w in [0] + list(widths):
                cost = 0 if w == 0 else s * w + header
                if used + cost <= budget:
                    rec(i + s, used + cost, err + errors.change(i, s, w))
    rec(0, 0, float(errors.energy[:p].sum()))
    return best[0]


@pytest.mark.parametrize("seed,p,budget", [(1, 6, 20), (2, 8, 33), (3, 8, 12), (4, 7, 48), (5, 8, 0), (6, 8, 64)])
def test_dp_matches_brute_force_on_tiny_problems(seed, p, budget):
    """The recurrence is optimal under its constraints (paper, appendix on the dynamic
    programme, proof sketch): every partition into allowed blocks and every width
    assignment within the budget is enumerated here."""
    rng = np.random.default_rng(seed)
    P = (rng.standard_normal((64, p)) * (np.arange(1, p + 1) ** -1.0)[None, :] * 3).astype(np.float32)
    errors = ko.BlockErrors(P)
    sizes, widths, header = (1, 2, 4), (1, 2, 3), 5
    blocks, best = ko.dp_allocate(errors, p, budget, sizes, widths, header_bits=header, unit=1)
    want = _brute_force(errors, p, budget, sizes, widths, header)
    assert best == pytest.approx(want, rel=1e-12, abs=1e-12)
    assert ko.allocation_error(errors, p, blocks) == pytest.approx(best, rel=1e-12, abs=1e-12)
    assert ko.allocation_bits(blocks, header) <= budget
    assert sum(b.n for b in blocks) == p and blocks[0].start == 0
    assert all(blocks[k].start + blocks[k].n == blocks[k + 1].start for k in range(len(blocks) - 1))


def test_dp_restricted_grid_matches_brute_force():
    """Same check on the 16-aligned grid the plans use (unit = 16)."""
    rng = np.random.default_rng(12)
    p = 96
    P = (rng.standard_normal((128, p)) * (np.arange(1, p + 1) ** -1.1)[None, :] * 4).astype(np.float32)
    errors = ko.BlockErrors(P)
    for budget in (0, 48, 160, 400, 1000):
        blocks, best = ko.dp_allocate(errors, p, budget, (16, 64), (1, 2, 4, 8), header_bits=32, unit=16)
        want = _brute_force(errors, p, budget, (16, 64), (1, 2, 4, 8), 32)
        assert best == pytest.approx(want, rel=1e-12)
        assert ko.allocation_bits(blocks) <= budget


def test_dp_properties_and_budget_on_power_law_spectrum():
    wl = ks.WORKLOADS["c1"]
    L = ks.make_layer(ks.layer_spec("c1", 0, 0))
    C = ko.bf16_round(ks.draw_f32(L, wl.n_calib, ks.CALIB_DRAW))
    mu, V, S = ko.pca(C)
    errors = ko.dp_errors(C, mu, V)
    prev = np.inf
    for cr in (16.0, 8.0, 4.0, 2.0):
        plan, info = ko.calibrate_from_pca(C, mu, V, S, cr, errors=errors)
        B = info["budget_bits"]
        assert B == 32 * int(16 * 128 // (32 * cr))
        used = 32 * plan.n_groups + int((plan.group_n * plan.group_bits).sum())
        assert used == ko.allocation_bits(info["blocks"]) <= B
        assert plan.record_bytes * 8 == 32 * ((used + 31) // 32) <= B
        assert 2 * 128 / plan.record_bytes >= cr           # achieved ratio >= target
        assert info["dp_error"] <= prev                     # more budget never hurts
        prev = info["dp_error"]
        assert ko.allocation_error(errors, 128, info["blocks"]) == pytest.approx(info["dp_error"], rel=1e-12)
        # high-variance coordinates get at least as many bits as trailing ones, and trailing
        # coordinates are dropped (paper, end of Section "Quantization")
        w = np.zeros(128, dtype=int)
        w[plan.kept] = plan.coef_bits
        assert w[:16].mean() >= w[-16:].mean()
        if cr >= 4:
            assert w[-16:].sum() == 0 and plan.r < 128
        assert np.all(plan.group_n % 16 == 0) and np.all(plan.kept % 16 == np.arange(plan.r) % 16)


def test_budget_formula_for_the_named_ratios():
    assert ko.bit_budget(1024, 8) == 2048 and ko.bit_budget(1024, 16) == 1024
    assert ko.bit_budget(1024, 20) == 800 and ko.bit_budget(1024, 40) == 384
    assert ko.bit_budget(128, 4) == 512


# ---- whole coder ---------------------------------------------------------------

def test_encode_decode_config1_end_to_end():
    wl = ks.WORKLOADS["c1"]
    L = ks.make_layer(ks.layer_spec("c1", 0, 0))
    C = ko.bf16_round(ks.draw_f32(L, wl.n_calib, ks.CALIB_DRAW))
    X = ko.bf16_round(ks.draw_f32(L, wl.n_tokens, ks.TEST_DRAW))
    plan, info = ko.calibrate(C, 4.0)
    rec = ko.encode(plan, X)
    assert rec.shape == (wl.n_tokens, plan.record_bytes) and plan.record_bytes <= 64
    x_hat = ko.decode(plan, rec)
    rng_x = X.max() - X.min()
    assert np.abs(x_hat - X).max() <= 2e-2 * rng_x
    # decode error in feature space equals quantisation + truncation error in coefficient
    # space up to the non-orthonormality of the bf16 basis
    rel = np.linalg.norm(x_hat - X) / np.linalg.norm(X - plan.mu32)
    assert rel < 0.05
    # the bf16-operand variant differs from the definition by operand rounding only
    x_m = ko.decode(plan, rec, operand_bf16=True)
    assert np.abs(x_m - x_hat).max() <= 2 ** -8 * np.abs(X - plan.mu32).max() * 2
    cr_raw, cr_z = ko.compression_ratios(plan, wl.n_tokens, rec)
    assert cr_raw >= 4.0 and cr_z > 0
    # centring matters: dropping mu from the projection must change the codes
    d_wrong = (X.astype(np.float64) @ plan.v64).astype(np.float32)
    assert not np.array_equal(ko.quantise(plan, d_wrong)[2], ko.quantise(plan, ko.project(plan, X))[2])


def test_decode_is_a_plain_matrix_product():
    rng = np.random.default_rng(3)
    p = 32
    V = np.linalg.qr(rng.standard_normal((p, p)))[0]
    mu = rng.standard_normal(p)
    plan = ko.compile_plan(mu, V, [ko.Block(0, 16, 8), ko.Block(16, 16, 0)])
    assert plan.r == 16 and plan.kept.tolist() == list(range(16))
    x = ko.bf16_round(rng.standard_normal((10, p)).astype(np.float32))
    rec = ko.encode(plan, x)
    sh, sc, co = ko.unpack(plan, rec)
    d_hat = sh.astype(np.float64) + co * sc.astype(np.float64)
    want = np.einsum("tj,fj->tf", d_hat, ko.bf16_round(V[:, :16]).astype(np.float64)) + mu.astype(np.float32)
    np.testing.assert_allclose(ko.decode(plan, rec), want, rtol=0, atol=1e-12)
    # zero-bit block in the middle is dropped, kept indices need not be a prefix
    plan2 = ko.compile_plan(mu, V, [ko.Block(0, 16, 0), ko.Block(16, 16, 3)])
    assert plan2.kept.tolist() == list(range(16, 32)) and plan2.record_bytes == 12   # 32 + 16*3 = 80 bits -> 3 dwords


def test_committed_bundle_is_what_the_calibration_script_writes():
    """The calibration bundles the benchmark loads are stored values; they must be exactly what the
    oracle's calibration (PCA + DP allocation on the seeded config-2 calibration draw) produces -- every
    ratio of the K tensor -- and the hand-set full-rank bundle must keep every coordinate of the same basis."""
    import os
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    plans_dir = os.path.join(root, "paper_2511_01815_amd", "plans")
    wl = ks.WORKLOADS["c2"]
    L = ks.make_layer(ks.layer_spec("c2", 0, 0))
    C = ks.bf16_bits_to_f32(ks.draw_bf16(L, wl.n_calib, ks.CALIB_DRAW))
    mu, V, S = ko.pca(C)
    plan, info = ko.calibrate_from_pca(C, mu, V, S, 16.0, errors=ko.dp_errors(C, mu, V))
    z = np.load(os.path.join(plans_dir, "c2_K_cr16.npz"))
    np.testing.assert_array_equal(z["v_bits"], plan.v_bits)
    np.testing.assert_array_equal(z["mu32"], plan.mu32)
    assert z["group_n"].tolist() == plan.group_n.tolist() and z["group_bits"].tolist() == plan.group_bits.tolist()
    assert plan.record_bytes * 8 <= info["budget_bits"] == 1024
    errors = info["errors"]
    for cr in (8, 20, 40):
        pl, inf = ko.calibrate_from_pca(C, mu, V, S, float(cr), errors=errors)
        zz = np.load(os.path.join(plans_dir, f"c2_K_cr{cr}.npz"))
        np.testing.assert_array_equal(zz["v_bits"], pl.v_bits)
        np.testing.assert_array_equal(zz["mu32"], pl.mu32)
        assert zz["group_n"].tolist() == pl.group_n.tolist() and zz["group_bits"].tolist() == pl.group_bits.tolist()
        assert pl.record_bytes * 8 <= inf["budget_bits"]
    full = np.load(os.path.join(plans_dir, "c2_K_full.npz"))
    assert full["v_bits"].shape == (1024, 1024) and int(full["group_n"].sum()) == 1024
    np.testing.assert_array_equal(full["v_bits"][:, :16], plan.v_bits[:, :16])      # same leading PCA directions
    np.testing.assert_array_equal(full["mu32"], plan.mu32)


def _c3_file(layer, kv):
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    return np.load(os.path.join(root, "paper_2511_01815_amd", "plans", f"c3_L{layer:02d}_{kv}.npz"))


@pytest.mark.parametrize("layer,kvi", [(3, 0), (20, 1)])
def test_committed_cache_bundles_are_what_the_calibration_script_writes(layer, kvi):
    """Two of the 64 per-tensor files of the 32-layer cache, recomputed from scratch (PCA + allocation at 8x, 16x
    and 20x on the tensor's seeded calibration draw): every stored array must come out again."""
    wl = ks.WORKLOADS["c3"]
    L = ks.make_layer(ks.layer_spec("c3", layer, kvi))
    C = ks.bf16_bits_to_f32(ks.draw_bf16(L, wl.n_calib, ks.CALIB_DRAW))
    mu, V, S = ko.pca(C)
    errors = ko.dp_errors(C, mu, V)
    z = _c3_file(layer, wl.kv[kvi])
    for cr in (8, 16, 20):
        plan, info = ko.calibrate_from_pca(C, mu, V, S, float(cr), errors=errors)
        np.testing.assert_array_equal(z[f"cr{cr}_kept"], plan.kept)
        np.testing.assert_array_equal(z["v_bits"][:, plan.kept], plan.v_bits)
        np.testing.assert_array_equal(z["mu32"], plan.mu32)
        assert z[f"cr{cr}_group_n"].tolist() == plan.group_n.tolist()
        assert z[f"cr{cr}_group_bits"].tolist() == plan.group_bits.tolist()
        assert plan.record_bytes * 8 <= info["budget_bits"]


def test_every_committed_cache_bundle_is_the_pca_of_its_calibration_draw_within_budget():
    """All 64 files, without re-running the SVD or the allocation: the stored mean is the mean of the tensor's
    seeded calibration draw; the stored columns are unit eigenvectors of that draw's covariance with
    descending eigenvalues (residual of Cov v = lambda v at bf16 storage precision); each ratio's kept
    groups fill at most the bit budget and more than the budget minus one smallest group; the 16x and 20x
    kept sets nest inside the 8x one."""
    wl = ks.WORKLOADS["c3"]
    for layer in range(wl.n_layers):
        for kvi, kv_name in enumerate(wl.kv):
            z = _c3_file(layer, kv_name)
            spec = ks.layer_spec("c3", layer, kvi)
            assert int(z["seed"]) == spec.seed and float(z["alpha"]) == spec.alpha
            L = ks.make_layer(spec)
            C = ks.bf16_bits_to_f32(ks.draw_bf16(L, wl.n_calib, ks.CALIB_DRAW)).astype(np.float64)
            mu = C.mean(axis=0)
            np.testing.assert_array_equal(z["mu32"], mu.astype(np.float32))
            Vk = ko.bf16_to_f32(z["v_bits"]).astype(np.float64)
            A = C - mu[None, :]
            Y = A @ Vk
            lam = (Y * Y).sum(axis=0) / (np.linalg.norm(Vk, axis=0) ** 2)       # Rayleigh quotients (times n)
            resid = A.T @ Y - Vk * lam[None, :]
            assert np.all(np.abs(np.linalg.norm(Vk, axis=0) - 1.0) < 4e-3), (layer, kv_name)
            assert np.all(np.linalg.norm(resid, axis=0) <= 1.5e-2 * lam[0]), (layer, kv_name, float((np.linalg.norm(resid, axis=0) / lam[0]).max()))
            # descending: checked on the leading 32 (bf16 storage leaks ~2^-9 of a vector's norm onto the leading
            # directions, whose eigenvalues are 10^7 times the trailing ones, so small Rayleigh quotients are noisy)
            assert np.all(np.diff(lam[:32]) <= 1e-2 * lam[:31]) and lam[32:].max() <= lam[31], (layer, kv_name)
            kept8 = set(z["cr8_kept"].tolist())
            for cr in (8, 16, 20):
                n, b, kept = z[f"cr{cr}_group_n"], z[f"cr{cr}_group_bits"], z[f"cr{cr}_kept"]
                assert int(n.sum()) == kept.size and np.all(n % 16 == 0) and np.all((b >= 1) & (b <= 8))
                used = 32 * n.size + int((n * b).sum())
                B = ko.bit_budget(wl.p, cr)
                assert B - (32 + 16) < used <= B, (layer, kv_name, cr, used, B)
                assert set(kept.tolist()) <= kept8 or cr == 8
                assert kept.max() < z["v_bits"].shape[1]


def test_reciprocal_form_of_the_code_decision_against_the_divide_form():
    """The quantiser decides a code as rint((d - shift) * (1/scale)) with a correctly rounded fp32 reciprocal (a
    fixed choice of this build; the plain statement of min-max quantisation divides).  The two forms can differ
    only where the quotient lies within a few fp32 ulps of a rounding boundary: never by more than one code, and
    on a tiny fraction of entries, which this test measures in exact (fp64) arithmetic for both forms over all
    widths and a spread of magnitudes."""
    rng = np.random.default_rng(20)
    worst_rate = 0.0
    for bits in range(1, 9):
        for mag in (1e-3, 1.0, 300.0):
            d = (rng.standard_normal((4000, 64)) * mag).astype(np.float32)
            shift, scale, codes = ko.quantise_group(d, bits)
            sh, sc = shift.astype(np.float64)[:, None], scale.astype(np.float64)[:, None]
            qmax = float((1 << bits) - 1)
            with np.errstate(divide="ignore", invalid="ignore"):
                exact = np.where(sc > 0, (d.astype(np.float64) - sh) / sc, 0.0)      # the divide form, no intermediate rounding
            divide_codes = np.clip(np.rint(exact), 0.0, qmax).astype(np.int64)
            diff = np.abs(codes.astype(np.int64) - divide_codes)
            assert diff.max() <= 1, (bits, mag)
            # a differing entry sits on a rounding boundary of the exact quotient to within fp32 resolution of its size
            rows, cols = np.nonzero(diff)
            if rows.size:
                frac = np.abs(exact[rows, cols] - np.floor(exact[rows, cols]) - 0.5)
                assert np.all(frac <= 4.0 * 2.0 ** -24 * np.maximum(exact[rows, cols], 1.0)), (bits, mag, frac.max())
            worst_rate = max(worst_rate, float((diff != 0).mean()))
    print(f"reciprocal vs divide form: at most {worst_rate:.2e} of entries differ, each by one code")
    assert worst_rate <= 2e-5


def test_committed_single_layer_bundle_is_what_the_calibration_script_writes():
    """The bundle of the ragged-batch configuration's layer 9 (K, 40x) that the benchmark loads equals the oracle's
    calibration on that layer's seeded calibration draw."""
    import os
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    wl = ks.WORKLOADS["c5"]
    L = ks.make_layer(ks.layer_spec("c5", 9, 0))
    C = ks.bf16_bits_to_f32(ks.draw_bf16(L, wl.n_calib, ks.CALIB_DRAW))
    mu, V, S = ko.pca(C)
    plan, info = ko.calibrate_from_pca(C, mu, V, S, 40.0, errors=ko.dp_errors(C, mu, V))
    z = np.load(os.path.join(root, "paper_2511_01815_amd", "plans", "c5_L09_K_cr40.npz"))
    np.testing.assert_array_equal(z["v_bits"], plan.v_bits)
    np.testing.assert_array_equal(z["mu32"], plan.mu32)
    assert z["group_n"].tolist() == plan.group_n.tolist() and z["group_bits"].tolist() == plan.group_bits.tolist()
    assert plan.record_bytes * 8 <= info["budget_bits"] == 384
