"""Pins for the oracle's number formats and PCA (CPU only)."""
import numpy as np
import pytest
import torch

import kvtc_oracle as ko
import kvtc_synth as ks


# ---- 16-bit formats ------------------------------------------------------

def _fp16_table():
    allv = np.arange(65536, dtype=np.uint32).astype(np.uint16).view(np.float16)
    fin = allv[np.isfinite(allv)].astype(np.float64)
    return np.unique(fin)          # sorted, +-0 merged


def _probe_values():
    rng = np.random.default_rng(5)
    tab = _fp16_table()
    xs = [rng.standard_normal(20000) * s for s in (1e-9, 1e-7, 1e-5, 1e-3, 1.0, 300.0, 7e4)]
    xs.append(tab)                                         # exact grid points
    xs.append(np.nextafter(tab.astype(np.float32), np.float32(np.inf)).astype(np.float64))
    xs.append(np.nextafter(tab.astype(np.float32), np.float32(-np.inf)).astype(np.float64))
    xs.append(np.array([0.0, -0.0, 65504.0, -65504.0, 65520.0, 1e30, -1e30, 6e-8, -6e-8, 2.9e-8]))
    return np.concatenate(xs).astype(np.float32)


def test_fp16_floor_ceil_against_exhaustive_table():
    """Directed roundings checked against a search in the sorted table of all 63 488
    finite fp16 values (a method that shares nothing with cast-and-nextafter)."""
    tab = _fp16_table()
    x = _probe_values()
    xc = np.clip(x.astype(np.float64), -65504.0, 65504.0)
    want_floor = tab[np.searchsorted(tab, xc, side="right") - 1]
    want_ceil = tab[np.searchsorted(tab, xc, side="left")]
    got_floor = ko.fp16_floor(x)
    got_ceil = ko.fp16_ceil(x)
    assert got_floor.dtype == np.float16 and got_ceil.dtype == np.float16
    np.testing.assert_array_equal(got_floor.astype(np.float64), want_floor)
    np.testing.assert_array_equal(got_ceil.astype(np.float64), want_ceil)
    assert np.all(got_floor.astype(np.float64) <= xc) and np.all(got_ceil.astype(np.float64) >= xc)


def test_bf16_round_matches_library_cast():
    rng = np.random.default_rng(11)
    x = np.concatenate([rng.standard_normal(100000) * s for s in (1e-20, 1e-3, 1.0, 1e4, 1e30)]).astype(np.float32)
    # exact ties: low 16 bits == 0x8000
    ties = (rng.integers(0, 2 ** 15, 1000).astype(np.uint32) << 16 | np.uint32(0x8000)).view(np.float32)
    x = np.concatenate([x, ties])
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(ko.bf16_round(x), want)
    np.testing.assert_array_equal(ko.bf16_to_f32(ko.bf16_bits(x)), want)
    # the input generator's cast is the same rounding
    np.testing.assert_array_equal(ks.bf16_bits_to_f32(ks.f32_to_bf16_bits(x)), want)


# ---- PCA ------------------------------------------------------------------

def test_pca_is_an_orthonormal_diagonalising_basis():
    L = ks.make_layer(ks.LayerSpec(p=48, alpha=1.0, seed=3))
    C = ks.draw(L, 4000, 1)
    mu, V, S = ko.pca(C)
    np.testing.assert_allclose(mu, C.mean(0), atol=1e-13)
    np.testing.assert_allclose(V.T @ V, np.eye(48), atol=1e-12)
    assert np.all(np.diff(S) <= 1e-12)
    P = (C - mu) @ V
    gram = P.T @ P
    np.testing.assert_allclose(np.diag(gram), S ** 2, rtol=1e-10)
    off = gram - np.diag(np.diag(gram))
    assert np.abs(off).max() <= 1e-9 * S[0] ** 2
    # full rank: X = D V^T + mu exactly (eq. 3 of the paper)
    np.testing.assert_allclose(P @ V.T + mu, C, atol=1e-12)
    # a transposed basis must not pass: its coefficients are not decorrelated
    Pt = (C - mu) @ V.T
    gt = Pt.T @ Pt
    assert np.abs(gt - np.diag(np.diag(gt))).max() > 1e-3 * S[0] ** 2
    # sign convention
    assert np.all(V[np.argmax(np.abs(V), axis=0), np.arange(48)] > 0)


def test_pca_recovers_closed_form_covariance_of_the_generator():
    """Without outliers the generator's covariance is Q diag(sigma^2) Q^T exactly, so the
    sample spectrum tends to sigma_i^2 and leading basis vectors to +-Q's columns."""
    p, n = 24, 200000
    L = ks.make_layer(ks.LayerSpec(p=p, alpha=1.2, seed=17))
    C = ks.draw(L, n, 2)
    mu, V, S = ko.pca(C)
    lam = S ** 2 / (n - 1)
    np.testing.assert_allclose(lam, L.sigma ** 2, rtol=0.03)
    np.testing.assert_allclose(mu, L.mu, atol=5 * L.sigma[0] / np.sqrt(n))
    for i in range(6):
        assert abs(V[:, i] @ L.Q[:, i]) > 0.995, i
    # and it equals the library eigendecomposition of the sample covariance
    w, _ = np.linalg.eigh(np.cov(C.T))
    np.testing.assert_allclose(lam, w[::-1], rtol=1e-9)


def test_truncation_error_equals_discarded_spectrum_mass():
    """Eckart-Young on the calibration set: ||(C-mu) - (C-mu) V_r V_r^T||_F^2 = sum_{i>r} s_i^2."""
    L = ks.make_layer(ks.LayerSpec(p=64, alpha=1.0, seed=23))
    C = ks.draw(L, 3000, 3)
    mu, V, S = ko.pca(C)
    A = C - mu
    for r in (1, 7, 32, 63, 64):
        Vr = V[:, :r]
        err = np.linalg.norm(A - A @ Vr @ Vr.T) ** 2
        want = (S[r:] ** 2).sum()
        assert abs(err - want) <= 1e-10 * (S ** 2).sum()
    # fresh draw: equality in expectation with the population tail sum(sigma_i^2)
    X = ks.draw(L, 40000, 4)
    r = 16
    err = np.linalg.norm((X - mu) - (X - mu) @ V[:, :r] @ V[:, :r].T) ** 2 / X.shape[0]
    assert err == pytest.approx((L.sigma[r:] ** 2).sum(), rel=0.08)


def test_generator_is_seeded_and_shaped():
    spec = ks.layer_spec("c2", 0, 1)
    assert spec.p == 1024 and spec.outlier_frac == 0.05 and spec.alpha == 1.0
    L = ks.make_layer(ks.LayerSpec(p=32, alpha=1.0, seed=9, outlier_frac=0.05))
    a = ks.draw(L, 500, 1)
    b = ks.draw(L, 500, 1)
    c = ks.draw(L, 500, 2)
    np.testing.assert_array_equal(a, b)
    assert np.abs(a - c).max() > 0.1
    np.testing.assert_allclose(L.Q.T @ L.Q, np.eye(32), atol=1e-12)
    # sizes the paper's KV-size table implies for Llama-3.1-8B: 32 layers x 8 KV heads x 128
    w = ks.WORKLOADS["c3"]
    assert 2 * w.n_layers * w.p * 2 == 131072            # bytes per token
    assert 2 * w.n_layers * w.p * 2 * 1024 == 128 * 2 ** 20   # 128 MiB per 1K tokens
    lens = ks.ragged_lengths("c5")
    assert lens.shape == (256,) and lens.min() >= 512 and lens.max() <= 16384
    assert ks.layer_spec("c3", 5, 0).alpha == ks.layer_spec("c3", 5, 1).alpha
    assert 0.8 <= ks.layer_spec("c3", 5, 0).alpha <= 1.4
