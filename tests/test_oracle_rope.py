"""Pins of the rotary-embedding oracle (CPU only): things the mathematics fixes, none of them a re-typing
of the oracle's own formula."""
import numpy as np
import pytest

import kvtc_rope as kr


def test_hand_computed_pair():
    """One head of two features at position 3, base irrelevant (theta_0 = 1): the vector (1, 0) turned by
    3 rad is (cos 3, sin 3) = (-0.9899924966..., 0.1411200080...); (0, 2) becomes (-2 sin 3, 2 cos 3)."""
    y = kr.rope(np.array([[1.0, 0.0]]), [3], 1, 2, base=123.0)
    np.testing.assert_allclose(y, [[-0.9899924966004454, 0.1411200080598672]], rtol=0, atol=1e-15)
    y = kr.rope(np.array([[0.0, 2.0]]), [3], 1, 2)
    np.testing.assert_allclose(y, [[-0.2822400161197344, -1.9799849932008908]], rtol=0, atol=1e-15)
    # four features, "half" pairs (0,2),(1,3); theta_1 = base^(-1/2) = 0.1 for base 100: position 5 -> angles 5 and 0.5
    y = kr.rope(np.array([[1.0, 1.0, 0.0, 0.0]]), [5], 1, 4, base=100.0, pairing="half")
    np.testing.assert_allclose(y, [[np.cos(5.0), np.cos(0.5), np.sin(5.0), np.sin(0.5)]], atol=1e-15)
    # the same pairs laid out interleaved: (0,1),(2,3)
    y = kr.rope(np.array([[1.0, 0.0, 1.0, 0.0]]), [5], 1, 4, base=100.0, pairing="interleaved")
    np.testing.assert_allclose(y, [[np.cos(5.0), np.sin(5.0), np.cos(0.5), np.sin(0.5)]], atol=1e-15)


@pytest.mark.parametrize("pairing", ["half", "interleaved"])
def test_identities(pairing):
    rng = np.random.default_rng(4)
    H, d, T = 8, 128, 50
    x = rng.standard_normal((T, H * d))
    pos = rng.integers(0, 131072, size=T)
    pos[0] = 0
    y = kr.rope(x, pos, H, d, pairing=pairing)
    np.testing.assert_array_equal(y[0], x[0])                                     # position 0: identity
    back = kr.rope(y, pos, H, d, pairing=pairing, inverse=True)
    np.testing.assert_allclose(back, x, rtol=0, atol=1e-12)                       # undo after redo
    ia, ib = kr.pair_indices(d, pairing)
    xh, yh = x.reshape(T, H, d), y.reshape(T, H, d)
    np.testing.assert_allclose(yh[:, :, ia] ** 2 + yh[:, :, ib] ** 2, xh[:, :, ia] ** 2 + xh[:, :, ib] ** 2, rtol=1e-12)
    # the complex form, by another route: (a + i b) * exp(i m theta_j) with theta_j from logarithms
    theta = np.exp(-2.0 * np.arange(d // 2) / d * np.log(10000.0))
    z = (xh[:, :, ia] + 1j * xh[:, :, ib]) * np.exp(1j * pos[:, None, None] * theta[None, None, :])
    np.testing.assert_allclose(yh[:, :, ia], z.real, rtol=0, atol=1e-9)
    np.testing.assert_allclose(yh[:, :, ib], z.imag, rtol=0, atol=1e-9)
    # rotations add
    p1, p2 = rng.integers(0, 5000, size=T), rng.integers(0, 5000, size=T)
    np.testing.assert_allclose(kr.rope(kr.rope(x, p1, H, d, pairing=pairing), p2, H, d, pairing=pairing),
                               kr.rope(x, p1 + p2, H, d, pairing=pairing), rtol=0, atol=1e-10)
    # a swapped sign or a transposed pair would break this: the score of a rotated query and key depends on m - n only
    q, k = rng.standard_normal((1, H * d)), rng.standard_normal((1, H * d))
    s1 = (kr.rope(q, [700], H, d, pairing=pairing) * kr.rope(k, [300], H, d, pairing=pairing)).sum()
    s2 = (kr.rope(q, [10400], H, d, pairing=pairing) * kr.rope(k, [10000], H, d, pairing=pairing)).sum()
    s3 = (kr.rope(q, [400], H, d, pairing=pairing) * k).sum()
    assert abs(s1 - s2) < 1e-8 and abs(s1 - s3) < 1e-9


def test_pairings_differ_only_by_a_permutation_of_features():
    rng = np.random.default_rng(5)
    H, d, T = 2, 16, 7
    x = rng.standard_normal((T, H * d))
    pos = np.arange(T) * 11
    perm = np.concatenate([np.stack(kr.pair_indices(d, "interleaved"), 1).ravel()])      # half layout -> interleaved layout
    # feature f of the interleaved layout is feature inv[f] of the half layout
    ia, ib = kr.pair_indices(d, "half")
    src = np.empty(d, dtype=int)
    src[0::2], src[1::2] = ia, ib
    xi = x.reshape(T, H, d)[:, :, src].reshape(T, H * d)
    yi = kr.rope(xi, pos, H, d, pairing="interleaved")
    yh = kr.rope(x, pos, H, d, pairing="half")
    np.testing.assert_allclose(yi, yh.reshape(T, H, d)[:, :, src].reshape(T, H * d), rtol=0, atol=1e-14)
    assert perm.shape == (d,)


def test_layout_helpers_round_trip():
    rng = np.random.default_rng(6)
    x = rng.standard_normal((5, 3 * 4))
    xh = kr.heads_first(x, 3, 4)
    assert xh.shape == (3, 5, 4) and xh[1, 2, 3] == x[2, 1 * 4 + 3]
    np.testing.assert_array_equal(kr.tokens_first(xh), x)
