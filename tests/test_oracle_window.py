"""Pins for oracle/kvtc_window.py: sinks, sliding window, FP8 sinks, compression ratio with window
(paper, Section "Sliding Windows and Sink Tokens"; Appendix "Compression ratio with sliding window")."""
import math
import os
import sys

import numpy as np
import pytest

sys.path.insert(0, os.path.join(os.path.dirname(__file__), "..", "oracle"))
import kvtc_window as kw  # noqa: E402


# ---- which tokens are coded -------------------------------------------------------------
def test_split_hand_counted_contexts():
    # s = 4 sinks, window w = 128, coder runs on 16 tokens whenever the window is full
    assert kw.window_split(0) == (0, 0, 0)
    assert kw.window_split(3) == (3, 0, 0)
    assert kw.window_split(4) == (4, 0, 0)
    assert kw.window_split(4 + 127) == (4, 0, 127)
    assert kw.window_split(4 + 128) == (4, 16, 112)          # the 128th window token triggers the coder
    assert kw.window_split(4 + 128 + 15) == (4, 16, 127)
    assert kw.window_split(4 + 128 + 16) == (4, 32, 112)
    assert kw.window_split(8192) == (4, 8064, 124)           # 8188 = 8064 + 124, 8064 = 16 * 504


@pytest.mark.parametrize("s,w,c", [(4, 128, 16), (0, 128, 16), (4, 64, 64), (1, 5, 2), (3, 7, 1)])
def test_split_invariants_and_closed_form(s, w, c):
    prev = (0, 0, 0)
    for ctx in range(0, 3 * w + 3 * s + 40):
        n_sink, n_coded, n_window = kw.window_split(ctx, s, w, c)
        assert n_sink + n_coded + n_window == ctx
        assert n_sink == min(ctx, s)
        assert n_coded % c == 0 and n_coded >= prev[1]
        assert 0 <= n_window < w                               # the paper's range: w - c .. w between coder runs
        if ctx >= s + w - c:
            assert n_window >= w - c
        # closed form, derived independently: the coder has run once for every c tokens beyond the first w - c of the window
        assert n_coded == c * max(0, (ctx - s - (w - c)) // c)
        prev = (n_sink, n_coded, n_window)


def test_split_rejects_nonsense():
    for bad in [(-1, 4, 128, 16), (10, -1, 128, 16), (10, 4, 0, 1), (10, 4, 8, 0), (10, 4, 8, 9)]:
        with pytest.raises(ValueError):
            kw.window_split(*bad)


# ---- FP8 E4M3 ---------------------------------------------------------------------------
def test_e4m3_table_matches_the_format():
    t = kw.e4m3_table()
    assert t[0x7E] == 448.0 and t[0xFE] == -448.0            # largest finite magnitude
    assert t[0x01] == 2.0 ** -9 and t[0x07] == 7 * 2.0 ** -9  # subnormals
    assert t[0x08] == 2.0 ** -6                               # smallest normal
    assert t[0x38] == 1.0 and t[0xC0] == -2.0 and t[0x3C] == 1.5
    assert t[0x00] == 0.0 and t[0x80] == 0.0 and math.copysign(1.0, t[0x80]) == -1.0
    assert np.isnan(t[0x7F]) and np.isnan(t[0xFF]) and np.isfinite(np.delete(t, [0x7F, 0xFF])).all()
    assert (np.diff(t[:0x7F]) > 0).all()                      # ascending in the code


def _e4m3_arith(v: float) -> int:
    """Independent arithmetic route: scale to the spacing of the binade, round half to even."""
    if math.isnan(v):
        return 0x7F
    sign = 0x80 if math.copysign(1.0, v) < 0 else 0
    a = min(abs(v), 448.0)
    if a < 2.0 ** -6:
        q = round(a / 2.0 ** -9)                              # Python rounds half to even
        return sign | q                                       # q == 8 is the smallest normal: code 0x08
    e = math.floor(math.log2(a))
    q = round(a / 2.0 ** (e - 3))                             # 8 .. 16 units of the binade's spacing
    if q == 16:
        e, q = e + 1, 8
    code = ((e + 7) << 3) | (q - 8)
    return sign | min(code, 0x7E)


def test_e4m3_encode_round_trips_every_code():
    t = kw.e4m3_table()
    finite = [c for c in range(256) if c not in (0x7F, 0xFF)]
    assert kw.e4m3_encode(t[finite]).tolist() == finite
    assert int(kw.e4m3_encode(np.array([np.nan]))[0]) == 0x7F


def test_e4m3_encode_midpoints_and_saturation():
    t = kw.e4m3_table()
    for k in range(0x7E):
        mid = 0.5 * (t[k] + t[k + 1])
        even = k if k % 2 == 0 else k + 1
        assert int(kw.e4m3_encode(np.array([mid]))[0]) == even
        assert int(kw.e4m3_encode(np.array([np.nextafter(mid, 0.0)]))[0]) == k
        assert int(kw.e4m3_encode(np.array([np.nextafter(mid, 1e9)]))[0]) == k + 1
        assert int(kw.e4m3_encode(np.array([-mid]))[0]) == 0x80 | even
    assert kw.e4m3_encode(np.array([449.0, 464.0, 480.0, 1e30, np.inf, -1e30])).tolist() == [0x7E] * 5 + [0xFE]


def test_e4m3_encode_equals_the_arithmetic_route():
    rng = np.random.default_rng(5)
    v = np.concatenate([rng.normal(0, 1, 4000), rng.normal(0, 60, 2000), rng.normal(0, 1e-2, 2000),
                        rng.uniform(-500, 500, 1000)])
    v = v.astype(np.float32).astype(np.float64)
    got = kw.e4m3_encode(v)
    want = np.array([_e4m3_arith(float(x)) for x in v], dtype=np.uint8)
    assert np.array_equal(got, want)
    # error bound of nearest rounding: half a spacing of the value's binade (or of the subnormal grid)
    err = np.abs(kw.e4m3_decode(got) - np.clip(v, -448, 448))
    spacing = np.maximum(2.0 ** (np.floor(np.log2(np.maximum(np.abs(v), 2.0 ** -6))) - 3), 2.0 ** -9)
    assert (err <= spacing / 2).all()


# ---- stored size ------------------------------------------------------------------------
@pytest.mark.parametrize("ctx", [132, 1000, 8192, 131072])
@pytest.mark.parametrize("R", [48, 100, 128, 256])
def test_counted_bytes_equal_the_appendix_formula(ctx, R):
    p = 1024
    n_sink, n_coded, n_window = kw.window_split(ctx)
    counted = kw.stored_bytes(ctx, p, R)
    assert counted == n_sink * p + n_coded * R + n_window * 2 * p
    cr = 2 * p / R                                            # ratio on the coded tokens alone
    # the appendix counts tokens in units of one 16-bit token: sinks weigh 1/2, window tokens 1, coded 1/cr
    assert 2 * p * ctx / counted == pytest.approx(kw.cr_with_window(ctx, n_window, n_sink, cr), rel=1e-12)


def test_cr_with_window_special_cases():
    assert kw.cr_with_window(1e6, 0, 0, 16.0) == pytest.approx(16.0)
    assert kw.cr_with_window(5000, 128, 0, 1.0) == pytest.approx(1.0)
    # the default setting of the paper's notation: four sinks in FP8 count as two tokens
    ctx, cr = 8192, 20.0
    assert kw.cr_with_window(ctx, 128, 4, cr) == pytest.approx(ctx / ((ctx - 128 - 4) / cr + 128 + 2))
    assert kw.cr_with_window(1e12, 128, 4, cr) == pytest.approx(cr, rel=1e-6)      # long contexts approach cr
