"""Sink tokens, sliding window and incremental compression on the CPU -- TEST INFRASTRUCTURE,
NOT A PRODUCT PATH.

The part of "KV Cache Transform Coding for Compact Storage in LLM Inference" that sits either
side of the coder in serving (Section "Sliding Windows and Sink Tokens"; Section "Experimental
setup", the paragraph on compressing every c tokens; Appendix "Compression ratio with sliding
window"): the s oldest tokens and the w most recent ones are not transform-coded, the sinks are
kept in FP8, and the coder runs every c new tokens so that the window stays between w - c and w.

Everything here is written as the plainest definition available: the split of a context into
sinks / coded tokens / window is found by replaying the arrival of the tokens one at a time, FP8
conversion is a nearest-neighbour search in the table of all values of the format, stored sizes
are counted array by array.  Only tests, the smoke check and the benchmark's CPU leg may import
this module; it shares no code with the GPU library and imports nothing from it.

Readings of the paper (it fixes none of these):
  * "FP8" for the sinks: OCP E4M3 (1 sign, 4 exponent bits with bias 7, 3 mantissa bits, no
    infinities, one NaN pattern per sign), a plain cast of each value with round-to-nearest-even
    and saturation to +-448, no scale factor;
  * "compress every c = 16 tokens, leaving the window in the 112-128 range" (w = 128): a token
    joins the window when it arrives; as soon as the window holds w tokens its c oldest are coded.
    Between arrivals the window therefore holds w - c .. w - 1 tokens once the context is long enough.

Pins (tests/test_oracle_window.py): the replay against hand-counted contexts and against the
closed form; the FP8 table against the format's published extremes and a handful of exact
values; the search against exhaustive round trips of all 256 codes and against midpoints; the
compression ratio with window against the appendix formula evaluated from counted bytes.
"""
from __future__ import annotations

from typing import Tuple

import numpy as np


# --------------------------------------------------------------------------
# which tokens are coded (Section "Sliding Windows and Sink Tokens"; compress every c tokens)
# --------------------------------------------------------------------------
def window_split(ctx: int, s: int = 4, w: int = 128, c: int = 16) -> Tuple[int, int, int]:
    """(sinks, coded tokens, window tokens) after ctx tokens have arrived, by replaying the arrivals."""
    if ctx < 0 or s < 0 or w < 1 or c < 1 or c > w:
        raise ValueError("need ctx >= 0, s >= 0, 1 <= c <= w")
    n_sink = n_coded = n_window = 0
    for _ in range(ctx):
        if n_sink < s:
            n_sink += 1            # the oldest tokens are the sinks; they are never coded
            continue
        n_window += 1              # a new token is recent: it joins the window
        if n_window == w:          # the window is full: its c oldest tokens go to the coder
            n_window -= c
            n_coded += c
    return n_sink, n_coded, n_window


# --------------------------------------------------------------------------
# FP8 (E4M3) for the sinks
# --------------------------------------------------------------------------
def e4m3_table() -> np.ndarray:
    """Value of each of the 256 codes (float64; NaN for the two NaN codes), from the format's definition."""
    t = np.empty(256, dtype=np.float64)
    for code in range(256):
        sign = -1.0 if code & 0x80 else 1.0
        e = (code >> 3) & 0xF
        m = code & 0x7
        if e == 0xF and m == 0x7:
            t[code] = np.nan
        elif e == 0:
            t[code] = sign * (m / 8.0) * 2.0 ** (1 - 7)          # subnormal
        else:
            t[code] = sign * (1.0 + m / 8.0) * 2.0 ** (e - 7)
    return t


def e4m3_encode(x: np.ndarray) -> np.ndarray:
    """Nearest E4M3 code of each value: ties go to the code with an even mantissa, magnitudes beyond the
    largest finite value (448) saturate to it, NaN gives the NaN code 0x7f, the sign of zero is kept."""
    x = np.asarray(x, dtype=np.float64)
    t = e4m3_table()
    pos = t[:0x7F]                                                # codes 0x00..0x7e: 0 .. 448, ascending
    out = np.empty(x.shape, dtype=np.uint8)
    flat = x.reshape(-1)
    o = out.reshape(-1)
    for i, v in enumerate(flat):
        if np.isnan(v):
            o[i] = 0x7F
            continue
        a = min(abs(v), pos[-1])
        d = np.abs(pos - a)
        k = int(np.argmin(d))                                    # first (smaller) code on a tie
        if k + 1 < len(pos) and d[k + 1] == d[k] and (k & 1):    # tie: take the even mantissa
            k += 1
        o[i] = k | (0x80 if np.signbit(v) else 0)
    return out


def e4m3_decode(codes: np.ndarray) -> np.ndarray:
    return e4m3_table()[np.asarray(codes, dtype=np.uint8)]


# --------------------------------------------------------------------------
# stored size with sinks and window (Appendix "Compression ratio with sliding window")
# --------------------------------------------------------------------------
def stored_bytes(ctx: int, p: int, record_bytes: int, s: int = 4, w: int = 128, c: int = 16) -> int:
    """Bytes one (layer, K or V) cache of ctx tokens occupies: sinks in FP8 (1 byte per value), coded
    tokens as records, window tokens in 16 bits."""
    n_sink, n_coded, n_window = window_split(ctx, s, w, c)
    return n_sink * p * 1 + n_coded * record_bytes + n_window * p * 2


def cr_with_window(ctx: float, w: float, s: float, cr: float) -> float:
    """The appendix's formula: ctx / ((ctx - w - s) / cr + w + s / 2)."""
    return ctx / ((ctx - w - s) / cr + w + s / 2.0)
