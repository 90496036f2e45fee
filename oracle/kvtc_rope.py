"""Rotary positional embeddings of keys, undone before coding and redone after decoding --
TEST INFRASTRUCTURE, NOT A PRODUCT PATH (same rules as kvtc_oracle.py: only tests, the smoke
check and the CPU-baseline leg of the benchmark may import it; it shares no code with the GPU path).

The paper removes the positional rotation from keys before they are transform-coded (Section
"Feature decorrelation": the rotation hides the low-rank structure of keys; the related-work section:
compression is applied before RoPE) and the decoded keys are rotated again before attention sees
them.  The rotation itself is the one of RoFormer: inside every head, features are paired and each
pair (a, b) of token position m is turned by the angle m * theta_j,

    theta_j = base ** (-2 j / d_head),  j = 0 .. d_head/2 - 1,
    a' = a cos(m theta_j) - b sin(m theta_j),   b' = a sin(m theta_j) + b cos(m theta_j),

and undoing it is the rotation by the opposite angle.  Which features form pair j is a convention of
the model code, not of the method; both common ones are here:
    "half"         pair j = (j, j + d_head/2)      (the rotate-half form)
    "interleaved"  pair j = (2j, 2j + 1)
Everything is float64; positions are integers.

Layouts: `x` is [T, H * d_head] (token-major, heads side by side: what the coder takes).
heads_first() / tokens_first() convert from and to the [H, T, d_head] layout caches are often kept in.

Pins (tests/test_oracle_rope.py): a hand-computed pair; position 0 is the identity; undo after redo is the
identity; every pair's norm is preserved; the complex-number form (a + i b) e^{i m theta} computed by
another route; R(m) R(n) = R(m + n); and the property the construction exists for:
<R(m) q, R(n) k> depends on m - n only.
"""
from __future__ import annotations

import numpy as np


def rope_angles(positions, d_head: int, base: float = 10000.0) -> np.ndarray:
    """[T, d_head/2] angles m * theta_j."""
    assert d_head % 2 == 0
    j = np.arange(d_head // 2, dtype=np.float64)
    theta = np.float64(base) ** (-2.0 * j / d_head)
    return np.asarray(positions, dtype=np.float64)[:, None] * theta[None, :]


def pair_indices(d_head: int, pairing: str):
    """(index of a, index of b) of every pair j inside a head."""
    half = d_head // 2
    if pairing == "half":
        return np.arange(half), np.arange(half) + half
    if pairing == "interleaved":
        return 2 * np.arange(half), 2 * np.arange(half) + 1
    raise ValueError(pairing)


def rope(x, positions, n_heads: int, d_head: int, base: float = 10000.0, pairing: str = "half",
         inverse: bool = False) -> np.ndarray:
    """Rotate (inverse=False) or un-rotate (inverse=True) every head of x [T, n_heads * d_head]."""
    x = np.asarray(x, dtype=np.float64)
    T = x.shape[0]
    assert x.shape == (T, n_heads * d_head)
    ang = rope_angles(positions, d_head, base)
    if inverse:
        ang = -ang
    c, s = np.cos(ang), np.sin(ang)                     # [T, d_head/2]
    ia, ib = pair_indices(d_head, pairing)
    xh = x.reshape(T, n_heads, d_head)
    out = np.empty_like(xh)
    a, b = xh[:, :, ia], xh[:, :, ib]
    out[:, :, ia] = a * c[:, None, :] - b * s[:, None, :]
    out[:, :, ib] = a * s[:, None, :] + b * c[:, None, :]
    return out.reshape(T, n_heads * d_head)


def heads_first(x, n_heads: int, d_head: int) -> np.ndarray:
    """[T, H * d] -> [H, T, d]."""
    x = np.asarray(x)
    return np.ascontiguousarray(x.reshape(x.shape[0], n_heads, d_head).transpose(1, 0, 2))


def tokens_first(xh) -> np.ndarray:
    """[H, T, d] -> [T, H * d]."""
    xh = np.asarray(xh)
    H, T, d = xh.shape
    return np.ascontiguousarray(xh.transpose(1, 0, 2)).reshape(T, H * d)
