"""Seeded synthetic KV-cache tensors that stand in for real model caches.

This module only *draws inputs*; it holds none of the coder's arithmetic
(no PCA, no quantiser, no packing).  Both the CPU oracle's callers and the
GPU path's callers take their tensors from here so that the two sides see
bit-identical inputs.

Recipe (one "layer" = one K or V tensor of one transformer layer):

    X = Z . diag(sigma) . Q^T + mu
    Z      ~ N(0, 1)                       [T, p], a fresh draw per call
    sigma_i = i ** (-alpha), i = 1..p       fast-decaying spectrum (low-rank KV)
    Q      = orthogonal factor of a seeded Gaussian p x p matrix
    mu     ~ N(0, 0.1**2)                  [p]
    outliers: a Bernoulli(outlier_frac) mask over tokens; the masked tokens'
              values on `n_outlier_channels` fixed (seeded) channels are
              multiplied by `outlier_gain` after generation.

The spectrum decay mimics the low effective rank of KV caches that the
paper's method exploits (Section "Feature decorrelation"); the few
high-magnitude channels mimic the channel outliers it reports in its
appendix on KV-cache properties.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional, Tuple

import numpy as np

BASE_SEED = 251101815


@dataclass(frozen=True)
class LayerSpec:
    """Parameters of one synthetic K or V tensor family."""
    p: int
    alpha: float
    seed: int
    outlier_frac: float = 0.0
    n_outlier_channels: int = 4
    outlier_gain: float = 10.0
    mu_std: float = 0.1


@dataclass
class Layer:
    """Materialised fixed parts (Q, sigma, mu, outlier channels) of a LayerSpec."""
    spec: LayerSpec
    Q: np.ndarray            # [p, p] float64, orthogonal
    sigma: np.ndarray        # [p] float64
    mu: np.ndarray           # [p] float64
    channels: np.ndarray     # [n_outlier_channels] int64
    _mix32: Optional[object] = field(default=None, repr=False)


def make_layer(spec: LayerSpec) -> Layer:
    rng = np.random.default_rng([spec.seed, 1])
    g = rng.standard_normal((spec.p, spec.p))
    q, r = np.linalg.qr(g)
    q = q * np.sign(np.diag(r))[None, :]          # make the factorisation unique
    sigma = np.arange(1, spec.p + 1, dtype=np.float64) ** (-spec.alpha)
    mu = rng.standard_normal(spec.p) * spec.mu_std
    channels = np.sort(rng.choice(spec.p, size=spec.n_outlier_channels, replace=False))
    return Layer(spec, q, sigma, mu, channels.astype(np.int64))


def draw(layer: Layer, n_tokens: int, draw_seed: int) -> np.ndarray:
    """A fresh [n_tokens, p] float64 draw of the layer (before any dtype cast)."""
    spec = layer.spec
    rng = np.random.default_rng([spec.seed, 2, draw_seed])
    z = rng.standard_normal((n_tokens, spec.p))
    x = (z * layer.sigma[None, :]) @ layer.Q.T + layer.mu[None, :]
    if spec.outlier_frac > 0.0:
        mask = rng.random(n_tokens) < spec.outlier_frac
        x[np.ix_(mask, layer.channels)] *= spec.outlier_gain
    return x


# ---- dtype casts of the *inputs* (bf16 is the cache dtype of configs 2-5) ----

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 values to bfloat16 (nearest even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def draw_bf16(layer: Layer, n_tokens: int, draw_seed: int) -> np.ndarray:
    """[n_tokens, p] uint16 bf16 bit patterns."""
    return f32_to_bf16_bits(draw(layer, n_tokens, draw_seed).astype(np.float32))


def draw_f32(layer: Layer, n_tokens: int, draw_seed: int) -> np.ndarray:
    return draw(layer, n_tokens, draw_seed).astype(np.float32)


# ---- device-side generation for tensors too large to build on the host ----

def draw_bf16_torch(layer: Layer, n_tokens: int, draw_seed: int, device, out=None, chunk: int = 32768):
    """[n_tokens, p] torch.bfloat16 tensor on `device`, generated there.

    A different random stream from `draw` (torch's generator, not numpy's);
    callers that need the oracle's view of these tensors copy the rows they
    check back to the host bit-for-bit.
    """
    import torch
    spec = layer.spec
    if layer._mix32 is None or layer._mix32[0].device != torch.device(device):
        mix = torch.from_numpy((layer.sigma[:, None] * layer.Q.T).astype(np.float32)).to(device)
        mu = torch.from_numpy(layer.mu.astype(np.float32)).to(device)
        ch = torch.from_numpy(layer.channels).to(device)
        layer._mix32 = (mix, mu, ch)
    mix, mu, ch = layer._mix32
    gen = torch.Generator(device=device)
    gen.manual_seed((spec.seed * 1000003 + draw_seed) % (2 ** 63 - 1))
    if out is None:
        out = torch.empty((n_tokens, spec.p), dtype=torch.bfloat16, device=device)
    for t0 in range(0, n_tokens, chunk):
        t1 = min(n_tokens, t0 + chunk)
        z = torch.randn((t1 - t0, spec.p), generator=gen, device=device, dtype=torch.float32)
        x = z @ mix + mu
        if spec.outlier_frac > 0.0:
            mask = torch.rand((t1 - t0,), generator=gen, device=device) < spec.outlier_frac
            gain = torch.where(mask, spec.outlier_gain, 1.0).to(torch.float32)
            x[:, ch] = x[:, ch] * gain[:, None]
        out[t0:t1] = x.to(torch.bfloat16)
    return out


# ---- the five workload shapes ----

@dataclass(frozen=True)
class Workload:
    name: str
    p: int
    n_layers: int
    n_tokens: int                 # per (layer, K/V) tensor; ragged workloads: see `ragged`
    n_calib: int
    cr: Tuple[float, ...]         # compression targets
    dtype: str                    # "f32" or "bf16"
    alpha: Tuple[float, float]    # (lo, hi): per-layer exponent ~ U[lo, hi]; lo == hi => fixed
    outlier_frac: float
    kv: Tuple[str, ...] = ("K", "V")
    ragged: Optional[Tuple[int, int, int]] = None   # (n_caches, min_len, max_len), log-uniform


WORKLOADS = {
    # tiny single head, fp32, 4x
    "c1": Workload("c1", 128, 1, 4096, 1024, (4.0,), "f32", (1.2, 1.2), 0.0, kv=("K",)),
    # Llama-3.1-8B-shaped single layer, K and V, 16x
    "c2": Workload("c2", 1024, 1, 32768, 8192, (16.0,), "bf16", (1.0, 1.0), 0.05),
    # full Llama-3.1-8B-shaped cache, per-layer exponent
    "c3": Workload("c3", 1024, 32, 32768, 8192, (8.0, 16.0, 20.0), "bf16", (0.8, 1.4), 0.05),
    # Mistral-NeMo-12B-shaped long context
    "c4": Workload("c4", 1024, 40, 131072, 8192, (20.0,), "bf16", (0.8, 1.4), 0.05),
    # Qwen2.5-32B-shaped ragged batch
    "c5": Workload("c5", 1024, 64, 0, 8192, (40.0,), "bf16", (0.8, 1.4), 0.05,
                   ragged=(256, 512, 16384)),
}
_WORKLOAD_INDEX = {"c1": 1, "c2": 2, "c3": 3, "c4": 4, "c5": 5}


def layer_spec(workload: str, layer: int, kv: int) -> LayerSpec:
    """LayerSpec of (layer, kv) in a workload; kv = 0 for K, 1 for V."""
    w = WORKLOADS[workload]
    base = BASE_SEED + _WORKLOAD_INDEX[workload]
    lo, hi = w.alpha
    if lo == hi:
        alpha = lo
    else:   # one exponent per layer, shared by its K and V
        alpha = float(np.random.default_rng([base, 7, layer]).uniform(lo, hi))
    return LayerSpec(p=w.p, alpha=alpha, seed=base + 1000 * layer + kv, outlier_frac=w.outlier_frac)


def ragged_lengths(workload: str, layer: int = 0) -> np.ndarray:
    """Token counts of the independent caches of a ragged workload (log-uniform, seeded)."""
    w = WORKLOADS[workload]
    n, lo, hi = w.ragged
    rng = np.random.default_rng([BASE_SEED + _WORKLOAD_INDEX[workload], 9])
    u = rng.uniform(np.log(lo), np.log(hi), size=n)
    return np.clip(np.rint(np.exp(u)), lo, hi).astype(np.int64)



def cross_layer_spec(n_layers: int, alpha: float = 1.0) -> LayerSpec:
    """The features of n_layers 8B-shaped layers (1024 each) side by side, correlated across layers: the recipe
    above over all n_layers * 1024 features at once (one spectrum, one rotation, a few outlier channels).  Stands in
    for the concatenated keys or values of several layers, whose cross-layer redundancy a single basis exploits
    (paper, Section "Feature decorrelation"; appendix "PCA feature concat size vs performance")."""
    return LayerSpec(p=1024 * n_layers, alpha=alpha, seed=BASE_SEED + 77_000 + n_layers, outlier_frac=0.05)

CALIB_DRAW = 1_000_001     # draw_seed of the calibration draw
TEST_DRAW = 1_000_002      # draw_seed of the evaluation draw
