"""GPU test of the error table of the bit allocation (paper, appendix "Dynamic programming algorithm": the simulated
quantisation of every candidate block at every width) against the oracle's BlockErrors, and the allocation that the oracle's
dynamic programme makes from the GPU's table against the one it makes from its own."""
import ctypes as C

import numpy as np
import pytest
import torch

import kvtc_oracle as ko
import kvtc_synth as ks
import paper_2511_01815_amd as kv

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _candidates(p, sizes=(16, 64, 256, 1024)):
    return [(s, n) for n in sizes if n <= p for s in range(0, p - n + 1, 16)]


class _TableErrors:
    """What dp_allocate reads, served from a table."""

    def __init__(self, energy, table):
        self.energy, self.table = energy, table

    def change(self, start, n, bits):
        return 0.0 if bits == 0 else self.table[(start, n, bits)]


@pytest.mark.parametrize("workload,n_tok", [("c1", 777), ("c2", 2048)])
def test_error_table_equals_the_oracles_and_gives_the_same_allocation(workload, n_tok):
    wl = ks.WORKLOADS[workload]
    L = ks.make_layer(ks.layer_spec(workload, 0, 0))
    C_ = ko.bf16_round(ks.draw_f32(L, max(n_tok, wl.p + 64), ks.CALIB_DRAW))
    mu, V, S = ko.pca(C_)
    errors = ko.dp_errors(C_, mu, V, n_dp_tokens=n_tok)
    P32 = errors.P32
    p = wl.p
    cand = _candidates(p) + [(0, 48), (16, 32), (p - 1024 if p >= 1024 else 0, min(p, 1024))]       # sizes the default set lacks, too
    blocks = torch.tensor(cand, dtype=torch.int32, device=DEV)
    out = torch.full((len(cand), 8), -7.0, dtype=torch.float64, device=DEV)
    pd = torch.from_numpy(P32).to(DEV)
    kv.kvtc_calib_block_errors(pd, n_tok, p, blocks, len(cand), 8, out)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    kv.kvtc_calib_block_errors(pd, n_tok, p, blocks, len(cand), 8, out)
    e1.record()
    torch.cuda.synchronize()
    gpu_ms = e0.elapsed_time(e1)
    got = out.cpu().numpy()
    worst = 0.0
    table = {}
    import time
    t_ref = time.perf_counter()
    for i, (s, n) in enumerate(cand):
        for b in range(1, 9):
            ref = errors.change(s, n, b)
            # the same exactly representable terms summed in another order: a few ulps of the larger of the two sums
            scale = errors.energy[s:s + n].sum()
            assert abs(got[i, b - 1] - ref) <= 1e-11 * scale, (s, n, b, got[i, b - 1], ref)
            worst = max(worst, abs(got[i, b - 1] - ref) / scale)
            table[(s, n, b)] = float(got[i, b - 1])
    t_ref = time.perf_counter() - t_ref
    # the allocation from the GPU's table is the oracle's own (16x for the 1024-feature layer, 4x for the small one)
    cr = 16.0 if p == 1024 else 4.0
    sizes = [s for s in (16, 64, 256, 1024) if s <= p]
    a_ref, e_ref = ko.dp_allocate(errors, p, ko.bit_budget(p, cr), sizes)
    a_gpu, e_gpu = ko.dp_allocate(_TableErrors(errors.energy, table), p, ko.bit_budget(p, cr), sizes)
    assert a_gpu == a_ref and abs(e_gpu - e_ref) <= 1e-9 * abs(e_ref)
    print(f"{workload}: {len(cand)} blocks x 8 widths over {n_tok} tokens, largest deviation {worst:.1e} of the block's energy; "
          f"GPU {gpu_ms:.2f} ms, oracle {t_ref:.1f} s")


def test_bad_blocks_and_arguments():
    L = kv.lib()
    P = torch.zeros((10, 64), dtype=torch.float32, device=DEV)
    P[:, 5] = 3.0
    blocks = torch.tensor([[0, 16], [60, 16], [-1, 16], [0, 0], [48, 16]], dtype=torch.int32, device=DEV)
    out = torch.zeros((5, 2), dtype=torch.float64, device=DEV)
    kv.kvtc_calib_block_errors(P, 10, 64, blocks, 5, 2, out)
    torch.cuda.synchronize()
    o = out.cpu().numpy()
    assert np.isfinite(o[0]).all() and np.isfinite(o[4]).all()
    assert np.isnan(o[1]).all() and np.isnan(o[2]).all() and np.isnan(o[3]).all()
    assert np.all(o[4] == 0.0)                                   # an all-zero block: nothing to gain, nothing to lose
    p = P.data_ptr()
    assert L.kvtc_calib_block_errors(p, 10, 64, blocks.data_ptr(), 5, 9, out.data_ptr(), None) == 1
    assert L.kvtc_calib_block_errors(p, 10, 64, blocks.data_ptr(), 5, 0, out.data_ptr(), None) == 1
    assert L.kvtc_calib_block_errors(p, -1, 64, blocks.data_ptr(), 5, 2, out.data_ptr(), None) == 1
    assert L.kvtc_calib_block_errors(None, 10, 64, blocks.data_ptr(), 5, 2, out.data_ptr(), None) == 1
    assert L.kvtc_calib_block_errors(p, 10, 64, blocks.data_ptr(), 0, 2, out.data_ptr(), None) == 0


def test_moments_give_the_oracles_pca():
    """Sum and second moments of a calibration draw on the GPU (bf16 tokens, token-major and heads-major), against NumPy in
    float64; the eigen-decomposition of the covariance formed from them against the oracle's SVD-based PCA."""
    L = ks.make_layer(ks.layer_spec("c2", 0, 0))
    n, p = 3000, 1024
    bits = ks.draw_bf16(L, n, ks.CALIB_DRAW)
    C_ = ks.bf16_bits_to_f32(bits).astype(np.float64)
    xd = torch.from_numpy(bits.view(np.int16)).to(DEV).view(torch.bfloat16)            # [n, 1024]
    s = torch.zeros(p, dtype=torch.float64, device=DEV)
    g = torch.zeros((p, p), dtype=torch.float64, device=DEV)
    kv.kvtc_calib_moments(xd, kv.KVTC_BF16, n, p, kv.layout(p), s, g)
    xh = xd.reshape(n, 8, 128).permute(1, 0, 2).contiguous()                            # [8][n][128]
    s2 = torch.zeros_like(s)
    g2 = torch.zeros_like(g)
    kv.kvtc_calib_moments(xh, kv.KVTC_BF16, n, p, kv.layout(128, 128, n * 128), s2, g2)
    torch.cuda.synchronize()
    assert torch.equal(s, s2) and torch.equal(g, g2)                                     # same sums in the same order
    S_, G_ = s.cpu().numpy(), g.cpu().numpy()
    ref_s, ref_g = C_.sum(axis=0), C_.T @ C_
    assert np.max(np.abs(S_ - ref_s)) <= 1e-12 * np.abs(C_).sum(axis=0).max()
    assert np.max(np.abs(G_ - ref_g)) <= 1e-12 * np.abs(ref_g).max()
    assert np.array_equal(G_, G_.T)
    # PCA from the moments (host: a 1024 x 1024 eigen-problem) against the oracle's SVD of the centred matrix
    mu = S_ / n
    lam, W = np.linalg.eigh(G_ / n - np.outer(mu, mu))
    lam, W = lam[::-1], W[:, ::-1]
    mu_o, V_o, S_o = ko.pca(C_)
    assert np.max(np.abs(mu - mu_o)) <= 1e-14
    k = 300                                                                              # beyond what any calibrated plan keeps at 16x
    assert np.max(np.abs(lam[:k] * n / S_o[:k] ** 2 - 1.0)) <= 1e-7
    dots = np.abs(np.sum(W[:, :k] * V_o[:, :k], axis=0))
    assert dots.min() >= 1.0 - 1e-6, dots.min()


def test_moments_fp32_input_and_arguments():
    L = ks.make_layer(ks.layer_spec("c1", 0, 0))
    n, p = 515, 128
    X = ks.draw_f32(L, n, ks.CALIB_DRAW)
    xd = torch.from_numpy(X).to(DEV)
    s = torch.zeros(p, dtype=torch.float64, device=DEV)
    g = torch.zeros((p, p), dtype=torch.float64, device=DEV)
    kv.kvtc_calib_moments(xd, kv.KVTC_F32, n, p, kv.layout(p), s, g)
    torch.cuda.synchronize()
    X64 = X.astype(np.float64)
    assert np.max(np.abs(s.cpu().numpy() - X64.sum(axis=0))) <= 1e-12 * np.abs(X64).sum(axis=0).max()
    assert np.max(np.abs(g.cpu().numpy() - X64.T @ X64)) <= 1e-12 * np.abs(X64.T @ X64).max()
    lib = kv.lib()
    lay = kv.layout(p)
    assert lib.kvtc_calib_moments(xd.data_ptr(), 1, n, 100, C.byref(lay), s.data_ptr(), g.data_ptr(), None) == 1      # p not a multiple of 64
    assert lib.kvtc_calib_moments(xd.data_ptr(), 1, n, p, None, s.data_ptr(), g.data_ptr(), None) == 1
    assert lib.kvtc_calib_moments(xd.data_ptr(), 1, n, p, C.byref(lay), None, g.data_ptr(), None) == 1
    short = kv.layout(64)
    assert lib.kvtc_calib_moments(xd.data_ptr(), 1, n, p, C.byref(short), s.data_ptr(), g.data_ptr(), None) == 1       # pitch below p
