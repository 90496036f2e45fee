"""GPU tests of plans over the concatenated features of several layers that keep more coordinates than one record
section holds (paper, Section "Feature decorrelation"; appendices "PCA matrix sizes" and "PCA feature concat size vs
performance"): kvtc_wide_* against oracle/kvtc_wide.py, section by section for the stream and over all kept
coordinates for the reconstruction."""
import ctypes as C

import numpy as np
import pytest
import torch

import kvtc_oracle as ko
import kvtc_synth as ks
import kvtc_wide as kw
import paper_2511_01815_amd as kv
from test_gpu_parity import _from_dev, _to_dev, check_stream

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _wide(oplan):
    groups = list(zip(oplan.group_n.tolist(), oplan.group_bits.tolist()))
    return kv.WidePlan(oplan.p, oplan.r, oplan.mu32, oplan.v_bits, groups)


def _check_wide(oplan, X, n_layers, label, fp32_in=False, hdr_bar=None):
    """X [T, p] host values (bf16-representable).  Encodes from per-layer tensors [L][T][1024], decodes to bf16 (through the fp32
    workspace) and to fp32 (summed in place), both into the per-layer layout."""
    T, p = X.shape
    w = _wide(oplan)
    secs = kw.sections_of(oplan)
    assert w.n_sections == len(secs) >= 2
    assert [kv.kvtc_wide_section_record_bytes(w.handle, i) for i in range(len(secs))] == [s.record_bytes for s in secs]
    assert w.record_bytes == kw.record_bytes(oplan)
    offs = kw.section_offsets([s.record_bytes for s in secs], T)
    n_bytes = kv.kvtc_wide_encoded_bytes(w.handle, T)
    assert n_bytes == offs[-1]
    in_dtype = kv.KVTC_F32 if fp32_in else kv.KVTC_BF16
    xl = _to_dev(X, in_dtype).reshape(T, n_layers, 1024).permute(1, 0, 2).contiguous()          # [L][T][1024]
    lay = kv.layout(1024, 1024, T * 1024)
    out = torch.full((n_bytes + 64,), 0xA5, dtype=torch.uint8, device=DEV)
    kv.kvtc_wide_encode(w.handle, xl, in_dtype, T, lay, out, n_bytes)
    torch.cuda.synchronize()
    o = out.cpu().numpy()
    assert np.all(o[n_bytes:] == 0xA5), "wrote past the stream"
    worst = 0.0
    for i, (s, off) in enumerate(zip(secs, offs)):
        end = off + T * s.record_bytes
        nxt = offs[i + 1] if i + 1 < len(secs) else n_bytes
        assert np.all(o[end:nxt] == 0xA5), "wrote into the gap between two sections"
        bars = dict(hdr_bar=hdr_bar) if hdr_bar is not None and i == len(secs) - 1 else {}        # the weakest coordinates are in the last section
        st = check_stream(s, X, o[off:end].reshape(T, s.record_bytes), f"{label}-sec{i}", **bars)
        worst = max(worst, st["code_rate"])
    stream = o[:n_bytes]
    ref = kw.decode_wide(oplan, stream, T)                                   # the definition, float64, all kept coordinates at once
    mirror = kw.decode_wide(oplan, stream, T, operand_bf16=True)
    rng_x = float(X.max() - X.min())
    # fp32 output, summed in place
    xf = torch.full((n_layers, T, 1024), 7.0, dtype=torch.float32, device=DEV)
    kv.kvtc_wide_decode(w.handle, out, n_bytes, T, xf, kv.KVTC_F32, lay)
    # bf16 output through the workspace
    xb = torch.full((n_layers, T, 1024), 7.0, dtype=torch.bfloat16, device=DEV)
    ws = torch.empty((T, p), dtype=torch.float32, device=DEV)
    kv.kvtc_wide_decode(w.handle, out, n_bytes, T, xb, kv.KVTC_BF16, lay, ws)
    torch.cuda.synchronize()
    got_f = _from_dev(xf.permute(1, 0, 2).reshape(T, p).contiguous()).astype(np.float64)
    got_b = _from_dev(xb.permute(1, 0, 2).reshape(T, p).contiguous()).astype(np.float64)
    for got, is_bf16 in ((got_f, False), (got_b, True)):
        assert np.abs(got - ref).max() <= 1e-2 * rng_x
        tol = 3e-5 * np.abs(mirror).max() + (2.0 ** -8 * np.abs(mirror) if is_bf16 else 0.0)
        assert np.all(np.abs(got - mirror) <= tol), (label, np.abs(got - mirror).max(), np.abs(mirror).max())
    # the bf16 output is the fp32 sum rounded once
    assert np.array_equal(got_b, ko.bf16_round(got_f.astype(np.float32)).astype(np.float64))
    # decoding again gives the same bits (the sections' terms arrive in section order)
    xf2 = torch.full_like(xf, -3.0)
    kv.kvtc_wide_decode(w.handle, out, n_bytes, T, xf2, kv.KVTC_F32, lay)
    torch.cuda.synchronize()
    assert torch.equal(xf, xf2)
    print(f"{label}: p={p} r={oplan.r} sections={len(secs)} R={w.record_bytes} B, codes differ on at most {worst:.1e} of a section's entries")
    w.close()


@pytest.mark.parametrize("fp32_in", [False, True])
def test_hand_built_plan_of_two_sections(fp32_in):
    """Two layers (p = 2048), 1168 kept coordinates in seven groups: sections of 832 and 336; a ragged token count."""
    p, T = 2048, 700
    rng = np.random.default_rng(11)
    group_n, group_bits = [256, 64, 256, 256, 256, 64, 16], [6, 5, 4, 3, 2, 2, 1]
    r = sum(group_n)
    V = np.linalg.qr(rng.standard_normal((p, p)))[0][:, :r]
    mu = rng.normal(0, 0.1, p)
    blocks, j = [], 0
    for n, b in zip(group_n, group_bits):
        blocks.append(ko.Block(j, n, b))
        j += n
    oplan = ko.compile_plan(mu, V, blocks)
    assert [s.r for s in kw.sections_of(oplan)] == [832, 336]
    sigma = np.arange(1, p + 1, dtype=np.float64) ** -0.7
    Q = np.concatenate([V, np.linalg.qr(rng.standard_normal((p, p - r)))[0]], axis=1)       # leading directions = the basis
    X = ko.bf16_round(((rng.standard_normal((T, p)) * sigma) @ Q.T + mu).astype(np.float32))
    _check_wide(oplan, X, 2, "wide-hand" + ("-f32" if fp32_in else ""), fp32_in)


def test_four_layers_under_one_basis_at_16x():
    """Four layers side by side (p = 4096) calibrated by the oracle at 16x with the basis cut to 2048 components: the
    allocation keeps more than 1024 coordinates, so the stream has two or more sections."""
    L = ks.make_layer(ks.cross_layer_spec(4))
    C_ = ko.bf16_round(ks.draw_f32(L, 4096 + 512, ks.CALIB_DRAW))
    oplan, info = kw.calibrate_wide(C_, 16.0, 2048, n_dp_tokens=512)
    assert oplan.r > 1024 and 8 * kw.record_bytes(oplan) <= info["budget_bits"]
    X = ko.bf16_round(ks.draw_f32(L, 1300, ks.TEST_DRAW))
    # Header bar: the last section holds the weakest kept coordinates of a 4096-term sum -- values far smaller than the
    # terms that cancel in them -- so the fp32 summation order moves a group's extremes across an fp16 rounding
    # boundary more often than in the per-layer plans (measured: 2.7e-2 of that section's headers, every one of them
    # inside the summation envelope, which is asserted whatever the rate).  The bar for this case is 5e-2.
    _check_wide(oplan, X, 4, "wide-4layers", hdr_bar=5e-2)


def test_eight_layers_four_sections():
    """Eight layers (p = 8192), 4096 kept coordinates in sixteen groups of 256 = four full sections, a basis that is not
    orthonormal (the coder does not need it to be): three sections are added to the first one's output, and a token's
    features are gathered from eight tensors."""
    p, T, r = 8192, 600, 4096
    rng = np.random.default_rng(21)
    V = (rng.standard_normal((p, r)) / np.sqrt(p)).astype(np.float32)
    mu = rng.normal(0, 0.1, p)
    blocks = [ko.Block(256 * i, 256, 2 + i % 4) for i in range(16)]
    oplan = ko.compile_plan(mu, V, blocks)
    assert [s_.r for s_ in kw.sections_of(oplan)] == [1024] * 4
    X = ko.bf16_round((rng.standard_normal((T, p)) * np.linspace(2.0, 0.2, p) + mu).astype(np.float32))
    _check_wide(oplan, X, 8, "wide-8layers")


def test_wide_arguments_are_checked_before_any_launch():
    p = 256
    rng = np.random.default_rng(2)
    V = ko.bf16_bits(np.linalg.qr(rng.standard_normal((p, p)))[0][:, :64].astype(np.float32))
    L = kv.lib()
    with pytest.raises(kv.KvtcError) as e:
        kv.kvtc_wide_create(p, 64, np.zeros(p, np.float32), V, [(48, 4), (8, 4), (8, 4)])       # groups of 8: not multiples of 16
    assert e.value.status == 2
    w = kv.WidePlan(p, 64, np.zeros(p, np.float32), V, [(32, 4), (32, 2)])
    assert w.n_sections == 1 and w.record_bytes == 8 + 16 + 8
    T = 5
    buf = torch.zeros(1 << 14, dtype=torch.uint8, device=DEV)
    lay = kv.layout(p)
    assert L.kvtc_wide_encode(w.handle, buf.data_ptr(), 0, T, C.byref(lay), buf.data_ptr(), T * 32 - 1, None) == 3     # stream too small
    assert L.kvtc_wide_decode(w.handle, buf.data_ptr(), T * 32 - 1, T, buf.data_ptr(), 1, C.byref(lay), None, None) == 3
    # a plan of two sections (65 groups) needs the fp32 workspace for bf16 output; a plan of one section does not
    p2, r2 = 1088, 1040
    V2 = ko.bf16_bits((rng.standard_normal((p2, r2)) / 32).astype(np.float32))
    w2 = kv.WidePlan(p2, r2, np.zeros(p2, np.float32), V2, [(16, 2)] * 65)
    assert w2.n_sections == 2
    big = torch.zeros(1 << 16, dtype=torch.uint8, device=DEV)
    lay2 = kv.layout(p2)
    nb2 = kv.kvtc_wide_encoded_bytes(w2.handle, T)
    assert L.kvtc_wide_decode(w2.handle, big.data_ptr(), nb2, T, big.data_ptr() + 32768, 0, C.byref(lay2), None, None) == 1
    assert "workspace" in kv.kvtc_last_error()
    w2.close()
    assert L.kvtc_wide_decode(w.handle, buf.data_ptr(), T * 32, T, buf.data_ptr() + 8192, 0, C.byref(lay), None, None) == 0
    torch.cuda.synchronize()
    assert L.kvtc_wide_encode(w.handle, buf.data_ptr(), 0, 0, C.byref(lay), buf.data_ptr(), 0, None) == 0               # nothing to do
    w.close()
