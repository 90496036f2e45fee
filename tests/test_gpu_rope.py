"""GPU parity of the positional rotation of keys (kvtc_rope) against the float64 oracle, and the whole
key path -- rotation undone, coded, decoded, rotated again -- against the oracle's."""
import numpy as np
import pytest
import torch

import kvtc_oracle as ko
import kvtc_rope as kr
import kvtc_synth as ks
import paper_2511_01815_amd as kv

pytestmark = pytest.mark.gpu
DEV = torch.device("cuda:0")


def _bf16_bits(a32):
    """bf16 bit patterns of float32 values that are exactly representable."""
    return (np.ascontiguousarray(a32, dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)


def _to_dev_bf16(a32):
    return torch.from_numpy(_bf16_bits(a32).view(np.int16)).to(DEV).view(torch.bfloat16)


def _from_dev_bf16(t):
    return (t.view(torch.int16).cpu().numpy().view(np.uint16).astype(np.uint32) << 16).view(np.float32)


@pytest.mark.parametrize("pairing", ["half", "interleaved"])
@pytest.mark.parametrize("inverse", [False, True])
def test_rotation_matches_the_oracle_bf16(pairing, inverse):
    """8 heads x 128 features, 1111 tokens at scattered positions up to 131071 (one at 0): the result, rounded once to
    bf16, must be the oracle's float64 rotation rounded to bf16 -- bit for bit up to the last-bit freedom of sin/cos
    (a result within 1e-15 relative of a bf16 rounding boundary), which may move at most 1e-6 of the entries by one ulp."""
    rng = np.random.default_rng(31)
    H, d, T = 8, 128, 1111
    x = ko.bf16_round((rng.standard_normal((T, H * d)) * np.exp(rng.normal(0, 1.5, (1, H * d)))).astype(np.float32))
    pos = rng.integers(0, 131072, size=T).astype(np.int32)
    pos[0], pos[1] = 0, 131071
    want64 = kr.rope(x, pos, H, d, base=10000.0, pairing=pairing, inverse=inverse)
    want = ko.bf16_round(want64)          # one rounding from float64
    xd = _to_dev_bf16(x).reshape(T, H * d).clone()
    kv.kvtc_rope(xd, kv.KVTC_BF16, T, H, d, H * d, d, torch.from_numpy(pos).to(DEV), 0, 10000.0,
                 kv.ROPE_HALF if pairing == "half" else kv.ROPE_INTERLEAVED, inverse)
    torch.cuda.synchronize()
    got = _from_dev_bf16(xd).reshape(T, H * d)
    np.testing.assert_array_equal(got[0], x[0])                    # position 0: identity
    ne = _bf16_bits(got) != _bf16_bits(want.astype(np.float32))
    assert ne.mean() <= 1e-6, ne.mean()
    if ne.any():
        assert np.abs(_bf16_bits(got)[ne].astype(np.int64) - _bf16_bits(want.astype(np.float32))[ne].astype(np.int64)).max() <= 1


def test_rotation_layouts_positions_and_fp32():
    """fp32 tensors (within one float ulp of the float64 result), consecutive positions from position0, a padded row
    pitch, and the heads-major [H][T][d] layout: all the same rotation."""
    rng = np.random.default_rng(32)
    H, d, T = 4, 64, 300
    x = rng.standard_normal((T, H * d)).astype(np.float32)
    pos0 = 70000
    want = kr.rope(x, np.arange(T) + pos0, H, d, base=500000.0, pairing="half")
    # token-major with a padded pitch
    ld = H * d + 32
    xd = torch.zeros((T, ld), dtype=torch.float32, device=DEV)
    xd[:, :H * d] = torch.from_numpy(x).to(DEV)
    kv.kvtc_rope(xd, kv.KVTC_F32, T, H, d, ld, d, None, pos0, 500000.0, kv.ROPE_HALF, False)
    torch.cuda.synchronize()
    got = xd.cpu().numpy()
    assert np.all(got[:, H * d:] == 0.0)                                           # padding untouched
    np.testing.assert_allclose(got[:, :H * d], want, rtol=2.0 ** -23, atol=1e-30)
    # heads-major
    xh = torch.from_numpy(kr.heads_first(x, H, d)).to(DEV).contiguous()           # [H, T, d]
    kv.kvtc_rope(xh, kv.KVTC_F32, T, H, d, d, T * d, None, pos0, 500000.0, kv.ROPE_HALF, False)
    torch.cuda.synchronize()
    np.testing.assert_allclose(kr.tokens_first(xh.cpu().numpy()), want, rtol=2.0 ** -23, atol=1e-30)
    # undo after redo returns the input to float accuracy
    kv.kvtc_rope(xh, kv.KVTC_F32, T, H, d, d, T * d, None, pos0, 500000.0, kv.ROPE_HALF, True)
    torch.cuda.synchronize()
    np.testing.assert_allclose(kr.tokens_first(xh.cpu().numpy()), x, rtol=0, atol=2e-6 * np.abs(x).max())


def test_key_path_rotation_undone_coded_decoded_rotated_again():
    """Keys of config 2's shape with the rotation applied (what a cache holds): kvtc_rope(inverse) + kvtc_encode must
    give the stream the oracle gives for the un-rotated keys (its bars for codes and headers), and kvtc_decode +
    kvtc_rope must give the oracle's decode rotated by the oracle, within the coder's reconstruction bar."""
    from test_gpu_parity import check_stream
    from paper_2511_01815_amd import bundles as kb
    H, d, T = 8, 128, 2000
    b = kb.load_plan_arrays("c2_K_cr16")
    L = ks.make_layer(ks.layer_spec("c2", 0, 0))
    k_plain = ko.bf16_round(ks.draw_f32(L, T, ks.TEST_DRAW))                      # keys before the rotation
    pos = np.arange(T) + 5000
    k_rot = ko.bf16_round(kr.rope(k_plain, pos, H, d).astype(np.float32))         # what the cache holds (bf16)
    # oracle path: undo in float64, round once to bf16 (the coder's input type), encode
    k_undone = ko.bf16_round(kr.rope(k_rot, pos, H, d, inverse=True).astype(np.float32))
    groups = list(zip(b["group_n"].tolist(), b["group_bits"].tolist()))
    oplan = ko.plan_from_arrays(b["mu32"], b["v_bits"], b["group_n"], b["group_bits"])
    plan = kv.Plan(1024, b["v_bits"].shape[1], b["mu32"], b["v_bits"], groups)
    xd = _to_dev_bf16(k_rot).reshape(T, H * d).clone()
    kv.kvtc_rope(xd, kv.KVTC_BF16, T, H, d, H * d, d, None, 5000, 10000.0, kv.ROPE_HALF, True)
    torch.cuda.synchronize()
    undone_gpu = _from_dev_bf16(xd).reshape(T, H * d)
    assert (_bf16_bits(undone_gpu) != _bf16_bits(k_undone)).mean() <= 1e-6
    out = torch.zeros(T * plan.record_bytes, dtype=torch.uint8, device=DEV)
    kv.kvtc_encode(plan.handle, xd, kv.KVTC_BF16, T, H * d, out, out.numel())
    xh = torch.empty_like(xd)
    kv.kvtc_decode(plan.handle, out, out.numel(), T, xh, kv.KVTC_BF16, H * d)
    kv.kvtc_rope(xh, kv.KVTC_BF16, T, H, d, H * d, d, None, 5000, 10000.0, kv.ROPE_HALF, False)
    torch.cuda.synchronize()
    recs = out.cpu().numpy().reshape(T, -1)
    check_stream(oplan, undone_gpu, recs, "keys-rope")
    want = kr.rope(ko.decode(oplan, recs), pos, H, d)                             # oracle decode, rotated again by the oracle
    got = _from_dev_bf16(xh).reshape(T, H * d)
    rng_x = float(k_rot.max() - k_rot.min())
    assert np.abs(got - want).max() <= 1e-2 * rng_x
    # and the point of it all: the round trip is as close to the cached keys as the coder is to the un-rotated ones
    rel = np.linalg.norm(got - k_rot) / np.linalg.norm(k_rot - k_rot.mean(0))
    assert rel < 0.3, rel
