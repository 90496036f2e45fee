"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, rejects bad
arguments before touching the GPU, and its scalar quantiser numerics (compiled from the same
header the kernels use) agree bit for bit with the oracle's."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import kvtc_oracle as ko
import paper_2511_01815_amd as kv

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    inc = os.path.join(ROOT, "include")
    headers = sorted(f for f in os.listdir(inc) if f.endswith(".h"))
    assert headers == ["kvtc.h", "kvtc_probe.h", "kvtc_test_hooks.h"]
    hdr = "\n".join(open(os.path.join(inc, f)).read() for f in headers)
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = sorted(set(re.findall(r"\b(kvtc_[a-z0-9_]+)\s*\(", hdr)))
    assert {"kvtc_plan_create", "kvtc_encode", "kvtc_decode", "kvtc_offsets", "kvtc_encode_batch",
            "kvtc_decode_batch", "kvtc_batch_create", "kvtc_last_error"} <= set(names)
    L = kv.lib()
    for n in names:
        assert hasattr(L, n), n


def _probe():
    rng = np.random.default_rng(2)
    tab = np.arange(65536, dtype=np.uint32).astype(np.uint16).view(np.float16)
    tab = tab[np.isfinite(tab)].astype(np.float32)
    xs = [rng.standard_normal(3000) * s for s in (1e-9, 1e-7, 3e-5, 1e-2, 1.0, 500.0, 8e4)]
    xs += [tab[::7], np.nextafter(tab[::11], np.float32(np.inf)), np.nextafter(tab[::13], np.float32(-np.inf))]
    xs.append(np.array([0.0, -0.0, 65504.0, -65504.0, 65519.9, 1e30, -1e30, np.inf, -np.inf, 5.9e-8, -2.9e-8, 2.98e-8]))
    return np.concatenate(xs).astype(np.float32)


def test_directed_fp16_rounding_matches_oracle_bits():
    L = kv.lib()
    x = _probe()
    want_dn = ko.fp16_floor(x).view(np.uint16)
    want_up = ko.fp16_ceil(x).view(np.uint16)
    got_dn = np.array([L.kvtc_host_f16_round_down(float(v)) for v in x], dtype=np.uint16)
    got_up = np.array([L.kvtc_host_f16_round_up(float(v)) for v in x], dtype=np.uint16)
    np.testing.assert_array_equal(got_dn, want_dn)
    np.testing.assert_array_equal(got_up, want_up)


@pytest.mark.parametrize("bits", [1, 2, 3, 4, 6, 8, 11, 16])
def test_header_and_code_decision_match_oracle(bits):
    L = kv.lib()
    rng = np.random.default_rng(bits)
    d = (rng.standard_normal((400, 16)) * rng.choice([1e-6, 1e-3, 0.3, 5.0, 900.0], (400, 1))).astype(np.float32)
    d[:5] = d[:5, :1]                      # zero-range groups
    d[5, :] = [70000.0, -70000.0] + [1.0] * 14   # saturating
    shift, scale, codes = ko.quantise_group(d, bits)
    sh = C.c_uint16()
    sc = C.c_uint16()
    for t in range(d.shape[0]):
        L.kvtc_host_group_header(float(d[t].min()), float(d[t].max()), bits, C.byref(sh), C.byref(sc))
        assert sh.value == int(shift.view(np.uint16)[t]) and sc.value == int(scale.view(np.uint16)[t]), t
        got = [L.kvtc_host_code(float(v), sh.value, sc.value, bits) for v in d[t]]
        assert got == codes[t].tolist(), t


def test_argument_errors_need_no_gpu():
    L = kv.lib()
    p, r = 64, 16
    mu = np.zeros(p, dtype=np.float32)
    v = np.zeros((p, r), dtype=np.uint16)
    with pytest.raises(kv.KvtcError) as e:
        kv.kvtc_plan_create(60, 16, np.zeros(60, np.float32), np.zeros((60, 16), np.uint16), [(16, 4)], stream=0)
    assert e.value.status == 1 and "multiple of 64" in str(e.value)
    with pytest.raises(kv.KvtcError) as e:
        kv.kvtc_plan_create(p, r, mu, v, [(16, 17)], stream=0)
    assert e.value.status == 1
    with pytest.raises(kv.KvtcError) as e:
        kv.kvtc_plan_create(p, r, mu, v, [(16, 0)], stream=0)
    assert e.value.status == 1
    with pytest.raises(kv.KvtcError) as e:
        kv.kvtc_plan_create(p, 32, mu, np.zeros((p, 32), np.uint16), [(16, 4)], stream=0)
    assert e.value.status == 1 and "sum" in str(e.value)
    with pytest.raises(kv.KvtcError) as e:          # group of 1: valid format, not served by the kernels
        kv.kvtc_plan_create(p, 17, mu, np.zeros((p, 17), np.uint16), [(16, 4), (1, 8)], stream=0)
    assert e.value.status == 2
    with pytest.raises(kv.KvtcError) as e:          # record too large for on-chip staging
        kv.kvtc_plan_create(1024, 1024, np.zeros(1024, np.float32), np.zeros((1024, 1024), np.uint16),
                            [(16, 16)] * 64, stream=0)
    assert e.value.status == 2
    # null handles
    assert L.kvtc_record_bytes(None) == 0 and L.kvtc_encoded_bytes(None, 5) == 0
    L.kvtc_plan_destroy(None)
    L.kvtc_batch_destroy(None)
    assert L.kvtc_encode(None, None, 0, 1, 64, None, 0, None) == 1
    assert L.kvtc_decode(None, None, 0, 1, None, 0, 64, None) == 1
    assert "null plan" in kv.kvtc_last_error()
    out = C.c_void_p()
    assert L.kvtc_batch_create(C.byref(out), None, 0, None) == 1


def test_job_struct_layout():
    assert kv.JOB_DTYPE.itemsize == 16
    j = kv.make_jobs([0, 1], [5, 7], [0, 5])
    assert j.tobytes() == (b"\x00\x00\x00\x00\x05\x00\x00\x00" + (0).to_bytes(8, "little") +
                           b"\x01\x00\x00\x00\x07\x00\x00\x00" + (5).to_bytes(8, "little"))


# ---- sinks / sliding window (host-only entry points) ------------------------------------------

def test_window_split_equals_the_replay():
    import kvtc_window as kw
    for s, w, c in [(4, 128, 16), (0, 128, 16), (4, 64, 64), (1, 5, 2), (3, 7, 1), (16, 256, 32)]:
        for ctx in list(range(0, 3 * w + 2 * s + 9)) + [8192, 131072, 10**9 + 7][: (3 if c > 1 else 0)]:
            if ctx > 10**6:
                # the replay is linear in ctx: check the closed form's invariants instead
                n_sink, n_coded, n_window = kv.kvtc_window_split(ctx, s, w, c)
                assert n_sink == s and n_coded % c == 0 and w - c <= n_window < w and n_sink + n_coded + n_window == ctx
            else:
                assert kv.kvtc_window_split(ctx, s, w, c) == kw.window_split(ctx, s, w, c), (ctx, s, w, c)


def test_window_split_and_ratio_reject_and_agree():
    import kvtc_window as kw
    for bad in [(-1, 4, 128, 16), (10, -1, 128, 16), (10, 4, 8, 0), (10, 4, 8, 9)]:
        with pytest.raises(kv.KvtcError) as e:
            kv.kvtc_window_split(*bad)
        assert e.value.status == 1
    st = kv.lib().kvtc_window_split(10, 4, 128, 16, None)
    assert st == 1 and "null" in kv.kvtc_last_error()
    for ctx, w, s, cr in [(8192, 128, 4, 20.0), (1000, 112, 4, 16.0), (131072, 127, 0, 40.0), (300, 128, 4, 8.0)]:
        assert kv.kvtc_cr_with_window(ctx, w, s, cr) == pytest.approx(kw.cr_with_window(ctx, w, s, cr), rel=1e-15)


def test_fp8_entry_points_reject_bad_arguments_before_any_launch():
    L = kv.lib()
    buf = np.zeros(4096, dtype=np.uint8)
    ptr = buf.ctypes.data & ~15
    assert L.kvtc_fp8_pack(None, 0, 0, 1024, 1024, None, 0, None) == 0                 # nothing to do
    assert L.kvtc_fp8_pack(None, 0, 4, 1024, 1024, ptr, 4096, None) == 1               # null input
    assert L.kvtc_fp8_pack(ptr, 0, 4, 1024, 512, ptr, 4096, None) == 1                 # pitch below p
    assert L.kvtc_fp8_pack(ptr, 7, 4, 1024, 1024, ptr, 4096, None) == 1                # unknown dtype
    assert L.kvtc_fp8_pack(ptr + 2, 0, 4, 1024, 1024, ptr, 4096, None) == 1            # misaligned
    assert L.kvtc_fp8_pack(ptr, 0, 4, 1024, 1024, ptr, 4095, None) == 3                # output too small
    assert L.kvtc_fp8_unpack(ptr, 4095, 4, 1024, ptr, 0, 1024, None) == 3
    assert L.kvtc_fp8_unpack(ptr, 4096, -1, 1024, ptr, 0, 1024, None) == 1
    assert L.kvtc_offsets_append(None, None, 0, None, None, None, None) == 1


def test_rope_rejects_bad_arguments_before_any_launch():
    L = kv.lib()
    buf = np.zeros(4096, dtype=np.uint8)
    ptr = buf.ctypes.data & ~15
    ok = dict(dtype=0, T=4, H=8, d=128, ts=1024, hs=128)

    def call(x=ptr, dtype=0, T=4, H=8, d=128, ts=1024, hs=128, base=10000.0, pairing=0, inverse=0):
        return L.kvtc_rope(x, dtype, T, H, d, ts, hs, None, 0, base, pairing, inverse, None)

    assert call(x=None, T=0) == 0                      # nothing to do
    assert call(x=None) == 1                           # null buffer
    assert call(dtype=5) == 1
    assert call(d=127) == 1 and call(d=0) == 1 and call(d=258) == 1
    assert call(H=0) == 1
    assert call(ts=1023) == 1                          # a token's heads would run into the next token
    assert call(ts=128, hs=3 * 128) == 1               # heads-major, but a head's slab is shorter than its tokens
    assert call(base=0.0) == 1 and call(base=float("inf")) == 1
    assert call(pairing=2) == 1 and call(inverse=2) == 1
    assert call(T=-1) == 1
    assert "kvtc_rope" in kv.kvtc_last_error()
    del ok


def test_later_entry_points_reject_bad_arguments_before_any_launch():
    """Sectioned plans, the lossless stage and the calibration passes: every argument error below is found on the host,
    before any allocation or launch, so it needs no GPU."""
    L = kv.lib()
    h = C.c_void_p()
    mu = np.zeros(256, np.float32)
    V = np.zeros((256, 64), np.uint16)
    grp = (kv.binding._Group * 2)(kv.binding._Group(32, 4, 0), kv.binding._Group(16, 4, 0))      # sums to 48, not 64
    assert L.kvtc_wide_create(C.byref(h), 256, 64, mu.ctypes.data, V.ctypes.data, 2, C.cast(grp, C.c_void_p), None) == 1
    assert "sum to" in kv.kvtc_last_error()
    assert L.kvtc_wide_create(C.byref(h), 250, 64, mu.ctypes.data, V.ctypes.data, 2, C.cast(grp, C.c_void_p), None) == 1
    assert L.kvtc_wide_create(C.byref(h), 256, 64, None, V.ctypes.data, 2, C.cast(grp, C.c_void_p), None) == 1
    big = (kv.binding._Group * 1)(kv.binding._Group(2048, 4, 0))
    assert L.kvtc_wide_create(C.byref(h), 4096, 2048, mu.ctypes.data, V.ctypes.data, 1, C.cast(big, C.c_void_p), None) == 1
    assert L.kvtc_wide_sections(None) == 0 and L.kvtc_wide_record_bytes(None) == 0 and L.kvtc_wide_encoded_bytes(None, 5) == 0
    lay = kv.layout(256)
    assert L.kvtc_wide_encode(None, 16, 0, 4, C.byref(lay), 16, 64, None) == 1
    assert L.kvtc_wide_decode(None, 16, 64, 4, 16, 0, C.byref(lay), None, None) == 1
    # lossless stage
    good = np.full((8, 256), 8, dtype=np.uint8)
    assert L.kvtc_entropy_create(C.byref(h), 6, 1, good.ctypes.data, None) == 1
    assert L.kvtc_entropy_create(C.byref(h), 580, 1, good.ctypes.data, None) == 2
    assert L.kvtc_entropy_create(C.byref(h), 8, 0, good.ctypes.data, None) == 1
    assert L.kvtc_entropy_create(C.byref(h), 8, 1, None, None) == 1
    bad = good.copy()
    bad[1, :2] = 1
    assert L.kvtc_entropy_create(C.byref(h), 8, 1, bad.ctypes.data, None) == 1 and "prefix code" in kv.kvtc_last_error()
    assert L.kvtc_entropy_bound(None, 100) == 0
    assert L.kvtc_entropy_encode(None, 0, 16, 4, 16, 64, 16, None) == 1
    assert L.kvtc_entropy_decode(None, 0, 16, 64, 4, 16, 64, None) == 1
    assert L.kvtc_entropy_encode_batch(None, 16, 1, 4, 16, 64, 16, 64, 16, None) == 1
    assert L.kvtc_entropy_decode_batch(None, 16, 1, 4, 16, 64, 16, 64, None) == 1
    assert kv.ENTROPY_JOB_DTYPE.itemsize == 32
    # calibration passes
    assert L.kvtc_calib_block_errors(16, 4, 64, 16, 1, 9, 16, None) == 1
    assert L.kvtc_calib_block_errors(None, 4, 64, 16, 1, 8, 16, None) == 1
    assert L.kvtc_calib_block_errors(16, 4, 64, 16, 1, 8, 20, None) == 1          # output not 8-byte aligned
    assert L.kvtc_calib_block_errors(16, 4, 64, 16, 0, 8, 16, None) == 0          # no blocks: nothing to do
    assert L.kvtc_calib_moments(16, 0, 4, 100, C.byref(lay), 16, 16, None) == 1
    assert L.kvtc_calib_moments(16, 0, 4, 256, None, 16, 16, None) == 1
    assert L.kvtc_calib_moments(16, 0, 4, 256, C.byref(kv.layout(128)), 16, 16, None) == 1
    assert L.kvtc_calib_moments(16, 0, 4, 256, C.byref(lay), 16, 20, None) == 1


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""
