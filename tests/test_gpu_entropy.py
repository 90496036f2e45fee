"""GPU tests of the lossless stage over the packed records (paper, Section "Entropy coding"): kvtc_entropy_* against
oracle/kvtc_entropy.py byte for byte, and exact round trips at full size."""
import ctypes as C

import numpy as np
import pytest
import torch

import kvtc_entropy as ke
import kvtc_oracle as ko
import kvtc_synth as ks
import paper_2511_01815_amd as kv
from paper_2511_01815_amd import bundles as kb

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _records(bundle, T, draw):
    b = kb.load_plan_arrays(bundle)
    oplan = ko.plan_from_arrays(b["mu32"], b["v_bits"], b["group_n"], b["group_bits"])
    L = ks.make_layer(ks.layer_spec("c2", 0, 0 if "_K_" in bundle else 1))
    return ko.encode(oplan, ko.bf16_round(ks.draw_f32(L, T, draw)))


def _gpu_encode(tab, rec, cap=None):
    T, R = rec.shape
    bound = kv.kvtc_entropy_bound(tab.handle, T)
    assert bound == ke.bound_bytes(T, R)
    cap = bound if cap is None else cap
    rd = torch.from_numpy(rec).to(DEV)
    out = torch.full((bound + 64,), 0xA5, dtype=torch.uint8, device=DEV)
    n = torch.zeros(1, dtype=torch.int64, device=DEV)
    kv.kvtc_entropy_encode(tab.handle, rd, T, out, cap, n)
    torch.cuda.synchronize()
    return out.cpu().numpy(), int(n.item()), bound


def _gpu_decode(tab, blob, T, R):
    bd = torch.from_numpy(np.frombuffer(blob, dtype=np.uint8).copy()).to(DEV)
    got = torch.full((T * R + 64,), 0x5A, dtype=torch.uint8, device=DEV)
    kv.kvtc_entropy_decode(tab.handle, bd, bd.numel(), T, got, T * R)
    torch.cuda.synchronize()
    g = got.cpu().numpy()
    assert np.all(g[T * R:] == 0x5A), "wrote past the records"
    return g[:T * R].reshape(T, R)


@pytest.mark.parametrize("bundle,T", [("c2_K_cr16", 1300), ("c2_V_cr20", 777), ("c2_K_cr16", 1), ("c2_K_cr16", 64), ("c2_V_cr16", 65),
                                      ("c2_K_cr8", 200)])
def test_container_equals_the_oracles_byte_for_byte(bundle, T):
    """Records of a calibrated plan (128, 100 and 256 bytes a token); tables from another draw's records, so the coded
    draw holds byte values the tables never saw."""
    rec = _records(bundle, T, ks.TEST_DRAW)
    lengths = ke.calibrate_tables(_records(bundle, 1024, ks.CALIB_DRAW))
    R = rec.shape[1]
    tab = kv.EntropyTables(R, lengths)
    ref = ke.encode(rec, lengths)
    out, n, bound = _gpu_encode(tab, rec)
    assert n == len(ref)
    assert out[:n].tobytes() == ref
    assert np.all(out[bound:] == 0xA5), "wrote past the bound"
    assert np.array_equal(_gpu_decode(tab, ref, T, R), rec)            # the oracle's container
    assert np.array_equal(_gpu_decode(tab, out[:n].tobytes(), T, R), rec)
    assert np.array_equal(ke.decode(out[:n].tobytes(), T, R, lengths), rec)
    print(f"{bundle} T={T}: {T * R} -> {n} bytes, ratio {T * R / n:.3f}")
    tab.close()


def test_short_buffer_is_reported_not_overrun():
    rec = _records("c2_K_cr16", 300, ks.TEST_DRAW)
    lengths = ke.calibrate_tables(rec)
    tab = kv.EntropyTables(128, lengths)
    ref = ke.encode(rec, lengths)
    cap = len(ref) - 4000                                  # the last chunk(s) do not fit
    out, n, bound = _gpu_encode(tab, rec, cap=cap)
    assert n == len(ref) > cap                             # the needed size is reported
    assert np.all(out[cap:] == 0xA5), "wrote past out_cap"
    n_chunks = (300 + 63) // 64
    hdr = 4 * (n_chunks + 1) + 128 * n_chunks
    assert out[:hdr].tobytes() == ref[:hdr]                # the directory is complete
    off = np.frombuffer(ref, dtype="<u4", count=n_chunks + 1)
    for c in range(n_chunks):                              # chunks that fit are written, the others untouched
        a, b = hdr + int(off[c]), hdr + int(off[c + 1])
        if b <= cap:
            assert out[a:b].tobytes() == ref[a:b]
        else:
            assert np.all(out[a:min(b, cap)] == 0xA5)
    tab.close()


def test_entropy_arguments_are_checked_before_any_launch():
    L = kv.lib()
    good = np.full((8, 256), 8, dtype=np.uint8)
    h = C.c_void_p()
    assert L.kvtc_entropy_create(C.byref(h), 6, 1, good.ctypes.data, None) == 1            # not a multiple of 4
    assert L.kvtc_entropy_create(C.byref(h), 580, 1, good.ctypes.data, None) == 2          # above the limit
    bad = good.copy(); bad[3, 7] = 0
    assert L.kvtc_entropy_create(C.byref(h), 8, 1, bad.ctypes.data, None) == 1             # a length of zero
    bad = good.copy(); bad[2, :3] = 1
    assert L.kvtc_entropy_create(C.byref(h), 8, 1, bad.ctypes.data, None) == 1             # Kraft sum above one
    assert "prefix code" in kv.kvtc_last_error()
    tab = kv.EntropyTables(8, good)
    buf = torch.zeros(4096, dtype=torch.uint8, device=DEV)
    n = torch.zeros(1, dtype=torch.int64, device=DEV)
    p = buf.data_ptr()
    assert L.kvtc_entropy_encode(tab.handle, 0, p, 10, p + 1024, 8, n.data_ptr(), None) == 3     # no room for the directory
    assert L.kvtc_entropy_encode(tab.handle, 0, p + 2, 10, p + 1024, 2048, n.data_ptr(), None) == 1
    assert L.kvtc_entropy_encode(tab.handle, 0, p, 10, p + 1024, 2048, None, None) == 1
    assert L.kvtc_entropy_decode(tab.handle, 0, p, 8, 10, p + 1024, 80, None) == 3               # container shorter than its directory
    assert L.kvtc_entropy_decode(tab.handle, 0, p, 1024, 10, p + 1024, 79, None) == 3
    assert L.kvtc_entropy_decode(tab.handle, 0, p, 1024, 0, None, 0, None) == 0
    assert L.kvtc_entropy_encode(tab.handle, 1, p, 10, p + 1024, 2048, n.data_ptr(), None) == 1             # one table set only
    assert L.kvtc_entropy_create(C.byref(h), 8, 0, good.ctypes.data, None) == 1
    # a container of zeros (a damaged one: every offset zero) decodes to something without a fault
    assert L.kvtc_entropy_decode(tab.handle, 0, p, 1024, 10, p + 2048, 80, None) == 0
    torch.cuda.synchronize()
    tab.close()


def test_full_size_round_trip_of_a_gpu_coded_tensor():
    """32768 tokens coded by the GPU coder at 16x, then through the lossless stage and back: exact; the container's
    length equals directory + padded chunk strings; the ratio is printed."""
    b = kb.load_plan_arrays("c2_K_cr16")
    groups = list(zip(b["group_n"].tolist(), b["group_bits"].tolist()))
    plan = kv.Plan(int(b["mu32"].shape[0]), int(b["v_bits"].shape[1]), b["mu32"], b["v_bits"], groups)
    R = plan.record_bytes
    Lr = ks.make_layer(ks.layer_spec("c2", 0, 0))
    T = 32768
    x = ks.draw_bf16_torch(Lr, T, 5, DEV)
    rec = torch.empty(T * R, dtype=torch.uint8, device=DEV)
    kv.kvtc_encode(plan.handle, x, kv.KVTC_BF16, T, 1024, rec, T * R)
    xc = ks.draw_bf16_torch(Lr, 4096, 6, DEV)
    rec_c = torch.empty(4096 * R, dtype=torch.uint8, device=DEV)
    kv.kvtc_encode(plan.handle, xc, kv.KVTC_BF16, 4096, 1024, rec_c, 4096 * R)
    torch.cuda.synchronize()
    lengths = ke.calibrate_tables(rec_c.cpu().numpy().reshape(4096, R))
    tab = kv.EntropyTables(R, lengths)
    bound = kv.kvtc_entropy_bound(tab.handle, T)
    out = torch.zeros(bound, dtype=torch.uint8, device=DEV)
    n = torch.zeros(1, dtype=torch.int64, device=DEV)
    kv.kvtc_entropy_encode(tab.handle, rec, T, out, bound, n)
    torch.cuda.synchronize()
    nb = int(n.item())
    back = torch.zeros_like(rec)
    kv.kvtc_entropy_decode(tab.handle, out, nb, T, back, T * R)
    torch.cuda.synchronize()
    assert torch.equal(back, rec)
    o = out[:nb].cpu().numpy()
    n_chunks = T // 64
    off = np.frombuffer(o.tobytes(), dtype="<u4", count=n_chunks + 1)
    lb = np.frombuffer(o.tobytes(), dtype="<u2", count=T, offset=4 * (n_chunks + 1)).astype(np.int64)
    assert nb == 4 * (n_chunks + 1) + 2 * T + int(off[-1])
    assert np.array_equal(np.diff(off.astype(np.int64)), (lb.reshape(n_chunks, 64).sum(axis=1) + 31) // 32 * 4)
    # the lengths are what the tables say for these bytes (sampled tokens)
    rh = rec.cpu().numpy().reshape(T, R)
    for t in (0, 1, 63, 64, 12345, T - 1):
        assert lb[t] == sum(int(lengths[k, rh[t, k]]) for k in range(R))
    print(f"32768 tokens at 16x: {T * R} -> {nb} bytes, lossless ratio {T * R / nb:.3f} (total {2048 * T / nb:.2f}x)")
    tab.close()
    plan.close()


def test_batched_jobs_equal_single_calls_and_bad_jobs_are_left_alone():
    """Four tensors in one call: two table sets, ragged lengths, containers at ragged (4-byte aligned) offsets; a fifth job
    names a table set that does not exist and a sixth is longer than max_tokens: both are reported and nothing of theirs
    is touched."""
    recs = [_records("c2_K_cr16", 300, ks.TEST_DRAW), _records("c2_V_cr16", 129, ks.TEST_DRAW),
            _records("c2_K_cr16", 64, 7), _records("c2_V_cr16", 1, 8)]
    tabs = np.stack([ke.calibrate_tables(_records("c2_K_cr16", 512, ks.CALIB_DRAW)), ke.calibrate_tables(_records("c2_V_cr16", 512, ks.CALIB_DRAW))])
    table_of = [0, 1, 0, 1]
    R = 128
    tab = kv.EntropyTables(R, tabs)
    refs = [ke.encode(r, tabs[t]) for r, t in zip(recs, table_of)]
    n_tok = [r.shape[0] for r in recs] + [10, 400]
    rec_off, pos = [], 0
    for n in n_tok:
        rec_off.append(pos)
        pos += n * R
    rec_all = np.full(pos, 0x11, dtype=np.uint8)
    for r, o in zip(recs, rec_off):
        rec_all[o:o + r.size] = r.reshape(-1)
    caps = [ke.bound_bytes(n, R) + 4 * i for i, n in enumerate(n_tok)]        # ragged room
    cod_off = np.concatenate([[0], np.cumsum(caps)[:-1]]).tolist()
    total = int(sum(caps))
    jobs = kv.make_entropy_jobs(table_of + [5, 0], n_tok, rec_off, cod_off, caps)
    jd = torch.from_numpy(jobs.view(np.uint8)).to(DEV)
    rd = torch.from_numpy(rec_all).to(DEV)
    coded = torch.full((total + 64,), 0xA5, dtype=torch.uint8, device=DEV)
    sizes = torch.zeros(6, dtype=torch.int64, device=DEV)
    kv.kvtc_entropy_encode_batch(tab.handle, jd, 6, 300, rd, rec_all.size, coded, total, sizes)
    torch.cuda.synchronize()
    c = coded.cpu().numpy()
    sz = sizes.cpu().numpy().view(np.uint64)
    assert sz[4] == sz[5] == np.uint64(2 ** 64 - 1)
    assert np.all(c[cod_off[4]:] == 0xA5), "a rejected job's room (or the guard) was written"
    for i, ref in enumerate(refs):
        assert int(sz[i]) == len(ref)
        assert c[cod_off[i]:cod_off[i] + len(ref)].tobytes() == ref
        assert np.all(c[cod_off[i] + ke.bound_bytes(n_tok[i], R):cod_off[i] + caps[i]] == 0xA5)
    # decode: the containers' true lengths as coded_cap
    jobs2 = kv.make_entropy_jobs(table_of + [5, 0], n_tok, rec_off, cod_off, [len(r) for r in refs] + [caps[4], caps[5]])
    jd2 = torch.from_numpy(jobs2.view(np.uint8)).to(DEV)
    back = torch.full((rec_all.size + 64,), 0x5A, dtype=torch.uint8, device=DEV)
    kv.kvtc_entropy_decode_batch(tab.handle, jd2, 6, 300, coded, total, back, rec_all.size)
    torch.cuda.synchronize()
    b = back.cpu().numpy()
    for r, o in zip(recs, rec_off):
        assert np.array_equal(b[o:o + r.size], r.reshape(-1))
    assert np.all(b[rec_off[4]:] == 0x5A), "a rejected job's records (or the guard) were written"
    tab.close()


@pytest.mark.parametrize("R,T", [(576, 130), (544, 64), (4, 1000), (36, 4097)])
def test_record_sizes_at_the_limits(R, T):
    """The largest record the stage takes (576 bytes: one wave per workgroup, 129 KB of LDS), the full-rank plans' 544, the
    smallest (4) and a size that is no power of two; synthetic bytes with a different skew at every position, tables from
    half of them."""
    rng = np.random.default_rng(R + T)
    rec = np.stack([np.minimum(255, rng.geometric(1.0 / (2 + (7 * k) % 90), T) - 1) for k in range(R)], axis=1).astype(np.uint8)
    lengths = ke.calibrate_tables(rec[:T // 2])
    tab = kv.EntropyTables(R, lengths)
    ref = ke.encode(rec, lengths)
    out, n, bound = _gpu_encode(tab, rec)
    assert n == len(ref) and out[:n].tobytes() == ref
    assert np.all(out[bound:] == 0xA5)
    assert np.array_equal(_gpu_decode(tab, ref, T, R), rec)
    tab.close()
