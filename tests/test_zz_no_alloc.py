"""The batched encode that allocates nothing (kvtc_encode_batch_static) against kvtc_encode_batch.

Two calls in a row on the same GPU, the second with a smaller input (fewer plans, fewer and shorter
jobs): each must write exactly the bytes, offsets and status the existing entry point writes for the
same jobs -- the shared work area inside the library keeps the first call's contents, and nothing of
them may leak into the second.  The existing entry point is itself checked against the oracle
elsewhere; one job here is checked against the oracle directly as well.
"""
import numpy as np
import pytest
import torch

import kvtc_oracle as ko
import kvtc_synth as ks
import paper_2511_01815_amd as kv
from test_gpu_parity import DEV, _gpu_plan, _manual, _to_dev, check_stream

pytestmark = pytest.mark.gpu


def _run_both(gplans, pidx, lens, xd, p, dtype):
    n_jobs = len(lens)
    row0 = np.concatenate([[0], np.cumsum(lens)[:-1]]).astype(np.int64)
    jobs_dev = torch.from_numpy(kv.make_jobs(pidx, lens, [int(r) for r in row0]).view(np.uint8)).to(DEV)
    # reference: batch object + offsets + encode
    batch = kv.Batch(gplans)
    offs = torch.zeros(n_jobs + 1, dtype=torch.int64, device=DEV)
    kv.kvtc_offsets(batch.handle, jobs_dev, n_jobs, offs)
    torch.cuda.synchronize()
    cap = int(offs[-1].item())
    ref = torch.full((cap + 64,), 0x5A, dtype=torch.uint8, device=DEV)
    st_ref = torch.zeros(1, dtype=torch.int32, device=DEV)
    kv.kvtc_encode_batch(batch.handle, jobs_dev, n_jobs, xd, dtype, p, offs, ref, cap, st_ref)
    # the call under test: host plan handles, no batch object, offsets returned on request
    out = torch.full((cap + 64,), 0x5A, dtype=torch.uint8, device=DEV)
    offs2 = torch.full((n_jobs + 1,), -1, dtype=torch.int64, device=DEV)
    st = torch.zeros(1, dtype=torch.int32, device=DEV)
    kv.kvtc_encode_batch_static([g.handle for g in gplans], jobs_dev, n_jobs, xd, dtype, p, out, cap, offs2, st)
    torch.cuda.synchronize()
    assert int(st.item()) == int(st_ref.item()) == 0
    assert torch.equal(offs2, offs), "offsets differ from kvtc_offsets"
    assert torch.equal(out, ref), "stream differs from kvtc_encode_batch"
    return out.cpu().numpy(), offs.cpu().numpy(), row0


def test_static_entry_point_matches_encode_batch_twice_in_a_row():
    p = 1024
    oplans = [_manual(p, [(16, 8), (16, 6), (64, 4), (64, 3), (64, 2)], 41),          # 224 coordinates
              _manual(p, [(16, 7), (64, 3)], 42),                                     # 80
              _manual(p, [(64, 6), (256, 3), (256, 2)], 43)]                          # 576: the 8-wave kernels
    gplans = [_gpu_plan(o) for o in oplans]
    rng = np.random.default_rng(44)
    scale = np.arange(1, p + 1, dtype=np.float64) ** -0.8
    Q = np.linalg.qr(rng.standard_normal((p, p)))[0]
    X = ko.bf16_round(((rng.standard_normal((3000, p)) * scale) @ Q + 0.03).astype(np.float32))
    xd = _to_dev(X, kv.KVTC_BF16)
    # first call: three plans, seven jobs (long, short, empty, one token)
    lens1, pidx1 = [700, 40, 0, 513, 1, 300, 65], [0, 1, 2, 2, 0, 1, 2]
    out1, offs1, row01 = _run_both(gplans, pidx1, lens1, xd, p, kv.KVTC_BF16)
    check_stream(oplans[0], X[row01[0]:row01[0] + 700], out1[offs1[0]:offs1[1]].reshape(700, -1), "static-job0")
    # second call, smaller: two plans (other handles, other order), three shorter jobs
    lens2, pidx2 = [130, 5, 64], [1, 0, 1]
    out2, offs2, row02 = _run_both([gplans[2], gplans[1]], pidx2, lens2, xd, p, kv.KVTC_BF16)
    check_stream(oplans[1], X[row02[0]:row02[0] + 130], out2[offs2[0]:offs2[1]].reshape(130, -1), "static-second-job0")
    # fp32 input through the same path
    xf = _to_dev(X, kv.KVTC_F32)
    _run_both(gplans[:2], [0, 1, 0], [200, 70, 3], xf, p, kv.KVTC_F32)


def test_static_entry_point_rejects_what_it_cannot_hold():
    p = 128
    oplan = _manual(p, [(16, 4)], 45)
    g = _gpu_plan(oplan)
    x = torch.zeros((8, p), dtype=torch.bfloat16, device=DEV)
    out = torch.zeros(1024, dtype=torch.uint8, device=DEV)
    st = torch.zeros(1, dtype=torch.int32, device=DEV)
    jobs = torch.from_numpy(kv.make_jobs([0], [8], [0]).view(np.uint8)).to(DEV)
    with pytest.raises(kv.KvtcError) as e:          # more plans than the fixed table holds
        kv.kvtc_encode_batch_static([g.handle] * 65, jobs, 1, x, kv.KVTC_BF16, p, out, 1024, None, st)
    assert e.value.status == 2 and "at most 64" in str(e.value)
    with pytest.raises(kv.KvtcError) as e:          # more jobs than one call takes
        kv.kvtc_encode_batch_static([g.handle], jobs, 1025, x, kv.KVTC_BF16, p, out, 1024, None, st)
    assert e.value.status == 2
    with pytest.raises(kv.KvtcError) as e:
        kv.kvtc_encode_batch_static([g.handle], None, 1, x, kv.KVTC_BF16, p, out, 1024, None, st)
    assert e.value.status == 1
    # capacity is checked on the device as in kvtc_encode_batch: the job is skipped and reported
    kv.kvtc_encode_batch_static([g.handle], jobs, 1, x, kv.KVTC_BF16, p, out, 8 * oplan.record_bytes - 1, None, st)
    torch.cuda.synchronize()
    assert int(st.item()) == 1 and int(out.sum().item()) == 0
    st.zero_()
    kv.kvtc_encode_batch_static([g.handle], jobs, 1, x, kv.KVTC_BF16, p, out, 8 * oplan.record_bytes, None, st)
    torch.cuda.synchronize()
    assert int(st.item()) == 0
