"""The batched path under HIP graph capture: offsets + encode + decode of a ragged batch recorded once and replayed with new
inputs in the same buffers must give what the eager calls give, on every replay (the launches allocate nothing, synchronise
nothing and clear nothing with memsets, so they can be recorded); the entry point that allocates nothing is recorded too."""
import numpy as np
import pytest
import torch

import kvtc_oracle as ko
import paper_2511_01815_amd as kv
from test_gpu_parity import DEV, _gpu_plan, _manual, _to_dev

pytestmark = pytest.mark.gpu


def test_recorded_batch_replays_like_eager_calls():
    p = 1024
    oplans = [_manual(p, [(16, 8), (16, 6), (64, 4), (64, 3), (64, 2)], 51), _manual(p, [(16, 7), (64, 3)], 52)]
    gplans = [_gpu_plan(o) for o in oplans]
    batch = kv.Batch(gplans)
    lens, pidx = [700, 40, 513], [0, 1, 0]
    T = sum(lens)
    row0 = [0, 700, 740]
    n_jobs = 3
    jobs_dev = torch.from_numpy(kv.make_jobs(pidx, lens, row0).view(np.uint8)).to(DEV)
    rng = np.random.default_rng(53)
    scale = np.arange(1, p + 1, dtype=np.float64) ** -0.9
    inputs = [_to_dev(ko.bf16_round((rng.standard_normal((T, p)) * scale + 0.05 * k).astype(np.float32)), kv.KVTC_BF16) for k in range(2)]
    cap = sum(n * gplans[i].record_bytes for n, i in zip(lens, pidx))
    handles = [g.handle for g in gplans]

    def run(x, offs, stream_buf, x_hat, status, out_static, offs_static):
        kv.kvtc_offsets(batch.handle, jobs_dev, n_jobs, offs)
        kv.kvtc_encode_batch(batch.handle, jobs_dev, n_jobs, x, kv.KVTC_BF16, p, offs, stream_buf, cap, status[0:1])
        kv.kvtc_decode_batch(batch.handle, jobs_dev, n_jobs, stream_buf, cap, offs, x_hat, kv.KVTC_BF16, p, status[1:2])
        kv.kvtc_encode_batch_static(handles, jobs_dev, n_jobs, x, kv.KVTC_BF16, p, out_static, cap, offs_static, status[2:3])

    def buffers():
        return (torch.zeros(n_jobs + 1, dtype=torch.int64, device=DEV), torch.zeros(cap, dtype=torch.uint8, device=DEV),
                torch.zeros((T, p), dtype=torch.bfloat16, device=DEV), torch.zeros(3, dtype=torch.int32, device=DEV),
                torch.zeros(cap, dtype=torch.uint8, device=DEV), torch.zeros(n_jobs + 1, dtype=torch.int64, device=DEV))

    # eager results for both inputs
    eager = []
    for x in inputs:
        b = buffers()
        run(x, *b)
        torch.cuda.synchronize()
        assert b[3].cpu().tolist() == [0, 0, 0]
        assert torch.equal(b[1], b[4]) and torch.equal(b[0], b[5])
        eager.append([t.clone() for t in b])
    assert not torch.equal(eager[0][1], eager[1][1])

    # record once: static input and output buffers
    x_static = inputs[0].clone()
    gb = buffers()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm-up on the side stream, as capture requires
        run(x_static, *gb)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run(x_static, *gb)
    # replays, with eager work and synchronisations in between
    for k in (0, 1, 0, 1):
        for t in gb:
            t.zero_()
        x_static.copy_(inputs[k])
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip(gb, eager[k]):
            assert torch.equal(got, ref), f"replay with input {k} differs from the eager calls"
        scratch = buffers()                            # the program's own eager work between replays
        run(inputs[1 - k], *scratch)
        torch.cuda.synchronize()
        assert torch.equal(scratch[1], eager[1 - k][1])
