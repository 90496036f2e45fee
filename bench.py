#!/usr/bin/env python3
"""Throughput of the KVTC hot path on one MI355X.

A step = one pass of the whole path over one batch: stream offsets (GPU prefix sum),
fused encode of every tensor (one launch), fused decode of every tensor (one launch).
Workload (default): the Llama-3.1-8B-shaped layer of the second BASELINE configuration
(K and V, 32768 tokens x 1024 features bf16, 16x plans from the calibration bundles),
replicated as 32 independent seeded draws so that one batch is the 4 GiB of a full
8B-shaped 32k-token cache and cannot sit in the 256 MB Infinity Cache.
Inputs are synthetic, generated on the GPU and resident in HBM before timing starts.

Prints ONE JSON line.  Roofline: a launch moves 2p + R algorithmic bytes and does 2 p r bf16
matrix-core flops per token; the bound is the larger of bytes / 8 TB/s and flops / 2.5 PFLOP/s, and
the fraction is quoted for the slower of the two kernels from its HIP-event duration.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0           # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16, published


def load_bundle(name: str):
    import numpy as np
    path = os.path.join(ROOT, "paper_2511_01815_amd", "plans", name + ".npz")
    z = np.load(path)
    return dict(mu32=z["mu32"], v_bits=z["v_bits"], group_n=z["group_n"], group_bits=z["group_bits"])


def cpu_baseline(bundles, x_host_by_kv, p):
    """The oracle's encode + decode, timed as it stands on this machine's host cores."""
    import numpy as np
    sys.path.insert(0, os.path.join(ROOT, "oracle"))
    import kvtc_oracle as ko
    try:
        from threadpoolctl import threadpool_info
        threads = max([int(i.get("num_threads", 1)) for i in threadpool_info()] or [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    best_e = best_d = 1e30
    raw = 0
    plans = [ko.plan_from_arrays(b["mu32"], b["v_bits"], b["group_n"], b["group_bits"]) for b in bundles]
    for _ in range(2):
        te = td = 0.0
        raw = 0
        for plan, x in zip(plans, x_host_by_kv):
            t0 = time.perf_counter()
            rec = ko.encode(plan, x)
            t1 = time.perf_counter()
            ko.decode(plan, rec, out="bf16")
            t2 = time.perf_counter()
            te += t1 - t0
            td += t2 - t1
            raw += x.shape[0] * p * 2
        best_e, best_d = min(best_e, te), min(best_d, td)
    return dict(value=2 * raw / (best_e + best_d) / 1e9, unit="GB/s", cores=threads, kind="oracle",
                sample=f"K and V of one layer, {x_host_by_kv[0].shape[0]} tokens each ({raw / 2**20:.0f} MiB raw bf16), "
                       f"encode {raw / best_e / 1e9:.3f} GB/s, decode {raw / best_d / 1e9:.3f} GB/s, best of 2, no DEFLATE",
                host_cpus=len(os.sched_getaffinity(0)))


def append_step_latency(kv, batch, x, T, n_jobs, R, stream_buf, dev, c=16, steps=60, warmup=10):
    """GPU time of kvtc_offsets_append + kvtc_encode_batch for c new tokens in each of n_jobs caches."""
    import numpy as np
    import torch
    if T < 2 * c:
        return None
    warmup = min(warmup, T // c - 1)
    steps = min(steps, T // c - warmup)
    room = [T * R[j % 2] for j in range(n_jobs)]
    region = torch.from_numpy(np.concatenate([[0], np.cumsum(room)]).astype(np.int64)).to(dev)
    cap = int(sum(room))
    offs = torch.zeros(n_jobs + 1, dtype=torch.int64, device=dev)
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    jobs = [torch.from_numpy(kv.make_jobs([j % 2 for j in range(n_jobs)], [c] * n_jobs,
                                          [j * T + k * c for j in range(n_jobs)]).view(np.uint8)).to(dev)
            for k in range(steps + warmup)]
    coded = [torch.full((n_jobs,), k * c, dtype=torch.int64, device=dev) for k in range(steps + warmup)]
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2 * (steps + warmup))]
    torch.cuda.synchronize()
    for k in range(steps + warmup):
        ev[2 * k].record()
        kv.kvtc_offsets_append(batch.handle, jobs[k], n_jobs, region, coded[k], offs)
        kv.kvtc_encode_batch(batch.handle, jobs[k], n_jobs, x, kv.KVTC_BF16, 1024, offs, stream_buf, cap, status)
        ev[2 * k + 1].record()
    torch.cuda.synchronize()
    assert int(status.item()) == 0, "an append did not fit its region"
    us = sorted(ev[2 * k].elapsed_time(ev[2 * k + 1]) * 1e3 for k in range(warmup, warmup + steps))
    return {"median_us": us[len(us) // 2], "min_us": us[0], "caches": n_jobs, "new_tokens_per_cache": c,
            "what": "kvtc_offsets_append + kvtc_encode_batch, GPU time between HIP events"}


def copy_ceiling(src, dst, reps=5):
    import torch
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2 * reps)]
    dst.copy_(src)
    for i in range(reps):
        ev[2 * i].record()
        dst.copy_(src)
        ev[2 * i + 1].record()
    torch.cuda.synchronize()
    ms = sorted(ev[2 * i].elapsed_time(ev[2 * i + 1]) for i in range(reps))[reps // 2]
    nbytes = 2 * src.numel() * src.element_size()
    return {"GBps": nbytes / (ms * 1e-3) / 1e9, "bytes": nbytes, "what": "torch copy of the input tensor, read + write, median of %d" % reps}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--cr", default="16", choices=["8", "16", "20", "40", "full"],
                    help="compression target of the calibrated plans; 'full' = hand-set full-rank plan (compute-bound)")
    ap.add_argument("--layers", type=int, default=32, help="independent draws of the layer per batch")
    ap.add_argument("--tokens", type=int, default=32768)
    ap.add_argument("--cpu-tokens", type=int, default=32768, help="tokens per tensor in the CPU-baseline sample")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--append", action="store_true",
                    help="also time one incremental step: 16 new tokens appended to each of the batch's caches")
    ap.add_argument("--copy-check", action="store_true",
                    help="also run one plain device copy of the whole input (known size) for scaling profiler byte counters")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (tokens and layers are independent, so the path "
              "shards with no exchange step); use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import kvtc_synth as ks
    import paper_2511_01815_amd as kv

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    kv.lib()      # fail loudly if the HIP library is missing: there is no other path
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    p, T, NL = 1024, args.tokens, args.layers

    tag = "full" if args.cr == "full" else f"cr{args.cr}"
    bundles = [load_bundle(f"c2_K_{tag}"), load_bundle(f"c2_V_{tag}")]
    plans = [kv.Plan(p, b["v_bits"].shape[1], b["mu32"], b["v_bits"],
                     list(zip(b["group_n"].tolist(), b["group_bits"].tolist()))) for b in bundles]
    batch = kv.Batch(plans)
    R = [pl.record_bytes for pl in plans]
    r = [pl.r for pl in plans]

    # ---- inputs, resident in HBM ----
    layers = [ks.make_layer(ks.layer_spec("c2", 0, kvi)) for kvi in (0, 1)]
    n_jobs = 2 * NL
    x = torch.empty((n_jobs * T, p), dtype=torch.bfloat16, device=dev)
    for j in range(n_jobs):
        ks.draw_bf16_torch(layers[j % 2], T, 10 + j // 2, dev, out=x[j * T:(j + 1) * T])
    jobs = kv.make_jobs([j % 2 for j in range(n_jobs)], [T] * n_jobs, [j * T for j in range(n_jobs)])
    jobs_dev = torch.from_numpy(jobs.view(np.uint8)).to(dev)
    offs = torch.zeros(n_jobs + 1, dtype=torch.int64, device=dev)
    cap = sum(T * R[j % 2] for j in range(n_jobs))
    stream_buf = torch.empty(cap, dtype=torch.uint8, device=dev)
    x_hat = torch.empty_like(x)
    status = torch.zeros(2, dtype=torch.int32, device=dev)
    torch.cuda.synchronize()

    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4 * (args.steps + args.warmup))]

    def step(i):
        e0, e1, e2, e3 = ev[4 * i:4 * i + 4]
        kv.kvtc_offsets(batch.handle, jobs_dev, n_jobs, offs)
        e0.record()
        kv.kvtc_encode_batch(batch.handle, jobs_dev, n_jobs, x, kv.KVTC_BF16, p, offs, stream_buf, cap, status[0:1])
        e1.record()
        e2.record()
        kv.kvtc_decode_batch(batch.handle, jobs_dev, n_jobs, stream_buf, cap, offs, x_hat, kv.KVTC_BF16, p, status[1:2])
        e3.record()

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.warmup, args.warmup + args.steps):
        step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    assert status.cpu().tolist() == [0, 0], "a job was skipped"
    if args.copy_check:        # 2 * raw bytes of traffic in one elementwise copy kernel
        scratch = torch.empty_like(x)
        scratch.copy_(x)
        torch.cuda.synchronize()
        del scratch
    assert int(offs[-1].item()) == cap

    enc_ms = [ev[4 * i].elapsed_time(ev[4 * i + 1]) for i in range(args.warmup, args.warmup + args.steps)]
    dec_ms = [ev[4 * i + 2].elapsed_time(ev[4 * i + 3]) for i in range(args.warmup, args.warmup + args.steps)]
    enc_avg, dec_avg = sum(enc_ms) / len(enc_ms), sum(dec_ms) / len(dec_ms)
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    raw_bytes = n_jobs * T * p * 2

    # sanity of the timed work: reconstruction error of the last step is what 16x should give
    with torch.no_grad():
        a = x[:T].float()
        b = x_hat[:T].float()
        rel = float((b - a).norm() / (a - a.mean(0)).norm())
    assert rel < (0.25 if args.cr in ("8", "16", "full") else 0.5), rel

    # ---- roofline of the dominant kernel (per launch) ----
    alg_bytes = sum(T * (2 * p + R[j % 2]) for j in range(n_jobs))
    flops = sum(T * 2 * p * r[j % 2] for j in range(n_jobs))
    dom, dom_ms = ("kvtc_encode_kernel", enc_avg) if enc_avg >= dec_avg else ("kvtc_decode_kernel", dec_avg)
    t_hbm = alg_bytes / (HBM_PEAK_GBPS * 1e9)
    t_mfma = flops / (MFMA_BF16_PEAK_TFLOPS * 1e12)
    if t_hbm >= t_mfma:
        roof = dict(bound="hbm", achieved=alg_bytes / (dom_ms * 1e-3) / 1e9, peak=HBM_PEAK_GBPS, unit="GB/s")
    else:
        roof = dict(bound="mfma", achieved=flops / (dom_ms * 1e-3) / 1e12, peak=MFMA_BF16_PEAK_TFLOPS, unit="TFLOP/s")
    roof["frac"] = roof["achieved"] / roof["peak"]
    # HBM bytes per launch of that kernel from rocprofv3 TCC counters (FETCH_SIZE + WRITE_SIZE, each scaled by
    # what the same counter reads for a 4 GiB copy): measured offline on the default workload only,
    # see profiles/kvtc_kernels_c2x32_cr16.md
    measured = {"kvtc_encode_kernel": 4.62 * 2**30, "kvtc_decode_kernel": 4.49 * 2**30}
    default_workload = args.cr == "16" and NL == 32 and T == 32768
    roof["traffic"] = measured[dom] if default_workload else None
    roof["kernel"] = dom
    roof["encode"] = dict(ms=enc_avg, raw_GBps=raw_bytes / enc_avg / 1e6,
                          hbm_frac=alg_bytes / (enc_avg * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                          mfma_frac=flops / (enc_avg * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS)
    roof["decode"] = dict(ms=dec_avg, raw_GBps=raw_bytes / dec_avg / 1e6,
                          hbm_frac=alg_bytes / (dec_avg * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                          mfma_frac=flops / (dec_avg * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS)

    result = {
        "metric": "encode/decode GB/s of bf16 KV at 16x (8B-shaped); % of binding roofline",
        "value": 2 * raw_bytes / (ms_per_step * 1e-3) / 1e9,
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"c2 layer (K+V, {T} tok x 1024 bf16, {args.cr if args.cr == 'full' else args.cr + 'x'}, r={r[0]}/{r[1]}, R={R[0]}/{R[1]} B) "
                               f"x {NL} seeded draws in one batch = {raw_bytes / 2**30:.2f} GiB raw KV; "
                               "step = offsets + encode + decode",
                   "compression": 2.0 * p / R[0], "n_jobs": n_jobs},
        "roofline": roof,
    }
    # Serving-side latency (not part of `value`): one incremental step of the paper's protocol, the coder
    # run on the 16 tokens that left each cache's sliding window, all n_jobs caches in one batched launch,
    # each cache appending to a region of its own in the stream buffer.
    # (on request only: it launches the encode kernels many more times, which would blur a profile of this run)
    if args.append:
        result["append_step"] = append_step_latency(kv, batch, x, T, n_jobs, R, stream_buf, dev)
    # What a plain device copy of the same input reaches on this machine (reads and writes 2 x raw bytes): the
    # achievable memory ceiling next to the published 8 TB/s the roofline fraction is quoted against.
    result["copy_ceiling"] = copy_ceiling(x, x_hat)
    if not args.no_cpu:
        nt = min(args.cpu_tokens, T)
        xs = [ks.bf16_bits_to_f32(x[j * T:j * T + nt].view(torch.int16).cpu().numpy().view(np.uint16)) for j in (0, 1)]
        result["cpu_baseline"] = cpu_baseline(bundles, xs, p)
    else:
        result["cpu_baseline"] = None
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
