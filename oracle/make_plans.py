"""Writes the calibration bundles the benchmark and the full-size tests load (paper, Section
"Method", mode "Calibration": PCA basis, mean and bit allocation are computed once per model
and compression ratio and reused).

Run from the repository root:  python oracle/make_plans.py [--only c2|c3|c45] [--procs N]
Calls only the oracle and the seeded input generator.  Output, under
paper_2511_01815_amd/plans/:
  c2_<K|V>_cr<ratio>.npz, c2_<K|V>_full.npz   one plan per file (mean, kept basis columns as
                                              bf16 bit patterns, kept groups);
  c4_L05_<K|V>_cr20.npz, c5_L09_<K|V>_cr40.npz one layer of the long-context and of the ragged-batch configuration at
                                              their ratios (one plan per file, as the c2 files);
  c3_L<layer>_<K|V>.npz                       one tensor of the 32-layer cache per file: the mean,
                                              the leading PCA directions (bf16 bit patterns) up to
                                              the last coordinate any ratio keeps, and for each
                                              ratio 8x / 16x / 20x the kept coordinates and groups
                                              (the ratios share one basis: calibration differs
                                              only in the bit allocation).
"""
import argparse
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "oracle"))

import kvtc_oracle as ko   # noqa: E402
import kvtc_synth as ks    # noqa: E402

OUT_DIR = os.path.join(ROOT, "paper_2511_01815_amd", "plans")
C3_RATIOS = (8.0, 16.0, 20.0)


def write_c2() -> None:
    wl = ks.WORKLOADS["c2"]
    for kvi, name in enumerate(wl.kv):
        spec = ks.layer_spec("c2", 0, kvi)
        layer = ks.make_layer(spec)
        C = ks.bf16_bits_to_f32(ks.draw_bf16(layer, wl.n_calib, ks.CALIB_DRAW))
        mu, V, S = ko.pca(C)
        errors = ko.dp_errors(C, mu, V)
        for cr in (8.0, 16.0, 20.0, 40.0):
            plan, info = ko.calibrate_from_pca(C, mu, V, S, cr, errors=errors)
            path = os.path.join(OUT_DIR, f"c2_{name}_cr{int(cr)}.npz")
            ko.save_plan(path, plan, cr=cr, budget_bits=info["budget_bits"], seed=spec.seed, alpha=spec.alpha)
            print(path, "r", plan.r, "R", plan.record_bytes,
                  list(zip(plan.group_n.tolist(), plan.group_bits.tolist())), flush=True)
        # a full-rank plan (every PCA coordinate kept, hand-set widths, about 3.8x) for the compute-bound
        # end of the roofline: the projection is then the whole p x p product
        blocks, start = [], 0
        for n, b in ((64, 8), (192, 6), (256, 4), (512, 3)):
            blocks.append(ko.Block(start, n, b))
            start += n
        plan = ko.compile_plan(mu, V, blocks)
        path = os.path.join(OUT_DIR, f"c2_{name}_full.npz")
        ko.save_plan(path, plan, cr=2.0 * wl.p / plan.record_bytes, budget_bits=8 * plan.record_bytes, seed=spec.seed, alpha=spec.alpha)
        print(path, "r", plan.r, "R", plan.record_bytes, flush=True)


def write_layer(workload: str, layer_idx: int, cr: float) -> None:
    """K and V plans of one layer of a multi-layer configuration at one ratio -> one-plan files."""
    wl = ks.WORKLOADS[workload]
    for kvi, name in enumerate(wl.kv):
        spec = ks.layer_spec(workload, layer_idx, kvi)
        layer = ks.make_layer(spec)
        C = ks.bf16_bits_to_f32(ks.draw_bf16(layer, wl.n_calib, ks.CALIB_DRAW))
        mu, V, S = ko.pca(C)
        plan, info = ko.calibrate_from_pca(C, mu, V, S, cr, errors=ko.dp_errors(C, mu, V))
        path = os.path.join(OUT_DIR, f"{workload}_L{layer_idx:02d}_{name}_cr{int(cr)}.npz")
        ko.save_plan(path, plan, cr=cr, budget_bits=info["budget_bits"], seed=spec.seed, alpha=spec.alpha)
        print(path, "r", plan.r, "R", plan.record_bytes, list(zip(plan.group_n.tolist(), plan.group_bits.tolist())), flush=True)


def calibrate_c3_tensor(layer_kv):
    """The plans of one tensor of the 32-layer cache at every ratio of the sweep -> one file."""
    layer_idx, kvi = layer_kv
    wl = ks.WORKLOADS["c3"]
    spec = ks.layer_spec("c3", layer_idx, kvi)
    layer = ks.make_layer(spec)
    C = ks.bf16_bits_to_f32(ks.draw_bf16(layer, wl.n_calib, ks.CALIB_DRAW))
    mu, V, S = ko.pca(C)
    errors = ko.dp_errors(C, mu, V)
    plans = {cr: ko.calibrate_from_pca(C, mu, V, S, cr, errors=errors)[0] for cr in C3_RATIOS}
    n_cols = 1 + max(int(pl.kept.max()) for pl in plans.values())
    arrays = dict(mu32=np.asarray(mu, dtype=np.float32), v_bits=ko.bf16_bits(V[:, :n_cols]),
                  seed=np.asarray(spec.seed), alpha=np.asarray(spec.alpha))
    for cr, pl in plans.items():
        tag = f"cr{int(cr)}"
        assert np.array_equal(arrays["v_bits"][:, pl.kept], pl.v_bits) and np.array_equal(arrays["mu32"], pl.mu32)
        arrays[tag + "_kept"] = pl.kept.astype(np.int32)
        arrays[tag + "_group_n"] = pl.group_n.astype(np.int32)
        arrays[tag + "_group_bits"] = pl.group_bits.astype(np.int32)
    path = os.path.join(OUT_DIR, f"c3_L{layer_idx:02d}_{wl.kv[kvi]}.npz")
    np.savez_compressed(path, **arrays)
    return path, spec.alpha, {cr: (pl.r, pl.record_bytes) for cr, pl in plans.items()}


def write_c3(procs: int) -> None:
    wl = ks.WORKLOADS["c3"]
    todo = [(l, kvi) for l in range(wl.n_layers) for kvi in range(len(wl.kv))]
    if procs > 1:
        import multiprocessing as mp
        with mp.Pool(procs) as pool:
            for res in pool.imap(calibrate_c3_tensor, todo):
                print(*res, flush=True)
    else:
        for t in todo:
            print(*calibrate_c3_tensor(t), flush=True)


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--only", choices=["c2", "c3", "c45"], default=None)
    ap.add_argument("--procs", type=int, default=1, help="worker processes for the 64 tensors of c3")
    args = ap.parse_args()
    os.makedirs(OUT_DIR, exist_ok=True)
    if args.only in (None, "c2"):
        write_c2()
    if args.only in (None, "c45"):
        write_layer("c4", 5, 20.0)
        write_layer("c5", 9, 40.0)
    if args.only in (None, "c3"):
        write_c3(args.procs)


if __name__ == "__main__":
    main()
