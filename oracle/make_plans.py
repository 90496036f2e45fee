"""Writes the calibration bundles the benchmark loads (paper, Section "Method", mode
"Calibration": PCA basis, mean and bit allocation are computed once and reused).

Run from the repository root:  python oracle/make_plans.py
Calls only the oracle and the seeded input generator.  Output:
paper_2511_01815_amd/plans/<workload>_<K|V>_cr<ratio>.npz  (mean, kept basis columns as
bf16 bit patterns, kept groups).
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "oracle"))

import kvtc_oracle as ko   # noqa: E402
import kvtc_synth as ks    # noqa: E402


def main() -> None:
    out_dir = os.path.join(ROOT, "paper_2511_01815_amd", "plans")
    os.makedirs(out_dir, exist_ok=True)
    wl = ks.WORKLOADS["c2"]
    for kvi, name in enumerate(wl.kv):
        spec = ks.layer_spec("c2", 0, kvi)
        layer = ks.make_layer(spec)
        C = ks.bf16_bits_to_f32(ks.draw_bf16(layer, wl.n_calib, ks.CALIB_DRAW))
        mu, V, S = ko.pca(C)
        errors = ko.dp_errors(C, mu, V)
        for cr in (8.0, 16.0, 20.0, 40.0):
            plan, info = ko.calibrate_from_pca(C, mu, V, S, cr, errors=errors)
            path = os.path.join(out_dir, f"c2_{name}_cr{int(cr)}.npz")
            ko.save_plan(path, plan, cr=cr, budget_bits=info["budget_bits"], seed=spec.seed, alpha=spec.alpha)
            print(path, "r", plan.r, "R", plan.record_bytes,
                  list(zip(plan.group_n.tolist(), plan.group_bits.tolist())))
        # a full-rank plan (every PCA coordinate kept, hand-set widths, about 3.8x) for the compute-bound
        # end of the roofline: the projection is then the whole p x p product
        blocks, start = [], 0
        for n, b in ((64, 8), (192, 6), (256, 4), (512, 3)):
            blocks.append(ko.Block(start, n, b))
            start += n
        plan = ko.compile_plan(mu, V, blocks)
        path = os.path.join(out_dir, f"c2_{name}_full.npz")
        ko.save_plan(path, plan, cr=2.0 * wl.p / plan.record_bytes, budget_bits=8 * plan.record_bytes, seed=spec.seed, alpha=spec.alpha)
        print(path, "r", plan.r, "R", plan.record_bytes)


if __name__ == "__main__":
    main()
