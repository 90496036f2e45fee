"""Writes the code-length tables of the lossless stage for the benchmark's cache (paper, Section "Entropy coding";
Section "Method", mode "Calibration": everything data-dependent is computed once on calibration data and reused).

Run from the repository root:  python oracle/make_entropy_tables.py
Calls only the oracle, the seeded input generator and the committed plan bundles (which the oracle wrote).
For every tensor of the 32-layer cache at 16x: the first 2048 tokens of the tensor's calibration draw are coded by the
oracle with the tensor's plan, and the records' per-position byte histograms give one prefix code per byte position
(oracle/kvtc_entropy.py).  Output: paper_2511_01815_amd/plans/c3_entropy_cr16.npz, code_len [64][128][256] uint8,
tensors in job order (layer-major, K before V)."""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "oracle"))

import kvtc_entropy as ke   # noqa: E402
import kvtc_oracle as ko    # noqa: E402
import kvtc_synth as ks     # noqa: E402
from paper_2511_01815_amd import bundles as kb   # noqa: E402  (data loader only)

N_TOKENS = 2048
CR = 16


def tables_of(layer_idx: int, kvi: int) -> np.ndarray:
    wl = ks.WORKLOADS["c3"]
    b = kb.load_tensor_plan_arrays("c3", layer_idx, wl.kv[kvi], CR)
    plan = ko.plan_from_arrays(b["mu32"], b["v_bits"], b["group_n"], b["group_bits"])
    layer = ks.make_layer(ks.layer_spec("c3", layer_idx, kvi))
    C = ks.bf16_bits_to_f32(ks.draw_bf16(layer, N_TOKENS, ks.CALIB_DRAW))
    return ke.calibrate_tables(ko.encode(plan, C))


def main() -> None:
    wl = ks.WORKLOADS["c3"]
    out = []
    for l in range(wl.n_layers):
        for kvi in range(len(wl.kv)):
            t = tables_of(l, kvi)
            assert t.shape == (128, 256), t.shape
            out.append(t)
            print(f"layer {l} {wl.kv[kvi]}: mean code length {t.mean():.2f} bits over the table", flush=True)
    path = os.path.join(kb.PLANS_DIR, f"c3_entropy_cr{CR}.npz")
    np.savez_compressed(path, code_len=np.stack(out).astype(np.uint8), n_tokens=np.asarray(N_TOKENS))
    print(path)


if __name__ == "__main__":
    main()
