"""Reads the calibration bundles under plans/ (data only: mean, kept basis columns as bf16 bit
patterns, kept groups).  Calibration itself is not part of this package; the files are written
by the calibration script that sits beside the CPU reference coder."""
from __future__ import annotations

import os
from typing import Dict, List, Tuple

import numpy as np

PLANS_DIR = os.path.join(os.path.dirname(os.path.abspath(__file__)), "plans")


def load_plan_arrays(name: str) -> Dict[str, np.ndarray]:
    """A one-plan bundle, e.g. "c2_K_cr16": mu32 [p], v_bits [p, r], group_n [G], group_bits [G]."""
    z = np.load(os.path.join(PLANS_DIR, name + ".npz"))
    return dict(mu32=z["mu32"], v_bits=z["v_bits"], group_n=z["group_n"], group_bits=z["group_bits"])


def load_tensor_plan_arrays(workload: str, layer: int, kv: str, cr: int) -> Dict[str, np.ndarray]:
    """One tensor of a multi-layer workload ("c3"), whose file holds one basis and the kept
    coordinates / groups of several ratios; returns the same arrays as load_plan_arrays."""
    z = np.load(os.path.join(PLANS_DIR, f"{workload}_L{layer:02d}_{kv}.npz"))
    tag = f"cr{int(cr)}"
    kept = z[tag + "_kept"]
    return dict(mu32=z["mu32"], v_bits=np.ascontiguousarray(z["v_bits"][:, kept]),
                group_n=z[tag + "_group_n"], group_bits=z[tag + "_group_bits"])


def cache_plan_arrays(workload: str, n_layers: int, cr: int, kvs: Tuple[str, ...] = ("K", "V")) -> List[Dict[str, np.ndarray]]:
    """All tensors of a cache in job order: layer-major, K before V."""
    return [load_tensor_plan_arrays(workload, l, kv, cr) for l in range(n_layers) for kv in kvs]


def entropy_tables(workload: str, cr: int):
    """Code lengths of the lossless stage, [tensors][record_bytes][256] uint8 in job order, or None when the bundle for
    this workload and ratio was not written."""
    path = os.path.join(PLANS_DIR, f"{workload}_entropy_cr{int(cr)}.npz")
    if not os.path.exists(path):
        return None
    return np.load(path)["code_len"]
