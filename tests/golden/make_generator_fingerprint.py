"""Writes generator_fingerprint.json: first values and moments of the seeded
tensors, as a regression fingerprint of the input generator.  Calls only the
workloads package (never the HIP library).  Run from the repo root:
    python tests/golden/make_generator_fingerprint.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import workloads as wl  # noqa: E402


def fingerprint():
    fp = {"seed": wl.MASTER_SEED, "tensors": {}}
    cases = {
        "normal_bf16_id1": ((64, 1024), wl.DTYPE_BF16, 1, "normal", 1.0),
        "normal_f16_id2": ((64, 1024), wl.DTYPE_F16, 2, "normal", 0.5),
        "uniform_f32_id3": ((64, 1024), wl.DTYPE_F32, 3, "uniform", 1.0),
    }
    for name, (shape, dtype, tid, dist, scale) in cases.items():
        t = wl.tensor(shape, dtype, tid, dist, scale)
        v = wl.widen(t, dtype)
        first = t.reshape(-1)[:16]
        fp["tensors"][name] = {
            "first16": [float(x) for x in first] if dtype == wl.DTYPE_F32 else [int(x) for x in first],
            "mean": float(v.mean()), "std": float(v.std()),
            "min": float(v.min()), "max": float(v.max()),
        }
    return fp


if __name__ == "__main__":
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "generator_fingerprint.json")
    with open(out, "w") as f:
        json.dump(fingerprint(), f, indent=1)
    print("wrote", out)
