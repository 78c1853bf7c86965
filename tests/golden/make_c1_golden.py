"""Writes tests/golden/c1_oracle.json from the CPU oracle alone.

The paper prints no worked example of an MoE layer, so this fixture is not a
pin of the oracle; it freezes the oracle's own answers on the tiny float32
workload so that an unintended change to the oracle or to the input generator
shows up as a diff.  Run:  python tests/golden/make_c1_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from moe_workloads import CONFIGS, make_inputs, oracle_view  # noqa: E402


def compute():
    cfg = CONFIGS["c1_tiny_f32"]
    v = {k: oracle_view(t) for k, t in make_inputs(cfg).items()}
    out = oracle.layer(v["x"], v["Wr"], v["W1"], v["W3"], v["W2"], cfg.k, cfg.dtype_code)
    return {
        "source": "oracle.layer on workload c1_tiny_f32 (seed 0); written by tests/golden/make_c1_golden.py",
        "counts": out["counts"].tolist(),
        "ids_first8": out["ids"][:8].tolist(),
        "w_first4": out["w"][:4].tolist(),
        "row_src_first16": out["row_src"][:16].tolist(),
        "y_first4x4": out["y"][:4, :4].tolist(),
        "y_sum": float(out["y"].sum()),
        "y_abs_sum": float(np.abs(out["y"]).sum()),
    }


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c1_oracle.json")
    with open(path, "w") as f:
        json.dump(compute(), f, indent=1)
    print("wrote", path)
