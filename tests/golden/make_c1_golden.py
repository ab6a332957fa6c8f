"""Writes c1_oracle.json from the CPU oracle alone (run from the repo root: python tests/golden/make_c1_golden.py)."""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle                      # noqa: E402
from workloads import make_workload  # noqa: E402

wl = make_workload("C1")
out = oracle.expanded_linear(wl.x, 80, wl.qw, wl.sw)
g = {
    "sx": [float(v) for v in out["sx"]],
    "qx_sum": int(out["qx"].astype(np.int64).sum()),
    "qx_abs_sum": int(np.abs(out["qx"].astype(np.int64)).sum()),
    "acc_sum": int(out["acc"].sum()),
    "acc_row0": [int(v) for v in out["acc"][0, :8]],
    "y_row0": [float(v) for v in out["y"][0, :8]],
}
with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "c1_oracle.json"), "w") as f:
    json.dump(g, f, indent=1)
print(g)
