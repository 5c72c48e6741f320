"""Writes tests/golden/unit16_oracle.txt: sampled fp64 oracle outputs for the
16x16 single-direction unit workload (seed 0).  Calls only the oracle and the
input generator, never the GPU path.  The paper prints no worked numeric
example of the recurrence, so this file is a regression guard for the oracle
and the generator (not a value from the paper); the hand-worked cases in
tests/test_oracle_forward.py are the independent pins.

Run from the repo root:  python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import gspn_oracle as O                      # noqa: E402
from paper_2512_07884_amd import workloads as WL         # noqa: E402

cfg = WL.CONFIGS["unit16"]
inp = WL.inputs_as_f64(WL.make_inputs(cfg), cfg.dtype)
y, h = O.scan_fwd(inp["x"], inp["w"], inp["lam"], inp["u"], cfg.dir_mask)
pts = [(0, 0, 0, 0), (0, 0, 1, 0), (0, 3, 7, 15), (0, 7, 15, 15), (0, 5, 15, 0), (0, 2, 8, 8)]
with open(os.path.join(os.path.dirname(__file__), "unit16_oracle.txt"), "w") as f:
    f.write("# b c i j y h  (fp64 oracle, workload unit16, seed 0); plus sum(y), sum(|y|)\n")
    for p in pts:
        f.write("%d %d %d %d %.17g %.17g\n" % (*p, y[p], h[(0,) + p]))
    f.write("sum %.17g %.17g\n" % (y.sum(), np.abs(y).sum()))
