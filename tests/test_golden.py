"""Regression guard: the oracle on the seed-0 unit workload reproduces the stored samples."""
import os

import numpy as np

from oracle import gspn_oracle as O
from paper_2512_07884_amd import workloads as WL


def test_unit16_oracle_samples():
    cfg = WL.CONFIGS["unit16"]
    inp = WL.inputs_as_f64(WL.make_inputs(cfg), cfg.dtype)
    y, h = O.scan_fwd(inp["x"], inp["w"], inp["lam"], inp["u"], cfg.dir_mask)
    path = os.path.join(os.path.dirname(__file__), "golden", "unit16_oracle.txt")
    for line in open(path):
        if line.startswith("#"):
            continue
        t = line.split()
        if t[0] == "sum":
            assert abs(y.sum() - float(t[1])) < 1e-10 and abs(np.abs(y).sum() - float(t[2])) < 1e-10
        else:
            p = tuple(int(v) for v in t[:4])
            assert abs(y[p] - float(t[4])) < 1e-13 and abs(h[(0,) + p] - float(t[5])) < 1e-13
