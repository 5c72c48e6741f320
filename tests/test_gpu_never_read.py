"""Weights that the recurrence never reads, on every kernel family, forward and backward.

The first line of a scan has no predecessor and the end positions of a line have no neighbour outside it (Eq. 1
with a zero initial state, Sec. 3.2).  Whatever w holds there -- NaN, infinities -- must reach neither the output
and the saved states nor any gradient, and the gradient with respect to those weights is exactly zero.
"""
import numpy as np
import pytest

from gpu_util import TOL, rel_inf_err, to_device, to_host_f64, empty_like_dev
from oracle import gspn_oracle as O
from paper_2512_07884_amd import workloads as WL

pytestmark = pytest.mark.gpu

# (B, C, H, W, G, dtype, forward plan, backward plan)
CASES = [
    (1, 16, 28, 28, 4, "bf16", "plane", "twopass"),
    (1, 8, 14, 14, 8, "f32", "plane", "plane"),
    (1, 4, 56, 56, 2, "f32", "tile", "twopass"),
    (1, 4, 128, 128, 2, "bf16", "pair", "twopass"),
    (1, 2, 128, 128, 2, "f32", "tile", "twopass"),
    (1, 4, 256, 256, 2, "bf16", "stream", "twopass"),      # two channels per workgroup, both horizontal directions at once
    (1, 2, 512, 512, 1, "bf16", "stream", "twopass"),      # two channels per workgroup, eight waves of rows
    (1, 3, 512, 256, 1, "bf16", "stream", "twopass"),      # one channel per workgroup
    (1, 2, 256, 256, 1, "f32", "stream", "twopass"),       # a row per lane
    (1, 2, 1024, 1024, 1, "bf16", "stream", "twopass"),    # vertical and horizontal pair as two launches
    (1, 1, 1024, 512, 1, "f32", "stream", "twopass"),
    (1, 3, 33, 70, 3, "bf16", "generic", "generic"),
]


def poison(w, dtype):
    nan, inf, ninf = ((np.nan, np.inf, -np.inf) if dtype == "f32" else
                      (np.uint16(0x7FC0), np.uint16(0x7F80), np.uint16(0xFF80)))
    w[0, :, :, :, 0, :] = nan; w[1, :, :, :, -1, :] = inf             # first line of each scan
    w[2, :, :, :, :, 0] = nan; w[3, :, :, :, :, -1] = ninf
    w[0, :, :, 0, :, 0] = nan; w[0, :, :, 2, :, -1] = inf             # out-of-line neighbours
    w[1, :, :, 0, :, 0] = inf; w[1, :, :, 2, :, -1] = nan
    w[2, :, :, 0, 0, :] = nan; w[2, :, :, 2, -1, :] = nan
    w[3, :, :, 0, 0, :] = inf; w[3, :, :, 2, -1, :] = nan


@pytest.mark.parametrize("case", CASES, ids=lambda s: "x".join(map(str, s[:6])))
def test_training_step_with_anything_in_the_weights_that_are_never_read(case):
    import torch
    import paper_2512_07884_amd as G
    B, C, H, W, Gr, dtype, fwd_plan, bwd_plan = case
    dt = 1 if dtype == "bf16" else 0
    assert G.gspn_fwd_plan(B, C, H, W, Gr, 15, dt, 0, True) == fwd_plan
    assert G.gspn_bwd_plan(B, C, H, W, Gr, 15, dt, 0) == bwd_plan
    cfg = WL.ScanConfig("poison", B, C, H, W, Gr, dtype, 15, 1.0, 3)
    inp = WL.make_inputs(cfg, with_gy=True)
    f = WL.inputs_as_f64(inp, dtype)
    y_ref, h_ref = O.scan_fwd(f["x"], f["w"], f["lam"], f["u"], 15)
    h_used = WL.storage_to_f64(WL.to_storage(h_ref, dtype), dtype)
    gx_r, gw_r, gl_r, gu_r = O.scan_bwd(f["gy"], f["x"], f["w"], f["lam"], f["u"], h_used, 15)
    poison(inp["w"], dtype)
    dev = {k: to_device(v, dtype) for k, v in inp.items()}
    nan = float("nan")
    y = empty_like_dev((B, C, H, W), dtype, nan)
    y_only = empty_like_dev((B, C, H, W), dtype, nan)
    hs = empty_like_dev((4, B, C, H, W), dtype, nan)
    gx = empty_like_dev((B, C, H, W), dtype, nan)
    gw = empty_like_dev((4, B, Gr, 3, H, W), dtype, nan)
    gl = empty_like_dev((4, B, C, H, W), dtype, nan)
    gu = empty_like_dev((4, B, C, H, W), dtype, nan)
    G.gspn_scan_fwd(dev["x"], dev["w"], dev["lam"], dev["u"], y_only, None, G=Gr, dir_mask=15)
    G.gspn_scan_fwd(dev["x"], dev["w"], dev["lam"], dev["u"], y, hs, G=Gr, dir_mask=15)
    G.gspn_scan_bwd(dev["gy"], dev["x"], dev["w"], dev["lam"], dev["u"], hs, gx, gw, gl, gu, G=Gr, dir_mask=15)
    torch.cuda.synchronize()
    tol = TOL[dtype]
    for name, got, ref in (("y without h_save", y_only, y_ref), ("y", y, y_ref), ("h", hs, h_ref), ("gx", gx, gx_r),
                           ("gw", gw, gw_r), ("glam", gl, gl_r), ("gu", gu, gu_r)):
        a = to_host_f64(got)
        assert np.all(np.isfinite(a)), (case, name)
        if ref.ndim == a.ndim and ref.shape[0] == 4:
            for d in range(4):
                assert rel_inf_err(a[d], ref[d]) <= tol, (case, name, d, rel_inf_err(a[d], ref[d]))
        else:
            assert rel_inf_err(a, ref) <= tol, (case, name, rel_inf_err(a, ref))
    g = to_host_f64(gw)
    for d in range(4):
        first = {0: g[d][:, :, :, 0, :], 1: g[d][:, :, :, -1, :], 2: g[d][:, :, :, :, 0], 3: g[d][:, :, :, :, -1]}[d]
        assert not first.any(), (case, d)
        if d < 2:
            assert not g[d][:, :, 0, :, 0].any() and not g[d][:, :, 2, :, -1].any(), (case, d)
        else:
            assert not g[d][:, :, 0, 0, :].any() and not g[d][:, :, 2, -1, :].any(), (case, d)
