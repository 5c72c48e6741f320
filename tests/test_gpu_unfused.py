"""The per-line-launch comparator (gspn_scan_fwd_unfused) against the oracle.

It is the structure the fused kernels replace (Sec. 3.3: one micro-launch per line, the hidden state through global
memory); it must compute the same scan, or a speed ratio against it would mean nothing.
"""
import numpy as np
import pytest

from gpu_util import TOL, rel_inf_err, to_device, to_host_f64, empty_like_dev
from oracle import gspn_oracle as O
from paper_2512_07884_amd import workloads as WL

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("shape", [(2, 6, 9, 13, 3, "f32", 15), (1, 4, 33, 70, 2, "bf16", 15), (1, 2, 64, 64, 1, "f32", 5),
                                   (1, 3, 40, 24, 3, "bf16", 10), (1, 4, 33, 70, 2, "f16", 15)], ids=lambda s: "x".join(map(str, s)))
def test_per_line_launch_comparator_matches_the_oracle(shape):
    import torch
    import paper_2512_07884_amd as G
    B, C, H, W, Gr, dtype, mask = shape
    cfg = WL.ScanConfig("unfused", B, C, H, W, Gr, dtype, mask, 1.0, 91)
    inp = WL.make_inputs(cfg, with_gy=False)
    f = WL.inputs_as_f64(inp, dtype)
    y_ref, h_ref = O.scan_fwd(f["x"], f["w"], f["lam"], f["u"], mask)
    dev = {k: to_device(v, dtype) for k, v in inp.items()}
    y = empty_like_dev((B, C, H, W), dtype, float("nan"))
    hs = empty_like_dev((4, B, C, H, W), dtype, float("nan"))
    ws = torch.empty(G.gspn_unfused_workspace_bytes(B, C, H, W), dtype=torch.uint8, device="cuda")
    G.gspn_scan_fwd_unfused(dev["x"], dev["w"], dev["lam"], dev["u"], y, hs, ws, G=Gr, dir_mask=mask)
    torch.cuda.synchronize()
    assert rel_inf_err(to_host_f64(y), y_ref) <= TOL[dtype]
    for d in range(4):
        if (mask >> d) & 1:
            assert rel_inf_err(to_host_f64(hs[d]), h_ref[d]) <= TOL[dtype]


def test_comparator_rejects_a_workspace_that_is_too_small():
    import torch
    import paper_2512_07884_amd as G
    cfg = WL.ScanConfig("unfusedws", 1, 2, 8, 8, 1, "f32", 15, 1.0, 93)
    inp = WL.make_inputs(cfg, with_gy=False)
    dev = {k: to_device(v, "f32") for k, v in inp.items()}
    y = empty_like_dev((1, 2, 8, 8), "f32", 7.0)
    ws = torch.empty(G.gspn_unfused_workspace_bytes(1, 2, 8, 8) - 16, dtype=torch.uint8, device="cuda")
    with pytest.raises(G.GspnError) as ei:
        G.gspn_scan_fwd_unfused(dev["x"], dev["w"], dev["lam"], dev["u"], y, None, ws, G=1)
    assert ei.value.status == 2
    assert torch.all(y == 7.0)
