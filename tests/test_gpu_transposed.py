"""GPU parity of gspn_scan_fwd_transposed (horizontal directions stored transposed, Sec. 4.3 layout) against the
fp64 oracle: the inputs of directions 2 and 3 are transposed on the host, the result must be the ordinary scan."""
import numpy as np
import pytest

from gpu_util import TOL, rel_inf_err, to_device, to_host_f64, empty_like_dev
from oracle import gspn_oracle as O
from paper_2512_07884_amd import workloads as WL

pytestmark = pytest.mark.gpu


def transposed_inputs(inp):
    """Slots 2 and 3 of w, lam, u rewritten so that the same memory holds the [.., W, H] layout; x transposed."""
    out = {k: v.copy() for k, v in inp.items()}
    for name in ("w", "lam", "u"):
        a = out[name]
        H, W = a.shape[-2:]
        for d in (2, 3):
            t = np.ascontiguousarray(np.swapaxes(inp[name][d], -1, -2))          # [.., W, H]
            a[d] = t.reshape(a[d].shape)                                            # same bytes, viewed as [.., H, W]
    out["xt"] = np.ascontiguousarray(np.swapaxes(inp["x"], -1, -2))
    return out


def check(shape, mask=15, plan=None, seed=113):
    import torch
    import paper_2512_07884_amd as G
    B, C, H, W, Gr, dtype = shape
    cfg = WL.ScanConfig("transposed", B, C, H, W, Gr, dtype, mask, 1.0, seed)
    inp = WL.make_inputs(cfg, with_gy=False)
    f = WL.inputs_as_f64(inp, dtype)
    y_ref, _ = O.scan_fwd(f["x"], f["w"], f["lam"], f["u"], mask)
    t = transposed_inputs(inp)
    if plan:
        assert G.gspn_fwd_transposed_plan(B, C, H, W, Gr, mask, int(dtype == "bf16"), 0) == plan
    dev = {k: to_device(v, dtype) for k, v in t.items()}
    y = empty_like_dev((B, C, H, W), dtype, float("nan"))
    G.gspn_scan_fwd_transposed(dev["x"], dev["xt"], dev["w"], dev["lam"], dev["u"], y, G=Gr, dir_mask=mask)
    torch.cuda.synchronize()
    assert rel_inf_err(to_host_f64(y), y_ref) <= TOL[dtype], rel_inf_err(to_host_f64(y), y_ref)


@pytest.mark.parametrize("shape,plan", [((1, 4, 128, 128, 2, "bf16"), "tile"), ((2, 8, 56, 56, 2, "bf16"), "tile"),
                                        ((1, 8, 64, 128, 2, "f32"), "tile"), ((1, 4, 96, 72, 2, "bf16"), "tile"),
                                        ((2, 6, 28, 40, 3, "f32"), "tile"), ((1, 4, 128, 128, 4, "bf16"), "tile"),
                                        ((1, 4, 33, 70, 2, "f32"), "generic"), ((2, 6, 9, 13, 3, "f32"), "generic"),
                                        ((1, 2, 256, 256, 1, "bf16"), "generic")],
                         ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else str(v))
def test_transposed_horizontal_layout(shape, plan):
    check(shape, plan=plan)


@pytest.mark.parametrize("mask", [4, 8, 12, 5, 10, 3, 14])
def test_transposed_horizontal_layout_direction_masks(mask):
    check((1, 4, 64, 96, 2, "bf16"), mask=mask)
    check((1, 3, 10, 7, 1, "f32"), mask=mask)
