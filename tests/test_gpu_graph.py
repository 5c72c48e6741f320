"""The library under HIP graph capture: forward + backward calls (including the zero-fill kernel of the
split-group backward and the two launches of the two-pass backward) recorded once and replayed several times with changed inputs; every replay must
equal the eager result bit for bit."""
import numpy as np
import pytest

from gpu_util import to_device
from paper_2512_07884_amd import workloads as WL

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("shape", [(2, 96, 28, 28, 2, "f32"), (2, 8, 56, 56, 2, "bf16"), (1, 4, 128, 128, 2, "bf16"),
                                   (1, 2, 256, 256, 1, "bf16")],
                         ids=lambda s: "x".join(map(str, s)))
def test_captured_training_step_replays_like_eager(shape):
    import torch
    import paper_2512_07884_amd as G
    B, C, H, W, Gr, dtype = shape
    cfg = WL.ScanConfig("graph", B, C, H, W, Gr, dtype, 15, 1.0, 71)
    inp = WL.make_inputs(cfg)
    d = {k: to_device(v, dtype) for k, v in inp.items()}
    outs = {k: torch.empty_like(d[s]) for k, s in (("y", "x"), ("hs", "lam"), ("gx", "x"), ("gw", "w"), ("gl", "lam"), ("gu", "lam"))}

    def step():
        G.gspn_scan_fwd(d["x"], d["w"], d["lam"], d["u"], outs["y"], outs["hs"], G=Gr)
        G.gspn_scan_bwd(d["gy"], d["x"], d["w"], d["lam"], d["u"], outs["hs"], outs["gx"], outs["gw"], outs["gl"],
                        outs["gu"], G=Gr)

    def snapshot():
        torch.cuda.synchronize()
        return {k: v.clone() for k, v in outs.items()}

    step()                                   # eager warm-up (also sets the kernels' LDS limits)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    gen = torch.Generator(device="cuda"); gen.manual_seed(5)
    for rep in range(3):
        # new inputs in place, eager reference, poison, replay, compare
        d["x"].copy_(torch.randn(d["x"].shape, device="cuda", generator=gen).to(d["x"].dtype))
        d["gy"].copy_(torch.randn(d["gy"].shape, device="cuda", generator=gen).to(d["gy"].dtype))
        step()
        ref = snapshot()
        for v in outs.values():
            v.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot()
        for k in outs:
            assert torch.equal(got[k].view(torch.int16 if dtype == "bf16" else torch.int32),
                               ref[k].view(torch.int16 if dtype == "bf16" else torch.int32)), (shape, rep, k)
