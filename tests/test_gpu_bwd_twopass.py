"""GPU parity of the two-pass backward scan (maps beyond the single-launch backward kernels) against the fp64 oracle.

Pass 1 runs the reverse sweep on the forward tile kernels (all four of their horizontal variants are covered here) or,
for maps beyond the LDS tile, on the forward stream kernel; pass 2 sums gw over the channels of a group; the shapes
below are ones the backward plane and tile kernels refuse."""
import numpy as np
import pytest

from gpu_util import to_device
from paper_2512_07884_amd import workloads as WL
from test_gpu_bwd import check_bwd, run_bwd_gpu
from gpu_util import TOL, rel_inf_err
from oracle import gspn_oracle as O

pytestmark = pytest.mark.gpu

# B, C, H, W, G, dtype: rows split over waves (2 and 3 parts), 64 B bursts, 16 B bursts, 112 B bursts with a group too
# large for one workgroup; per-channel and shared weights; several images
SHAPES = [(1, 4, 128, 128, 2, "bf16"), (2, 4, 128, 128, 4, "bf16"), (1, 2, 128, 64, 1, "f32"), (1, 3, 192, 128, 3, "bf16"),
          (1, 4, 96, 96, 2, "bf16"), (1, 2, 100, 48, 1, "f32"), (1, 4, 96, 72, 2, "bf16"), (1, 4, 70, 36, 2, "f32"),
          (1, 32, 56, 56, 1, "bf16"), (1, 32, 56, 56, 1, "f32"), (2, 6, 66, 40, 3, "f32"),
          # maps the single-launch tile kernel would take too (the two-pass backward comes first)
          (2, 8, 56, 56, 2, "bf16"), (2, 24, 56, 56, 2, "f32"), (1, 8, 64, 128, 2, "f32"), (2, 8, 40, 32, 8, "f32"),
          (1, 24, 16, 40, 2, "f32"), (1, 8, 64, 64, 8, "bf16"),
          # maps beyond the LDS tile: 4 / 8 / 16 positions per lane in the vertical passes, 1 to 5 waves per column
          (1, 2, 256, 256, 1, "bf16"), (1, 2, 128, 256, 2, "f32"), (1, 2, 64, 1024, 1, "bf16"), (2, 2, 320, 256, 2, "bf16"),
          (1, 2, 192, 512, 1, "f32"), (1, 4, 128, 512, 2, "bf16")]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_two_pass_backward_shapes(shape):
    import paper_2512_07884_amd as G
    B, C, H, W, Gr, dtype = shape
    assert G.gspn_bwd_plan(B, C, H, W, Gr, 15, int(dtype == "bf16"), 0) == "twopass", shape
    check_bwd(WL.ScanConfig("twopass", B, C, H, W, Gr, dtype, 15, 1.0, 71))


@pytest.mark.parametrize("mask", [1, 2, 4, 8, 5, 10, 7, 12])
@pytest.mark.parametrize("shape", [(1, 4, 128, 64, 2, "f32"), (1, 4, 96, 72, 2, "bf16"), (1, 2, 128, 256, 1, "bf16")],
                         ids=lambda s: "x".join(map(str, s)))
def test_two_pass_backward_direction_masks(mask, shape):
    import paper_2512_07884_amd as G
    B, C, H, W, Gr, dtype = shape
    assert G.gspn_bwd_plan(B, C, H, W, Gr, mask, int(dtype == "bf16"), 0) == "twopass"
    check_bwd(WL.ScanConfig("twopassmask", B, C, H, W, Gr, dtype, mask, 1.0, 73))


@pytest.mark.parametrize("bcg", [(1, 2, 1), (2, 12, 2)], ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("pair", [True, False], ids=["two-channel", "one-channel"])
def test_two_pass_backward_on_128x128_bf16_maps(bcg, pair, monkeypatch):
    """The reverse sweep of these maps runs on the two-channel kernel (and on the one-channel tile kernel when that is
    switched off): both against the oracle."""
    import paper_2512_07884_amd as G
    if not pair:
        monkeypatch.setenv("GSPN_FWD_NO_PAIR", "1")
    B, C, Gr = bcg
    assert G.gspn_bwd_plan(B, C, 128, 128, Gr, 15, 1, 0) == "twopass"
    check_bwd(WL.ScanConfig("twopass128", B, C, 128, 128, Gr, "bf16", 15, 3.0, 83))


def test_two_pass_backward_when_a_workgroup_of_the_reverse_sweep_works_through_several_pairs():
    """600 channels of 128x128: 300 pairs on 256 workgroups (a short second round) in the reverse sweep."""
    check_bwd(WL.ScanConfig("twopassrounds", 1, 600, 128, 128, 4, "bf16", 15, 2.0, 85))


def test_two_pass_backward_is_bitwise_repeatable():
    import torch
    import paper_2512_07884_amd as G
    cfg = WL.ScanConfig("twopassrep", 1, 8, 128, 128, 2, "bf16", 15, 1.0, 79)
    inp = WL.make_inputs(cfg)
    dev = {k: to_device(v, "bf16") for k, v in inp.items()}
    hs = torch.empty_like(dev["lam"]); y = torch.empty_like(dev["x"])
    G.gspn_scan_fwd(dev["x"], dev["w"], dev["lam"], dev["u"], y, hs, G=cfg.G)
    outs = []
    for rep in range(3):
        gx = torch.full_like(dev["x"], float("nan")); gw = torch.full_like(dev["w"], float("nan"))
        gl = torch.full_like(dev["lam"], float("nan")); gu = torch.full_like(dev["lam"], float("nan"))
        G.gspn_scan_bwd(dev["gy"], dev["x"], dev["w"], dev["lam"], dev["u"], hs, gx, gw, gl, gu, G=cfg.G)
        torch.cuda.synchronize()
        outs.append([t.view(torch.int16).cpu().numpy().copy() for t in (gx, gw, gl, gu)])
    for k in range(4):
        assert np.array_equal(outs[0][k], outs[1][k]) and np.array_equal(outs[0][k], outs[2][k])


def test_two_pass_backward_on_512x512_planes():
    """The high-resolution shape (512x512, 32 channels per group, bf16) with fewer channels: the same kernels and the same
    work per workgroup as bench.py's train512 workload."""
    import paper_2512_07884_amd as G
    cfg = WL.shrink(WL.CONFIGS["train512"], C=64, G=2)
    assert G.gspn_fwd_plan(cfg.B, cfg.C, cfg.H, cfg.W, cfg.G, 15, 1, 0, True) == "stream"
    assert G.gspn_bwd_plan(cfg.B, cfg.C, cfg.H, cfg.W, cfg.G, 15, 1, 0) == "twopass"
    check_bwd(cfg)


# GSPN-local and logits calls on the same maps: stretch lengths that divide the map, that do not, of one line, longer
# than a chunk of the horizontal phases; all four horizontal variants of the reverse sweep
@pytest.mark.parametrize("shape,kchunk", [((1, 4, 128, 128, 2, "bf16"), 32), ((1, 4, 128, 64, 2, "f32"), 48), ((1, 4, 96, 96, 2, "bf16"), 7),
                                          ((1, 4, 96, 72, 2, "bf16"), 20), ((1, 4, 70, 36, 2, "f32"), 1), ((1, 32, 56, 56, 1, "f32"), 9),
                                          ((2, 3, 192, 128, 3, "bf16"), 100),
                                          # maps beyond the LDS tile
                                          ((1, 2, 256, 256, 1, "bf16"), 37), ((1, 2, 128, 256, 2, "f32"), 100), ((1, 2, 64, 1024, 1, "bf16"), 300)],
                         ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else str(v))
def test_two_pass_backward_with_local_stretches(shape, kchunk):
    import paper_2512_07884_amd as G
    from test_gpu_local import check_local
    B, C, H, W, Gr, dtype = shape
    assert G.gspn_bwd_local_plan(B, C, H, W, Gr, kchunk, 15, int(dtype == "bf16"), 0) == "twopass"
    check_local(shape, kchunk)


@pytest.mark.parametrize("shape,kchunk", [((1, 4, 128, 128, 2, "bf16"), None), ((1, 4, 128, 64, 2, "f32"), None), ((1, 4, 96, 96, 2, "f32"), None),
                                          ((1, 4, 96, 72, 2, "bf16"), 20), ((1, 4, 70, 36, 2, "f32"), 16), ((1, 32, 56, 56, 1, "f32"), None),
                                          ((1, 2, 256, 256, 1, "bf16"), None), ((1, 2, 128, 256, 2, "f32"), 50), ((2, 2, 320, 256, 2, "bf16"), 64)],
                         ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else str(v))
def test_two_pass_backward_with_logits(shape, kchunk):
    from test_gpu_logits import check_logits
    check_logits(shape, kchunk=kchunk, bwd_plan="twopass")


@pytest.mark.parametrize("mask", [1, 2, 4, 8, 6, 9])
def test_two_pass_backward_with_logits_and_local_stretches_direction_masks(mask):
    from test_gpu_logits import check_logits
    check_logits((1, 4, 128, 64, 2, "f32"), kchunk=24, mask=mask, bwd_plan="twopass")


# small maps whose forward runs on the plane kernel and whose backward the plane kernel refuses: the reverse sweep runs on
# the plane kernel too (padded and unpadded LDS planes, 1 to 8 channels per wave, shared and per-channel weights --
# 7x7 and 14x14 with one weight map per channel are the original GSPN on the last stages of a classifier, Sec. 5.2)
PLANE_SWEEP_SHAPES = [(2, 16, 28, 28, 2, "bf16"), (1, 12, 16, 32, 3, "bf16"), (2, 24, 56, 56, 2, "bf16"), (1, 8, 64, 64, 8, "bf16"), (1, 6, 40, 24, 3, "bf16"), (2, 16, 14, 14, 16, "bf16"),
                      (2, 16, 7, 7, 16, "f32"), (2, 16, 7, 7, 16, "bf16"), (3, 8, 56, 56, 8, "bf16"), (1, 4, 64, 64, 1, "bf16")]


@pytest.mark.parametrize("shape", PLANE_SWEEP_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_two_pass_backward_with_the_reverse_sweep_on_the_plane_kernel(shape):
    import paper_2512_07884_amd as G
    B, C, H, W, Gr, dtype = shape
    dt = int(dtype == "bf16")
    assert G.gspn_fwd_plan(B, C, H, W, Gr, 15, dt, 0, True) == "plane"
    assert G.gspn_bwd_plan(B, C, H, W, Gr, 15, dt, 0) == "twopass"
    check_bwd(WL.ScanConfig("planesweep", B, C, H, W, Gr, dtype, 15, 1.0, 89))


@pytest.mark.parametrize("shape,kchunk", [((2, 24, 56, 56, 2, "bf16"), 14), ((1, 8, 64, 64, 8, "bf16"), 10), ((2, 16, 14, 14, 16, "bf16"), 5),
                                          ((2, 16, 7, 7, 16, "f32"), 3)],
                         ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else str(v))
def test_two_pass_backward_on_the_plane_kernel_with_local_stretches_and_logits(shape, kchunk):
    import paper_2512_07884_amd as G
    from test_gpu_local import check_local
    from test_gpu_logits import check_logits
    B, C, H, W, Gr, dtype = shape
    assert G.gspn_bwd_local_plan(B, C, H, W, Gr, kchunk, 15, int(dtype == "bf16"), 0) == "twopass"
    check_local(shape, kchunk)
    check_logits(shape, kchunk=kchunk, fwd_plan="plane", bwd_plan="twopass")
    check_logits(shape, fwd_plan="plane", bwd_plan="twopass")


@pytest.mark.parametrize("mask", [1, 2, 4, 8, 6, 9, 11])
def test_two_pass_backward_on_the_plane_kernel_direction_masks(mask):
    check_bwd(WL.ScanConfig("planesweepmask", 2, 8, 56, 56, 2, "bf16", mask, 1.0, 97))


@pytest.mark.parametrize("shape", [(2, 8, 28, 28, 2, "f32"), (1, 4, 128, 64, 2, "f32"), (2, 24, 56, 56, 2, "bf16"), (1, 2, 256, 256, 1, "bf16"),
                                   (2, 6, 17, 17, 3, "f32")], ids=lambda s: "x".join(map(str, s)))
def test_backward_with_one_parameter_set_for_all_directions(shape):
    """GSPN_FLAG_SHARED_PARAMS: w, lam, u have a single slot that every direction reads; the gradients keep four slots
    (plane, two-pass on the tile / plane / stream sweeps, generic kernels)."""
    B, C, H, W, Gr, dtype = shape
    cfg = WL.ScanConfig("sharedbwd", B, C, H, W, Gr, dtype, 15, 1.0, 101)
    inp = WL.make_inputs(cfg, with_gy=True)
    one = {"x": inp["x"], "gy": inp["gy"], "w": inp["w"][:1].copy(), "lam": inp["lam"][:1].copy(), "u": inp["u"][:1].copy()}
    rep = {"x": inp["x"], "gy": inp["gy"], "w": np.repeat(one["w"], 4, 0), "lam": np.repeat(one["lam"], 4, 0),
           "u": np.repeat(one["u"], 4, 0)}
    f = WL.inputs_as_f64(rep, dtype)
    _, h_ref = O.scan_fwd(f["x"], f["w"], f["lam"], f["u"], 15)
    h_used = WL.storage_to_f64(WL.to_storage(h_ref, dtype), dtype)
    gx, gw, glam, gu = O.scan_bwd(f["gy"], f["x"], f["w"], f["lam"], f["u"], h_used, 15)
    out = run_bwd_gpu(one, cfg, 15, flags=1)
    tol = TOL[dtype]
    assert rel_inf_err(out["gx"], gx) <= tol
    for d in range(4):
        for name, got, ref in (("gw", out["gw"], gw), ("glam", out["glam"], glam), ("gu", out["gu"], gu)):
            e = rel_inf_err(got[d], ref[d])
            assert e <= tol, (shape, name, d, e)
