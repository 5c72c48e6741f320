"""GPU parity of gspn_scan_bwd against the fp64 oracle, through the C ABI.

The forward call writes h_save, the backward call consumes it; every gradient
tensor is compared separately with the tolerance of its storage dtype.
"""
import numpy as np
import pytest

from gpu_util import TOL, rel_inf_err, to_device, to_host_f64, empty_like_dev
from oracle import gspn_oracle as O
from paper_2512_07884_amd import workloads as WL

pytestmark = pytest.mark.gpu


def run_bwd_gpu(inp, cfg, mask, flags=0):
    import torch
    import paper_2512_07884_amd as G
    dev = {k: to_device(v, cfg.dtype) for k, v in inp.items()}
    B, C, H, W = inp["x"].shape
    nan = float("nan")
    y = empty_like_dev((B, C, H, W), cfg.dtype, nan)
    hs = empty_like_dev((4, B, C, H, W), cfg.dtype, nan)
    G.gspn_scan_fwd(dev["x"], dev["w"], dev["lam"], dev["u"], y, hs, G=cfg.G, dir_mask=mask, flags=flags)
    gx = empty_like_dev((B, C, H, W), cfg.dtype, nan)
    gw = empty_like_dev((4, B, cfg.G, 3, H, W), cfg.dtype, nan)
    glam = empty_like_dev((4, B, C, H, W), cfg.dtype, nan)
    gu = empty_like_dev((4, B, C, H, W), cfg.dtype, nan)
    G.gspn_scan_bwd(dev["gy"], dev["x"], dev["w"], dev["lam"], dev["u"], hs, gx, gw, glam, gu,
                    G=cfg.G, dir_mask=mask, flags=flags)
    torch.cuda.synchronize()
    return {"h": to_host_f64(hs), "gx": to_host_f64(gx), "gw": to_host_f64(gw),
            "glam": to_host_f64(glam), "gu": to_host_f64(gu)}


def check_bwd(cfg, mask=None):
    mask = cfg.dir_mask if mask is None else mask
    inp = WL.make_inputs(cfg, with_gy=True)
    f = WL.inputs_as_f64(inp, cfg.dtype)
    out = run_bwd_gpu(inp, cfg, mask)
    # the oracle's backward consumes the oracle's own hidden states, rounded to storage like h_save is
    _, h_ref = O.scan_fwd(f["x"], f["w"], f["lam"], f["u"], mask)
    h_used = WL.storage_to_f64(WL.to_storage(h_ref, cfg.dtype), cfg.dtype)
    gx, gw, glam, gu = O.scan_bwd(f["gy"], f["x"], f["w"], f["lam"], f["u"], h_used, mask)
    tol = TOL[cfg.dtype]
    assert rel_inf_err(out["gx"], gx) <= tol, (cfg, "gx", rel_inf_err(out["gx"], gx))
    for d in range(4):
        for name, got, ref in (("gw", out["gw"], gw), ("glam", out["glam"], glam), ("gu", out["gu"], gu)):
            if (mask >> d) & 1:
                e = rel_inf_err(got[d], ref[d])
                assert e <= tol, (cfg, name, d, e)
            else:
                assert np.all(np.isnan(got[d])), (name, d, "slot of an unmasked direction was written")
    # exact zeros where a weight is never used
    for d in range(4):
        if not (mask >> d) & 1:
            continue
        g = out["gw"][d]
        first = {0: g[:, :, :, 0, :], 1: g[:, :, :, -1, :], 2: g[:, :, :, :, 0], 3: g[:, :, :, :, -1]}[d]
        assert not first.any()
        if d < 2:
            assert not g[:, :, 0, :, 0].any() and not g[:, :, 2, :, -1].any()
        else:
            assert not g[:, :, 0, 0, :].any() and not g[:, :, 2, -1, :].any()


BWD_SHAPES = [(2, 6, 9, 13, 3), (1, 4, 33, 70, 2), (1, 8, 65, 31, 8), (1, 2, 1, 37, 1), (1, 2, 37, 1, 2),
              (1, 1, 1, 1, 1), (1, 4, 130, 20, 1), (2, 8, 28, 28, 8), (2, 96, 28, 28, 2)]

# shapes the whole-plane backward kernel takes (H, W <= 32): per-channel weights with 8 / 4 / 2 channels
# per workgroup, a whole group per workgroup, a group split over two workgroups (atomic gw), several
# pairs per wave, one wave only, H != W, the 16 / 28 / 32 step variants
PLANE_BWD_SHAPES = [(2, 8, 28, 28, 8), (2, 96, 28, 28, 2), (1, 16, 28, 28, 4), (1, 24, 28, 28, 1), (1, 12, 16, 32, 3),
                    (3, 32, 2, 4, 32), (2, 4, 32, 32, 2), (1, 6, 12, 20, 3), (1, 8, 6, 10, 1), (1, 12, 28, 28, 12),
                    (1, 6, 8, 8, 6), (1, 2, 28, 28, 1), (1, 40, 28, 20, 1), (300, 16, 4, 4, 2)]

# shapes the line-by-line register-resident backward kernel takes (when the two-pass backward, which comes first in the
# dispatch, is switched off): larger maps, odd group sizes
# (56- and 112-wide maps read 56 / 112 B per row and request in the horizontal phases; twelve 56x56 channels in a
# group do not fit in LDS: two launches, the second adding onto the stored gw)
TILE_BWD_SHAPES = [(2, 8, 56, 56, 2), (1, 4, 56, 56, 4), (1, 8, 64, 128, 2), (1, 24, 16, 40, 2), (2, 8, 40, 32, 8),
                   (2, 8, 40, 32, 2), (2, 12, 56, 56, 1), (1, 4, 40, 112, 2)]


@pytest.mark.parametrize("shape", PLANE_BWD_SHAPES)
def test_backward_plane_kernel_shapes(shape):
    import paper_2512_07884_amd as G
    B, C, H, W, Gr = shape
    assert G.gspn_bwd_plan(B, C, H, W, Gr, 15, 0, 0) == "plane", shape
    check_bwd(WL.ScanConfig("bwdplane", B, C, H, W, Gr, "f32", 15, 1.0, 29))


# the same kernel in bf16 storage (H*W a multiple of 8; a group is never split: no atomics in bf16)
PLANE_BWD_BF16_SHAPES = [(2, 8, 28, 28, 8), (2, 16, 28, 28, 2), (1, 12, 16, 32, 3), (3, 32, 2, 4, 32), (2, 4, 32, 32, 2),
                         (1, 6, 12, 20, 3), (1, 24, 28, 28, 1), (1, 12, 28, 28, 12), (300, 16, 4, 4, 2)]


@pytest.mark.parametrize("shape", PLANE_BWD_BF16_SHAPES)
def test_backward_plane_kernel_shapes_bf16(shape, monkeypatch):
    import paper_2512_07884_amd as G
    monkeypatch.setenv("GSPN_BWD_NO_TWOPASS", "1")     # (the two-pass backward takes the larger of these maps first)
    B, C, H, W, Gr = shape
    assert G.gspn_bwd_plan(B, C, H, W, Gr, 15, 1, 0) == "plane", shape
    check_bwd(WL.ScanConfig("bwdplane16", B, C, H, W, Gr, "bf16", 15, 1.0, 53))


# lines of at most 16 / 8 positions with shared weights: four / eight channels per wave; planes that are not
# whole 16 B chunks, weight blocks moved in 16, 8, 4 and 2 B pieces, a group split over two workgroups
# (fp32, few groups), one to six waves, and the last stages of the paper's classifier (Sec. 5.2) with fewer images
PLANE_BWD_SMALL_SHAPES = [(2, 16, 14, 14, 2, "f32"), (2, 16, 7, 7, 2, "f32"), (1, 48, 7, 7, 1, "f32"), (1, 12, 14, 14, 1, "f32"),
                          (1, 8, 5, 6, 1, "f32"), (1, 4, 9, 9, 1, "f32"), (2, 8, 14, 10, 2, "f32"), (300, 16, 7, 7, 2, "f32"),
                          (2, 16, 14, 14, 2, "bf16"), (2, 16, 7, 7, 2, "bf16"), (3, 8, 5, 6, 1, "bf16"), (1, 24, 14, 14, 2, "bf16"),
                          (1, 8, 6, 14, 2, "bf16"), (1, 16, 8, 8, 2, "bf16"), (1, 48, 7, 7, 1, "bf16"),
                          (2, 384, 14, 14, 8, "f32"), (2, 768, 7, 7, 8, "f32"), (2, 384, 14, 14, 8, "bf16"), (2, 768, 7, 7, 8, "bf16")]


@pytest.mark.parametrize("shape", PLANE_BWD_SMALL_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_backward_plane_kernel_on_short_lines(shape):
    import paper_2512_07884_amd as G
    B, C, H, W, Gr, dtype = shape
    assert G.gspn_bwd_plan(B, C, H, W, Gr, 15, int(dtype == "bf16"), 0) == "plane", shape
    check_bwd(WL.ScanConfig("bwdsmall", B, C, H, W, Gr, dtype, 15, 1.0, 61))


@pytest.mark.parametrize("mask", [1, 2, 4, 8, 5, 10, 14])
@pytest.mark.parametrize("shape", [(2, 16, 7, 7, 2, "bf16"), (2, 8, 14, 14, 2, "f32")], ids=lambda s: "x".join(map(str, s)))
def test_backward_plane_kernel_direction_masks_on_short_lines(mask, shape):
    B, C, H, W, Gr, dtype = shape
    check_bwd(WL.ScanConfig("bwdsmallmask", B, C, H, W, Gr, dtype, mask, 1.0, 67))


@pytest.mark.parametrize("mask", [1, 2, 4, 8, 3, 12, 6, 9, 14])
def test_backward_plane_kernel_direction_masks_bf16(mask, monkeypatch):
    monkeypatch.setenv("GSPN_BWD_NO_TWOPASS", "1")
    check_bwd(WL.ScanConfig("bwdplane16mask", 2, 8, 28, 28, 2, "bf16", mask, 1.0, 59))


@pytest.mark.parametrize("shape", [(2, 8, 56, 56, 2), (1, 4, 56, 56, 4), (1, 8, 64, 128, 2), (1, 24, 16, 40, 2), (2, 8, 40, 32, 8),
                                   (2, 12, 56, 56, 1), (1, 4, 40, 112, 2)])
def test_backward_tile_kernel_shapes_bf16(shape, monkeypatch):
    import paper_2512_07884_amd as G
    monkeypatch.setenv("GSPN_BWD_NO_TWOPASS", "1")     # (the two-pass backward takes these maps first)
    B, C, H, W, Gr = shape
    assert G.gspn_bwd_plan(B, C, H, W, Gr, 15, 1, 0) == "tile", shape
    check_bwd(WL.ScanConfig("bwdtile16", B, C, H, W, Gr, "bf16", 15, 1.0, 61))


@pytest.mark.parametrize("mask", [1, 2, 4, 8, 3, 12, 6, 9])
def test_backward_tile_kernel_direction_masks_bf16(mask):
    check_bwd(WL.ScanConfig("bwdtile16mask", 1, 8, 40, 32, 2, "bf16", mask, 1.0, 67))


@pytest.mark.parametrize("shape", TILE_BWD_SHAPES)
def test_backward_tile_kernel_shapes(shape, monkeypatch):
    import paper_2512_07884_amd as G
    monkeypatch.setenv("GSPN_BWD_NO_TWOPASS", "1")
    B, C, H, W, Gr = shape
    assert G.gspn_bwd_plan(B, C, H, W, Gr, 15, 0, 0) == "tile", shape
    check_bwd(WL.ScanConfig("bwdtile", B, C, H, W, Gr, "f32", 15, 1.0, 29))


@pytest.mark.parametrize("shape", [(2, 8, 28, 28, 8), (2, 96, 28, 28, 2), (1, 16, 28, 28, 4), (1, 12, 16, 32, 3),
                                   (3, 32, 2, 4, 32)])
def test_backward_tile_kernel_on_shapes_the_plane_kernel_normally_takes(shape, monkeypatch):
    import paper_2512_07884_amd as G
    monkeypatch.setenv("GSPN_BWD_NO_PLANE", "1")
    monkeypatch.setenv("GSPN_BWD_NO_TWOPASS", "1")
    B, C, H, W, Gr = shape
    assert G.gspn_bwd_plan(B, C, H, W, Gr, 15, 0, 0) == "tile", shape
    check_bwd(WL.ScanConfig("bwdtile2", B, C, H, W, Gr, "f32", 15, 1.0, 29))


@pytest.mark.parametrize("mask", [1, 2, 4, 8, 3, 12, 5, 10, 14])
@pytest.mark.parametrize("G_", [8, 2])
@pytest.mark.parametrize("hw", [(28, 28), (40, 32)])
def test_backward_fast_kernels_direction_masks(mask, G_, hw, monkeypatch):
    import paper_2512_07884_amd as G
    monkeypatch.setenv("GSPN_BWD_NO_TWOPASS", "1")
    assert G.gspn_bwd_plan(2, 8, hw[0], hw[1], G_, mask, 0, 0) == ("plane" if hw[0] <= 32 else "tile")
    check_bwd(WL.ScanConfig("bwdmask2", 2, 8, hw[0], hw[1], G_, "f32", mask, 1.0, 31))


def test_backward_generic_kernel_on_tile_shapes(monkeypatch):
    import paper_2512_07884_amd as G
    monkeypatch.setenv("GSPN_FORCE_GENERIC", "1")
    assert G.gspn_bwd_plan(2, 8, 28, 28, 2, 15, 0, 0) == "generic"
    check_bwd(WL.ScanConfig("bwdgen", 2, 8, 28, 28, 2, "f32", 15, 1.0, 37))


@pytest.mark.parametrize("kernel", ["plane", "tile"])
def test_backward_is_bitwise_repeatable_with_split_groups(kernel, monkeypatch):
    import torch
    import paper_2512_07884_amd as G
    if kernel == "tile":
        monkeypatch.setenv("GSPN_BWD_NO_PLANE", "1")
        monkeypatch.setenv("GSPN_BWD_NO_TWOPASS", "1")
    assert G.gspn_bwd_plan(2, 96, 28, 28, 2, 15, 0, 0) == kernel
    cfg = WL.ScanConfig("bwdrep", 2, 96, 28, 28, 2, "f32", 15, 1.0, 41)     # 48 channels per group: two workgroups per group
    inp = WL.make_inputs(cfg)
    dev = {k: to_device(v, "f32") for k, v in inp.items()}
    hs = torch.empty_like(dev["lam"]); y = torch.empty_like(dev["x"])
    G.gspn_scan_fwd(dev["x"], dev["w"], dev["lam"], dev["u"], y, hs, G=cfg.G)
    outs = []
    for rep in range(3):
        gx = torch.full_like(dev["x"], float("nan")); gw = torch.full_like(dev["w"], float("nan"))
        gl = torch.full_like(dev["lam"], float("nan")); gu = torch.full_like(dev["lam"], float("nan"))
        G.gspn_scan_bwd(dev["gy"], dev["x"], dev["w"], dev["lam"], dev["u"], hs, gx, gw, gl, gu, G=cfg.G)
        torch.cuda.synchronize()
        outs.append([t.cpu().numpy().copy() for t in (gx, gw, gl, gu)])
    for k in range(4):
        assert np.array_equal(outs[0][k], outs[1][k]) and np.array_equal(outs[0][k], outs[2][k])


@pytest.mark.parametrize("shape", BWD_SHAPES)
def test_backward_fp32_shapes(shape):
    B, C, H, W, G = shape
    check_bwd(WL.ScanConfig("bwd", B, C, H, W, G, "f32", 15, 1.0, 13))


@pytest.mark.parametrize("mask", [1, 2, 4, 8, 6, 9])
def test_backward_direction_masks(mask):
    check_bwd(WL.ScanConfig("bwdmask", 2, 4, 14, 18, 2, "f32", mask, 1.0, 17))


def test_backward_generic_kernel_bf16(monkeypatch):
    import paper_2512_07884_amd as G
    monkeypatch.setenv("GSPN_FORCE_GENERIC", "1")
    assert G.gspn_bwd_plan(2, 6, 24, 20, 6, 15, 1, 0) == "generic"
    check_bwd(WL.ScanConfig("bwdgenbf16", 2, 6, 24, 20, 6, "bf16", 15, 1.0, 19))


@pytest.mark.parametrize("shape", [(2, 24, 57, 57, 2), (1, 64, 33, 70, 1), (1, 8, 1, 56, 2)], ids=lambda s: "x".join(map(str, s)))
def test_backward_generic_kernel_bf16_large_groups(shape):
    """Odd widths (and single rows) run the generic kernels; the sum of gw over the 12 / 64 channels of a group is taken
    in fp32 and rounded once, so the bf16 tolerance holds at any group size."""
    import paper_2512_07884_amd as G
    B, C, H, W, Gr = shape
    assert G.gspn_bwd_plan(B, C, H, W, Gr, 15, 1, 0) == "generic", shape
    check_bwd(WL.ScanConfig("bwdgenbig", B, C, H, W, Gr, "bf16", 15, 1.0, 83))


def test_backward_single_row_fp32():
    check_bwd(WL.ScanConfig("bwdonerow", 1, 8, 1, 28, 2, "f32", 15, 1.0, 89))


def test_backward_bf16_per_channel_weights():
    # bf16 storage with one channel per group: every gradient is rounded once
    check_bwd(WL.ScanConfig("bwdbf16", 2, 6, 24, 20, 6, "bf16", 15, 1.0, 19))


def test_backward_adjoint_identity_on_the_gpu():
    # <gy, scan(v)> == <gx, v> for the linear map x -> y, evaluated entirely on the GPU path
    import torch
    import paper_2512_07884_amd as G
    cfg = WL.ScanConfig("adj", 2, 8, 28, 28, 2, "f32", 15, 1.0, 23)
    inp = WL.make_inputs(cfg)
    out = run_bwd_gpu(inp, cfg, 15)
    v = np.random.default_rng(1).standard_normal(inp["x"].shape).astype(np.float32)
    dev = {k: to_device(a, "f32") for k, a in inp.items()}
    yv = torch.empty_like(dev["x"])
    G.gspn_scan_fwd(to_device(v, "f32"), dev["w"], dev["lam"], dev["u"], yv, None, G=cfg.G)
    lhs = float((to_host_f64(yv) * inp["gy"].astype(np.float64)).sum())
    rhs = float((out["gx"] * v.astype(np.float64)).sum())
    assert abs(lhs - rhs) <= 1e-4 * max(1.0, abs(lhs))
