"""GPU parity of gspn_scan_fwd against the fp64 oracle, through the C ABI.

Tolerances (max|gpu - oracle| / max|oracle| per tensor): 1e-5 for fp32 storage,
1e-2 for bf16 storage.  Both sides consume the same storage-rounded inputs.
"""
import numpy as np
import pytest

from gpu_util import TOL, rel_inf_err, run_fwd_gpu, to_device, to_host_f64, empty_like_dev
from oracle import gspn_oracle as O
from paper_2512_07884_amd import workloads as WL

pytestmark = pytest.mark.gpu


def check_case(cfg, dir_mask=None, save_h=True, slots_nan=True):
    mask = cfg.dir_mask if dir_mask is None else dir_mask
    inp = WL.make_inputs(cfg, with_gy=False)
    f = WL.inputs_as_f64(inp, cfg.dtype)
    y_ref, h_ref = O.scan_fwd(f["x"], f["w"], f["lam"], f["u"], mask)
    if slots_nan:   # slots of unmasked directions must never be read
        nanv = np.float32(np.nan) if cfg.dtype == "f32" else np.uint16(0x7FC0)
        for d in range(4):
            if not (mask >> d) & 1:
                for k in ("w", "lam", "u"):
                    inp[k][d] = nanv
    y, h, *_ = run_fwd_gpu(inp, cfg, mask, save_h=save_h)
    tol = TOL[cfg.dtype]
    assert np.all(np.isfinite(y)), cfg
    err = rel_inf_err(y, y_ref)
    assert err <= tol, (cfg, mask, "y", err)
    if save_h:
        for d in range(4):
            if (mask >> d) & 1:
                e = rel_inf_err(h[d], h_ref[d])
                assert e <= tol, (cfg, mask, "h", d, e)
            else:
                assert np.all(np.isnan(h[d])), "slot of an unmasked direction was written"
    return err


def test_unit16_single_direction_fp32():
    check_case(WL.CONFIGS["unit16"])


SHAPES = [  # B, C, H, W, G
    (2, 6, 9, 13, 3), (1, 4, 33, 70, 2), (1, 8, 65, 31, 8), (2, 4, 130, 67, 1),
    (1, 2, 1, 37, 1), (1, 2, 37, 1, 2), (1, 1, 1, 1, 1), (1, 3, 300, 5, 3), (1, 2, 5, 300, 1),
    (3, 5, 2, 2, 5), (1, 2, 64, 64, 1), (1, 2, 63, 65, 2),
    # lines longer than one wave at one row per lane: rows split over 2, 3, 4 waves (even and ragged parts)
    (1, 4, 128, 64, 2), (1, 2, 192, 128, 1), (1, 2, 256, 64, 2), (2, 3, 96, 64, 1), (1, 2, 130, 64, 1),
    # rows of 224 B in bf16: two bursts of 112 B per row
    (1, 4, 40, 112, 2),
    # maps too large for an on-chip output tile: output accumulated in global memory
    (1, 2, 256, 256, 1), (1, 3, 192, 512, 3), (1, 2, 64, 1024, 1), (2, 2, 320, 256, 2),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", SHAPES)
def test_ragged_shapes_all_directions(shape, dtype):
    B, C, H, W, G = shape
    check_case(WL.ScanConfig("ragged", B, C, H, W, G, dtype, 15, 1.0, 7))
    check_case(WL.ScanConfig("ragged", B, C, H, W, G, dtype, 15, 1.0, 8), save_h=False)


@pytest.mark.parametrize("mask", [1, 2, 4, 8, 3, 12, 5, 10, 7, 14])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_direction_masks(mask, dtype):
    check_case(WL.ScanConfig("mask", 2, 4, 20, 24, 2, dtype, mask, 1.0, 11))


SHRUNK = [
    WL.shrink(WL.CONFIGS["cls56"], B=2, C=24, G=2),               # 56x56, 12 channels per group
    WL.shrink(WL.CONFIGS["cls56"], B=2, C=24, G=2, dtype="f32"),
    WL.shrink(WL.CONFIGS["diff128"], B=1, C=128, G=2),            # 128x128, cpg 64, peaked weights
    WL.shrink(WL.CONFIGS["long512"], C=4, G=2),
    WL.shrink(WL.CONFIGS["long256x1024"], C=4, G=2),
    WL.shrink(WL.CONFIGS["long256x1024"], C=2, G=1, H=1024, W=256),
    WL.shrink(WL.CONFIGS["train28_gc"], B=2, C=16, G=16),
    WL.shrink(WL.CONFIGS["train28_g4"], B=2, C=96, G=2),
    WL.shrink(WL.CONFIGS["train28_g4"], B=2, C=96, G=2, dtype="bf16"),
]


@pytest.mark.parametrize("cfg", SHRUNK, ids=lambda c: f"{c.name}-{c.B}x{c.C}x{c.H}x{c.W}-G{c.G}-{c.dtype}")
def test_benchmark_shapes_with_fewer_channels(cfg):
    check_case(cfg)
    check_case(cfg, save_h=False)


def test_kernel_families_by_shape():
    import paper_2512_07884_amd as G
    assert G.gspn_fwd_plan(2, 1024, 128, 128, 16, 15, 1, 0, False) == "pair"
    assert G.gspn_fwd_plan(2, 1024, 128, 128, 1024, 15, 1, 0, False) == "tile"      # one channel per group: nothing to share
    assert G.gspn_fwd_plan(2, 1024, 128, 128, 16, 7, 1, 0, False) == "tile"        # not all four directions
    assert G.gspn_fwd_plan(2, 1024, 128, 128, 16, 15, 0, 0, False) == "tile"       # fp32 storage
    assert G.gspn_fwd_plan(64, 96, 56, 56, 8, 15, 1, 0, False) == "plane"
    assert G.gspn_fwd_plan(32, 192, 28, 28, 4, 15, 0, 0, True) == "plane"
    assert G.gspn_fwd_plan(32, 192, 28, 28, 192, 15, 0, 0, True) == "plane"
    assert G.gspn_fwd_plan(2, 8, 56, 56, 2, 15, 0, 0, False) == "tile"          # fp32 56x56 planes exceed the plane kernel's 8 KB
    assert G.gspn_fwd_plan(1, 512, 512, 512, 16, 15, 1, 0, False) == "stream"
    assert G.gspn_fwd_plan(1, 512, 256, 1024, 16, 15, 1, 0, False) == "stream"
    assert G.gspn_fwd_plan(1, 2, 256, 256, 1, 15, 0, 0, False) == "stream"
    assert G.gspn_fwd_plan(1, 2, 256, 256, 1, 15, 0, 0, True) == "stream"       # ... with h_save too (global scan)
    assert G.gspn_fwd_plan(1, 2, 130, 67, 1, 15, 0, 0, False) == "generic"


@pytest.mark.parametrize("mask", [1, 2, 4, 8, 3, 12, 6, 9, 14])
def test_direction_masks_on_large_maps(mask):
    check_case(WL.ScanConfig("maskbig", 1, 2, 256, 256, 1, "bf16", mask, 1.0, 15), save_h=False)
    check_case(WL.ScanConfig("maskbig", 1, 2, 128, 256, 2, "f32", mask, 1.0, 16), save_h=False)


@pytest.mark.parametrize("shape", [(1, 4, 12, 10, 2, "f32"), (1, 16, 7, 7, 2, "bf16"), (1, 8, 14, 14, 8, "f32"),
                                   (1, 4, 28, 24, 2, "bf16"), (1, 2, 40, 40, 1, "f32"), (1, 3, 9, 11, 3, "bf16"),
                                   (1, 4, 128, 128, 2, "bf16")],
                         ids=lambda s: "x".join(map(str, s)))
def test_weights_that_are_never_read_may_hold_anything(shape):
    """The first line of a scan has no predecessor and the end positions of a line have no neighbour outside
    it (Eq. 1 with a zero initial state, Sec. 3.2): what w holds there must not reach the output."""
    B, C, H, W, Gr, dtype = shape
    cfg = WL.ScanConfig("poison", B, C, H, W, Gr, dtype, 15, 1.0, 3)
    inp = WL.make_inputs(cfg, with_gy=False)
    f = WL.inputs_as_f64(inp, cfg.dtype)
    y_ref, _ = O.scan_fwd(f["x"], f["w"], f["lam"], f["u"], 15)
    w = inp["w"]
    nan, inf, ninf = ((np.nan, np.inf, -np.inf) if dtype == "f32" else
                      (np.uint16(0x7FC0), np.uint16(0x7F80), np.uint16(0xFF80)))
    w[0, :, :, :, 0, :] = nan; w[1, :, :, :, -1, :] = inf             # first line of each scan
    w[2, :, :, :, :, 0] = nan; w[3, :, :, :, :, -1] = ninf
    w[0, :, :, 0, :, 0] = nan; w[0, :, :, 2, :, -1] = inf             # out-of-line neighbours
    w[1, :, :, 0, :, 0] = inf; w[1, :, :, 2, :, -1] = nan
    w[2, :, :, 0, 0, :] = nan; w[2, :, :, 2, -1, :] = nan
    w[3, :, :, 0, 0, :] = inf; w[3, :, :, 2, -1, :] = nan
    y, *_ = run_fwd_gpu(inp, cfg, 15)
    assert np.all(np.isfinite(y)) and rel_inf_err(y, y_ref) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_shared_parameter_flag(dtype):
    cfg = WL.ScanConfig("shared", 2, 6, 17, 17, 3, dtype, 15, 1.0, 5)
    inp = WL.make_inputs(cfg, with_gy=False)
    # one parameter set for all directions: plain (not border-renormalised) weights are fine for parity
    one = {"x": inp["x"], "w": inp["w"][:1].copy(), "lam": inp["lam"][:1].copy(), "u": inp["u"][:1].copy()}
    rep = {"x": inp["x"], "w": np.repeat(one["w"], 4, 0), "lam": np.repeat(one["lam"], 4, 0),
           "u": np.repeat(one["u"], 4, 0)}
    f = WL.inputs_as_f64(rep, dtype)
    y_ref, _ = O.scan_fwd(f["x"], f["w"], f["lam"], f["u"], 15)
    y, *_ = run_fwd_gpu(one, cfg, 15, flags=1)
    assert rel_inf_err(y, y_ref) <= TOL[dtype]


def test_runs_on_a_side_stream_and_is_bitwise_repeatable():
    import torch
    import paper_2512_07884_amd as G
    cfg = WL.ScanConfig("stream", 2, 8, 40, 36, 2, "bf16", 15, 1.0, 9)
    inp = WL.make_inputs(cfg, with_gy=False)
    dev = {k: to_device(v, cfg.dtype) for k, v in inp.items()}
    outs = []
    s = torch.cuda.Stream()
    for rep in range(3):
        y = empty_like_dev(inp["x"].shape, cfg.dtype, float("nan"))
        torch.cuda.synchronize()
        with torch.cuda.stream(s):
            G.gspn_scan_fwd(dev["x"], dev["w"], dev["lam"], dev["u"], y, None, G=cfg.G, stream=s)
        s.synchronize()
        outs.append(y.view(torch.int16).cpu().numpy())
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])
    f = WL.inputs_as_f64(inp, cfg.dtype)
    y_ref, _ = O.scan_fwd(f["x"], f["w"], f["lam"], f["u"], 15)
    assert rel_inf_err(to_host_f64(y), y_ref) <= TOL["bf16"]


def test_library_reports_shape_errors_through_the_binding():
    import torch
    import paper_2512_07884_amd as G
    x = torch.zeros(1, 4, 8, 8, device="cuda")
    w = torch.zeros(4, 1, 3, 3, 8, 8, device="cuda")      # G = 3 does not divide C = 4
    lam = torch.zeros(4, 1, 4, 8, 8, device="cuda")
    y = torch.full((1, 4, 8, 8), 7.0, device="cuda")
    with pytest.raises(G.GspnError) as ei:
        G.gspn_scan_fwd(x, w, lam, lam, y, None)
    assert ei.value.status == 2
    assert torch.all(y == 7.0)                               # outputs untouched on argument errors


@pytest.mark.parametrize("cfg", [SHRUNK[0], SHRUNK[2], SHRUNK[6], SHRUNK[7]],
                         ids=lambda c: f"{c.name}-{c.dtype}")
def test_generic_kernel_on_shapes_the_fast_kernels_normally_take(cfg, monkeypatch):
    import paper_2512_07884_amd as G
    dt = int(cfg.dtype == "bf16")
    assert G.gspn_fwd_plan(cfg.B, cfg.C, cfg.H, cfg.W, cfg.G, 15, dt, 0, True) in ("tile", "plane", "pair")
    monkeypatch.setenv("GSPN_FORCE_GENERIC", "1")
    assert G.gspn_fwd_plan(cfg.B, cfg.C, cfg.H, cfg.W, cfg.G, 15, dt, 0, True) == "generic"
    check_case(cfg)


def test_both_kernel_families_agree_closely(monkeypatch):
    # the tile kernel (one rounding of the merged sum) and the generic kernel (one per direction)
    # must agree to storage precision on the same inputs
    cfg = SHRUNK[0]
    inp = WL.make_inputs(cfg, with_gy=False)
    y_tile, *_ = run_fwd_gpu(inp, cfg, 15)
    monkeypatch.setenv("GSPN_FORCE_GENERIC", "1")
    y_gen, *_ = run_fwd_gpu(inp, cfg, 15)
    assert rel_inf_err(y_gen, y_tile) <= 1e-2


# shapes the whole-plane forward kernel takes (lines <= 64, planes <= 8 KB): shared weights with 1 / 2
# channels per wave, per-channel weights, several waves, H != W, ragged last chunk, a single wave
PLANE_FWD_SHAPES = [(2, 24, 56, 56, 2, "bf16"), (2, 16, 28, 28, 2, "f32"), (2, 8, 28, 28, 8, "f32"), (1, 12, 16, 32, 3, "f32"),
                    (1, 6, 40, 24, 3, "bf16"), (3, 32, 2, 4, 32, "f32"), (1, 8, 64, 64, 8, "bf16"), (1, 4, 12, 20, 2, "f32"),
                    (1, 3, 28, 28, 3, "f32"), (2, 10, 8, 16, 5, "bf16"), (1, 2, 33, 40, 1, "bf16"), (5, 7, 20, 8, 1, "f32"),
                    # small groups: more weight chunks than the threads prefetch
                    (2, 8, 28, 28, 2, "f32"), (1, 2, 64, 64, 1, "bf16"), (1, 4, 56, 56, 2, "bf16"), (1, 1, 32, 32, 1, "f32")]


@pytest.mark.parametrize("shape", PLANE_FWD_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_forward_plane_kernel_shapes(shape):
    import paper_2512_07884_amd as G
    B, C, H, W, Gr, dtype = shape
    dt = int(dtype == "bf16")
    assert G.gspn_fwd_plan(B, C, H, W, Gr, 15, dt, 0, True) == "plane", shape
    cfg = WL.ScanConfig("fwdplane", B, C, H, W, Gr, dtype, 15, 1.0, 43)
    check_case(cfg)
    check_case(cfg, save_h=False)


# maps whose rows are not whole 16 B chunks (unpadded planes in LDS, 2 / 4 / 8 channels per wave): shared
# weights fetched in 16, 8, 4 and 2 B pieces, per-channel weights, H != W, one to six waves, and the later
# stages of the paper's classifier (Sec. 5.2: 28x28, 14x14, 7x7) with fewer images
FLAT_FWD_SHAPES = [(2, 16, 28, 28, 2, "bf16"), (2, 8, 14, 14, 2, "f32"), (2, 16, 14, 14, 2, "bf16"), (2, 16, 7, 7, 2, "bf16"),
                   (2, 16, 7, 7, 2, "f32"), (1, 8, 7, 7, 8, "f32"), (2, 16, 7, 7, 16, "bf16"), (1, 8, 14, 14, 8, "bf16"),
                   (3, 8, 5, 6, 1, "bf16"), (1, 4, 9, 9, 1, "f32"), (1, 24, 14, 14, 2, "bf16"), (2, 2, 28, 28, 1, "bf16"),
                   (1, 8, 6, 14, 2, "bf16"), (1, 4, 12, 10, 2, "f32"), (1, 2, 30, 30, 2, "f32"), (1, 4, 28, 28, 4, "bf16"),
                   (2, 192, 28, 28, 8, "bf16"), (2, 384, 14, 14, 8, "bf16"), (2, 384, 14, 14, 8, "f32"),
                   (2, 768, 7, 7, 8, "bf16"), (2, 768, 7, 7, 8, "f32")]


@pytest.mark.parametrize("shape", FLAT_FWD_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_forward_plane_kernel_on_maps_with_ragged_rows(shape):
    import paper_2512_07884_amd as G
    B, C, H, W, Gr, dtype = shape
    assert G.gspn_fwd_plan(B, C, H, W, Gr, 15, int(dtype == "bf16"), 0, True) == "plane", shape
    cfg = WL.ScanConfig("fwdflat", B, C, H, W, Gr, dtype, 15, 1.0, 53)
    check_case(cfg)
    check_case(cfg, save_h=False)


@pytest.mark.parametrize("mask", [1, 2, 4, 8, 5, 10, 7])
@pytest.mark.parametrize("shape", [(2, 8, 14, 14, 2, "bf16"), (1, 8, 7, 7, 8, "f32")], ids=lambda s: "x".join(map(str, s)))
def test_forward_plane_kernel_direction_masks_on_ragged_rows(mask, shape):
    B, C, H, W, Gr, dtype = shape
    check_case(WL.ScanConfig("fwdflatmask", B, C, H, W, Gr, dtype, mask, 1.0, 59))


@pytest.mark.parametrize("mask", [1, 2, 4, 8, 3, 12, 6, 9, 14])
@pytest.mark.parametrize("G_", [8, 2])
def test_forward_plane_kernel_direction_masks(mask, G_):
    check_case(WL.ScanConfig("fwdplanemask", 2, 8, 28, 24, G_, "bf16", mask, 1.0, 47))


@pytest.mark.parametrize("shape", [(2, 24, 56, 56, 2, "bf16"), (2, 16, 28, 28, 2, "f32"), (2, 8, 28, 28, 8, "f32"),
                                   (1, 12, 16, 32, 3, "f32")], ids=lambda s: "x".join(map(str, s)))
def test_tile_kernel_on_shapes_the_plane_kernel_normally_takes(shape, monkeypatch):
    import paper_2512_07884_amd as G
    monkeypatch.setenv("GSPN_FWD_NO_PLANE", "1")
    B, C, H, W, Gr, dtype = shape
    assert G.gspn_fwd_plan(B, C, H, W, Gr, 15, int(dtype == "bf16"), 0, True) == "tile", shape
    cfg = WL.ScanConfig("fwdtile2", B, C, H, W, Gr, dtype, 15, 1.0, 43)
    check_case(cfg)
    check_case(cfg, save_h=False)


@pytest.mark.parametrize("bcg", [(1, 2, 1), (2, 12, 2), (1, 6, 1), (3, 4, 2)], ids=lambda s: "x".join(map(str, s)))
def test_two_channel_kernel_on_128x128_maps(bcg):
    """128x128 bf16 maps with an even number of channels per weight group: two channels of a group per workgroup,
    the merged output accumulated in storage precision on chip (four roundings, inside the 1e-2 of the tolerance)."""
    import paper_2512_07884_amd as G
    B, C, Gr = bcg
    assert G.gspn_fwd_plan(B, C, 128, 128, Gr, 15, 1, 0, True) == "pair" and G.gspn_fwd_plan(B, C, 128, 128, Gr, 15, 1, 0, False) == "pair"
    cfg = WL.ScanConfig("pair128", B, C, 128, 128, Gr, "bf16", 15, 3.0, 61)
    check_case(cfg)
    check_case(cfg, save_h=False)


@pytest.mark.parametrize("bcg", [(1, 600, 4), (3, 344, 2)], ids=lambda s: "x".join(map(str, s)))
def test_two_channel_kernel_when_a_workgroup_works_through_several_pairs(bcg):
    """More pairs of channels than workgroups in the launch (one per compute unit): every workgroup works through
    several pairs, the last round is short (300 and 516 pairs on 256 workgroups), and the requests for the next pair
    are already on their way while the current one finishes."""
    B, C, Gr = bcg
    cfg = WL.ScanConfig("pairrounds", B, C, 128, 128, Gr, "bf16", 15, 2.0, 71)
    check_case(cfg)
    check_case(cfg, save_h=False)


def test_two_channel_kernel_with_one_parameter_set_for_all_directions():
    import paper_2512_07884_amd as G
    cfg = WL.ScanConfig("pairshared", 1, 4, 128, 128, 2, "bf16", 15, 1.0, 67)
    assert G.gspn_fwd_plan(cfg.B, cfg.C, cfg.H, cfg.W, cfg.G, 15, 1, 1, False) == "pair"
    inp = WL.make_inputs(cfg, with_gy=False)
    one = {"x": inp["x"], "w": inp["w"][:1].copy(), "lam": inp["lam"][:1].copy(), "u": inp["u"][:1].copy()}
    rep = {"x": inp["x"], "w": np.repeat(one["w"], 4, 0), "lam": np.repeat(one["lam"], 4, 0), "u": np.repeat(one["u"], 4, 0)}
    f = WL.inputs_as_f64(rep, "bf16")
    y_ref, _ = O.scan_fwd(f["x"], f["w"], f["lam"], f["u"], 15)
    y, *_ = run_fwd_gpu(one, cfg, 15, flags=1)
    assert rel_inf_err(y, y_ref) <= TOL["bf16"]


def test_one_channel_tile_kernel_on_the_maps_the_two_channel_kernel_normally_takes(monkeypatch):
    import paper_2512_07884_amd as G
    monkeypatch.setenv("GSPN_FWD_NO_PAIR", "1")
    assert G.gspn_fwd_plan(1, 4, 128, 128, 2, 15, 1, 0, True) == "tile"
    cfg = WL.ScanConfig("tile128", 1, 4, 128, 128, 2, "bf16", 15, 3.0, 63)
    check_case(cfg)
    check_case(cfg, save_h=False)


@pytest.mark.parametrize("shape", [(1, 2, 2, 16384), (1, 2, 16384, 2)], ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_longest_supported_line(shape, dtype):
    """GSPN_MAX_LINE positions per line / lines per scan (generic kernel).  In fp32 storage the bound on the
    error of S sequential fp32 steps with non-expanding weights is S * 2^-24 (1e-3 here), which replaces the
    1e-5 of the short scans.  In bf16 storage a plane of this size does not fit the kernel's fp32 output tile
    beside its two line buffers, so the running sum of the directions is rounded in place once per direction:
    the k-th rounding is at most 2^-8 (half a unit in the last of bf16's 8 significant bits) of the largest
    partial sum after k directions, and the tolerance is the sum of those four bounds, taken from the oracle's
    per-direction outputs (1e-2 where it is smaller)."""
    import paper_2512_07884_amd as G
    B, C, H, W = shape
    assert G.gspn_fwd_plan(B, C, H, W, 1, 15, int(dtype == "bf16"), 0, False) == "generic"
    cfg = WL.ScanConfig("maxline", B, C, H, W, 1, dtype, 15, 1.0, 73)
    inp = WL.make_inputs(cfg, with_gy=False)
    f = WL.inputs_as_f64(inp, dtype)
    y_ref, _ = O.scan_fwd(f["x"], f["w"], f["lam"], f["u"], 15)
    y, *_ = run_fwd_gpu(inp, cfg, 15)
    if dtype == "bf16":
        partial, bound = np.zeros_like(y_ref), 0.0
        for d in range(4):
            partial = partial + O.scan_fwd(f["x"], f["w"], f["lam"], f["u"], 1 << d)[0]
            bound += 2.0 ** -8 * np.max(np.abs(partial))
        tol = max(TOL["bf16"], bound / np.max(np.abs(y_ref)))
    else:
        tol = max(TOL["f32"], 16384 * 2.0 ** -24)
    assert np.all(np.isfinite(y))
    assert rel_inf_err(y, y_ref) <= tol


@pytest.mark.parametrize("shape", [(1, 8, 1, 56, 2, "bf16"), (1, 8, 1, 28, 2, "f32"), (2, 4, 1, 112, 4, "bf16")],
                         ids=lambda s: "x".join(map(str, s)))
def test_maps_of_a_single_row(shape):
    """H = 1 with rows the register-resident kernels would otherwise accept: the vertical pair has no mid-scan
    meeting on such a map, so it must run elsewhere (all four directions, with and without h_save)."""
    import paper_2512_07884_amd as G
    B, C, H, W, Gr, dtype = shape
    assert G.gspn_fwd_plan(B, C, H, W, Gr, 15, int(dtype == "bf16"), 0, True) in ("generic", "plane"), shape
    cfg = WL.ScanConfig("onerow", B, C, H, W, Gr, dtype, 15, 1.0, 79)
    check_case(cfg)
    check_case(cfg, save_h=False)
