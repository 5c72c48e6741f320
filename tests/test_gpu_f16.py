"""GPU parity of the scan calls in fp16 (IEEE binary16) storage against the fp64 oracle, through the C ABI.

fp16 storage runs every kernel family bf16 storage does except the single-launch backward tile kernel (the two passes,
else the generic kernel); the tile kernels in workgroups of at most four waves.  Tolerance: 1.25e-3 (max|gpu - oracle| / max|oracle| per
tensor): the bf16 bound scaled by the ratio of the two formats' rounding units; both sides consume the same
storage-rounded inputs, and the oracle's backward consumes its own states rounded to fp16 like h_save is.
"""
import numpy as np
import pytest

from gpu_util import TOL, rel_inf_err, to_device, to_host_f64, empty_like_dev
from oracle import gspn_oracle as O
from paper_2512_07884_amd import workloads as WL
from test_gpu_fwd import check_case
from test_gpu_bwd import check_bwd
from test_gpu_local import check_local
from test_gpu_logits import check_logits
from test_gpu_transposed import check as check_transposed

pytestmark = pytest.mark.gpu

F16 = 2   # GSPN_F16


def plans(B, C, H, W, Gr, mask=15):
    import paper_2512_07884_amd as G
    return (G.gspn_fwd_plan(B, C, H, W, Gr, mask, F16, 0, True), G.gspn_bwd_plan(B, C, H, W, Gr, mask, F16, 0))


# the whole-plane kernels: standard and flat layouts (rows that are no multiple of 16 B), shared and per-channel weights,
# the single-launch backward of the shortest lines and of per-channel weights, the two passes on the others
PLANE_SHAPES = [((2, 8, 56, 56, 2), "twopass"), ((2, 16, 28, 28, 2), "twopass"), ((2, 8, 14, 14, 8), "twopass"),
                ((2, 16, 7, 7, 2), "plane"), ((2, 48, 28, 28, 48), "plane"), ((2, 64, 32, 32, 2), "twopass"),
                ((1, 6, 40, 24, 3), "twopass"), ((1, 4, 2, 56, 2), "twopass"), ((2, 12, 56, 56, 1), "twopass"),
                ((3, 8, 5, 6, 1), "plane")]


@pytest.mark.parametrize("shape,bwd_plan", PLANE_SHAPES, ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else v)
def test_f16_on_the_plane_kernels(shape, bwd_plan):
    B, C, H, W, Gr = shape
    assert plans(B, C, H, W, Gr) == ("plane", bwd_plan)
    cfg = WL.ScanConfig("f16plane", B, C, H, W, Gr, "f16", 15, 2.0, 127)
    check_case(cfg)
    check_case(cfg, save_h=False)
    check_bwd(cfg)


def test_f16_on_the_single_launch_plane_backward(monkeypatch):
    monkeypatch.setenv("GSPN_BWD_NO_TWOPASS", "1")
    assert plans(2, 16, 28, 28, 2) == ("plane", "plane")
    check_bwd(WL.ScanConfig("f16bplane", 2, 16, 28, 28, 2, "f16", 15, 2.0, 129))
    check_local((2, 16, 28, 28, 2, "f16"), 9, poison_starts=True)
    check_logits((2, 16, 28, 28, 2, "f16"), kchunk=None, poison=True)


# the tile kernels' horizontal variants (rows of 112 B, rows split over waves, 64 B and 16 B bursts), shared and
# per-channel weights, many small planes per workgroup, maps of two rows, a group of twelve channels; the smaller maps
# with the plane kernels switched off
TILE_SHAPES = [(2, 8, 56, 56, 2), (1, 3, 128, 128, 1), (1, 8, 64, 64, 8), (2, 8, 40, 32, 2), (1, 6, 40, 24, 3),
               (2, 64, 32, 32, 2), (1, 8, 64, 128, 2), (1, 4, 96, 72, 2), (1, 4, 2, 56, 2), (2, 12, 56, 56, 1)]


@pytest.mark.parametrize("shape", TILE_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_f16_on_the_tile_kernels(shape, monkeypatch):
    monkeypatch.setenv("GSPN_FWD_NO_PLANE", "1")
    monkeypatch.setenv("GSPN_BWD_NO_PLANE", "1")
    B, C, H, W, Gr = shape
    assert plans(B, C, H, W, Gr) == ("tile", "twopass")
    cfg = WL.ScanConfig("f16tile", B, C, H, W, Gr, "f16", 15, 2.0, 131)
    check_case(cfg)
    check_case(cfg, save_h=False)
    check_bwd(cfg)


# the two-channel kernel of the 128 x 128 maps (an even number of channels per group): forward, h_save, reverse sweep;
# several pairs per workgroup; GSPN-local and logits on it
@pytest.mark.parametrize("shape", [(1, 4, 128, 128, 2), (2, 12, 128, 128, 2), (1, 8, 128, 128, 1)], ids=lambda s: "x".join(map(str, s)))
def test_f16_on_the_two_channel_kernel(shape, monkeypatch):
    monkeypatch.setenv("GSPN_FWD_NO_CHUNK", "1")
    B, C, H, W, Gr = shape
    assert plans(B, C, H, W, Gr) == ("pair", "twopass")
    cfg = WL.ScanConfig("f16pair", B, C, H, W, Gr, "f16", 15, 3.0, 163)
    check_case(cfg)
    check_case(cfg, save_h=False)
    check_bwd(cfg)
    check_local((B, C, H, W, Gr, "f16"), 37, poison_starts=True)
    check_local((B, C, H, W, Gr, "f16"), 32)
    check_logits((B, C, H, W, Gr, "f16"), kchunk=None, poison=True)
    check_logits((B, C, H, W, Gr, "f16"), kchunk=48, poison=True)


def test_f16_on_the_tile_kernel_for_128_rows(monkeypatch):
    monkeypatch.setenv("GSPN_FWD_NO_PAIR", "1")
    assert plans(1, 4, 128, 128, 2) == ("tile", "twopass")
    cfg = WL.ScanConfig("f16tile128", 1, 4, 128, 128, 2, "f16", 15, 3.0, 167)
    check_case(cfg)
    check_bwd(cfg)


# the stream kernels (maps beyond the LDS tile: rows and columns in multiples of 64): the whole-line variant with one and
# with two channels per workgroup, on 512, 256 and fewer rows; the general kernel with the variant switched off
@pytest.mark.parametrize("general", [False, None, True], ids=["whole-line-two-channels", "whole-line", "general"])
@pytest.mark.parametrize("shape", [(1, 2, 256, 256, 1), (1, 4, 128, 256, 2), (1, 2, 192, 512, 2), (1, 2, 512, 512, 2),
                                   (1, 2, 256, 1024, 1), (1, 3, 512, 512, 1), (1, 2, 256, 512, 2)], ids=lambda s: "x".join(map(str, s)))
def test_f16_on_the_stream_kernels(shape, general, monkeypatch):
    if general:
        monkeypatch.setenv("GSPN_STREAM_NO_STAGED", "1")
    elif general is False:
        monkeypatch.setenv("GSPN_STREAM_TWO_CHANNELS", "1")    # (so few planes keep one channel per workgroup otherwise)
    B, C, H, W, Gr = shape
    assert plans(B, C, H, W, Gr) == ("stream", "twopass")
    cfg = WL.ScanConfig("f16stream", B, C, H, W, Gr, "f16", 15, 1.0, 137)
    check_case(cfg)
    check_case(cfg, save_h=False)
    check_bwd(cfg)


# maps of 1024 rows (two launches: the vertical pair, then the horizontal pair; backward in two passes on them) and of
# 2048 rows (forward only; the backward call takes the generic kernel)
@pytest.mark.parametrize("shape,bwd_plan", [((1, 2, 1024, 256, 1), "twopass"), ((1, 2, 640, 512, 2), "twopass"),
                                            ((1, 2, 2048, 256, 1), "generic")],
                         ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else v)
def test_f16_on_maps_beyond_512_rows(shape, bwd_plan):
    B, C, H, W, Gr = shape
    assert plans(B, C, H, W, Gr) == ("stream", bwd_plan)
    cfg = WL.ScanConfig("f16big", B, C, H, W, Gr, "f16", 15, 1.0, 173)
    check_case(cfg)
    check_case(cfg, save_h=False)
    if bwd_plan == "twopass":
        check_bwd(cfg)


# GSPN-local with few planes: the stretches as work items (one workgroup per stretch), forward and reverse sweep
@pytest.mark.parametrize("shape,kchunk", [((1, 4, 128, 128, 2, "f16"), 32), ((1, 2, 256, 256, 1, "f16"), 64), ((1, 8, 64, 128, 2, "f16"), 8)],
                         ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else str(v))
def test_f16_local_scans_on_the_chunk_axis(shape, kchunk):
    import paper_2512_07884_amd as G
    B, C, H, W, Gr, _ = shape
    assert G.gspn_fwd_local_plan(B, C, H, W, Gr, kchunk, 15, F16, 0, True) == "chunk"
    check_local(shape, kchunk, poison_starts=True)


# every other shape: odd widths, a single row or column, lines longer than a wave, more than 512 rows that are no
# multiple of 64, 64 channels per group (the channel sum of gw is fp32 and rounded once)
@pytest.mark.parametrize("shape", [(2, 6, 9, 13, 3), (1, 4, 33, 70, 2), (1, 2, 1, 37, 1), (1, 2, 37, 1, 2), (1, 1, 1, 1, 1),
                                   (1, 3, 300, 5, 3), (1, 64, 33, 35, 1), (1, 2, 640, 64, 1)], ids=lambda s: "x".join(map(str, s)))
def test_f16_on_the_generic_kernels(shape):
    B, C, H, W, Gr = shape
    assert plans(B, C, H, W, Gr) == ("generic", "generic")
    cfg = WL.ScanConfig("f16generic", B, C, H, W, Gr, "f16", 15, 1.0, 139)
    check_case(cfg)
    check_bwd(cfg)


@pytest.mark.parametrize("mask", [1, 2, 4, 8, 6, 9, 14])
@pytest.mark.parametrize("hw", [(56, 56), (128, 256), (9, 13)], ids=lambda v: "x".join(map(str, v)))
def test_f16_direction_masks(mask, hw):
    cfg = WL.ScanConfig("f16mask", 1, 4, hw[0], hw[1], 2, "f16", mask, 1.0, 149)
    check_case(cfg)
    check_bwd(cfg)


def test_f16_with_shared_parameter_slots():
    import paper_2512_07884_amd as G
    cfg = WL.ScanConfig("f16shared", 1, 4, 56, 56, 2, "f16", 15, 1.0, 151)
    inp = WL.make_inputs(cfg, with_gy=False)
    one = {k: (v[:1].copy() if k in ("w", "lam", "u") else v) for k, v in inp.items()}
    rep = {k: (np.repeat(v, 4, axis=0) if k in ("w", "lam", "u") else v) for k, v in one.items()}
    f = WL.inputs_as_f64(rep, "f16")
    y_ref, _ = O.scan_fwd(f["x"], f["w"], f["lam"], f["u"], 15)
    import torch
    dev = {k: to_device(v, "f16") for k, v in one.items()}
    y = empty_like_dev((1, 4, 56, 56), "f16", float("nan"))
    G.gspn_scan_fwd(dev["x"], dev["w"], dev["lam"], dev["u"], y, None, G=2, dir_mask=15, flags=1)   # GSPN_FLAG_SHARED_PARAMS
    torch.cuda.synchronize()
    assert rel_inf_err(to_host_f64(y), y_ref) <= TOL["f16"]


# GSPN-local and weights as logits: the local instantiations of the tile and stream kernels, the generic kernels;
# stretch lengths that divide the map and that do not; the first line of every stretch never read
@pytest.mark.parametrize("shape,kchunk", [((2, 8, 56, 56, 2, "f16"), 14), ((1, 3, 128, 128, 1, "f16"), 37), ((1, 2, 256, 256, 1, "f16"), 64),
                                          ((2, 6, 9, 13, 3, "f16"), 4), ((2, 8, 28, 28, 8, "f16"), 1)],
                         ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else str(v))
def test_f16_local_scans(shape, kchunk, monkeypatch):
    monkeypatch.setenv("GSPN_FWD_NO_CHUNK", "1")
    check_local(shape, kchunk, poison_starts=True)


@pytest.mark.parametrize("shape,kchunk", [((2, 8, 56, 56, 2, "f16"), None), ((1, 3, 128, 128, 1, "f16"), 32), ((1, 2, 128, 256, 2, "f16"), None),
                                          ((2, 6, 9, 13, 3, "f16"), None), ((2, 8, 28, 28, 8, "f16"), 9)],
                         ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else str(v))
def test_f16_weights_as_logits(shape, kchunk):
    check_logits(shape, kchunk=kchunk, poison=True)


# the forward scan with the horizontal directions stored transposed (tile kernel in its transposed layout, generic kernel)
@pytest.mark.parametrize("shape", [(1, 4, 128, 128, 2, "f16"), (2, 8, 56, 56, 2, "f16"), (1, 4, 33, 70, 2, "f16")],
                         ids=lambda s: "x".join(map(str, s)))
def test_f16_with_the_horizontal_directions_stored_transposed(shape):
    check_transposed(shape)


def test_f16_values_beyond_bf16_resolution_survive():
    """Inputs that differ only below bf16's resolution give different outputs: the call does not pass through bf16."""
    cfg = WL.ScanConfig("f16res", 1, 2, 56, 56, 1, "f16", 15, 1.0, 157)
    inp = WL.make_inputs(cfg, with_gy=False)
    x = WL.storage_to_f64(inp["x"], "f16")
    inp2 = dict(inp)
    inp2["x"] = WL.to_storage(x * (1.0 + 2.0 ** -9), "f16")            # one or two fp16 steps, half a bf16 step
    assert np.any(inp2["x"] != inp["x"])
    from gpu_util import run_fwd_gpu
    y1, *_ = run_fwd_gpu(inp, cfg, 15)
    y2, *_ = run_fwd_gpu(inp2, cfg, 15)
    f2 = WL.inputs_as_f64(inp2, "f16")
    y2_ref, _ = O.scan_fwd(f2["x"], f2["w"], f2["lam"], f2["u"], 15)
    assert rel_inf_err(y2, y2_ref) <= TOL["f16"]
    assert np.any(y1 != y2)
