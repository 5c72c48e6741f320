"""GPU parity of the GSPN-local calls (Sec. 3.2: propagation confined to stretches of kchunk lines)
against the fp64 oracle, through the C ABI, forward and backward, on every kernel family."""
import numpy as np
import pytest

from gpu_util import TOL, rel_inf_err, to_device, to_host_f64, empty_like_dev
from oracle import gspn_oracle as O
from paper_2512_07884_amd import workloads as WL

pytestmark = pytest.mark.gpu


def run_local(inp, cfg, kchunk, mask, backward):
    import torch
    import paper_2512_07884_amd as G
    dev = {k: to_device(v, cfg.dtype) for k, v in inp.items()}
    B, C, H, W = inp["x"].shape
    nan = float("nan")
    y = empty_like_dev((B, C, H, W), cfg.dtype, nan)
    hs = empty_like_dev((4, B, C, H, W), cfg.dtype, nan)
    G.gspn_scan_fwd_local(dev["x"], dev["w"], dev["lam"], dev["u"], y, hs, kchunk=kchunk, G=cfg.G, dir_mask=mask)
    y2 = empty_like_dev((B, C, H, W), cfg.dtype, nan)
    G.gspn_scan_fwd_local(dev["x"], dev["w"], dev["lam"], dev["u"], y2, None, kchunk=kchunk, G=cfg.G, dir_mask=mask)
    out = {"y": to_host_f64(y), "y_nosave": to_host_f64(y2), "h": to_host_f64(hs)}
    if backward:
        gx = empty_like_dev((B, C, H, W), cfg.dtype, nan)
        gw = empty_like_dev((4, B, cfg.G, 3, H, W), cfg.dtype, nan)
        glam = empty_like_dev((4, B, C, H, W), cfg.dtype, nan)
        gu = empty_like_dev((4, B, C, H, W), cfg.dtype, nan)
        G.gspn_scan_bwd_local(dev["gy"], dev["x"], dev["w"], dev["lam"], dev["u"], hs, gx, gw, glam, gu,
                              kchunk=kchunk, G=cfg.G, dir_mask=mask)
        out.update(gx=to_host_f64(gx), gw=to_host_f64(gw), glam=to_host_f64(glam), gu=to_host_f64(gu))
    torch.cuda.synchronize()
    return out


def check_local(shape, kchunk, mask=15, backward=True, seed=83, poison_starts=False):
    B, C, H, W, Gr, dtype = shape
    cfg = WL.ScanConfig("local", B, C, H, W, Gr, dtype, mask, 1.0, seed)
    inp = WL.make_inputs(cfg, with_gy=True)
    f = WL.inputs_as_f64(inp, dtype)
    y_ref, h_ref = O.scan_fwd_local(f["x"], f["w"], f["lam"], f["u"], kchunk, mask)
    if poison_starts:
        # the weights of a stretch's first line in scan order are never read: they may hold anything
        nan = np.nan if dtype == "f32" else np.uint16(0x7FC0)
        w = inp["w"]
        for lo in range(0, H, kchunk):
            w[0, :, :, :, lo, :] = nan
            w[1, :, :, :, min(lo + kchunk, H) - 1, :] = nan
        for lo in range(0, W, kchunk):
            w[2, :, :, :, :, lo] = nan
            w[3, :, :, :, :, min(lo + kchunk, W) - 1] = nan
    out = run_local(inp, cfg, kchunk, mask, backward)
    tol = TOL[dtype]
    assert rel_inf_err(out["y"], y_ref) <= tol, ("y", rel_inf_err(out["y"], y_ref))
    assert rel_inf_err(out["y_nosave"], y_ref) <= tol
    for d in range(4):
        if (mask >> d) & 1:
            assert rel_inf_err(out["h"][d], h_ref[d]) <= tol, ("h", d)
        else:
            assert np.all(np.isnan(out["h"][d]))
    if not backward:
        return
    h_used = WL.storage_to_f64(WL.to_storage(h_ref, dtype), dtype)
    gx, gw, glam, gu = O.scan_bwd_local(f["gy"], f["x"], f["w"], f["lam"], f["u"], h_used, kchunk, mask)
    assert rel_inf_err(out["gx"], gx) <= tol, ("gx", rel_inf_err(out["gx"], gx))
    for d in range(4):
        for name, got, ref in (("gw", out["gw"], gw), ("glam", out["glam"], glam), ("gu", out["gu"], gu)):
            if (mask >> d) & 1:
                e = rel_inf_err(got[d], ref[d])
                assert e <= tol, (name, d, e)
            else:
                assert np.all(np.isnan(got[d])), (name, d)
    # gw is exactly zero on the first line of every stretch
    for d in range(4):
        if not (mask >> d) & 1:
            continue
        S = H if d < 2 else W
        starts = [lo if d in (0, 2) else min(lo + kchunk, S) - 1 for lo in range(0, S, kchunk)]
        g = out["gw"][d]
        assert not (g[:, :, :, starts, :] if d < 2 else g[:, :, :, :, starts]).any(), d


# (B, C, H, W, G, dtype), kchunk -- plane kernels, padded and unpadded LDS planes, 1 to 8 channels per wave,
# shared and per-channel weights, kchunk dividing the axis or not, kchunk between H and W
PLANE_LOCAL = [((2, 16, 28, 28, 2, "f32"), 7), ((2, 8, 28, 28, 8, "f32"), 5), ((2, 16, 28, 28, 2, "bf16"), 14),
               ((2, 16, 14, 14, 2, "bf16"), 7), ((2, 16, 7, 7, 2, "f32"), 3), ((1, 12, 16, 32, 3, "f32"), 20),
               ((1, 8, 6, 14, 2, "bf16"), 4), ((1, 8, 14, 14, 8, "f32"), 2), ((2, 8, 28, 24, 2, "f32"), 1),
               ((1, 4, 32, 32, 2, "f32"), 31), ((2, 96, 28, 28, 2, "f32"), 4), ((300, 16, 4, 4, 2, "bf16"), 2)]


@pytest.mark.parametrize("shape,kchunk", PLANE_LOCAL, ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else str(v))
def test_local_scans_on_the_plane_kernels(shape, kchunk, monkeypatch):
    import paper_2512_07884_amd as G
    monkeypatch.setenv("GSPN_BWD_NO_TWOPASS", "1")     # (the two-pass backward takes the larger bf16 maps first)
    B, C, H, W, Gr, dtype = shape
    dt = int(dtype == "bf16")
    assert G.gspn_fwd_local_plan(B, C, H, W, Gr, kchunk, 15, dt, 0, True) == "plane"
    assert G.gspn_bwd_local_plan(B, C, H, W, Gr, kchunk, 15, dt, 0) == "plane"
    check_local(shape, kchunk)


# larger maps: forward plane kernel with the backward tile kernel (lines of 33..64 positions), the tile kernels'
# horizontal variants (whole rows, 64 B and 16 B bursts, rows split over waves), the stream kernel, per-channel
# and shared weights, and ragged shapes on the generic kernels (whose bf16 gw is summed in storage precision
# channel by channel: small groups there)
@pytest.mark.parametrize("shape,kchunk,plans", [
    ((2, 8, 56, 56, 2, "bf16"), 14, ("plane", "tile")), ((1, 8, 64, 64, 8, "bf16"), 10, ("plane", "tile")),
    ((1, 6, 40, 24, 3, "bf16"), 16, ("plane", "twopass")), ((2, 8, 56, 56, 2, "f32"), 9, ("tile", "tile")),
    ((1, 4, 128, 128, 2, "bf16"), 32, ("pair", "twopass")), ((1, 4, 128, 128, 4, "bf16"), 5, ("tile", "twopass")),
    ((1, 8, 64, 128, 2, "f32"), 48, ("tile", "tile")), ((1, 24, 16, 40, 2, "f32"), 3, ("plane", "tile")),
    ((2, 8, 40, 32, 8, "f32"), 7, ("plane", "tile")), ((1, 4, 96, 72, 2, "bf16"), 20, ("tile", "twopass")),
    ((1, 4, 33, 70, 2, "f32"), 9, ("generic", "generic")), ((2, 6, 9, 13, 3, "f32"), 4, ("generic", "generic")),
    ((1, 2, 1, 37, 1, "f32"), 5, ("generic", "generic")), ((1, 2, 64, 256, 1, "bf16"), 100, ("stream", "twopass")),
    ((1, 4, 40, 112, 2, "bf16"), 30, ("tile", "tile"))],
    ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else str(v))
def test_local_scans_on_larger_and_ragged_maps(shape, kchunk, plans, monkeypatch):
    import paper_2512_07884_amd as G
    monkeypatch.setenv("GSPN_FWD_NO_CHUNK", "1")           # (the per-stretch kernels take 128x128 with kchunk 32 first)
    if plans[1] == "tile":
        monkeypatch.setenv("GSPN_BWD_NO_TWOPASS", "1")     # (the two-pass backward takes these maps first)
    B, C, H, W, Gr, dtype = shape
    dt = int(dtype == "bf16")
    assert G.gspn_fwd_local_plan(B, C, H, W, Gr, kchunk, 15, dt, 0, True) == plans[0]
    assert G.gspn_bwd_local_plan(B, C, H, W, Gr, kchunk, 15, dt, 0) == plans[1]
    check_local(shape, kchunk)


@pytest.mark.parametrize("shape,kchunk", [((2, 8, 56, 56, 2, "bf16"), 9), ((2, 16, 28, 28, 2, "f32"), 5),
                                          ((1, 12, 16, 32, 3, "f32"), 6), ((2, 8, 28, 28, 8, "f32"), 14)],
                         ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else str(v))
def test_local_scans_on_the_tile_kernels_for_small_maps(shape, kchunk, monkeypatch):
    """Shapes the plane kernels normally take, on the tile kernels (whole-row bursts among them)."""
    import paper_2512_07884_amd as G
    monkeypatch.setenv("GSPN_FWD_NO_PLANE", "1")
    monkeypatch.setenv("GSPN_BWD_NO_PLANE", "1")
    monkeypatch.setenv("GSPN_BWD_NO_TWOPASS", "1")
    B, C, H, W, Gr, dtype = shape
    dt = int(dtype == "bf16")
    assert G.gspn_fwd_local_plan(B, C, H, W, Gr, kchunk, 15, dt, 0, True) == "tile"
    assert G.gspn_bwd_local_plan(B, C, H, W, Gr, kchunk, 15, dt, 0) == "tile"
    check_local(shape, kchunk)


# calls with few planes: one workgroup per (plane, stretch) -- the stretch as a work item (Sec. 4.1: grid indexed by
# (chunk, n, c)); every positions-per-lane / rows-per-lane variant in both storage types, forward with and without
# h_save and the two-pass backward whose reverse sweep runs on the same kernels
CHUNK_LOCAL = [((1, 32, 128, 128, 4, "f32"), 32), ((1, 32, 128, 128, 2, "bf16"), 32), ((2, 6, 64, 128, 3, "f32"), 16),
               ((1, 4, 256, 128, 2, "bf16"), 64), ((1, 3, 128, 256, 1, "bf16"), 8), ((1, 2, 256, 256, 2, "f32"), 64),
               ((1, 4, 64, 64, 2, "f32"), 4), ((1, 2, 64, 256, 1, "bf16"), 32), ((1, 4, 128, 64, 4, "f32"), 64),
               ((1, 2, 256, 64, 1, "f32"), 32), ((1, 2, 64, 128, 2, "bf16"), 8), ((1, 8, 64, 128, 2, "bf16"), 8)]


@pytest.mark.parametrize("shape,kchunk", CHUNK_LOCAL, ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else str(v))
def test_local_scans_with_one_workgroup_per_stretch(shape, kchunk):
    import paper_2512_07884_amd as G
    B, C, H, W, Gr, dtype = shape
    dt = int(dtype == "bf16")
    assert G.gspn_fwd_local_plan(B, C, H, W, Gr, kchunk, 15, dt, 0, True) == "chunk"
    assert G.gspn_fwd_local_plan(B, C, H, W, Gr, kchunk, 15, dt, 0, False) == "chunk"
    assert G.gspn_bwd_local_plan(B, C, H, W, Gr, kchunk, 15, dt, 0) == "twopass"
    check_local(shape, kchunk, poison_starts=True)


def test_per_stretch_kernels_are_for_calls_with_few_planes(monkeypatch):
    import paper_2512_07884_amd as G
    assert G.gspn_fwd_local_plan(1, 32, 128, 128, 4, 32, 15, 0, 0, False) == "chunk"
    assert G.gspn_fwd_local_plan(2, 1024, 128, 128, 16, 32, 15, 1, 0, False) == "pair"      # planes fill the chip
    assert G.gspn_fwd_local_plan(1, 128, 128, 128, 4, 32, 15, 0, 0, False) == "chunk"       # 512 stretches per launch
    assert G.gspn_fwd_local_plan(1, 256, 128, 128, 4, 32, 15, 0, 0, False) == "tile"        # 1024: more than two per CU
    assert G.gspn_fwd_local_plan(1, 32, 128, 128, 4, 24, 15, 0, 0, False) == "tile"         # kchunk does not divide
    assert G.gspn_fwd_local_plan(1, 32, 128, 128, 4, 128, 15, 0, 0, False) == "tile"        # a single stretch
    assert G.gspn_fwd_local_plan(1, 32, 128, 128, 4, 32, 5, 0, 0, False) == "tile"          # not all four directions
    assert G.gspn_fwd_plan(1, 32, 128, 128, 4, 15, 0, 0, False) == "tile"                   # the global scan
    monkeypatch.setenv("GSPN_FWD_NO_CHUNK", "1")
    assert G.gspn_fwd_local_plan(1, 32, 128, 128, 4, 32, 15, 0, 0, False) == "tile"


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_per_stretch_kernels_with_one_parameter_set_for_all_directions(dtype):
    import torch
    import paper_2512_07884_amd as G
    B, C, H, W, Gr, k = 1, 4, 128, 128, 2, 32
    cfg = WL.ScanConfig("chunkshared", B, C, H, W, Gr, dtype, 15, 1.0, 93)
    inp = WL.make_inputs(cfg, with_gy=False)
    one = {"x": inp["x"], "w": inp["w"][:1].copy(), "lam": inp["lam"][:1].copy(), "u": inp["u"][:1].copy()}
    rep = {"x": inp["x"], "w": np.repeat(one["w"], 4, 0), "lam": np.repeat(one["lam"], 4, 0), "u": np.repeat(one["u"], 4, 0)}
    f = WL.inputs_as_f64(rep, dtype)
    y_ref, h_ref = O.scan_fwd_local(f["x"], f["w"], f["lam"], f["u"], k, 15)
    assert G.gspn_fwd_local_plan(B, C, H, W, Gr, k, 15, int(dtype == "bf16"), 1, True) == "chunk"
    dev = {n: to_device(v, dtype) for n, v in one.items()}
    y = empty_like_dev((B, C, H, W), dtype, float("nan"))
    hs = empty_like_dev((4, B, C, H, W), dtype, float("nan"))
    G.gspn_scan_fwd_local(dev["x"], dev["w"], dev["lam"], dev["u"], y, hs, kchunk=k, G=Gr, flags=1)
    torch.cuda.synchronize()
    assert rel_inf_err(to_host_f64(y), y_ref) <= TOL[dtype]
    assert rel_inf_err(to_host_f64(hs), h_ref) <= TOL[dtype]


@pytest.mark.parametrize("shape,kchunk", [((1, 2, 256, 256, 1, "bf16"), 37), ((1, 2, 512, 512, 2, "bf16"), 64),
                                          ((1, 2, 128, 256, 2, "f32"), 100), ((1, 2, 256, 1024, 1, "bf16"), 300)],
                         ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else str(v))
def test_local_scans_on_the_stream_kernel(shape, kchunk):
    import paper_2512_07884_amd as G
    B, C, H, W, Gr, dtype = shape
    assert G.gspn_fwd_local_plan(B, C, H, W, Gr, kchunk, 15, int(dtype == "bf16"), 0, False) == "stream"
    cfg = WL.ScanConfig("localstream", B, C, H, W, Gr, dtype, 15, 1.0, 87)
    inp = WL.make_inputs(cfg, with_gy=False)
    f = WL.inputs_as_f64(inp, dtype)
    y_ref, _ = O.scan_fwd_local(f["x"], f["w"], f["lam"], f["u"], kchunk, 15)
    import torch
    dev = {k: to_device(v, dtype) for k, v in inp.items()}
    y = empty_like_dev((B, C, H, W), dtype, float("nan"))
    G.gspn_scan_fwd_local(dev["x"], dev["w"], dev["lam"], dev["u"], y, None, kchunk=kchunk, G=Gr)
    torch.cuda.synchronize()
    assert rel_inf_err(to_host_f64(y), y_ref) <= TOL[dtype]


# the two limits on every kernel family: kchunk = 1 (every line starts a stretch: no propagation at all) and a
# stretch longer than one axis only
@pytest.mark.parametrize("shape,kchunk", [((1, 4, 56, 56, 2, "f32"), 1), ((1, 2, 128, 128, 2, "bf16"), 1),
                                          ((2, 8, 28, 28, 2, "f32"), 1), ((1, 2, 40, 70, 1, "f32"), 1),
                                          ((1, 8, 40, 32, 2, "f32"), 36), ((1, 2, 64, 128, 2, "f32"), 64)],
                         ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else str(v))
def test_local_scans_at_the_limits_of_kchunk(shape, kchunk):
    check_local(shape, kchunk)


@pytest.mark.parametrize("mask", [1, 2, 4, 8, 6, 9, 13])
@pytest.mark.parametrize("shape,kchunk", [((2, 8, 28, 28, 2, "f32"), 6), ((1, 4, 20, 36, 2, "bf16"), 8)],
                         ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else str(v))
def test_local_scans_direction_masks(shape, kchunk, mask):
    check_local(shape, kchunk, mask=mask)


@pytest.mark.parametrize("shape,kchunk", [((1, 8, 28, 28, 2, "f32"), 7), ((1, 8, 14, 14, 2, "bf16"), 5),
                                          ((1, 4, 12, 10, 4, "f32"), 4), ((1, 2, 40, 70, 1, "f32"), 16),
                                          ((1, 4, 56, 56, 2, "f32"), 8), ((1, 2, 128, 128, 1, "bf16"), 24)],
                         ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else str(v))
def test_weights_on_the_first_line_of_a_stretch_are_never_read(shape, kchunk):
    check_local(shape, kchunk, poison_starts=True)


def test_a_stretch_that_covers_the_map_is_the_global_scan_bit_for_bit():
    import torch
    import paper_2512_07884_amd as G
    cfg = WL.ScanConfig("localglobal", 2, 8, 28, 28, 2, "f32", 15, 1.0, 5)
    inp = WL.make_inputs(cfg, with_gy=False)
    dev = {k: to_device(v, cfg.dtype) for k, v in inp.items()}
    y0 = empty_like_dev((2, 8, 28, 28), "f32", float("nan"))
    y1 = empty_like_dev((2, 8, 28, 28), "f32", float("nan"))
    G.gspn_scan_fwd(dev["x"], dev["w"], dev["lam"], dev["u"], y0, None, G=2)
    G.gspn_scan_fwd_local(dev["x"], dev["w"], dev["lam"], dev["u"], y1, None, kchunk=28, G=2)
    torch.cuda.synchronize()
    assert torch.equal(y0, y1)


def test_local_training_stage_at_full_size_on_sampled_slices():
    """The 28x28 training shape of the benchmark (B=32, C=192, G=4, fp32) with kchunk = 7, launch shape as
    timed; the oracle computes a few (b, g) slices, which are independent given the group's weights."""
    import torch
    import paper_2512_07884_amd as G
    B, C, H, W, Gr, k = 32, 192, 28, 28, 4, 7
    cfg = WL.ScanConfig("localfull", B, C, H, W, Gr, "f32", 15, 1.0, 91)
    inp = WL.make_inputs(cfg, with_gy=True)
    out = run_local(inp, cfg, k, 15, True)
    cpg = C // Gr
    for b, g in ((0, 0), (17, 2), (31, 3)):
        cs = slice(g * cpg, (g + 1) * cpg)
        f = {n: np.asarray(inp[n][:, b:b + 1, cs] if n in ("lam", "u") else
                           inp[n][:, b:b + 1, g:g + 1] if n == "w" else inp[n][b:b + 1, cs], dtype=np.float64)
             for n in ("x", "w", "lam", "u", "gy")}
        y_ref, h_ref = O.scan_fwd_local(f["x"], f["w"], f["lam"], f["u"], k, 15)
        assert rel_inf_err(out["y"][b:b + 1, cs], y_ref) <= TOL["f32"]
        h_used = h_ref.astype(np.float32).astype(np.float64)
        gx, gw, glam, gu = O.scan_bwd_local(f["gy"], f["x"], f["w"], f["lam"], f["u"], h_used, k, 15)
        assert rel_inf_err(out["gx"][b:b + 1, cs], gx) <= TOL["f32"]
        assert rel_inf_err(out["gw"][:, b:b + 1, g:g + 1], gw) <= TOL["f32"]
        assert rel_inf_err(out["glam"][:, b:b + 1, cs], glam) <= TOL["f32"]
        assert rel_inf_err(out["gu"][:, b:b + 1, cs], gu) <= TOL["f32"]


# the two-channel kernel of the 128x128 bf16 maps (even channel groups, all four directions) with stretches: lengths that
# divide the map and that do not, a single line per stretch, a stretch longer than the map; several pairs per workgroup
@pytest.mark.parametrize("shape,kchunk", [((1, 4, 128, 128, 2, "bf16"), 1), ((1, 4, 128, 128, 2, "bf16"), 7),
                                          ((2, 8, 128, 128, 4, "bf16"), 32), ((1, 4, 128, 128, 1, "bf16"), 50),
                                          ((1, 2, 128, 128, 1, "bf16"), 128), ((1, 2, 128, 128, 1, "bf16"), 300),
                                          ((1, 600, 128, 128, 4, "bf16"), 24)],
                         ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else str(v))
def test_local_scans_on_the_two_channel_kernel(shape, kchunk, monkeypatch):
    import paper_2512_07884_amd as G
    monkeypatch.setenv("GSPN_FWD_NO_CHUNK", "1")           # (the per-stretch kernels take few planes first)
    B, C, H, W, Gr, dtype = shape
    assert G.gspn_fwd_local_plan(B, C, H, W, Gr, kchunk, 15, 1, 0, True) == "pair"
    assert G.gspn_fwd_local_plan(B, C, H, W, Gr, kchunk, 15, 1, 0, False) == "pair"
    assert G.gspn_bwd_local_plan(B, C, H, W, Gr, kchunk, 15, 1, 0) == "twopass"
    check_local(shape, kchunk, poison_starts=True)


# GSPN-local on the whole-line stream kernel of the 16-bit maps: one channel per workgroup (calls with few planes) and
# two channels of a group per workgroup (forced here: both take the same 64 steps of a chunk and share the walk's state);
# maps of 512 rows (one horizontal direction at a time) and of 256 rows (both at once, each first on its own half of the
# columns); forward with and without h_save and the two-pass backward; stretches that divide the map and that do not
@pytest.mark.parametrize("two_channels", [False, True], ids=["one-channel", "two-channels"])
@pytest.mark.parametrize("shape,kchunk", [((1, 4, 512, 512, 2, "bf16"), 64), ((1, 2, 256, 512, 1, "bf16"), 100),
                                          ((1, 4, 256, 1024, 2, "f16"), 37), ((1, 2, 512, 256, 1, "f16"), 1),
                                          ((1, 2, 256, 256, 1, "bf16"), 255)],
                         ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else str(v))
def test_local_scans_on_the_whole_line_stream_kernel(shape, kchunk, two_channels, monkeypatch):
    import paper_2512_07884_amd as G
    monkeypatch.setenv("GSPN_FWD_NO_CHUNK", "1")           # (short stretches on few planes would go to the chunk-axis kernels)
    if two_channels:
        monkeypatch.setenv("GSPN_STREAM_TWO_CHANNELS", "1")
    B, C, H, W, Gr, dtype = shape
    dt = {"f32": 0, "bf16": 1, "f16": 2}[dtype]
    assert G.gspn_fwd_local_plan(B, C, H, W, Gr, kchunk, 15, dt, 0, True) == "stream"
    assert G.gspn_bwd_local_plan(B, C, H, W, Gr, kchunk, 15, dt, 0) == "twopass"
    check_local(shape, kchunk, poison_starts=True)
