"""GPU parity of the calls that take the weights as raw logits (normalisation of Sec. 3.2 inside the call)
against the fp64 oracle, through the C ABI, forward and backward."""
import numpy as np
import pytest

from gpu_util import TOL, rel_inf_err, to_device, to_host_f64, empty_like_dev
from oracle import gspn_oracle as O
from paper_2512_07884_amd import workloads as WL

pytestmark = pytest.mark.gpu


def check_logits(shape, kchunk=None, mask=15, seed=101, scale=1.5, poison=False, fwd_plan=None, bwd_plan=None):
    import torch
    import paper_2512_07884_amd as G
    B, C, H, W, Gr, dtype = shape
    cfg = WL.ScanConfig("logits", B, C, H, W, Gr, dtype, mask, scale, seed)
    inp = WL.make_inputs(cfg, with_gy=True)
    inp["w"] = WL.make_logits(cfg)
    f = WL.inputs_as_f64(inp, dtype)
    y_ref, h_ref = O.scan_fwd_logits(f["x"], f["w"], f["lam"], f["u"], mask, kchunk)
    if poison:
        # logits that are never read: taps that point outside the line, first line of each scan
        nan = np.nan if dtype == "f32" else np.uint16(0x7FC0)
        z = inp["w"]
        z[0, :, :, 0, :, 0] = nan; z[1, :, :, 2, :, -1] = nan; z[2, :, :, 0, 0, :] = nan; z[3, :, :, 2, -1, :] = nan
        z[0, :, :, :, 0, :] = nan; z[1, :, :, :, -1, :] = nan; z[2, :, :, :, :, 0] = nan; z[3, :, :, :, :, -1] = nan
        if kchunk:
            # GSPN-local: the first line of every stretch in scan order (cuts at image lines 0, kchunk, 2*kchunk, ...)
            for r in range(0, H, kchunk):
                z[0, :, :, :, r, :] = nan
                if r > 0:
                    z[1, :, :, :, r - 1, :] = nan
            for r in range(0, W, kchunk):
                z[2, :, :, :, :, r] = nan
                if r > 0:
                    z[3, :, :, :, :, r - 1] = nan
    k = kchunk if kchunk else 1 << 14
    dt = {"f32": 0, "bf16": 1, "f16": 2}[dtype]
    if fwd_plan:
        assert G.gspn_fwd_logits_plan(B, C, H, W, Gr, k, mask, dt, 0, True) == fwd_plan
    if bwd_plan:
        assert G.gspn_bwd_logits_plan(B, C, H, W, Gr, k, mask, dt, 0) == bwd_plan
    dev = {n: to_device(v, dtype) for n, v in inp.items()}
    nanf = float("nan")
    y = empty_like_dev((B, C, H, W), dtype, nanf)
    y2 = empty_like_dev((B, C, H, W), dtype, nanf)
    hs = empty_like_dev((4, B, C, H, W), dtype, nanf)
    gx = empty_like_dev((B, C, H, W), dtype, nanf)
    gz = empty_like_dev((4, B, Gr, 3, H, W), dtype, nanf)
    glam = empty_like_dev((4, B, C, H, W), dtype, nanf)
    gu = empty_like_dev((4, B, C, H, W), dtype, nanf)
    G.gspn_scan_fwd_logits(dev["x"], dev["w"], dev["lam"], dev["u"], y, hs, kchunk=k, G=Gr, dir_mask=mask)
    G.gspn_scan_fwd_logits(dev["x"], dev["w"], dev["lam"], dev["u"], y2, None, kchunk=k, G=Gr, dir_mask=mask)
    G.gspn_scan_bwd_logits(dev["gy"], dev["x"], dev["w"], dev["lam"], dev["u"], hs, gx, gz, glam, gu, kchunk=k, G=Gr,
                           dir_mask=mask)
    torch.cuda.synchronize()
    tol = TOL[dtype]
    assert rel_inf_err(to_host_f64(y), y_ref) <= tol, ("y", rel_inf_err(to_host_f64(y), y_ref))
    assert rel_inf_err(to_host_f64(y2), y_ref) <= tol
    h_used = WL.storage_to_f64(WL.to_storage(h_ref, dtype), dtype)
    gx_r, gz_r, glam_r, gu_r = O.scan_bwd_logits(f["gy"], f["x"], f["w"], f["lam"], f["u"], h_used, mask, kchunk)
    assert rel_inf_err(to_host_f64(gx), gx_r) <= tol, ("gx", rel_inf_err(to_host_f64(gx), gx_r))
    got = {"gz": to_host_f64(gz), "glam": to_host_f64(glam), "gu": to_host_f64(gu), "h": to_host_f64(hs)}
    ref = {"gz": gz_r, "glam": glam_r, "gu": gu_r, "h": h_ref}
    for d in range(4):
        for n in got:
            if (mask >> d) & 1:
                e = rel_inf_err(got[n][d], ref[n][d])
                assert e <= tol, (n, d, e)
            else:
                assert np.all(np.isnan(got[n][d])), (n, d)
    # exact zeros of gz: taps that point outside the line, first line of each scan
    g = got["gz"]
    for d in range(4):
        if not (mask >> d) & 1:
            continue
        if d < 2:
            assert not g[d][:, :, 0, :, 0].any() and not g[d][:, :, 2, :, -1].any()
        else:
            assert not g[d][:, :, 0, 0, :].any() and not g[d][:, :, 2, -1, :].any()
        if kchunk is None:
            first = {0: g[d][:, :, :, 0, :], 1: g[d][:, :, :, -1, :], 2: g[d][:, :, :, :, 0], 3: g[d][:, :, :, :, -1]}[d]
            assert not first.any()


GENERIC_SHAPES = [(2, 6, 9, 13, 3, "f32"), (1, 4, 33, 70, 2, "f32"), (1, 2, 1, 37, 1, "f32"), (1, 2, 37, 1, 2, "f32"),
                  (1, 4, 41, 73, 2, "bf16"), (1, 2, 130, 67, 2, "bf16"), (1, 1, 1, 1, 1, "f32")]


@pytest.mark.parametrize("shape", GENERIC_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_logits_on_the_generic_kernels(shape):
    check_logits(shape, fwd_plan="generic", bwd_plan="generic")


@pytest.mark.parametrize("shape,kchunk", [((2, 6, 9, 13, 3, "f32"), 4), ((1, 4, 41, 73, 2, "bf16"), 16)],
                         ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else str(v))
def test_logits_with_local_stretches_on_the_generic_kernels(shape, kchunk):
    check_logits(shape, kchunk=kchunk, fwd_plan="generic", bwd_plan="generic")


# shapes of the plane kernels: padded and unpadded LDS planes, shared and per-channel weights, 1 to 8 channels
# per wave, small groups (weights not prefetched), bf16 and fp32
PLANE_SHAPES = [(2, 16, 28, 28, 2, "f32"), (2, 8, 28, 28, 8, "f32"), (2, 24, 56, 56, 2, "bf16"), (2, 16, 28, 28, 2, "bf16"),
                (2, 16, 14, 14, 2, "bf16"), (2, 16, 7, 7, 2, "f32"), (1, 8, 14, 14, 8, "f32"), (1, 12, 16, 32, 3, "f32"),
                (2, 8, 28, 28, 2, "f32"), (1, 4, 12, 10, 2, "f32"), (1, 8, 64, 64, 8, "bf16"), (300, 16, 4, 4, 2, "bf16")]


@pytest.mark.parametrize("shape", PLANE_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_logits_on_the_plane_kernels(shape, monkeypatch):
    monkeypatch.setenv("GSPN_BWD_NO_TWOPASS", "1")     # (the two-pass backward takes the larger bf16 maps first)
    B, C, H, W, Gr, dtype = shape
    small = max(H, W) <= 32 and (C // Gr) % 2 == 0 or C == Gr and (H * W) % (4 if dtype == "f32" else 8) == 0 and max(H, W) <= 32
    check_logits(shape, fwd_plan="plane", bwd_plan="plane" if small else None)


# the backward plane kernel's own variants: 16 / 28 / 32 steps, two / four / eight channels per wave, a group
# split over two workgroups (fp32, few groups), per-channel weights with 8 / 4 / 2 channels per workgroup
@pytest.mark.parametrize("shape", [(2, 96, 28, 28, 2, "f32"), (1, 16, 28, 28, 4, "f32"), (2, 4, 32, 32, 2, "f32"),
                                   (1, 6, 12, 20, 3, "f32"), (1, 12, 28, 28, 12, "f32"), (1, 2, 28, 28, 1, "f32"),
                                   (1, 48, 7, 7, 1, "f32"), (2, 16, 14, 14, 2, "f32"), (2, 16, 7, 7, 2, "bf16"),
                                   (1, 24, 28, 28, 1, "bf16"), (3, 32, 2, 4, 32, "bf16"), (2, 4, 32, 32, 4, "f32")],
                         ids=lambda s: "x".join(map(str, s)))
def test_logits_on_the_backward_plane_kernel_variants(shape, monkeypatch):
    monkeypatch.setenv("GSPN_BWD_NO_TWOPASS", "1")     # (the two-pass backward takes the larger bf16 maps first)
    check_logits(shape, bwd_plan="plane")


@pytest.mark.parametrize("shape,kchunk", [((2, 16, 28, 28, 2, "f32"), 7), ((2, 8, 28, 28, 8, "f32"), 5),
                                          ((2, 24, 56, 56, 2, "bf16"), 14), ((2, 16, 7, 7, 2, "f32"), 3),
                                          ((2, 8, 28, 28, 2, "f32"), 6)],
                         ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else str(v))
def test_logits_with_local_stretches_on_the_plane_kernels(shape, kchunk):
    check_logits(shape, kchunk=kchunk, fwd_plan="plane", bwd_plan="plane" if max(shape[2], shape[3]) <= 32 else None)


@pytest.mark.parametrize("shape", [(1, 8, 28, 28, 2, "f32"), (1, 4, 12, 10, 4, "f32"), (1, 4, 40, 70, 2, "f32"),
                                   (1, 8, 14, 14, 2, "bf16")], ids=lambda s: "x".join(map(str, s)))
def test_logits_that_are_never_read_may_hold_anything(shape):
    check_logits(shape, poison=True)


@pytest.mark.parametrize("shape,kchunk", [((1, 8, 128, 128, 2, "f32"), None), ((2, 24, 56, 56, 2, "bf16"), None),
                                          ((1, 8, 128, 128, 2, "f32"), 32), ((2, 24, 56, 56, 2, "bf16"), 14),
                                          ((1, 2, 256, 256, 1, "bf16"), None)],
                         ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else str(v))
def test_unread_logits_may_hold_anything_in_the_two_pass_backward(shape, kchunk):
    """The channel-sum pass of the two-pass backward normalises the logits of every pixel once more; on lines without a
    predecessor (first line of a scan, of a stretch) the stored logits must stay out of it and gz must be an exact 0."""
    check_logits(shape, kchunk=kchunk, poison=True, bwd_plan="twopass")


@pytest.mark.parametrize("mask", [1, 2, 4, 8, 6, 9])
def test_logits_direction_masks(mask):
    check_logits((2, 8, 28, 28, 2, "f32"), mask=mask)


# the tile kernels (forward: rows split over waves, 64 B and 16 B bursts; backward: 4 and 8 columns per request,
# shared and per-channel weights) and the stream kernel (forward without h_save)
@pytest.mark.parametrize("shape,plans", [
    ((1, 4, 128, 128, 2, "bf16"), ("pair", "twopass")), ((1, 4, 128, 128, 2, "bf16"), ("tile", "twopass")),
    ((2, 8, 56, 56, 2, "f32"), ("tile", "tile")),
    ((1, 8, 64, 128, 2, "f32"), ("tile", "tile")), ((1, 4, 96, 72, 2, "bf16"), ("tile", "twopass")),
    ((2, 8, 56, 56, 2, "bf16"), ("plane", "tile")), ((1, 4, 56, 56, 4, "f32"), ("tile", "tile")),
    ((1, 24, 16, 40, 2, "f32"), ("plane", "tile")), ((2, 8, 40, 32, 8, "f32"), ("plane", "tile")),
    ((2, 8, 40, 32, 2, "bf16"), ("plane", "tile"))],
    ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else str(v))
def test_logits_on_the_tile_kernels(shape, plans, monkeypatch):
    if plans[1] == "tile":
        monkeypatch.setenv("GSPN_BWD_NO_TWOPASS", "1")     # (the two-pass backward takes these maps first)
    if plans[0] == "tile" and shape[2:4] == (128, 128) and shape[5] == "bf16":
        monkeypatch.setenv("GSPN_FWD_NO_PAIR", "1")        # (... and the two-channel kernel the 128 x 128 bf16 maps)
    check_logits(shape, fwd_plan=plans[0], bwd_plan=plans[1])


# the two-channel kernel of the 128 x 128 bf16 maps normalises the logits as it unpacks them (forward, forward with
# h_save, and the reverse sweep of the two-pass backward): global and GSPN-local, stretch lengths that divide the map and
# that do not, an odd number of pairs, and taps that are never read
@pytest.mark.parametrize("shape,kchunk,mask", [
    ((1, 4, 128, 128, 2, "bf16"), None, 15), ((2, 12, 128, 128, 3, "bf16"), None, 15), ((1, 8, 128, 128, 1, "bf16"), 32, 15),
    ((1, 4, 128, 128, 2, "bf16"), 37, 15), ((1, 4, 128, 128, 2, "bf16"), 1, 15), ((2, 6, 128, 128, 1, "bf16"), 16, 15),
    ((1, 4, 128, 128, 2, "bf16"), 127, 15)],
    ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else str(v))
def test_logits_on_the_two_channel_kernel(shape, kchunk, mask, monkeypatch):
    monkeypatch.setenv("GSPN_FWD_NO_CHUNK", "1")           # (short stretches would go to the chunk-parallel kernel)
    check_logits(shape, kchunk=kchunk, mask=mask, poison=True, fwd_plan="pair", bwd_plan="twopass")


@pytest.mark.parametrize("shape,kchunk", [((2, 8, 56, 56, 2, "f32"), 9), ((1, 4, 128, 128, 2, "bf16"), 32),
                                          ((2, 8, 40, 32, 8, "f32"), 7)],
                         ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else str(v))
def test_logits_with_local_stretches_on_the_tile_kernels(shape, kchunk):
    check_logits(shape, kchunk=kchunk)


@pytest.mark.parametrize("shape", [(2, 8, 56, 56, 2, "bf16"), (2, 16, 28, 28, 2, "f32"), (2, 8, 28, 28, 8, "f32")],
                         ids=lambda s: "x".join(map(str, s)))
def test_logits_on_the_tile_kernels_for_small_maps(shape, monkeypatch):
    monkeypatch.setenv("GSPN_FWD_NO_PLANE", "1")
    monkeypatch.setenv("GSPN_BWD_NO_PLANE", "1")
    monkeypatch.setenv("GSPN_BWD_NO_TWOPASS", "1")
    check_logits(shape, fwd_plan="tile", bwd_plan="tile")


@pytest.mark.parametrize("shape", [(1, 2, 256, 256, 1, "bf16"), (1, 2, 128, 256, 2, "f32"), (1, 2, 256, 1024, 1, "bf16")],
                         ids=lambda s: "x".join(map(str, s)))
def test_logits_on_the_stream_kernel(shape):
    import torch
    import paper_2512_07884_amd as G
    B, C, H, W, Gr, dtype = shape
    big = 1 << 14
    assert G.gspn_fwd_logits_plan(B, C, H, W, Gr, big, 15, int(dtype == "bf16"), 0, False) == "stream"
    cfg = WL.ScanConfig("logitsstream", B, C, H, W, Gr, dtype, 15, 1.5, 103)
    inp = WL.make_inputs(cfg, with_gy=False)
    inp["w"] = WL.make_logits(cfg)
    f = WL.inputs_as_f64(inp, dtype)
    y_ref, _ = O.scan_fwd_logits(f["x"], f["w"], f["lam"], f["u"], 15)
    dev = {k: to_device(v, dtype) for k, v in inp.items()}
    y = empty_like_dev((B, C, H, W), dtype, float("nan"))
    G.gspn_scan_fwd_logits(dev["x"], dev["w"], dev["lam"], dev["u"], y, None, G=Gr)
    torch.cuda.synchronize()
    assert rel_inf_err(to_host_f64(y), y_ref) <= TOL[dtype]


def test_logits_training_stage_at_full_size_on_sampled_slices():
    """The 28x28 training shape of the benchmark with per-channel weights (B=32, C=192, G=192, fp32) -- the case the
    fused normalisation is for -- in the launch shape the benchmark times; the oracle computes a few (b, g) slices."""
    import torch
    import paper_2512_07884_amd as G
    B, C, H, W, Gr = 32, 192, 28, 28, 192
    cfg = WL.ScanConfig("logitsfull", B, C, H, W, Gr, "f32", 15, 1.5, 107)
    inp = WL.make_inputs(cfg, with_gy=True)
    inp["w"] = WL.make_logits(cfg)
    dev = {n: to_device(v, "f32") for n, v in inp.items()}
    nanf = float("nan")
    y = empty_like_dev((B, C, H, W), "f32", nanf)
    hs = empty_like_dev((4, B, C, H, W), "f32", nanf)
    gx = empty_like_dev((B, C, H, W), "f32", nanf)
    gz = empty_like_dev((4, B, Gr, 3, H, W), "f32", nanf)
    glam = empty_like_dev((4, B, C, H, W), "f32", nanf)
    gu = empty_like_dev((4, B, C, H, W), "f32", nanf)
    assert G.gspn_fwd_logits_plan(B, C, H, W, Gr, 1 << 14, 15, 0, 0, True) == "plane"
    assert G.gspn_bwd_logits_plan(B, C, H, W, Gr, 1 << 14, 15, 0, 0) == "plane"
    G.gspn_scan_fwd_logits(dev["x"], dev["w"], dev["lam"], dev["u"], y, hs, G=Gr)
    G.gspn_scan_bwd_logits(dev["gy"], dev["x"], dev["w"], dev["lam"], dev["u"], hs, gx, gz, glam, gu, G=Gr)
    torch.cuda.synchronize()
    got = {"y": to_host_f64(y), "gx": to_host_f64(gx), "gz": to_host_f64(gz), "glam": to_host_f64(glam), "gu": to_host_f64(gu)}
    for b, c0 in ((0, 0), (13, 77), (31, 184)):
        cs = slice(c0, c0 + 8)                       # eight channels = eight weight groups
        f = {n: np.asarray(inp[n][:, b:b + 1, cs] if n in ("lam", "u", "w") else inp[n][b:b + 1, cs], dtype=np.float64)
             for n in ("x", "w", "lam", "u", "gy")}
        y_ref, h_ref = O.scan_fwd_logits(f["x"], f["w"], f["lam"], f["u"], 15)
        assert rel_inf_err(got["y"][b:b + 1, cs], y_ref) <= TOL["f32"]
        h_used = h_ref.astype(np.float32).astype(np.float64)
        gx_r, gz_r, glam_r, gu_r = O.scan_bwd_logits(f["gy"], f["x"], f["w"], f["lam"], f["u"], h_used, 15)
        assert rel_inf_err(got["gx"][b:b + 1, cs], gx_r) <= TOL["f32"]
        assert rel_inf_err(got["gz"][:, b:b + 1, cs], gz_r) <= TOL["f32"]
        assert rel_inf_err(got["glam"][:, b:b + 1, cs], glam_r) <= TOL["f32"]
        assert rel_inf_err(got["gu"][:, b:b + 1, cs], gu_r) <= TOL["f32"]


@pytest.mark.parametrize("shape", [(1, 2, 2, 4096, 1, "f32"), (1, 2, 4096, 2, 2, "f32")], ids=lambda s: "x".join(map(str, s)))
def test_logits_at_the_longest_supported_line(shape):
    """GSPN_MAX_LINE_LOGITS positions per line / lines per scan (generic kernels, 128 KB of LDS in the backward).
    The bound on the error of S sequential fp32 steps with non-expanding weights is S * 2^-24 (2.4e-4 here), which
    replaces the 1e-5 of the short scans."""
    import torch
    import paper_2512_07884_amd as G
    B, C, H, W, Gr, dtype = shape
    big = 1 << 14
    assert G.gspn_fwd_logits_plan(B, C, H, W, Gr, big, 15, 0, 0, True) == "generic"
    assert G.gspn_bwd_logits_plan(B, C, H, W, Gr, big, 15, 0, 0) == "generic"
    cfg = WL.ScanConfig("logitsmax", B, C, H, W, Gr, dtype, 15, 1.0, 109)
    inp = WL.make_inputs(cfg, with_gy=True)
    inp["w"] = WL.make_logits(cfg)
    f = WL.inputs_as_f64(inp, dtype)
    dev = {n: to_device(v, dtype) for n, v in inp.items()}
    y = empty_like_dev((B, C, H, W), dtype, float("nan"))
    hs = empty_like_dev((4, B, C, H, W), dtype, float("nan"))
    gx = empty_like_dev((B, C, H, W), dtype, float("nan"))
    gz = empty_like_dev((4, B, Gr, 3, H, W), dtype, float("nan"))
    glam = empty_like_dev((4, B, C, H, W), dtype, float("nan"))
    gu = empty_like_dev((4, B, C, H, W), dtype, float("nan"))
    G.gspn_scan_fwd_logits(dev["x"], dev["w"], dev["lam"], dev["u"], y, hs, G=Gr)
    G.gspn_scan_bwd_logits(dev["gy"], dev["x"], dev["w"], dev["lam"], dev["u"], hs, gx, gz, glam, gu, G=Gr)
    torch.cuda.synchronize()
    tol = 4096 * 2.0 ** -24
    y_ref, h_ref = O.scan_fwd_logits(f["x"], f["w"], f["lam"], f["u"], 15)
    assert rel_inf_err(to_host_f64(y), y_ref) <= tol
    h_used = h_ref.astype(np.float32).astype(np.float64)
    gx_r, gz_r, glam_r, gu_r = O.scan_bwd_logits(f["gy"], f["x"], f["w"], f["lam"], f["u"], h_used, 15)
    assert rel_inf_err(to_host_f64(gx), gx_r) <= tol
    assert rel_inf_err(to_host_f64(gz), gz_r) <= tol
    assert rel_inf_err(to_host_f64(glam), glam_r) <= tol and rel_inf_err(to_host_f64(gu), gu_r) <= tol


# the whole-line stream kernel of the 16-bit maps normalises the logits where it unpacks a step's taps: one channel per
# workgroup (calls with few planes) and two channels of a group per workgroup (forced here); maps of 512 and of 256 rows;
# global and GSPN-local; forward with and without h_save and the two-pass backward; taps that are never read poisoned
@pytest.mark.parametrize("two_channels", [False, True], ids=["one-channel", "two-channels"])
@pytest.mark.parametrize("shape,kchunk", [((1, 4, 512, 512, 2, "bf16"), None), ((1, 2, 256, 512, 1, "bf16"), 100),
                                          ((1, 4, 256, 1024, 2, "f16"), None), ((1, 2, 512, 256, 1, "f16"), 64)],
                         ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else str(v))
def test_logits_on_the_whole_line_stream_kernel(shape, kchunk, two_channels, monkeypatch):
    monkeypatch.setenv("GSPN_FWD_NO_CHUNK", "1")
    if two_channels:
        monkeypatch.setenv("GSPN_STREAM_TWO_CHANNELS", "1")
    check_logits(shape, kchunk=kchunk, poison=True, fwd_plan="stream", bwd_plan="twopass")
