"""GPU parity on maps beyond 512 rows / 1024 columns (the 1024x1024 shapes of the paper's scaling experiments, Sec. 5.1,
and of high-resolution generation, App. B) against the fp64 oracle, through the C ABI: forward, h_save, direction
masks and the two-pass backward whose reverse sweep runs on the same kernels."""
import numpy as np
import pytest

from gpu_util import TOL, rel_inf_err, run_fwd_gpu
from oracle import gspn_oracle as O
from paper_2512_07884_amd import workloads as WL
from test_gpu_fwd import check_case
from test_gpu_bwd import check_bwd

pytestmark = pytest.mark.gpu

# (B, C, H, W, G, dtype): 16, 9 and 1 waves of rows; lines of 256 to 2048 positions
BIG = [(1, 4, 1024, 1024, 2, "f32"), (1, 4, 1024, 1024, 2, "bf16"), (2, 2, 576, 1024, 1, "f32"), (1, 2, 1024, 256, 2, "bf16"),
       (1, 2, 512, 2048, 1, "bf16"), (1, 2, 64, 1024, 1, "f32"), (1, 3, 704, 512, 3, "f32"), (1, 2, 1024, 2048, 2, "bf16")]


def _cfg(shape, seed, mask=15):
    B, C, H, W, G, dtype = shape
    return WL.ScanConfig("big", B, C, H, W, G, dtype, mask, 1.0, seed)


@pytest.mark.parametrize("shape", BIG, ids=lambda v: "x".join(map(str, v)))
def test_forward_on_maps_beyond_the_stream_kernel(shape):
    import paper_2512_07884_amd as G
    B, C, H, W, Gr, dtype = shape
    for save in (False, True):
        assert G.gspn_fwd_plan(B, C, H, W, Gr, 15, int(dtype == "bf16"), 0, save) == "stream"
    check_case(_cfg(shape, 101), save_h=True)
    check_case(_cfg(shape, 102), save_h=False)


@pytest.mark.parametrize("mask", [1, 2, 4, 8, 12, 6, 11])
@pytest.mark.parametrize("shape", [(1, 2, 640, 512, 1, "f32"), (1, 2, 1024, 256, 2, "bf16")], ids=lambda v: "x".join(map(str, v)))
def test_direction_masks_on_maps_beyond_the_stream_kernel(shape, mask):
    check_case(_cfg(shape, 103, mask), dir_mask=mask)


@pytest.mark.parametrize("shape", [(1, 4, 1024, 512, 2, "f32"), (1, 4, 1024, 1024, 2, "bf16"), (1, 2, 640, 1024, 1, "f32")],
                         ids=lambda v: "x".join(map(str, v)))
def test_backward_on_maps_beyond_the_stream_kernel(shape):
    import paper_2512_07884_amd as G
    B, C, H, W, Gr, dtype = shape
    assert G.gspn_bwd_plan(B, C, H, W, Gr, 15, int(dtype == "bf16"), 0) == "twopass"
    check_bwd(_cfg(shape, 104))


# more than 1024 rows: two image rows per lane in the horizontal pair (forward only; the backward call takes the generic kernel)
TALL = [(1, 2, 2048, 2048, 1, "bf16"), (1, 1, 2048, 1024, 1, "f32"), (1, 2, 1152, 256, 2, "f32"), (1, 2, 1280, 512, 1, "bf16"),
        (1, 1, 2048, 2048, 1, "f32")]


@pytest.mark.parametrize("shape", TALL, ids=lambda v: "x".join(map(str, v)))
def test_forward_on_maps_of_more_than_1024_rows(shape):
    import paper_2512_07884_amd as G
    B, C, H, W, Gr, dtype = shape
    dt = int(dtype == "bf16")
    assert G.gspn_fwd_plan(B, C, H, W, Gr, 15, dt, 0, True) == "stream"
    assert G.gspn_bwd_plan(B, C, H, W, Gr, 15, dt, 0) == "generic"
    check_case(_cfg(shape, 106), save_h=True)
    check_case(_cfg(shape, 107), save_h=False)


@pytest.mark.parametrize("mask", [4, 8, 12, 7])
def test_direction_masks_on_maps_of_more_than_1024_rows(mask):
    check_case(_cfg((1, 2, 1280, 256, 1, "f32"), 108, mask), dir_mask=mask)


# bf16 maps of 512 rows: the whole-line stream kernel with two channels of a weight group per workgroup (the weights of
# the horizontal phases fetched once for both; calls with at most 256 planes pair their channels only under the knob),
# with one channel per workgroup, and the row-per-lane stream kernel
@pytest.mark.parametrize("knob", ["GSPN_STREAM_TWO_CHANNELS", None, "GSPN_STREAM_NO_STAGED"], ids=["two-channel", "one-channel", "row-per-lane"])
@pytest.mark.parametrize("shape", [(1, 4, 512, 512, 2, "bf16"), (1, 4, 512, 1024, 1, "bf16"), (2, 2, 512, 256, 1, "bf16"),
                                   (1, 3, 512, 256, 1, "bf16"), (1, 4, 256, 1024, 2, "bf16"), (2, 2, 256, 256, 1, "bf16"),
                                   (1, 4, 256, 512, 1, "bf16")], ids=lambda v: "x".join(map(str, v)))
def test_stream_kernel_variants_on_maps_of_256_and_512_rows(shape, knob, monkeypatch):
    import paper_2512_07884_amd as G
    if knob:
        monkeypatch.setenv(knob, "1")
    B, C, H, W, Gr, dtype = shape
    assert G.gspn_fwd_plan(B, C, H, W, Gr, 15, 1, 0, True) == "stream"
    check_case(_cfg(shape, 109), save_h=True)
    check_case(_cfg(shape, 110), save_h=False)


# the reverse sweep of the two-pass backward on the same three kernels (two channels per workgroup: eight waves of rows on
# 512-row maps, both horizontal directions at once on 256-row maps)
@pytest.mark.parametrize("knob", ["GSPN_STREAM_TWO_CHANNELS", None, "GSPN_STREAM_NO_STAGED"], ids=["two-channel", "one-channel", "row-per-lane"])
@pytest.mark.parametrize("shape", [(1, 4, 512, 512, 2, "bf16"), (1, 4, 256, 512, 2, "bf16")], ids=lambda s: "x".join(map(str, s)))
def test_backward_on_maps_of_256_and_512_rows_bf16(shape, knob, monkeypatch):
    if knob:
        monkeypatch.setenv(knob, "1")
    check_bwd(_cfg(shape, 111))


def test_scaling_shape_1024x1024_on_sampled_slices():
    """1024x1024 with 8 channels per image in fp32 (the shape of the paper's step-by-step comparison, Sec. 5.1; batch 4
    here), launch shape as timed; the oracle computes a few (b, g) slices, which are independent given the group's weights."""
    import paper_2512_07884_amd as G
    cfg = WL.ScanConfig("big1024", 4, 8, 1024, 1024, 2, "f32", 15, 1.0, 105)
    assert G.gspn_fwd_plan(cfg.B, cfg.C, cfg.H, cfg.W, cfg.G, 15, 0, 0, False) == "stream"
    inp = WL.make_inputs(cfg, with_gy=False)
    y, *_ = run_fwd_gpu(inp, cfg, 15, save_h=False)
    cpg = cfg.cpg
    for b, g in ((0, 0), (2, 1), (3, 0)):
        cs = slice(g * cpg, (g + 1) * cpg)
        f = {n: np.asarray(inp[n][:, b:b + 1, cs] if n in ("lam", "u") else
                           inp[n][:, b:b + 1, g:g + 1] if n == "w" else inp[n][b:b + 1, cs], dtype=np.float64)
             for n in ("x", "w", "lam", "u")}
        y_ref, _ = O.scan_fwd(f["x"], f["w"], f["lam"], f["u"], 15)
        assert rel_inf_err(y[b:b + 1, cs], y_ref) <= TOL["f32"], (b, g)


# GSPN-local and logits calls on maps of 513 to 1024 rows: the same two launches with the stretch bookkeeping and the
# softmax of the line objects; forward with and without h_save and the two-pass backward; stretch lengths that divide
# the map and that do not; the first line of every stretch and the taps that point outside a line never read
@pytest.mark.parametrize("shape,kchunk", [((1, 2, 1024, 256, 1, "bf16"), 64), ((1, 2, 640, 512, 2, "f32"), 100),
                                          ((1, 2, 1024, 256, 1, "f16"), 37), ((1, 4, 576, 256, 2, "bf16"), 1)],
                         ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else str(v))
def test_local_scans_on_maps_beyond_512_rows(shape, kchunk):
    import paper_2512_07884_amd as G
    from test_gpu_local import check_local
    B, C, H, W, Gr, dtype = shape
    dt = {"f32": 0, "bf16": 1, "f16": 2}[dtype]
    assert G.gspn_fwd_local_plan(B, C, H, W, Gr, kchunk, 15, dt, 0, True) == "stream"
    assert G.gspn_bwd_local_plan(B, C, H, W, Gr, kchunk, 15, dt, 0) == "twopass"
    check_local(shape, kchunk, poison_starts=True)


@pytest.mark.parametrize("shape,kchunk", [((1, 2, 1024, 256, 1, "bf16"), None), ((1, 2, 640, 256, 2, "f32"), None),
                                          ((1, 2, 1024, 256, 1, "f16"), 128), ((1, 4, 576, 256, 2, "bf16"), 50)],
                         ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else str(v))
def test_logits_on_maps_beyond_512_rows(shape, kchunk):
    from test_gpu_logits import check_logits
    check_logits(shape, kchunk=kchunk, poison=True, fwd_plan="stream", bwd_plan="twopass")
