"""GPU parity of the compressive proxy projection (Sec. 4.2) against the fp64 oracle, through the C ABI:
matrix-core kernel (bf16) and the plain FMA kernel (fp32, ragged shapes), and the whole wrapper
project down -> scan -> project up."""
import numpy as np
import pytest

from gpu_util import TOL, rel_inf_err, to_device, to_host_f64, empty_like_dev
from oracle import gspn_oracle as O
from paper_2512_07884_amd import workloads as WL

pytestmark = pytest.mark.gpu


def run_project(x_st, P_st, dtype):
    import torch
    import paper_2512_07884_amd as G
    B, K, H, W = x_st.shape
    M = P_st.shape[0]
    out = empty_like_dev((B, M, H, W), dtype, float("nan"))
    G.gspn_proxy_project(to_device(x_st, dtype), to_device(P_st, dtype), out)
    torch.cuda.synchronize()
    return to_host_f64(out)


# (B, K, M, H, W, dtype): down- and up-projections of the paper's shapes (C_proxy = 2 and 8 at classifier widths,
# 1152 -> 144 of the diffusion study, Sec. 4.2 / App. "low rank"), several row tiles, ragged pixel and row tiles
SHAPES = [(2, 96, 8, 56, 56, "bf16"), (2, 8, 96, 56, 56, "bf16"), (1, 96, 2, 28, 28, "bf16"), (1, 1152, 144, 16, 16, "bf16"),
          (1, 144, 1152, 16, 16, "bf16"), (3, 40, 33, 12, 10, "bf16"), (1, 8, 1, 2, 4, "bf16"), (1, 64, 70, 24, 40, "bf16"),
          (2, 96, 8, 28, 28, "f32"), (1, 7, 5, 9, 13, "f32"), (1, 12, 3, 5, 7, "bf16"), (1, 10, 4, 8, 8, "bf16"),
          (2, 96, 8, 56, 56, "f16"), (2, 8, 96, 56, 56, "f16"), (1, 1152, 144, 16, 16, "f16"), (3, 40, 33, 12, 10, "f16"),
          (1, 12, 3, 5, 7, "f16")]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_projection_matches_the_oracle(shape):
    import paper_2512_07884_amd as G
    B, K, M, H, W, dtype = shape
    rng = np.random.default_rng([11, K, M, H])
    x = WL.to_storage(rng.standard_normal((B, K, H, W)), dtype)
    P = WL.to_storage(rng.standard_normal((M, K)) / np.sqrt(K), dtype)
    want = "mfma" if dtype != "f32" and K % 8 == 0 and (H * W) % 8 == 0 else "fma"
    assert G.gspn_proxy_plan(B, K, M, H, W, {"f32": 0, "bf16": 1, "f16": 2}[dtype]) == want
    ref = O.proxy_project(WL.storage_to_f64(x, dtype), WL.storage_to_f64(P, dtype))
    got = run_project(x, P, dtype)
    assert rel_inf_err(got, ref) <= TOL[dtype], rel_inf_err(got, ref)


@pytest.mark.parametrize("K", [64, 40], ids=["k16_steps", "k8_steps"])
def test_every_output_element_comes_from_its_own_row_and_pixel(K):
    """P with a single 1 per row copies input channels: the output must equal them bit for bit, which pins the
    operand and accumulator layout of the matrix-core kernel (both instruction shapes) element by element."""
    rng = np.random.default_rng(5)
    B, M, H, W = 2, 40, 16, 24
    x = WL.to_storage(rng.standard_normal((B, K, H, W)), "bf16")
    pick = rng.integers(0, K, size=M)
    P = np.zeros((M, K))
    P[np.arange(M), pick] = 1.0
    got = run_project(x, WL.to_storage(P, "bf16"), "bf16")
    assert np.array_equal(got, WL.storage_to_f64(x, "bf16")[:, pick])


def test_scan_wrapped_in_the_proxy():
    import torch
    import paper_2512_07884_amd as G
    B, C, Cp, H, W, dtype = 2, 96, 8, 56, 56, "bf16"
    cfg = WL.ScanConfig("proxy", B, Cp, H, W, 1, dtype, 15, 1.0, 21)        # the scan runs on the proxy channels
    inp = WL.make_inputs(cfg, with_gy=False)
    rng = np.random.default_rng(22)
    x = WL.to_storage(rng.standard_normal((B, C, H, W)), dtype)
    Pd = WL.to_storage(rng.standard_normal((Cp, C)) / np.sqrt(C), dtype)
    Pu = WL.to_storage(rng.standard_normal((C, Cp)) / np.sqrt(Cp), dtype)
    dev = {k: to_device(v, dtype) for k, v in inp.items()}
    xp = empty_like_dev((B, Cp, H, W), dtype)
    yp = empty_like_dev((B, Cp, H, W), dtype)
    y = empty_like_dev((B, C, H, W), dtype, float("nan"))
    G.gspn_proxy_project(to_device(x, dtype), to_device(Pd, dtype), xp)
    G.gspn_scan_fwd(xp, dev["w"], dev["lam"], dev["u"], yp, None, G=1)
    G.gspn_proxy_project(yp, to_device(Pu, dtype), y)
    torch.cuda.synchronize()
    f = WL.inputs_as_f64(inp, dtype)
    ref = O.proxy_scan_fwd(WL.storage_to_f64(x, dtype), WL.storage_to_f64(Pd, dtype), f["w"], f["lam"], f["u"],
                           WL.storage_to_f64(Pu, dtype))
    # three roundings to bf16 on the way (x_proxy, y_proxy, y): 3 * 2^-9 relative to intermediate maxima
    assert rel_inf_err(to_host_f64(y), ref) <= 2e-2


# ---- gradients of the projection ------------------------------------------------------------------------------------
def run_project_bwd(g_st, x_st, P_st, dtype, want_gin=True, want_gp=True):
    import torch
    import paper_2512_07884_amd as G
    B, K, H, W = x_st.shape
    M = P_st.shape[0]
    gin = empty_like_dev((B, K, H, W), dtype, float("nan")) if want_gin else None
    gP = torch.full((M, K), float("nan"), device="cuda", dtype=torch.float32) if want_gp else None
    partial = torch.full((B, M, K), float("nan"), device="cuda", dtype=torch.float32) if want_gp else None
    G.gspn_proxy_project_bwd(to_device(g_st, dtype), to_device(x_st, dtype), to_device(P_st, dtype), gin, gP, partial)
    torch.cuda.synchronize()
    return (to_host_f64(gin) if want_gin else None), (gP.double().cpu().numpy() if want_gp else None)


# (B, K, M, H, W, dtype) as above: matrix-core kernels (M a multiple of 16 / of 8 for gin, H*W a multiple of 16 for gP),
# plain kernels (fp32, C_proxy = 2, ragged pixel counts), several tiles of gP with ragged edges
BWD_SHAPES = [(2, 96, 8, 56, 56, "bf16"), (2, 8, 96, 56, 56, "bf16"), (1, 96, 2, 28, 28, "bf16"), (1, 1152, 144, 16, 16, "bf16"),
              (1, 144, 1152, 16, 16, "bf16"), (3, 40, 33, 12, 10, "bf16"), (1, 64, 70, 24, 40, "bf16"), (2, 96, 8, 28, 28, "f32"),
              (1, 7, 5, 9, 13, "f32"), (1, 12, 3, 5, 7, "bf16"), (2, 40, 16, 12, 12, "bf16"), (2, 70, 24, 8, 6, "f32"),
              (2, 96, 8, 56, 56, "f16"), (2, 8, 96, 56, 56, "f16"), (1, 144, 1152, 16, 16, "f16"), (3, 40, 33, 12, 10, "f16"),
              (1, 12, 3, 5, 7, "f16")]


@pytest.mark.parametrize("shape", BWD_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_projection_gradients_match_the_oracle(shape):
    B, K, M, H, W, dtype = shape
    rng = np.random.default_rng([13, K, M, H])
    x = WL.to_storage(rng.standard_normal((B, K, H, W)), dtype)
    P = WL.to_storage(rng.standard_normal((M, K)) / np.sqrt(K), dtype)
    g = WL.to_storage(rng.standard_normal((B, M, H, W)), dtype)
    gin_ref, gP_ref = O.proxy_project_bwd(WL.storage_to_f64(g, dtype), WL.storage_to_f64(x, dtype), WL.storage_to_f64(P, dtype))
    gin, gP = run_project_bwd(g, x, P, dtype)
    assert rel_inf_err(gin, gin_ref) <= TOL[dtype], ("gin", rel_inf_err(gin, gin_ref))
    # gP is accumulated and returned in fp32 whatever the storage type
    assert rel_inf_err(gP, gP_ref) <= 1e-5, ("gP", rel_inf_err(gP, gP_ref))


@pytest.mark.parametrize("K,M", [(40, 33), (200, 130)], ids=["8_waves_per_tile", "4_waves_per_tile"])
def test_weight_gradient_with_either_wave_count_and_more_images_than_one_batch_of_the_sum(K, M):
    # 19 images: the kernel that adds the per-image sums asks for 16 at a time and has a ragged second batch;
    # 76 tiles run the tile kernel's eight-wave instantiation, 665 tiles (512 and more) the four-wave one
    B, H, W = 19, 12, 12
    rng = np.random.default_rng([19, K])
    x = WL.to_storage(rng.standard_normal((B, K, H, W)), "bf16")
    P = WL.to_storage(rng.standard_normal((M, K)) / np.sqrt(K), "bf16")
    g = WL.to_storage(rng.standard_normal((B, M, H, W)), "bf16")
    _, gP_ref = O.proxy_project_bwd(WL.storage_to_f64(g, "bf16"), WL.storage_to_f64(x, "bf16"), WL.storage_to_f64(P, "bf16"))
    _, gP = run_project_bwd(g, x, P, "bf16", want_gin=False)
    assert rel_inf_err(gP, gP_ref) <= 1e-5, rel_inf_err(gP, gP_ref)
    _, gP2 = run_project_bwd(g, x, P, "bf16", want_gin=False)
    assert np.array_equal(gP, gP2)


def test_projection_gradients_one_at_a_time_and_bitwise_repeatable():
    rng = np.random.default_rng(17)
    B, K, M, H, W = 3, 96, 8, 28, 28
    x = WL.to_storage(rng.standard_normal((B, K, H, W)), "bf16")
    P = WL.to_storage(rng.standard_normal((M, K)) / np.sqrt(K), "bf16")
    g = WL.to_storage(rng.standard_normal((B, M, H, W)), "bf16")
    gin, gP = run_project_bwd(g, x, P, "bf16")
    gin_only, none = run_project_bwd(g, x, P, "bf16", want_gp=False)
    none2, gP_only = run_project_bwd(g, x, P, "bf16", want_gin=False)
    assert none is None and none2 is None
    assert np.array_equal(gin, gin_only) and np.array_equal(gP, gP_only)
    for _ in range(2):
        gin2, gP2 = run_project_bwd(g, x, P, "bf16")
        assert np.array_equal(gin, gin2) and np.array_equal(gP, gP2)


def test_input_gradient_of_a_selection_matrix_is_a_copy():
    """P with a single 1 per row: gin of the picked channels equals gout bit for bit, the other channels get 0 -- pins the
    transposed read of P in the matrix-core kernel."""
    rng = np.random.default_rng(19)
    B, K, M, H, W = 2, 64, 16, 16, 24
    g = WL.to_storage(rng.standard_normal((B, M, H, W)), "bf16")
    x = WL.to_storage(rng.standard_normal((B, K, H, W)), "bf16")
    pick = rng.permutation(K)[:M]
    P = np.zeros((M, K))
    P[np.arange(M), pick] = 1.0
    gin, _ = run_project_bwd(g, x, WL.to_storage(P, "bf16"), "bf16", want_gp=False)
    assert np.array_equal(gin[:, pick], WL.storage_to_f64(g, "bf16"))
    rest = np.setdiff1d(np.arange(K), pick)
    assert not gin[:, rest].any()


def test_training_step_through_the_wrapped_scan():
    """project down -> scan -> project up, and the gradients back through the three stages, all on the GPU path, against
    the oracle's chain (fp32 storage: the intermediate tensors are rounded nowhere)."""
    import torch
    import paper_2512_07884_amd as G
    B, C, Cp, H, W, dtype = 2, 24, 8, 28, 28, "f32"
    cfg = WL.ScanConfig("proxytrain", B, Cp, H, W, 2, dtype, 15, 1.0, 23)
    inp = WL.make_inputs(cfg, with_gy=False)
    rng = np.random.default_rng(24)
    x = WL.to_storage(rng.standard_normal((B, C, H, W)), dtype)
    Pd = WL.to_storage(rng.standard_normal((Cp, C)) / np.sqrt(C), dtype)
    Pu = WL.to_storage(rng.standard_normal((C, Cp)) / np.sqrt(Cp), dtype)
    gy = WL.to_storage(rng.standard_normal((B, C, H, W)), dtype)
    d = {k: to_device(v, dtype) for k, v in inp.items()}
    dx, dPd, dPu, dgy = (to_device(a, dtype) for a in (x, Pd, Pu, gy))
    new = lambda *shape: torch.full(shape, float("nan"), device="cuda", dtype=torch.float32)
    xp, yp, y, hs = new(B, Cp, H, W), new(B, Cp, H, W), new(B, C, H, W), new(4, B, Cp, H, W)
    G.gspn_proxy_project(dx, dPd, xp)
    G.gspn_scan_fwd(xp, d["w"], d["lam"], d["u"], yp, hs, G=cfg.G)
    G.gspn_proxy_project(yp, dPu, y)
    gyp, gPu, part_u = new(B, Cp, H, W), new(C, Cp), new(B, C, Cp)
    G.gspn_proxy_project_bwd(dgy, yp, dPu, gyp, gPu, part_u)
    gxp, gw, glam, gu = new(B, Cp, H, W), torch.full_like(d["w"], float("nan")), new(4, B, Cp, H, W), new(4, B, Cp, H, W)
    G.gspn_scan_bwd(gyp, xp, d["w"], d["lam"], d["u"], hs, gxp, gw, glam, gu, G=cfg.G)
    gx, gPd, part_d = new(B, C, H, W), new(Cp, C), new(B, Cp, C)
    G.gspn_proxy_project_bwd(gxp, dx, dPd, gx, gPd, part_d)
    torch.cuda.synchronize()
    f = WL.inputs_as_f64(inp, dtype)
    ref = O.proxy_scan_bwd(gy.astype(np.float64), x.astype(np.float64), Pd.astype(np.float64), f["w"], f["lam"], f["u"],
                           Pu.astype(np.float64))
    got = (gx, gPd, gw, glam, gu, gPu)
    for name, a, r in zip(("gx", "gPd", "gw", "glam", "gu", "gPu"), got, ref):
        e = rel_inf_err(a.double().cpu().numpy(), r)
        assert e <= 2e-5, (name, e)
