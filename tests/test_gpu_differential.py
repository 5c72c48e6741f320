"""Seeded random shapes, masks, stretch lengths and call forms: what the fast kernels return (plane, tile, stream,
two-pass backward) against what the generic kernels return for the same device tensors.  The generic kernels are held
against the oracle elsewhere (test_gpu_fwd / test_gpu_bwd / test_gpu_local / test_gpu_logits with GSPN_FORCE_GENERIC);
this test spreads over many more shapes than the oracle could check in the same time."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _rel(a, b):
    m = float(b.abs().max())
    return float((a - b).abs().max()) / (m if m > 0 else 1.0)


def _run(G, inp, Gr, mask, kchunk, logits):
    import torch
    nan = float("nan")
    out = {"y": torch.full_like(inp["x"], nan), "hs": torch.full_like(inp["lam"], nan), "gx": torch.full_like(inp["x"], nan),
           "gw": torch.full_like(inp["w"], nan), "gl": torch.full_like(inp["lam"], nan), "gu": torch.full_like(inp["lam"], nan)}
    a = (inp["x"], inp["w"], inp["lam"], inp["u"])
    g = (out["gx"], out["gw"], out["gl"], out["gu"])
    k = kchunk if kchunk else G.binding.GLOBAL_SCAN
    if logits:
        G.gspn_scan_fwd_logits(*a, out["y"], out["hs"], kchunk=k, G=Gr, dir_mask=mask)
        G.gspn_scan_bwd_logits(inp["gy"], *a, out["hs"], *g, kchunk=k, G=Gr, dir_mask=mask)
    elif kchunk:
        G.gspn_scan_fwd_local(*a, out["y"], out["hs"], kchunk=k, G=Gr, dir_mask=mask)
        G.gspn_scan_bwd_local(inp["gy"], *a, out["hs"], *g, kchunk=k, G=Gr, dir_mask=mask)
    else:
        G.gspn_scan_fwd(*a, out["y"], out["hs"], G=Gr, dir_mask=mask)
        G.gspn_scan_bwd(inp["gy"], *a, out["hs"], *g, G=Gr, dir_mask=mask)
    torch.cuda.synchronize()
    return out


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_fast_kernels_agree_with_the_generic_kernels_on_random_cases(seed, monkeypatch):
    import torch
    import paper_2512_07884_amd as G
    from paper_2512_07884_amd import binding
    G.binding = binding
    rng = np.random.default_rng(seed)
    for it in range(16):
        dtype = "bf16" if rng.random() < 0.5 else "f32"
        cls = int(rng.integers(0, 5))
        if cls == 0:   H, W = int(rng.integers(2, 65)), int(rng.integers(1, 17)) * 4          # up to 64 lines
        elif cls == 1: H, W = int(rng.integers(1, 5)) * 32, int(rng.integers(1, 5)) * 32      # rows split over waves
        elif cls == 2: H, W = int(rng.integers(1, 4)) * 64, int(rng.choice([256, 512]))       # beyond the LDS tile
        elif cls == 3: H, W = int(rng.integers(2, 33)), int(rng.integers(2, 33))              # small, ragged
        else:          H, W = int(rng.integers(33, 130)), int(rng.integers(1, 17)) * 8
        cpg = int(rng.choice([1, 2, 3, 4, 6, 8, 12]))
        Gr = int(rng.integers(1, 4)); C = cpg * Gr; B = int(rng.integers(1, 3))
        if H * W * C * B > 2_000_000:
            C, Gr, B = cpg, 1, 1
        mask = int(rng.integers(1, 16)) if rng.random() < 0.3 else 15
        kchunk = int(rng.integers(1, max(H, W))) if rng.random() < 0.35 else 0
        logits = bool(rng.random() < 0.3)
        td = torch.bfloat16 if dtype == "bf16" else torch.float32
        g = torch.Generator(device="cuda"); g.manual_seed(1000 * seed + it)
        z = torch.randn((4, B, Gr, 3, H, W), generator=g, device="cuda")
        if logits:
            w = z.to(td)
        else:       # rows stochastic over the neighbours that exist
            z[:2, :, :, 0, :, 0] = -1e30; z[:2, :, :, 2, :, -1] = -1e30; z[2:, :, :, 0, 0, :] = -1e30; z[2:, :, :, 2, -1, :] = -1e30
            w = torch.softmax(z.double(), dim=3).to(td)
        inp = {"x": torch.randn((B, C, H, W), generator=g, device="cuda").to(td), "w": w,
               "lam": torch.rand((4, B, C, H, W), generator=g, device="cuda").to(td),
               "u": torch.rand((4, B, C, H, W), generator=g, device="cuda").to(td),
               "gy": torch.randn((B, C, H, W), generator=g, device="cuda").to(td)}
        monkeypatch.delenv("GSPN_FORCE_GENERIC", raising=False)
        fast = _run(G, inp, Gr, mask, kchunk, logits)
        monkeypatch.setenv("GSPN_FORCE_GENERIC", "1")
        ref = _run(G, inp, Gr, mask, kchunk, logits)
        monkeypatch.delenv("GSPN_FORCE_GENERIC", raising=False)
        # bf16: both sides round every stored value once (two storage roundings apart at most, plus the generic
        # forward's per-direction rounding of y on maps beyond its LDS tile)
        tol = 2e-2 if dtype == "bf16" else 2e-5
        case = (seed, it, B, C, H, W, Gr, dtype, mask, kchunk, logits)
        for n in fast:
            a, b = fast[n].float(), ref[n].float()
            na, nb = torch.isnan(a), torch.isnan(b)
            assert torch.equal(na, nb), (case, n, "slots of unmasked directions differ")
            e = _rel(torch.where(na, torch.zeros_like(a), a), torch.where(nb, torch.zeros_like(b), b))
            assert e <= tol, (case, n, e)
