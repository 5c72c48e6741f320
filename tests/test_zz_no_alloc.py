"""The proxy-projection backward call for callers that cannot allocate (gspn_proxy_project_bwd_static: per-image sums in
a static device array of the library's) against the call that takes the workspace from the caller: same kernels, so
the results must agree bit for bit -- on two calls in a row, the second with a smaller input, so that what the first
call left in the array is there when the second runs."""
import numpy as np
import pytest

from gpu_util import to_device, empty_like_dev
from paper_2512_07884_amd import workloads as WL

pytestmark = pytest.mark.gpu


def _both(shape, seed):
    import torch
    import paper_2512_07884_amd as G
    B, K, M, H, W, dtype = shape
    rng = np.random.default_rng([seed, K, M])
    x = to_device(WL.to_storage(rng.standard_normal((B, K, H, W)), dtype), dtype)
    P = to_device(WL.to_storage(rng.standard_normal((M, K)) / np.sqrt(K), dtype), dtype)
    g = to_device(WL.to_storage(rng.standard_normal((B, M, H, W)), dtype), dtype)
    nan = float("nan")
    gin_a = empty_like_dev((B, K, H, W), dtype, nan); gin_b = empty_like_dev((B, K, H, W), dtype, nan)
    gP_a = torch.full((M, K), nan, device="cuda"); gP_b = torch.full((M, K), nan, device="cuda")
    partial = torch.full((B, M, K), nan, device="cuda")
    G.gspn_proxy_project_bwd(g, x, P, gin_a, gP_a, partial)
    G.gspn_proxy_project_bwd_static(g, x, P, gin_b, gP_b)
    torch.cuda.synchronize()
    assert torch.isfinite(gP_a).all() and torch.isfinite(gin_a.float()).all()
    assert torch.equal(gP_a, gP_b), shape
    assert torch.equal(gin_a.view(torch.int16 if dtype == "bf16" else torch.int32),
                       gin_b.view(torch.int16 if dtype == "bf16" else torch.int32)), shape


def test_static_workspace_call_matches_the_workspace_call_on_two_calls_in_a_row():
    _both((4, 96, 8, 28, 28, "bf16"), 1)       # matrix-core kernels, 3072 floats of per-image sums
    _both((2, 40, 5, 12, 12, "bf16"), 2)       # smaller: the array still holds the first call's sums beyond these
    _both((3, 7, 5, 9, 13, "f32"), 3)          # plain kernels, fp32 storage
    _both((2, 96, 8, 28, 28, "bf16"), 1)       # and a larger one again


def test_static_workspace_call_rejects_what_does_not_fit_and_needs_no_weight_gradient():
    import torch
    import paper_2512_07884_amd as G
    # B*M*K = 2 * 1024 * 1024 floats: twice the array
    B, K, M, H, W = 2, 1024, 1024, 4, 4
    x = torch.zeros((B, K, H, W), device="cuda", dtype=torch.bfloat16)
    P = torch.zeros((M, K), device="cuda", dtype=torch.bfloat16)
    g = torch.zeros((B, M, H, W), device="cuda", dtype=torch.bfloat16)
    gP = torch.full((M, K), 7.0, device="cuda")
    with pytest.raises(G.GspnError):
        G.gspn_proxy_project_bwd_static(g, x, P, None, gP)
    torch.cuda.synchronize()
    assert bool((gP == 7.0).all())             # nothing was launched
    gin = torch.full((B, K, H, W), float("nan"), device="cuda", dtype=torch.bfloat16)
    G.gspn_proxy_project_bwd_static(g, x, P, gin, None)     # without gP the size does not matter
    torch.cuda.synchronize()
    assert bool((gin == 0).all())
