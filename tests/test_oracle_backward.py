"""Pins for the fp64 oracle's backward scan (CPU only).

The paper gives no backward algorithm; the oracle's formulas are the chain rule
on Eq. 1-2.  They are pinned here by central finite differences on every input
(single weight entries perturbed independently), by the adjoint identity, and
by the transposed dense operator built in image coordinates.
"""
import numpy as np
import pytest

from oracle import gspn_oracle as O
from test_oracle_forward import rand_problem


def loss(x, w, lam, u, gy, mask):
    y, _ = O.scan_fwd(x, w, lam, u, mask)
    return float((y * gy).sum())


@pytest.mark.parametrize("mask", [1, 2, 4, 8, 15])
@pytest.mark.parametrize("G", [1, 2, 4])
def test_gradients_match_central_finite_differences(mask, G):
    rng = np.random.default_rng(40 + mask + G)
    B, C, H, W = 1, 4, 4, 3
    x, w, lam, u = rand_problem(rng, B, C, H, W, G)
    gy = rng.standard_normal(x.shape)
    _, h = O.scan_fwd(x, w, lam, u, mask)
    gx, gw, glam, gu = O.scan_bwd(gy, x, w, lam, u, h, mask)
    eps = 1e-6
    for name, arr, grad in (("x", x, gx), ("w", w, gw), ("lam", lam, glam), ("u", u, gu)):
        flat = arr.reshape(-1)
        idx = rng.choice(flat.size, size=min(flat.size, 60), replace=False)
        for k in idx:
            old = flat[k]
            flat[k] = old + eps; lp = loss(x, w, lam, u, gy, mask)
            flat[k] = old - eps; lm = loss(x, w, lam, u, gy, mask)
            flat[k] = old
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - grad.reshape(-1)[k]) < 1e-7 * (1 + abs(fd)), (name, k, fd, grad.reshape(-1)[k])


def test_gw_is_zero_where_the_weight_is_never_used():
    rng = np.random.default_rng(50)
    B, C, H, W, G = 1, 2, 4, 5, 1
    x, w, lam, u = rand_problem(rng, B, C, H, W, G)
    gy = rng.standard_normal(x.shape)
    _, h = O.scan_fwd(x, w, lam, u, 15)
    _, gw, _, _ = O.scan_bwd(gy, x, w, lam, u, h, 15)
    # first scan line of every direction, and the out-of-line planes
    assert not gw[0][:, :, :, 0, :].any() and not gw[1][:, :, :, -1, :].any()
    assert not gw[2][:, :, :, :, 0].any() and not gw[3][:, :, :, :, -1].any()
    for d in (0, 1):
        assert not gw[d][:, :, 0, :, 0].any() and not gw[d][:, :, 2, :, -1].any()
    for d in (2, 3):
        assert not gw[d][:, :, 0, 0, :].any() and not gw[d][:, :, 2, -1, :].any()
    # and non-zero elsewhere
    assert np.count_nonzero(gw[0][:, :, 1, 1:, :]) == gw[0][:, :, 1, 1:, :].size


def test_adjoint_identity_for_x():
    rng = np.random.default_rng(51)
    B, C, H, W, G = 2, 3, 5, 6, 3
    x, w, lam, u = rand_problem(rng, B, C, H, W, G)
    gy = rng.standard_normal(x.shape)
    v = rng.standard_normal(x.shape)
    _, h = O.scan_fwd(x, w, lam, u, 15)
    gx, _, _, _ = O.scan_bwd(gy, x, w, lam, u, h, 15)
    jv, _ = O.scan_fwd(v, w, lam, u, 15)              # the map x -> y is linear
    assert abs((gy * jv).sum() - (gx * v).sum()) < 1e-10


def test_gx_matches_transposed_dense_operator():
    rng = np.random.default_rng(52)
    B, C, H, W, G = 1, 2, 4, 3, 2
    x, w, lam, u = rand_problem(rng, B, C, H, W, G)
    gy = rng.standard_normal(x.shape)
    _, h = O.scan_fwd(x, w, lam, u, 15)
    gx, _, glam, gu = O.scan_bwd(gy, x, w, lam, u, h, 15)
    eye = np.eye(H * W)
    for c in range(C):
        acc = np.zeros(H * W)
        for d in range(4):
            A = O.one_step_matrix_image(w[d, 0, c], d, H, W)      # G == C here
            # y_d = diag(u) (I-A)^{-1} diag(lam) x  =>  gx_d = diag(lam) (I-A)^{-T} diag(u) gy
            e = np.linalg.solve((eye - A).T, (u[d, 0, c] * gy[0, c]).reshape(-1))
            acc += lam[d, 0, c].reshape(-1) * e
            assert np.allclose(glam[d, 0, c].reshape(-1), x[0, c].reshape(-1) * e, atol=1e-12)
            assert np.allclose(gu[d, 0, c], gy[0, c] * h[d, 0, c], atol=1e-12)
        assert np.allclose(gx[0, c].reshape(-1), acc, atol=1e-12)


def test_unmasked_directions_get_zero_gradients():
    rng = np.random.default_rng(53)
    x, w, lam, u = rand_problem(rng, 1, 2, 3, 4, 1)
    gy = rng.standard_normal(x.shape)
    _, h = O.scan_fwd(x, w, lam, u, 9)
    gx, gw, glam, gu = O.scan_bwd(gy, x, w, lam, u, h, 9)
    for d in (1, 2):
        assert not gw[d].any() and not glam[d].any() and not gu[d].any()
    assert gw[0].any() and gw[3].any()
