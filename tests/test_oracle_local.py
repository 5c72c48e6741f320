"""Pins for the oracle's GSPN-local scans (CPU only).

GSPN-local (Sec. 3.2) confines propagation to stretches of kchunk lines along the scan axis.  The
oracle writes that as one global scan per stretch; here it is held against forms that do not slice:
the dense solve with the links between stretches removed, the two limits of kchunk, the fact that a
perturbation stays inside its stretch, and for the backward central finite differences, the adjoint
identity and the zeros of gw on the first line of every stretch.
"""
import numpy as np
import pytest

from oracle import gspn_oracle as O
from test_oracle_forward import rand_problem


@pytest.mark.parametrize("kchunk", [1, 2, 3, 4, 7])
@pytest.mark.parametrize("mask", [1, 2, 4, 8, 15])
def test_local_scan_equals_dense_solve_without_links_between_stretches(kchunk, mask):
    rng = np.random.default_rng(100 + kchunk + mask)
    B, C, H, W, G = 1, 2, 5, 6, 2                       # 5 and 6 lines: ragged last stretch for 2, 3, 4
    x, w, lam, u = rand_problem(rng, B, C, H, W, G)
    y, h = O.scan_fwd_local(x, w, lam, u, kchunk, mask)
    yd, hd = O.dense_fwd(x, w, lam, u, mask, kchunk=kchunk)
    assert np.abs(y - yd).max() < 1e-12 and np.abs(h - hd).max() < 1e-12


def test_kchunk_of_one_line_leaves_no_propagation():
    rng = np.random.default_rng(7)
    x, w, lam, u = rand_problem(rng, 2, 4, 5, 4, 2)
    y, h = O.scan_fwd_local(x, w, lam, u, 1, 15)
    assert np.array_equal(h, lam * x[None])
    assert np.allclose(y, (u * lam * x[None]).sum(axis=0), rtol=0, atol=1e-15)


@pytest.mark.parametrize("kchunk", [6, 7, 100])
def test_kchunk_of_at_least_the_scan_length_is_the_global_scan(kchunk):
    rng = np.random.default_rng(8)
    x, w, lam, u = rand_problem(rng, 1, 4, 6, 5, 2)
    y, h = O.scan_fwd_local(x, w, lam, u, kchunk, 15)
    yg, hg = O.scan_fwd(x, w, lam, u, 15)
    assert np.array_equal(y, yg) and np.array_equal(h, hg)
    gy = rng.standard_normal(x.shape)
    for a, b in zip(O.scan_bwd_local(gy, x, w, lam, u, h, kchunk, 15), O.scan_bwd(gy, x, w, lam, u, hg, 15)):
        assert np.array_equal(a, b)


def test_mixed_limits_when_only_one_axis_is_shorter_than_kchunk():
    """H = 3 < kchunk = 4 <= W = 8: the vertical scans are global, the horizontal ones local."""
    rng = np.random.default_rng(9)
    x, w, lam, u = rand_problem(rng, 1, 2, 3, 8, 1)
    _, h = O.scan_fwd_local(x, w, lam, u, 4, 15)
    _, hg = O.scan_fwd(x, w, lam, u, 15)
    assert np.array_equal(h[:2], hg[:2]) and not np.allclose(h[2:], hg[2:])


@pytest.mark.parametrize("d", [0, 1, 2, 3])
def test_a_perturbation_stays_inside_its_stretch(d):
    rng = np.random.default_rng(10 + d)
    H, W, k = 7, 8, 3
    x, w, lam, u = rand_problem(rng, 1, 2, H, W, 1)
    _, h0 = O.scan_fwd_local(x, w, lam, u, k, 1 << d)
    x2 = x.copy()
    pos = (4, 2) if d < 2 else (2, 4)                   # line 4 of the scan axis: stretch [3, 6)
    x2[0, 0, pos[0], pos[1]] += 1.0
    _, h1 = O.scan_fwd_local(x2, w, lam, u, k, 1 << d)
    diff = np.abs(h1 - h0)[d, 0, 0]
    lines = diff.any(axis=1) if d < 2 else diff.any(axis=0)
    inside = np.zeros_like(lines)
    inside[3:6] = True
    assert not lines[~inside].any()
    # ... and does reach the rest of the stretch downstream of it, in scan order
    downstream = 5 if d in (0, 2) else 3
    assert lines[downstream]
    upstream = 3 if d in (0, 2) else 5
    assert not lines[upstream]


def loss(x, w, lam, u, gy, k, mask):
    y, _ = O.scan_fwd_local(x, w, lam, u, k, mask)
    return float((y * gy).sum())


@pytest.mark.parametrize("mask", [1, 2, 4, 8, 15])
@pytest.mark.parametrize("kchunk", [2, 3])
def test_local_gradients_match_central_finite_differences(mask, kchunk):
    rng = np.random.default_rng(60 + mask + kchunk)
    B, C, H, W, G = 1, 4, 5, 4, 2
    x, w, lam, u = rand_problem(rng, B, C, H, W, G)
    gy = rng.standard_normal(x.shape)
    _, h = O.scan_fwd_local(x, w, lam, u, kchunk, mask)
    gx, gw, glam, gu = O.scan_bwd_local(gy, x, w, lam, u, h, kchunk, mask)
    eps = 1e-6
    for name, arr, grad in (("x", x, gx), ("w", w, gw), ("lam", lam, glam), ("u", u, gu)):
        flat = arr.reshape(-1)
        idx = rng.choice(flat.size, size=min(flat.size, 80), replace=False)
        for i in idx:
            old = flat[i]
            flat[i] = old + eps; lp = loss(x, w, lam, u, gy, kchunk, mask)
            flat[i] = old - eps; lm = loss(x, w, lam, u, gy, kchunk, mask)
            flat[i] = old
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - grad.reshape(-1)[i]) < 1e-7 * (1 + abs(fd)), (name, i, fd, grad.reshape(-1)[i])


def test_local_adjoint_identity_for_x():
    rng = np.random.default_rng(70)
    x, w, lam, u = rand_problem(rng, 2, 4, 6, 7, 2)
    gy = rng.standard_normal(x.shape)
    v = rng.standard_normal(x.shape)
    k = 3
    _, h = O.scan_fwd_local(x, w, lam, u, k, 15)
    gx, *_ = O.scan_bwd_local(gy, x, w, lam, u, h, k, 15)
    jv, _ = O.scan_fwd_local(v, w, lam, u, k, 15)       # the scan is linear in x
    assert abs((gy * jv).sum() - (gx * v).sum()) < 1e-10 * (1 + abs((gx * v).sum()))


def test_local_gw_is_zero_on_the_first_line_of_every_stretch():
    rng = np.random.default_rng(71)
    H, W, k = 7, 5, 3
    x, w, lam, u = rand_problem(rng, 1, 2, H, W, 1)
    gy = rng.standard_normal(x.shape)
    _, h = O.scan_fwd_local(x, w, lam, u, k, 15)
    _, gw, _, _ = O.scan_bwd_local(gy, x, w, lam, u, h, k, 15)
    # stretches of the rows: [0,3) [3,6) [6,7); of the columns: [0,3) [3,5)
    assert not gw[0][:, :, :, [0, 3, 6], :].any() and gw[0][:, :, 1, [1, 2, 4, 5], :].all()
    assert not gw[1][:, :, :, [2, 5, 6], :].any() and gw[1][:, :, 1, [0, 1, 3, 4], :].all()
    assert not gw[2][:, :, :, :, [0, 3]].any() and gw[2][:, :, 1, :, [1, 2, 4]].all()
    assert not gw[3][:, :, :, :, [2, 4]].any() and gw[3][:, :, 1, :, [0, 1, 3]].all()
