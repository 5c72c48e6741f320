"""Pins for the oracle's handling of weights given as raw logits (CPU only): the normalisation the paper
asks for (Sec. 3.2: weights normalised so that every row of T_i sums to 1), taken as a softmax over the
three taps with the taps that point outside the line left out."""
import numpy as np
import pytest
from scipy.special import softmax

from oracle import gspn_oracle as O


def rand_logits_problem(rng, B, C, H, W, G):
    x = rng.standard_normal((B, C, H, W))
    z = 2.0 * rng.standard_normal((4, B, G, 3, H, W))
    lam = rng.uniform(0, 1, (4, B, C, H, W))
    u = rng.uniform(0, 1, (4, B, C, H, W))
    return x, z, lam, u


def test_interior_positions_are_the_library_softmax_and_ends_use_the_two_taps_that_exist():
    rng = np.random.default_rng(1)
    z = rng.standard_normal((4, 2, 3, 3, 5, 6))
    w = O.weights_from_logits(z)
    for d in range(4):
        inner = (slice(None), slice(None), slice(None), slice(None), slice(1, -1)) if d < 2 else \
                (slice(None), slice(None), slice(None), slice(1, -1), slice(None))
        assert np.allclose(w[d][inner], softmax(z[d], axis=2)[inner], rtol=0, atol=1e-15)
    # left end of a row (vertical scans): taps 1 and 2 only
    assert np.allclose(w[0][:, :, 1:, :, 0], softmax(z[0][:, :, 1:, :, 0], axis=2), rtol=0, atol=1e-15)
    assert not w[0][:, :, 0, :, 0].any() and not w[1][:, :, 2, :, -1].any()
    # top end of a column (horizontal scans): taps 1 and 2 only; bottom end: taps 0 and 1
    assert np.allclose(w[2][:, :, 1:, 0, :], softmax(z[2][:, :, 1:, 0, :], axis=2), rtol=0, atol=1e-15)
    assert np.allclose(w[3][:, :, :2, -1, :], softmax(z[3][:, :, :2, -1, :], axis=2), rtol=0, atol=1e-15)
    assert not w[2][:, :, 0, 0, :].any() and not w[3][:, :, 2, -1, :].any()


def test_every_row_of_the_assembled_tridiagonal_sums_to_one():
    rng = np.random.default_rng(2)
    z = 3.0 * rng.standard_normal((4, 1, 2, 3, 4, 5))
    w = O.weights_from_logits(z)
    assert (w >= 0).all()
    for d in range(4):
        wc = O._to_canonical(w[d], d)                     # [B, G, 3, S, L]
        for g in range(2):
            for i in range(wc.shape[3]):
                T = O.tridiagonal(wc[0, g, :, i, :])
                assert np.allclose(T.sum(axis=1), 1.0, rtol=0, atol=1e-14)


def test_shift_of_the_logits_and_content_of_masked_logits_do_not_matter():
    rng = np.random.default_rng(3)
    x, z, lam, u = rand_logits_problem(rng, 1, 4, 5, 4, 2)
    y0, h0 = O.scan_fwd_logits(x, z, lam, u)
    shift = rng.standard_normal((4, 1, 2, 1, 5, 4))
    y1, _ = O.scan_fwd_logits(x, z + shift, lam, u)
    assert np.allclose(y0, y1, rtol=0, atol=1e-12)
    z2 = z.copy()
    z2[0, :, :, 0, :, 0] = np.nan; z2[1, :, :, 2, :, -1] = np.inf
    z2[2, :, :, 0, 0, :] = -np.inf; z2[3, :, :, 2, -1, :] = np.nan
    y2, h2 = O.scan_fwd_logits(x, z2, lam, u)
    assert np.array_equal(y0, y2) and np.array_equal(h0, h2)


def test_constant_state_is_kept_by_the_normalised_weights():
    """Row-stochastic weights map a constant line to itself (the stability condition of Sec. 3.2): with
    x = c, lam = 1 the state on scan step s is (s + 1) c for every position, whatever the logits."""
    rng = np.random.default_rng(4)
    B, C, H, W, G = 1, 2, 6, 5, 1
    z = 4.0 * rng.standard_normal((4, B, G, 3, H, W))
    x = np.full((B, C, H, W), 0.75)
    one = np.ones((4, B, C, H, W))
    _, h = O.scan_fwd_logits(x, z, one, one)
    steps_v = np.arange(1, H + 1)[:, None] * np.ones((1, W))
    steps_h = np.ones((H, 1)) * np.arange(1, W + 1)[None, :]
    assert np.allclose(h[0][0, 0], 0.75 * steps_v) and np.allclose(h[1][0, 0], 0.75 * steps_v[::-1])
    assert np.allclose(h[2][0, 0], 0.75 * steps_h) and np.allclose(h[3][0, 0], 0.75 * steps_h[:, ::-1])


def loss(x, z, lam, u, gy, mask, k):
    y, _ = O.scan_fwd_logits(x, z, lam, u, mask, k)
    return float((y * gy).sum())


@pytest.mark.parametrize("mask,kchunk", [(1, None), (2, None), (4, None), (8, None), (15, None), (15, 2), (5, 3)])
def test_gradients_through_the_logits_match_central_finite_differences(mask, kchunk):
    rng = np.random.default_rng(20 + mask + (kchunk or 0))
    x, z, lam, u = rand_logits_problem(rng, 1, 4, 4, 5, 2)
    gy = rng.standard_normal(x.shape)
    _, h = O.scan_fwd_logits(x, z, lam, u, mask, kchunk)
    gx, gz, glam, gu = O.scan_bwd_logits(gy, x, z, lam, u, h, mask, kchunk)
    eps = 1e-6
    for name, arr, grad in (("x", x, gx), ("z", z, gz), ("lam", lam, glam), ("u", u, gu)):
        flat = arr.reshape(-1)
        idx = rng.choice(flat.size, size=min(flat.size, 120), replace=False)
        for i in idx:
            old = flat[i]
            flat[i] = old + eps; lp = loss(x, z, lam, u, gy, mask, kchunk)
            flat[i] = old - eps; lm = loss(x, z, lam, u, gy, mask, kchunk)
            flat[i] = old
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - grad.reshape(-1)[i]) < 2e-7 * (1 + abs(fd)), (name, i, fd, grad.reshape(-1)[i])


def test_logit_gradients_sum_to_zero_over_the_taps_and_vanish_where_nothing_is_read():
    rng = np.random.default_rng(30)
    x, z, lam, u = rand_logits_problem(rng, 2, 4, 5, 6, 2)
    gy = rng.standard_normal(x.shape)
    _, h = O.scan_fwd_logits(x, z, lam, u)
    _, gz, _, _ = O.scan_bwd_logits(gy, x, z, lam, u, h)
    assert np.abs(gz.sum(axis=3)).max() < 1e-12                   # softmax: a common shift changes nothing
    assert not gz[0][:, :, 0, :, 0].any() and not gz[1][:, :, 2, :, -1].any()
    assert not gz[2][:, :, 0, 0, :].any() and not gz[3][:, :, 2, -1, :].any()
    assert not gz[0][:, :, :, 0, :].any() and not gz[1][:, :, :, -1, :].any()     # first line of each scan
    assert not gz[2][:, :, :, :, 0].any() and not gz[3][:, :, :, :, -1].any()
    assert gz[0][:, :, 1, 1:, 1:-1].all()
