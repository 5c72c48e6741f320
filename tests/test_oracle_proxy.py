"""Pins for the oracle's compressive proxy projection (Sec. 4.2), CPU only: the einsum is held against the
definition written as loops, against matrices whose effect is known, and against composition."""
import numpy as np

from oracle import gspn_oracle as O


def test_projection_equals_the_sum_written_out():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((2, 5, 3, 4))
    P = rng.standard_normal((3, 5))
    got = O.proxy_project(x, P)
    ref = np.zeros((2, 3, 3, 4))
    for b in range(2):
        for m in range(3):
            for k in range(5):
                for h in range(3):
                    for w in range(4):
                        ref[b, m, h, w] += P[m, k] * x[b, k, h, w]
    assert np.allclose(got, ref, rtol=0, atol=1e-14)


def test_identity_selection_and_summing_matrices():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((2, 6, 4, 5))
    assert np.array_equal(O.proxy_project(x, np.eye(6)), x)
    sel = np.zeros((2, 6)); sel[0, 4] = 1.0; sel[1, 1] = -2.0
    out = O.proxy_project(x, sel)
    assert np.array_equal(out[:, 0], x[:, 4]) and np.array_equal(out[:, 1], -2.0 * x[:, 1])
    assert np.allclose(O.proxy_project(x, np.ones((1, 6)))[:, 0], x.sum(axis=1), rtol=0, atol=1e-14)


def test_two_projections_compose_like_their_matrix_product_and_the_wrapper_is_linear_in_x():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((1, 8, 3, 3))
    Pd = rng.standard_normal((2, 8)); Pu = rng.standard_normal((8, 2))
    assert np.allclose(O.proxy_project(O.proxy_project(x, Pd), Pu), O.proxy_project(x, Pu @ Pd), rtol=0, atol=1e-13)
    from test_oracle_forward import rand_problem
    _, w, lam, u = rand_problem(rng, 1, 2, 3, 3, 1)
    x2 = rng.standard_normal(x.shape)
    y = O.proxy_scan_fwd(x, Pd, w, lam, u, Pu)
    y2 = O.proxy_scan_fwd(x2, Pd, w, lam, u, Pu)
    y12 = O.proxy_scan_fwd(0.5 * x - 2.0 * x2, Pd, w, lam, u, Pu)
    assert np.allclose(y12, 0.5 * y - 2.0 * y2, rtol=0, atol=1e-12)
    # with identity projections the wrapper is the scan itself
    xs = rng.standard_normal((1, 2, 3, 3))
    assert np.array_equal(O.proxy_scan_fwd(xs, np.eye(2), w, lam, u, np.eye(2)), O.scan_fwd(xs, w, lam, u)[0])


def test_projection_gradients_equal_the_sums_written_out():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((2, 5, 3, 4)); P = rng.standard_normal((3, 5)); g = rng.standard_normal((2, 3, 3, 4))
    gin, gP = O.proxy_project_bwd(g, x, P)
    rin = np.zeros_like(x); rP = np.zeros_like(P)
    for b in range(2):
        for m in range(3):
            for k in range(5):
                for h in range(3):
                    for w in range(4):
                        rin[b, k, h, w] += P[m, k] * g[b, m, h, w]
                        rP[m, k] += g[b, m, h, w] * x[b, k, h, w]
    assert np.allclose(gin, rin, rtol=0, atol=1e-14) and np.allclose(gP, rP, rtol=0, atol=1e-13)


def test_projection_gradients_against_finite_differences_and_the_adjoint_identity():
    rng = np.random.default_rng(4)
    x = rng.standard_normal((2, 4, 2, 3)); P = rng.standard_normal((3, 4)); g = rng.standard_normal((2, 3, 2, 3))
    gin, gP = O.proxy_project_bwd(g, x, P)
    loss = lambda xx, PP: float(np.sum(g * O.proxy_project(xx, PP)))
    eps = 1e-6
    for idx in [(0, 0, 0, 0), (1, 3, 1, 2), (0, 2, 1, 1)]:
        d = np.zeros_like(x); d[idx] = eps
        assert abs((loss(x + d, P) - loss(x - d, P)) / (2 * eps) - gin[idx]) < 1e-8
    for idx in [(0, 0), (2, 3), (1, 2)]:
        d = np.zeros_like(P); d[idx] = eps
        assert abs((loss(x, P + d) - loss(x, P - d)) / (2 * eps) - gP[idx]) < 1e-8
    # <g, P x> = <P^T g, x> and = <gP, P>: the loss is bilinear
    assert np.isclose(np.sum(g * O.proxy_project(x, P)), np.sum(gin * x), rtol=1e-13)
    assert np.isclose(np.sum(g * O.proxy_project(x, P)), np.sum(gP * P), rtol=1e-13)
    # the input gradient is the projection with the transposed matrix
    assert np.allclose(gin, O.proxy_project(g, P.T), rtol=0, atol=1e-14)


def test_projection_gradient_of_a_selection_matrix():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((1, 6, 2, 2)); g = rng.standard_normal((1, 2, 2, 2))
    sel = np.zeros((2, 6)); sel[0, 4] = 1.0; sel[1, 1] = -2.0
    gin, gP = O.proxy_project_bwd(g, x, sel)
    assert np.array_equal(gin[:, 4], g[:, 0]) and np.array_equal(gin[:, 1], -2.0 * g[:, 1])
    assert not gin[:, [0, 2, 3, 5]].any()
    assert np.isclose(gP[0, 4], np.sum(g[:, 0] * x[:, 4])) and np.isclose(gP[1, 0], np.sum(g[:, 1] * x[:, 0]))


def test_gradients_through_the_wrapped_scan_against_finite_differences():
    from test_oracle_forward import rand_problem
    rng = np.random.default_rng(6)
    B, C, Cp, H, W = 1, 5, 2, 3, 4
    x = rng.standard_normal((B, C, H, W))
    Pd = rng.standard_normal((Cp, C)); Pu = rng.standard_normal((C, Cp))
    _, w, lam, u = rand_problem(rng, B, Cp, H, W, 1)
    gy = rng.standard_normal((B, C, H, W))
    gx, gPd, gw, glam, gu, gPu = O.proxy_scan_bwd(gy, x, Pd, w, lam, u, Pu)
    loss = lambda **kw: float(np.sum(gy * O.proxy_scan_fwd(kw.get("x", x), kw.get("Pd", Pd), kw.get("w", w), kw.get("lam", lam),
                                                           kw.get("u", u), kw.get("Pu", Pu))))
    eps = 1e-6
    for name, base, grad in (("x", x, gx), ("Pd", Pd, gPd), ("Pu", Pu, gPu), ("lam", lam, glam), ("u", u, gu)):
        for _ in range(4):
            idx = tuple(int(rng.integers(n)) for n in base.shape)
            d = np.zeros_like(base); d[idx] = eps
            fd = (loss(**{name: base + d}) - loss(**{name: base - d})) / (2 * eps)
            assert abs(fd - grad[idx]) < 1e-7 * max(1.0, abs(fd)), (name, idx, fd, grad[idx])
