"""Pins for the oracle's LayerNorm forward and backward (Sec. IV-B).

Expected values come from the mathematics, never from the oracle's own loops:
row statistics of the output, exact special cases, brute force with numpy's own
mean/var on tiny rows, central finite differences of the forward, and the
paper's second (rearranged) statement of the gradient.
"""
import numpy as np
import pytest

import oracle
from workloads import decode, encode


def _rand(shape, seed, std=1.0, mean=0.0):
    return np.random.default_rng(seed).standard_normal(shape) * std + mean


@pytest.mark.parametrize("dt", ["f32", "f16", "bf16"])
def test_fwd_unit_affine_rows_are_standardised(dt):
    T, H, eps = 7, 96, 1e-5
    x = encode(_rand((T, H), 0, 2.0, 0.5), dt)
    y, mean, rstd = oracle.layernorm_fwd(x, encode(np.ones(H), dt), encode(np.zeros(H), dt), eps, dt)
    xd = decode(x, dt)
    var = xd.var(axis=1)  # numpy's biased variance
    assert np.allclose(y.mean(axis=1), 0, atol=1e-12)
    assert np.allclose(y.var(axis=1), var / (var + np.float32(eps)), rtol=1e-12)
    assert np.allclose(mean, xd.mean(axis=1), rtol=1e-13, atol=1e-15)
    assert np.allclose(rstd, 1 / np.sqrt(var + np.float64(np.float32(eps))), rtol=1e-13)


def test_fwd_bruteforce_tiny_rows():
    # H <= 8, every term written out with numpy primitives
    for H in (1, 2, 3, 8):
        x = _rand((5, H), H).astype(np.float32)
        g = _rand((H,), 10 + H, 0.1, 1.0).astype(np.float32)
        b = _rand((H,), 20 + H, 0.1).astype(np.float32)
        y, _, _ = oracle.layernorm_fwd(x, g, b, 1e-5, "f32")
        xd, gd, bd = x.astype(np.float64), g.astype(np.float64), b.astype(np.float64)
        exp = np.empty_like(xd)
        for r in range(5):
            mu = sum(xd[r]) / H
            var = sum((v - mu) ** 2 for v in xd[r]) / H
            for i in range(H):
                exp[r, i] = gd[i] * (xd[r, i] - mu) / np.sqrt(var + np.float64(np.float32(1e-5))) + bd[i]
        assert np.allclose(y, exp, rtol=1e-13, atol=1e-15)


def test_fwd_special_cases():
    H = 33
    g = _rand((H,), 1, 0.1, 1.0).astype(np.float32)
    b = _rand((H,), 2, 0.1).astype(np.float32)
    # constant row -> y == beta exactly (x - mean is exactly 0)
    x = np.full((2, H), 3.25, dtype=np.float32)
    y, _, _ = oracle.layernorm_fwd(x, g, b, 1e-5, "f32")
    assert np.array_equal(y, np.broadcast_to(b.astype(np.float64), (2, H)))
    # hidden == 1 -> y == beta
    y1, m1, _ = oracle.layernorm_fwd(np.array([[7.0]], np.float32), g[:1], b[:1], 1e-5, "f32")
    assert y1[0, 0] == np.float64(b[0]) and m1[0] == 7.0
    # affine: y(gamma, beta) = gamma * y(1, 0) + beta
    x = _rand((4, H), 3).astype(np.float32)
    y0, _, _ = oracle.layernorm_fwd(x, np.ones(H, np.float32), np.zeros(H, np.float32), 1e-5, "f32")
    y, _, _ = oracle.layernorm_fwd(x, g, b, 1e-5, "f32")
    assert np.allclose(y, g.astype(np.float64) * y0 + b.astype(np.float64), rtol=1e-14, atol=1e-15)
    # permutation equivariance along the hidden axis
    perm = np.random.default_rng(4).permutation(H)
    yp, _, _ = oracle.layernorm_fwd(np.ascontiguousarray(x[:, perm]), np.ascontiguousarray(g[perm]),
                                    np.ascontiguousarray(b[perm]), 1e-5, "f32")
    assert np.allclose(yp, y[:, perm], rtol=1e-12, atol=1e-14)


def test_fwd_one_pass_variance_identity():
    # the paper's sigma^2 = mu(x^2) - mu(x)^2 is the same number in exact arithmetic
    x = _rand((6, 512), 5).astype(np.float32)
    _, mean, rstd = oracle.layernorm_fwd(x, np.ones(512, np.float32), np.zeros(512, np.float32), 0.0, "f32")
    xd = x.astype(np.float64)
    one_pass = (xd ** 2).mean(axis=1) - xd.mean(axis=1) ** 2
    assert np.allclose(1 / rstd ** 2, one_pass, rtol=1e-10)


def _loss(x32, g32, b32, c, eps):
    y, _, _ = oracle.layernorm_fwd(x32, g32, b32, eps, "f32")
    return float((c * y).sum())


def test_bwd_matches_finite_differences_of_fwd():
    T, H, eps = 3, 12, 1e-5
    # inputs on a coarse binary grid so that +-h perturbations stay exactly representable in float32
    x = np.round(_rand((T, H), 6) * 64) / 64
    g = np.round(_rand((H,), 7, 0.1, 1.0) * 64) / 64
    b = np.round(_rand((H,), 8, 0.1) * 64) / 64
    c = _rand((T, H), 9)
    c32 = np.round(c * 64) / 64  # upstream gradient dy, exactly representable
    x32, g32, b32 = x.astype(np.float32), g.astype(np.float32), b.astype(np.float32)
    dx, dgamma, dbeta = oracle.layernorm_bwd(c32.astype(np.float32), x32, g32, eps, "f32")
    h = 2.0 ** -10
    for (r, i) in [(0, 0), (1, 5), (2, 11), (0, 7)]:
        xp, xm = x32.copy(), x32.copy()
        xp[r, i] += h; xm[r, i] -= h
        fd = (_loss(xp, g32, b32, c32, eps) - _loss(xm, g32, b32, c32, eps)) / (2 * h)
        assert fd == pytest.approx(dx[r, i], rel=2e-5, abs=1e-7)
    for i in (0, 3, 11):
        gp, gm = g32.copy(), g32.copy()
        gp[i] += h; gm[i] -= h
        fd = (_loss(x32, gp, b32, c32, eps) - _loss(x32, gm, b32, c32, eps)) / (2 * h)
        assert fd == pytest.approx(dgamma[i], rel=1e-8, abs=1e-9)   # linear in gamma: FD exact
        bp, bm = b32.copy(), b32.copy()
        bp[i] += h; bm[i] -= h
        fd = (_loss(x32, g32, bp, c32, eps) - _loss(x32, g32, bm, c32, eps)) / (2 * h)
        assert fd == pytest.approx(dbeta[i], rel=1e-8, abs=1e-9)


def test_bwd_row_invariants_and_special_cases():
    T, H = 5, 64
    x = _rand((T, H), 11).astype(np.float32)
    dy = _rand((T, H), 12).astype(np.float32)
    g = _rand((H,), 13, 0.1, 1.0).astype(np.float32)
    dx, dgamma, dbeta = oracle.layernorm_bwd(dy, x, g, 0.0, "f32")
    xd = x.astype(np.float64)
    xhat = (xd - xd.mean(1, keepdims=True)) / xd.std(1, keepdims=True)
    # with eps = 0 the gradient is orthogonal to 1 and to xhat in every row
    assert np.allclose(dx.sum(axis=1), 0, atol=1e-12)
    assert np.allclose((dx * xhat).sum(axis=1), 0, atol=1e-11)
    # column sums by numpy
    assert np.allclose(dgamma, (dy.astype(np.float64) * xhat).sum(0), rtol=1e-12, atol=1e-13)
    assert np.allclose(dbeta, dy.astype(np.float64).sum(0), rtol=1e-13, atol=1e-14)
    # gamma == 0 -> dx == 0
    dx0, _, _ = oracle.layernorm_bwd(dy, x, np.zeros(H, np.float32), 1e-5, "f32")
    assert np.array_equal(dx0, np.zeros((T, H)))
    # dres_in is added on top
    res = _rand((T, H), 14).astype(np.float32)
    dxr, _, _ = oracle.layernorm_bwd(dy, x, g, 0.0, "f32", dres_in=res)
    assert np.allclose(dxr, dx + res.astype(np.float64), rtol=1e-15, atol=1e-15)
    # a single row: dgamma = dy * xhat
    _, dg1, db1 = oracle.layernorm_bwd(dy[:1], x[:1], g, 0.0, "f32")
    assert np.allclose(dg1, dy[0].astype(np.float64) * xhat[0], rtol=1e-12, atol=1e-14)
    assert np.array_equal(db1, dy[0].astype(np.float64))


@pytest.mark.parametrize("dt", ["f32", "f16"])
def test_bwd_agrees_with_the_papers_rearranged_form(dt):
    T, H, eps = 6, 80, 1e-5
    x = encode(_rand((T, H), 21, 1.0, 0.3), dt)
    dy = encode(_rand((T, H), 22), dt)
    g = encode(_rand((H,), 23, 0.1, 1.0), dt)
    dx, _, _ = oracle.layernorm_bwd(dy, x, g, eps, dt)
    dx2 = oracle.layernorm_bwd_rearranged(dy, x, g, eps, dt)
    assert np.allclose(dx, dx2, rtol=1e-9, atol=1e-10)
