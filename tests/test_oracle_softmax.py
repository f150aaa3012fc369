"""Pins for the oracle's masked attention softmax (Sec. IV-B Softmax; Jacobian of Sec. IV-A)."""
import numpy as np
import pytest

import oracle
from workloads import decode, encode


def _rand(shape, seed, std=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * std


def _allowed(B, N, Lq, Lk, key_len, causal):
    j = np.arange(Lk)[None, None, None, :]
    i = np.arange(Lq)[None, None, :, None]
    kl = (np.full(B, Lk) if key_len is None else np.clip(key_len, 0, Lk))[:, None, None, None]
    a = j < kl
    if causal:
        a = a & (j <= i + (Lk - Lq))
    return np.broadcast_to(a, (B, N, Lq, Lk))


@pytest.mark.parametrize("dt", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("causal", [False, True])
def test_fwd_rows_sum_to_one_and_masked_are_exact_zero(dt, causal):
    B, N, Lq, Lk = 3, 2, 10, 10
    x = encode(_rand((B, N, Lq, Lk), 0, 2.0), dt)
    key_len = np.array([10, 4, 1], np.int32)
    y, _ = oracle.softmax_fwd(x, key_len, causal, 0.5, dt)
    a = _allowed(B, N, Lq, Lk, key_len, causal)
    assert np.allclose(y.sum(-1), 1.0, atol=1e-12)
    assert np.all(y[~a] == 0.0) and not np.signbit(y[~a]).any()
    assert np.all(y[a] > 0.0)
    # against scipy-free numpy log-sum-exp on the allowed set
    xs = 0.5 * decode(x, dt)
    xs = np.where(a, xs, -np.inf)
    ref = np.exp(xs - np.log(np.exp(xs - xs.max(-1, keepdims=True)).sum(-1, keepdims=True)) - xs.max(-1, keepdims=True))
    assert np.allclose(y, ref, rtol=1e-12, atol=1e-300)


def test_fwd_bruteforce_tiny():
    x = np.array([[[[0.5, -1.0, 2.0, 0.25]]]], np.float32)
    y, _ = oracle.softmax_fwd(x, None, False, 1.0, "f32")
    e = [np.exp(v) for v in (0.5, -1.0, 2.0, 0.25)]
    assert np.allclose(y[0, 0, 0], np.array(e) / sum(e), rtol=1e-14)
    y, _ = oracle.softmax_fwd(x, np.array([2], np.int32), False, 1.0, "f32")
    assert np.allclose(y[0, 0, 0], [e[0] / (e[0] + e[1]), e[1] / (e[0] + e[1]), 0, 0], rtol=1e-14)


def test_fwd_special_cases():
    B, N, L = 2, 2, 8
    x = _rand((B, N, L, L), 1).astype(np.float32)
    # shift invariance (shift by a value that keeps float32 inputs exact: a power of two on a coarse grid)
    xg = (np.round(x * 16) / 16).astype(np.float32)
    y0, _ = oracle.softmax_fwd(xg, None, False, 1.0, "f32")
    y1, _ = oracle.softmax_fwd(xg + np.float32(4.0), None, False, 1.0, "f32")
    assert np.allclose(y0, y1, rtol=1e-13)
    # all-equal row -> 1/|A|
    c = np.full((1, 1, 4, 8), 1.5, np.float32)
    y, _ = oracle.softmax_fwd(c, np.array([5], np.int32), False, 1.0, "f32")
    assert np.allclose(y[0, 0, :, :5], 0.2, rtol=1e-15) and np.all(y[0, 0, :, 5:] == 0)
    # causal: row 0 sees one key; |A| = 1 -> exactly 1
    y, _ = oracle.softmax_fwd(x, None, True, 1.0, "f32")
    assert np.all(y[:, :, 0, 0] == 1.0) and np.all(y[:, :, 0, 1:] == 0)
    # empty allowed set -> all-zero row, no NaN
    y, _ = oracle.softmax_fwd(x, np.array([0, 3], np.int32), False, 1.0, "f32")
    assert np.all(y[0] == 0) and np.isfinite(y).all()
    # scale argument == pre-scaled input
    ys, _ = oracle.softmax_fwd(xg, None, False, 0.25, "f32")
    yp, _ = oracle.softmax_fwd((xg * np.float32(0.25)).astype(np.float32), None, False, 1.0, "f32")
    assert np.allclose(ys, yp, rtol=1e-14)
    # monotone: argmax preserved
    assert np.array_equal(y0.argmax(-1), xg.argmax(-1))
    # causal with Lq != Lk is end-aligned: query i sees keys j <= i + (Lk - Lq)
    xr = _rand((1, 1, 3, 5), 2).astype(np.float32)
    y, _ = oracle.softmax_fwd(xr, None, True, 1.0, "f32")
    assert np.all(y[0, 0, 0, 3:] == 0) and y[0, 0, 0, 2] > 0 and np.all(y[0, 0, 2] > 0)


def test_fwd_dropout_output_is_mask_times_y():
    B, N, L, p = 2, 3, 8, 0.25
    x = _rand((B, N, L, L), 3).astype(np.float32)
    y, yd = oracle.softmax_fwd(x, None, True, 1.0, "f32", p=p, seed=11, offset=5)
    keep = oracle.dropout_mask(x.size, p, 11, 5).reshape(x.shape)
    assert np.allclose(yd, keep * y / (1 - np.float64(np.float32(p))), rtol=1e-15)
    # a slice of batches addresses the same global elements
    _, yd1 = oracle.softmax_fwd(x[1:], None, True, 1.0, "f32", p=p, seed=11, offset=5, e0=N * L * L)
    assert np.array_equal(yd1, yd[1:])


@pytest.mark.parametrize("p", [0.0, 0.25])
def test_bwd_matches_finite_differences_of_fwd(p):
    B, N, Lq, Lk = 1, 2, 4, 6
    x = (np.round(_rand((B, N, Lq, Lk), 4) * 32) / 32).astype(np.float32)
    c = (np.round(_rand((B, N, Lq, Lk), 5) * 32) / 32).astype(np.float32)
    key_len = np.array([5], np.int32)
    scale = 0.5
    y, yd = oracle.softmax_fwd(x, key_len, True, scale, "f32", p=p, seed=3, offset=1)
    # the backward takes the STORED y: here float64 y rounded to float32 storage
    dx = oracle.softmax_bwd(c, y.astype(np.float32), key_len, True, scale, "f32", p=p, seed=3, offset=1)

    def loss(xx):
        yy, yyd = oracle.softmax_fwd(xx, key_len, True, scale, "f32", p=p, seed=3, offset=1)
        return float((c.astype(np.float64) * (yyd if p > 0 else yy)).sum())

    h = 2.0 ** -9
    for idx in [(0, 0, 3, 1), (0, 1, 2, 0), (0, 0, 3, 4), (0, 1, 3, 5), (0, 0, 0, 3)]:
        xp, xm = x.copy(), x.copy()
        xp[idx] += h; xm[idx] -= h
        fd = (loss(xp) - loss(xm)) / (2 * h)
        assert fd == pytest.approx(dx[idx], rel=1e-4, abs=2e-7)


def test_bwd_invariants():
    B, N, L = 2, 2, 12
    x = _rand((B, N, L, L), 6).astype(np.float32)
    key_len = np.array([12, 7], np.int32)
    y, _ = oracle.softmax_fwd(x, key_len, True, 1.0, "f32")
    y32 = y.astype(np.float32)
    dy = _rand((B, N, L, L), 7).astype(np.float32)
    dx = oracle.softmax_bwd(dy, y32, key_len, True, 0.7, "f32")
    a = _allowed(B, N, L, L, key_len, True)
    assert np.allclose(dx.sum(-1), 0, atol=1e-7)   # y32 rows sum to 1 only to float32 rounding
    assert np.all(dx[~a] == 0)
    # constant upstream gradient -> zero (up to the rounding of the stored y)
    dxc = oracle.softmax_bwd(np.full_like(dy, 2.0), y32, key_len, True, 1.0, "f32")
    assert np.abs(dxc).max() < 1e-6
    # numpy statement of the contraction
    yd = y32.astype(np.float64); g = dy.astype(np.float64)
    ref = 0.7 * np.float64(np.float32(0.7)) / 0.7 * yd * (g - (g * yd).sum(-1, keepdims=True))
    assert np.allclose(dx, ref, rtol=1e-12, atol=1e-15)
