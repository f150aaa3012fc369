"""Pins for the oracle's bias + dropout + residual (Sec. IV-A, Transformer layers)."""
import numpy as np
import pytest

import oracle
from workloads import decode, encode


def _rand(shape, seed, std=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * std


@pytest.mark.parametrize("dt", ["f32", "f16", "bf16"])
def test_fwd_p_zero_is_a_plain_sum(dt):
    T, H = 5, 40
    x, b, r = encode(_rand((T, H), 0), dt), encode(_rand((H,), 1, 0.1), dt), encode(_rand((T, H), 2), dt)
    out = oracle.bias_dropout_residual_fwd(x, b, r, 0.0, 1, 0, dt)
    assert np.array_equal(out, decode(x, dt) + decode(b, dt) + decode(r, dt))
    out_nb = oracle.bias_dropout_residual_fwd(x, None, r, 0.0, 1, 0, dt)
    assert np.array_equal(out_nb, decode(x, dt) + decode(r, dt))


def test_fwd_is_mask_times_scaled_sum_plus_residual():
    # assembled from the separately pinned mask
    T, H, p, seed, off = 9, 24, 0.3, 77, 4
    x, b, r = _rand((T, H), 3).astype(np.float32), _rand((H,), 4).astype(np.float32), _rand((T, H), 5).astype(np.float32)
    out = oracle.bias_dropout_residual_fwd(x, b, r, p, seed, off, "f32")
    keep = oracle.dropout_mask(T * H, p, seed, off).reshape(T, H).astype(np.float64)
    scale = 1.0 / (1.0 - np.float64(np.float32(p)))
    exp = r.astype(np.float64) + keep * (x.astype(np.float64) + b.astype(np.float64)) * scale
    assert np.allclose(out, exp, rtol=1e-15, atol=0)
    # dropped positions pass the residual through untouched
    assert np.array_equal(out[keep == 0], r.astype(np.float64)[keep == 0])
    assert 0 < (keep == 0).sum() < T * H


def test_row_slices_use_the_global_element_index():
    T, H, p = 16, 24, 0.5
    x, r = _rand((T, H), 6).astype(np.float32), _rand((T, H), 7).astype(np.float32)
    full = oracle.bias_dropout_residual_fwd(x, None, r, p, 5, 0, "f32")
    part = oracle.bias_dropout_residual_fwd(x[3:9], None, r[3:9], p, 5, 0, "f32", e0=3 * H)
    assert np.array_equal(full[3:9], part)


def test_bwd_is_the_frozen_mask_derivative_of_fwd():
    T, H, p, seed, off = 6, 16, 0.25, 9, 2
    x = (np.round(_rand((T, H), 8) * 32) / 32).astype(np.float32)
    b = (np.round(_rand((H,), 9) * 32) / 32).astype(np.float32)
    r = (np.round(_rand((T, H), 10) * 32) / 32).astype(np.float32)
    c = (np.round(_rand((T, H), 11) * 32) / 32).astype(np.float32)  # upstream dy
    dx, dbias = oracle.bias_dropout_residual_bwd(c, p, seed, off, "f32")

    def loss(xx, bb):
        return float((c.astype(np.float64) * oracle.bias_dropout_residual_fwd(xx, bb, r, p, seed, off, "f32")).sum())

    h = 2.0 ** -6
    for (t, i) in [(0, 0), (2, 7), (5, 15), (3, 3)]:
        xp, xm = x.copy(), x.copy()
        xp[t, i] += h; xm[t, i] -= h
        assert (loss(xp, b) - loss(xm, b)) / (2 * h) == pytest.approx(dx[t, i], rel=1e-10, abs=1e-12)
    for i in (0, 5, 15):
        bp, bm = b.copy(), b.copy()
        bp[i] += h; bm[i] -= h
        assert (loss(x, bp) - loss(x, bm)) / (2 * h) == pytest.approx(dbias[i], rel=1e-10, abs=1e-12)


def test_bwd_special_cases():
    T, H = 7, 24
    dy = _rand((T, H), 12).astype(np.float32)
    dx, dbias = oracle.bias_dropout_residual_bwd(dy, 0.0, 1, 0, "f32")
    assert np.array_equal(dx, dy.astype(np.float64))
    assert np.allclose(dbias, dy.astype(np.float64).sum(0), rtol=1e-14, atol=1e-15)
    dx, dbias = oracle.bias_dropout_residual_bwd(dy, 0.4, 3, 1, "f32")
    keep = oracle.dropout_mask(T * H, 0.4, 3, 1).reshape(T, H)
    assert np.array_equal(dx == 0, keep == 0)      # dy has no exact zeros
    assert np.allclose(dbias, dx.sum(0), rtol=1e-14, atol=1e-15)
