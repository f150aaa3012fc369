"""Pins for the oracle's bias + activation + dropout (the FFN half of Sec. IV-A's fused element-wise ops)."""
import math

import numpy as np
import pytest
from scipy import special, stats

import oracle
from workloads import decode, encode


def _rand(shape, seed, std=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * std


@pytest.mark.parametrize("dt", ["f32", "f16", "bf16"])
def test_fwd_p_zero_closed_forms(dt):
    T, H = 6, 40
    x, b = encode(_rand((T, H), 0, 2.0), dt), encode(_rand((H,), 1, 0.5), dt)
    z = decode(x, dt) + decode(b, dt)
    relu = oracle.bias_act_dropout_fwd(x, b, "relu", 0.0, 1, 0, dt)
    assert np.array_equal(relu, np.maximum(z, 0.0))
    # GELU(z) = z * Phi(z): scipy's normal CDF is an independent statement of the erf form
    gelu = oracle.bias_act_dropout_fwd(x, b, "gelu", 0.0, 1, 0, dt)
    assert np.allclose(gelu, z * stats.norm.cdf(z), rtol=1e-13, atol=1e-300)
    gt = oracle.bias_act_dropout_fwd(x, b, "gelu_tanh", 0.0, 1, 0, dt)
    ref = 0.5 * z * (1 + np.tanh(math.sqrt(2 / math.pi) * (z + 0.044715 * z ** 3)))
    # 1 + tanh(u) cancels in the negative tail: both sides carry ~1e-16*|z| of absolute error there
    assert np.allclose(gt, ref, rtol=1e-12, atol=1e-15)
    # the two GELUs differ by less than 1e-3 everywhere (the approximation's known error bound)
    assert np.abs(gt - gelu).max() < 1e-3
    # no bias
    nb = oracle.bias_act_dropout_fwd(x, None, "relu", 0.0, 1, 0, dt)
    assert np.array_equal(nb, np.maximum(decode(x, dt), 0.0))


def test_fwd_dropout_is_the_pinned_mask_times_activation():
    T, H, p, seed, off = 8, 24, 0.3, 5, 2
    x, b = _rand((T, H), 2).astype(np.float32), _rand((H,), 3).astype(np.float32)
    out = oracle.bias_act_dropout_fwd(x, b, "gelu", p, seed, off, "f32")
    keep = oracle.dropout_mask(T * H, p, seed, off).reshape(T, H)
    z = x.astype(np.float64) + b.astype(np.float64)
    ref = keep * (0.5 * z * (1 + special.erf(z / math.sqrt(2)))) / (1 - np.float64(np.float32(p)))
    assert np.allclose(out, ref, rtol=1e-13, atol=0)
    part = oracle.bias_act_dropout_fwd(x[2:5], b, "gelu", p, seed, off, "f32", e0=2 * H)
    assert np.array_equal(part, out[2:5])


@pytest.mark.parametrize("act", ["relu", "gelu", "gelu_tanh"])
def test_bwd_matches_finite_differences_of_fwd(act):
    T, H, p, seed, off = 5, 16, 0.25, 9, 1
    x = (np.round(_rand((T, H), 4, 1.5) * 32) / 32 + 1 / 64).astype(np.float32)   # never exactly at ReLU's kink
    b = (np.round(_rand((H,), 5, 0.5) * 32) / 32).astype(np.float32)
    c = (np.round(_rand((T, H), 6) * 32) / 32).astype(np.float32)
    dx, dbias = oracle.bias_act_dropout_bwd(c, x, b, act, p, seed, off, "f32")

    def loss(xx, bb):
        return float((c.astype(np.float64) * oracle.bias_act_dropout_fwd(xx, bb, act, p, seed, off, "f32")).sum())

    h = 2.0 ** -13      # central differences: truncation error ~h^2 |f'''|/6, summed over rows for dbias
    for (t, i) in [(0, 0), (1, 7), (4, 15), (2, 3), (3, 9)]:
        xp, xm = x.copy(), x.copy()
        xp[t, i] += h; xm[t, i] -= h
        assert (loss(xp, b) - loss(xm, b)) / (2 * h) == pytest.approx(dx[t, i], rel=1e-5, abs=1e-8)
    for i in (0, 6, 15):
        bp, bm = b.copy(), b.copy()
        bp[i] += h; bm[i] -= h
        assert (loss(x, bp) - loss(x, bm)) / (2 * h) == pytest.approx(dbias[i], rel=1e-5, abs=1e-8)
    assert np.allclose(dbias, dx.sum(0), rtol=1e-14, atol=1e-15)


def test_bwd_special_cases():
    T, H = 4, 16
    x = _rand((T, H), 7).astype(np.float32)
    dy = _rand((T, H), 8).astype(np.float32)
    dx, _ = oracle.bias_act_dropout_bwd(dy, x, None, "relu", 0.0, 1, 0, "f32")
    assert np.array_equal(dx, np.where(x > 0, dy.astype(np.float64), 0.0))
    # GELU slope: Phi(z) + z*phi(z)
    dxg, _ = oracle.bias_act_dropout_bwd(dy, x, None, "gelu", 0.0, 1, 0, "f32")
    z = x.astype(np.float64)
    assert np.allclose(dxg, dy * (stats.norm.cdf(z) + z * stats.norm.pdf(z)), rtol=1e-12)
    # slope at 0: ReLU 0 (left derivative), GELU 1/2
    z0 = np.zeros((1, 8), np.float32)
    one = np.ones((1, 8), np.float32)
    assert np.all(oracle.bias_act_dropout_bwd(one, z0, None, "relu", 0.0, 1, 0, "f32")[0] == 0)
    assert np.allclose(oracle.bias_act_dropout_bwd(one, z0, None, "gelu", 0.0, 1, 0, "f32")[0], 0.5)
    assert np.allclose(oracle.bias_act_dropout_bwd(one, z0, None, "gelu_tanh", 0.0, 1, 0, "f32")[0], 0.5)
