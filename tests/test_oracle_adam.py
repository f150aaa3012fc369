"""Pins for the oracle's Adam step (Sec. IV-C; update rule = textbook Adam)."""
import numpy as np
import pytest

import oracle
from workloads import decode, encode

HY = dict(lr=1e-3, beta1=0.9, beta2=0.98, eps=1e-8)
f32 = lambda v: np.float64(np.float32(v))


def _state(n, seed, g_dt="f16"):
    r = np.random.default_rng(seed)
    p = (r.standard_normal(n) * 0.02).astype(np.float32)
    g = encode(r.standard_normal(n) * 1e-3, g_dt)
    return p, g


@pytest.mark.parametrize("g_dt", ["f16", "bf16", "f32"])
def test_first_step_closed_form(g_dt):
    # t = 1, m = v = 0  ->  p1 = p0 - lr * g / (|g| + eps)
    n = 1000
    p, g = _state(n, 0, g_dt)
    z = np.zeros(n, np.float32)
    po, mo, vo = oracle.adam_step(p, z, z, g, g_dt, step=1, **HY)
    gd = decode(g, g_dt)
    exp = p.astype(np.float64) - f32(HY["lr"]) * gd / (np.abs(gd) + f32(HY["eps"]))
    assert np.allclose(po, exp, rtol=1e-12, atol=1e-18)
    assert np.allclose(mo, (1 - f32(0.9)) * gd, rtol=1e-14)
    assert np.allclose(vo, (1 - f32(0.98)) * gd * gd, rtol=1e-14)


def test_zero_lr_zero_grad_and_zero_betas():
    n = 257
    p, g = _state(n, 1)
    r = np.random.default_rng(2)
    m = (r.standard_normal(n) * 1e-3).astype(np.float32)
    v = (r.random(n) * 1e-6).astype(np.float32)
    hy = dict(HY, lr=0.0)
    po, mo, vo = oracle.adam_step(p, m, v, g, "f16", step=3, **hy)
    assert np.array_equal(po, p.astype(np.float64))
    assert not np.array_equal(mo, m.astype(np.float64))
    # g = 0 -> pure decay of the moments
    g0 = encode(np.zeros(n), "f16")
    _, mo, vo = oracle.adam_step(p, m, v, g0, "f16", step=3, **HY)
    assert np.allclose(mo, f32(0.9) * m.astype(np.float64), rtol=1e-15)
    assert np.allclose(vo, f32(0.98) * v.astype(np.float64), rtol=1e-15)
    # beta1 = beta2 = 0 -> the t = 1 closed form at any step
    hy = dict(HY, beta1=0.0, beta2=0.0)
    po, _, _ = oracle.adam_step(p, m, v, g, "f16", step=17, **hy)
    gd = decode(g, "f16")
    assert np.allclose(po, p.astype(np.float64) - f32(1e-3) * gd / (np.abs(gd) + f32(1e-8)), rtol=1e-12)


def test_constant_gradient_geometric_closed_form():
    # feeding float64 outputs back as float32 state would round; use values that stay exact: beta = 0.5
    n, steps = 8, 6
    g = encode(np.full(n, 0.25), "f16")
    p = np.zeros(n, np.float32); m = np.zeros(n, np.float32); v = np.zeros(n, np.float32)
    hy = dict(lr=0.125, beta1=0.5, beta2=0.5, eps=0.0)
    pos = 0.0
    for t in range(1, steps + 1):
        po, mo, vo = oracle.adam_step(p, m, v, g, "f16", step=t, **hy)
        # m_t = g (1 - 0.5^t), v_t = g^2 (1 - 0.5^t): bias-corrected ratio is exactly 1 -> p moves by lr
        assert np.allclose(mo, 0.25 * (1 - 0.5 ** t), rtol=1e-15)
        assert np.allclose(vo, 0.0625 * (1 - 0.5 ** t), rtol=1e-15)
        pos -= 0.125
        assert np.allclose(po, pos, rtol=1e-14)
        p, m, v = po.astype(np.float32), mo.astype(np.float32), vo.astype(np.float32)


def test_flags_weight_decay_scale_and_bias_correction():
    n = 64
    p, g = _state(n, 3)
    r = np.random.default_rng(4)
    m = (r.standard_normal(n) * 1e-3).astype(np.float32)
    v = (r.random(n) * 1e-6).astype(np.float32)
    pd, md, vd, gd = (a.astype(np.float64) for a in (p, m, v, decode(g, "f16")))
    b1, b2, lr, eps, wd = f32(0.9), f32(0.98), f32(1e-3), f32(1e-8), f32(0.01)
    t = 5
    # L2 regularisation folded into the gradient, gradient un-scaling by 1/128
    po, mo, vo = oracle.adam_step(p, m, v, g, "f16", step=t, weight_decay=0.01, adamw=False,
                                  inv_grad_scale=1 / 128, **HY)
    gh = gd * f32(1 / 128) + wd * pd
    me = b1 * md + (1 - b1) * gh; ve = b2 * vd + (1 - b2) * gh * gh
    pe = pd - lr * (me / (1 - b1 ** t)) / (np.sqrt(ve / (1 - b2 ** t)) + eps)
    assert np.allclose(po, pe, rtol=1e-12) and np.allclose(mo, me, rtol=1e-13) and np.allclose(vo, ve, rtol=1e-13)
    # decoupled decay, no bias correction
    po, mo, vo = oracle.adam_step(p, m, v, g, "f16", step=t, weight_decay=0.01, adamw=True,
                                  bias_correction=False, **HY)
    me = b1 * md + (1 - b1) * gd; ve = b2 * vd + (1 - b2) * gd * gd
    pe = pd - lr * (me / (np.sqrt(ve) + eps) + wd * pd)
    assert np.allclose(po, pe, rtol=1e-12)


def test_split_invariance():
    n = 1001
    p, g = _state(n, 5)
    z = np.zeros(n, np.float32)
    full = oracle.adam_step(p, z, z, g, "f16", step=1, **HY)
    a = oracle.adam_step(p[:400], z[:400], z[:400], g[:400], "f16", step=1, **HY)
    b = oracle.adam_step(p[400:], z[400:], z[400:], g[400:], "f16", step=1, **HY)
    for f, x, y in zip(full, a, b):
        assert np.array_equal(f, np.concatenate([x, y]))
