"""Pins for the oracle's trainer variants: Adam against torch.optim (an independent library
implementation run in float64), the low-precision-parameter Adam, and SGD."""
import numpy as np
import pytest
import torch

import oracle
from workloads import decode, encode

f32 = lambda v: float(np.float32(v))


def _torch_run(opt_cls, p0, grads, **kw):
    p = torch.tensor(p0, dtype=torch.float64, requires_grad=True)
    opt = opt_cls([p], **kw)
    for g in grads:
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
    return p.detach().numpy()


@pytest.mark.parametrize("mode", ["adam", "adam_l2", "adamw"])
def test_adam_matches_torch_optim_in_float64(mode):
    n, steps = 257, 4
    r = np.random.default_rng(0)
    p0 = (r.standard_normal(n) * 0.02).astype(np.float32)
    grads = [decode(encode(r.standard_normal(n) * 1e-3, "f16"), "f16") for _ in range(steps)]
    lr, b1, b2, eps, wd = 1e-3, 0.9, 0.98, 1e-8, 0.0 if mode == "adam" else 0.01
    cls = torch.optim.AdamW if mode == "adamw" else torch.optim.Adam
    ref = _torch_run(cls, p0.astype(np.float64), grads, lr=f32(lr), betas=(f32(b1), f32(b2)), eps=f32(eps),
                     weight_decay=f32(wd))
    # the oracle takes float32 state in and gives float64 out; carry float64 between steps by hand
    p, m, v = p0.astype(np.float64), np.zeros(n), np.zeros(n)
    for t, g in enumerate(grads, 1):
        # state is fed back through float32, as the device keeps it; torch keeps float64, so compare loosely
        po, mo, vo = oracle.adam_step(p.astype(np.float32), m.astype(np.float32), v.astype(np.float32),
                                      encode(g, "f16"), "f16", lr, b1, b2, eps, t, weight_decay=wd,
                                      adamw=(mode == "adamw"))
        p, m, v = po, mo, vo
    assert np.allclose(p, ref, rtol=2e-6, atol=2e-9)     # float32 round trips of the state, 4 steps
    # a single step from float32-exact state agrees to float64 accuracy
    po, _, _ = oracle.adam_step(p0, np.zeros(n, np.float32), np.zeros(n, np.float32), encode(grads[0], "f16"), "f16",
                                lr, b1, b2, eps, 1, weight_decay=wd, adamw=(mode == "adamw"))
    ref1 = _torch_run(cls, p0.astype(np.float64), grads[:1], lr=f32(lr), betas=(f32(b1), f32(b2)), eps=f32(eps),
                      weight_decay=f32(wd))
    assert np.allclose(po, ref1, rtol=1e-12, atol=1e-15)


@pytest.mark.parametrize("dt", ["f16", "bf16"])
def test_adam_lp_is_adam_on_the_decoded_parameter(dt):
    n = 300
    r = np.random.default_rng(1)
    p_lp = encode(r.standard_normal(n) * 0.02, dt)
    g = encode(r.standard_normal(n) * 1e-3, dt)
    m = (r.standard_normal(n) * 1e-3).astype(np.float32)
    v = ((r.random(n) * 0.9 + 0.1) * 1e-6).astype(np.float32)
    hy = dict(lr=1e-3, beta1=0.9, beta2=0.98, eps=1e-8, step=3, weight_decay=0.01, adamw=True)
    a = oracle.adam_step_lp(p_lp, m, v, g, dt, **hy)
    b = oracle.adam_step(decode(p_lp, dt).astype(np.float32), m, v, g, dt, **hy)   # lp values are exact in float32
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
    # first step closed form on the low-precision parameter
    z = np.zeros(n, np.float32)
    po, _, _ = oracle.adam_step_lp(p_lp, z, z, g, dt, lr=1e-3, beta1=0.9, beta2=0.98, eps=1e-8, step=1)
    gd = decode(g, dt)
    assert np.allclose(po, decode(p_lp, dt) - f32(1e-3) * gd / (np.abs(gd) + f32(1e-8)), rtol=1e-12, atol=1e-18)


@pytest.mark.parametrize("kw", [dict(momentum=0.0), dict(momentum=0.9), dict(momentum=0.9, nesterov=True),
                                dict(momentum=0.5, weight_decay=0.01), dict(momentum=0.0, weight_decay=0.1)])
def test_sgd_matches_torch_optim_in_float64(kw):
    n, steps = 129, 5
    r = np.random.default_rng(2)
    p0 = (r.standard_normal(n) * 0.02).astype(np.float32)
    grads = [decode(encode(r.standard_normal(n) * 1e-2, "f16"), "f16") for _ in range(steps)]
    tkw = dict(lr=f32(0.1), momentum=f32(kw.get("momentum", 0.0)), weight_decay=f32(kw.get("weight_decay", 0.0)),
               nesterov=kw.get("nesterov", False))
    # one step from zero momentum: float64-exact agreement
    ref1 = _torch_run(torch.optim.SGD, p0.astype(np.float64), grads[:1], **tkw)
    po, bo = oracle.sgd_step(p0, np.zeros(n, np.float32), encode(grads[0], "f16"), "f16", 0.1, **kw)
    assert np.allclose(po, ref1, rtol=1e-13, atol=1e-16)
    # several steps (state round-trips through float32 between the oracle's steps)
    ref = _torch_run(torch.optim.SGD, p0.astype(np.float64), grads, **tkw)
    p, buf = p0.astype(np.float64), np.zeros(n)
    for g in grads:
        p, b = oracle.sgd_step(p.astype(np.float32), buf.astype(np.float32), encode(g, "f16"), "f16", 0.1, **kw)
        buf = b if b is not None else buf
    assert np.allclose(p, ref, rtol=2e-6, atol=2e-8)


def test_sgd_closed_forms():
    n = 16
    g = encode(np.full(n, 0.25), "f16")
    p = np.ones(n, np.float32)
    # plain: p - lr*g; grad scale; constant gradient with momentum: buf_t = g (1 - mu^t)/(1 - mu)
    po, bo = oracle.sgd_step(p, None, g, "f16", 0.5)
    assert bo is None and np.array_equal(po, np.full(n, 1 - 0.125))
    po, _ = oracle.sgd_step(p, None, g, "f16", 0.5, inv_grad_scale=0.5)
    assert np.array_equal(po, np.full(n, 1 - 0.0625))
    buf = np.zeros(n, np.float32)
    for t in range(1, 5):
        po, bo = oracle.sgd_step(p, buf, g, "f16", 0.0, momentum=0.5)
        assert np.allclose(bo, 0.25 * (1 - 0.5 ** t) / 0.5, rtol=1e-15)
        assert np.array_equal(po, p.astype(np.float64))      # lr = 0 leaves p alone
        buf = bo.astype(np.float32)
