"""GPU parity: the trainer variants (low-precision-parameter Adam, SGD) through the C-ABI against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2110_05722_amd as L
from tests._util import LP_TOL, assert_close_f32, assert_close_store, dev, say
from workloads import ADAM_HYPER as HY
from workloads import CONFIGS, adam_tensors, decode, device_normal, encode, from_torch, to_torch

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dt", ["f16", "bf16"])
@pytest.mark.parametrize("n", [1 << 20, 1000003, 5, 2049, 4199427])
def test_adam_lp_three_steps(n, dt):
    say(f"[adam_lp] n={n} dt={dt}")
    d = dev()
    t = adam_tensors(CONFIGS[0], dt, n=n)
    p_host = encode(t["p"], dt)
    p = to_torch(p_host, dt, d)
    m = torch.zeros(n, dtype=torch.float32, device=d)
    v = torch.zeros(n, dtype=torch.float32, device=d)
    hm, hv = np.zeros(n, np.float32), np.zeros(n, np.float32)
    for step in range(1, 4):
        g_host = adam_tensors(CONFIGS[0], dt, n=n, stream=60 + step)["g"]
        L.lsq_adam_step_lp(p, m, v, to_torch(g_host, dt, d), step=step, **HY)
        rp, rm, rv = oracle.adam_step_lp(p_host, hm, hv, g_host, dt, step=step, **HY)
        # the parameter is stored in low precision: one ulp of the storage type (the paper's trade-off)
        assert_close_store(p, rp, dt, "p_lp")
        a, r = LP_TOL[dt]
        assert np.abs(decode(from_torch(p, dt), dt) - rp).max() <= r * np.abs(rp).max() + 1e-12
        floor_m = 2.0 ** -23 * (HY["beta1"] * np.abs(hm.astype(np.float64)) + (1 - HY["beta1"]) * np.abs(decode(g_host, dt)))
        assert_close_f32(m, rm, "m", rel=1e-6, floor=floor_m)
        assert_close_f32(v, rv, "v", rel=1e-6, floor=1e-30)
        p_host, hm, hv = from_torch(p, dt), m.cpu().numpy(), v.cpu().numpy()


@pytest.mark.parametrize("kw", [dict(momentum=0.0), dict(momentum=0.9), dict(momentum=0.9, nesterov=True),
                                dict(momentum=0.5, weight_decay=0.01, inv_grad_scale=0.25)])
@pytest.mark.parametrize("g_dt,lp_dt", [("f16", "f16"), ("bf16", "bf16"), ("f32", None)])
@pytest.mark.parametrize("n", [1 << 20, 1000003, 3, 4199427])
def test_sgd_three_steps(n, g_dt, lp_dt, kw):
    say(f"[sgd] n={n} g={g_dt} p_lp={lp_dt} {kw}")
    d = dev()
    t = adam_tensors(CONFIGS[0], g_dt, n=n)
    p = torch.from_numpy(t["p"].copy()).to(d)
    mom = kw.get("momentum", 0.0)
    buf = torch.zeros(n, dtype=torch.float32, device=d) if mom else None
    p_lp = None if lp_dt is None else torch.empty(n, dtype=torch.float16 if lp_dt == "f16" else torch.bfloat16, device=d)
    hp, hb = t["p"].copy(), np.zeros(n, np.float32)
    for step in range(3):
        g_host = adam_tensors(CONFIGS[0], g_dt, n=n, stream=70 + step)["g"]
        L.lsq_sgd_step(p, buf, to_torch(g_host, g_dt, d), p_lp, lr=0.1, **kw)
        rp, rb = oracle.sgd_step(hp, hb, g_host, g_dt, 0.1, **kw)
        assert_close_f32(p, rp, "p", rel=1e-6, floor=1e-9)
        if mom:
            # buf = momentum*buf + g': the two terms can cancel; floor = fp32 rounding of the terms
            gd = np.abs(decode(g_host, g_dt)) * kw.get("inv_grad_scale", 1.0) + kw.get("weight_decay", 0.0) * np.abs(hp)
            assert_close_f32(buf, rb, "buf", rel=1e-6, floor=2.0 ** -23 * (mom * np.abs(hb.astype(np.float64)) + gd))
            hb = buf.cpu().numpy()
        if p_lp is not None:
            assert torch.equal(p_lp, p.to(p_lp.dtype))
        hp = p.cpu().numpy()


def test_trainers_full_size_transformer_big():
    """Config 3's 210 M-parameter workspace through both variants, sampled chunks against the oracle."""
    cfg, dt, d = CONFIGS[2], "f16", dev()
    n = cfg.adam_n
    say(f"[adam_lp / sgd] full size n={n}")
    p = device_normal((n,), 0.02, "f32", seed=11, device=d)
    g = device_normal((n,), 1e-3, dt, seed=12, device=d)
    rng = np.random.default_rng(5)
    starts = np.unique(np.concatenate([[0, n - 4099], rng.integers(0, n - 4099, size=20)]))
    # SGD with momentum
    buf = torch.zeros(n, dtype=torch.float32, device=d)
    p_lp = torch.empty(n, dtype=torch.float16, device=d)
    before = [(s, p[s:s + 4099].cpu().numpy(), from_torch(g[s:s + 4099], dt)) for s in starts]
    L.lsq_sgd_step(p, buf, g, p_lp, lr=0.1, momentum=0.9)
    for s, hp, hg in before:
        rp, rb = oracle.sgd_step(hp, np.zeros(4099, np.float32), hg, dt, 0.1, momentum=0.9)
        assert_close_f32(p[s:s + 4099], rp, "p", rel=1e-6, floor=1e-9)
        assert_close_f32(buf[s:s + 4099], rb, "buf", rel=1e-6, floor=1e-12)
    assert torch.equal(p_lp, p.to(torch.float16))
    # low-precision-parameter Adam
    q = p.to(torch.float16)
    m = torch.zeros(n, dtype=torch.float32, device=d)
    v = torch.zeros(n, dtype=torch.float32, device=d)
    before = [(s, from_torch(q[s:s + 4099], dt), from_torch(g[s:s + 4099], dt)) for s in starts]
    L.lsq_adam_step_lp(q, m, v, g, step=1, **HY)
    z = np.zeros(4099, np.float32)
    for s, hq, hg in before:
        rq, rm, rv = oracle.adam_step_lp(hq, z, z, hg, dt, step=1, **HY)
        assert_close_store(q[s:s + 4099], rq, dt, "p_lp")
        assert_close_f32(v[s:s + 4099], rv, "v", rel=1e-6, floor=1e-30)
    assert torch.isfinite(q).all()
