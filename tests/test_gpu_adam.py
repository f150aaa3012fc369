"""GPU parity: fused mixed-precision Adam through the C-ABI against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2110_05722_amd as L
from tests._util import assert_close_f32, dev, say
from workloads import ADAM_HYPER as HY
from workloads import CONFIGS, adam_tensors, decode, device_normal, from_torch, to_torch

pytestmark = pytest.mark.gpu


def _check(p, m, v, rp, rm, rv, m_old, g64, b1=HY["beta1"], extra=0.0):
    """Master weights: 1e-6 relative (+1e-9: the update, of size lr, carries ~1e-10 of fp32 error even when
    |p| << lr).  Second moment: 1e-6 relative (a sum of positives).  First moment: beta1*m and (1-beta1)*g
    may cancel, so the fp32 rounding of the two TERMS (2^-23 of their magnitudes) is the floor, not the result's."""
    assert_close_f32(p, rp, "p", rel=1e-6, floor=1e-9)
    floor_m = 2.0 ** -23 * (b1 * np.abs(m_old.astype(np.float64)) + (1 - b1) * (np.abs(g64) + extra))
    assert_close_f32(m, rm, "m", rel=1e-6, floor=floor_m)
    assert_close_f32(v, rv, "v", rel=1e-6, floor=1e-30)


@pytest.mark.parametrize("g_dt,lp_dt", [("f16", "f16"), ("bf16", "bf16"), ("f32", "f16"), ("f16", None)])
# 4199427 = two full groups of XCD runs (2 x 2048 tiles of 1024 elements), five more tiles and a ragged end
@pytest.mark.parametrize("n", [1 << 20, 1000003, 8, 7, 1, 2049, 4199427])
def test_adam_four_steps(n, g_dt, lp_dt):
    """Config 1: state from zero moments, step 1 then three more, fresh gradient each step."""
    say(f"[adam] n={n} g={g_dt} p_lp={lp_dt}")
    d = dev()
    t = adam_tensors(CONFIGS[0], g_dt, n=n)
    p, m, v = (torch.from_numpy(t[k].copy()).to(d) for k in ("p", "m", "v"))
    hp, hm, hv = t["p"].copy(), t["m"].copy(), t["v"].copy()
    p_lp = None if lp_dt is None else torch.empty(n, dtype=torch.float16 if lp_dt == "f16" else torch.bfloat16, device=d)
    for step in range(1, 5):
        g_host = adam_tensors(CONFIGS[0], g_dt, n=n, stream=40 + step)["g"]
        g = to_torch(g_host, g_dt, d)
        L.lsq_adam_step(p, m, v, g, p_lp, step=step, **HY)
        rp, rm, rv = oracle.adam_step(hp, hm, hv, g_host, g_dt, step=step, **HY)
        _check(p, m, v, rp, rm, rv, hm, decode(g_host, g_dt))
        if p_lp is not None:
            # the low-precision copy is the round-to-nearest-even image of the fp32 parameter, bit for bit
            assert torch.equal(p_lp, p.to(p_lp.dtype))
        # carry the GPU's own fp32 state forward on both sides: each step is compared in isolation
        hp, hm, hv = p.cpu().numpy(), m.cpu().numpy(), v.cpu().numpy()


def test_adam_flags_and_split_invariance():
    say("[adam] weight decay / AdamW / no bias correction / grad scale; split invariance")
    d, n = dev(), 100003
    t = adam_tensors(CONFIGS[0], "f16", n=n)
    rng = np.random.default_rng(3)
    m0 = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    # second moments bounded away from zero, as (1-beta2)*g^2 history makes them: a vanishing v would
    # amplify the first moment's rounding floor through the division, which says nothing about the kernel
    v0 = ((rng.random(n) * 0.9 + 0.1) * 1e-6).astype(np.float32)
    g = to_torch(t["g"], "f16", d)
    for kw in (dict(weight_decay=0.01, adamw=False, inv_grad_scale=1 / 128),
               dict(weight_decay=0.01, adamw=True, bias_correction=False),
               dict(weight_decay=0.0, adamw=False, inv_grad_scale=0.5, bias_correction=True)):
        p, m, v = (torch.from_numpy(a.copy()).to(d) for a in (t["p"], m0, v0))
        L.lsq_adam_step(p, m, v, g, None, step=5, **HY, **kw)
        rp, rm, rv = oracle.adam_step(t["p"], m0, v0, t["g"], "f16", step=5, **HY, **kw)
        wd_term = 0.01 * np.abs(t["p"].astype(np.float64)) if not kw.get("adamw", False) else 0.0
        _check(p, m, v, rp, rm, rv, m0, decode(t["g"], "f16") * kw.get("inv_grad_scale", 1.0), extra=wd_term)
    # one call on n == two calls on the halves, bit for bit (cut on a pack boundary and off it)
    for cut in (40000, 40003):
        pa, ma, va = (torch.from_numpy(a.copy()).to(d) for a in (t["p"], m0, v0))
        L.lsq_adam_step(pa, ma, va, g, None, step=2, **HY)
        pb, mb, vb = (torch.from_numpy(a.copy()).to(d) for a in (t["p"], m0, v0))
        if cut % 8 == 0:
            L.lsq_adam_step(pb[:cut], mb[:cut], vb[:cut], g[:cut], None, step=2, **HY)
            L.lsq_adam_step(pb[cut:], mb[cut:], vb[cut:], g[cut:], None, step=2, **HY)
        else:   # an unaligned cut needs aligned base pointers: copy the second half out and back
            L.lsq_adam_step(pb[:cut], mb[:cut], vb[:cut], g[:cut], None, step=2, **HY)
            p2, m2, v2, g2 = (x[cut:].clone() for x in (pb, mb, vb, g))
            L.lsq_adam_step(p2, m2, v2, g2, None, step=2, **HY)
            pb[cut:], mb[cut:], vb[cut:] = p2, m2, v2
        assert torch.equal(pa, pb) and torch.equal(ma, mb) and torch.equal(va, vb)
    # lr = 0 leaves p untouched bit for bit; the moments still move
    p, m, v = (torch.from_numpy(a.copy()).to(d) for a in (t["p"], m0, v0))
    L.lsq_adam_step(p, m, v, g, None, step=3, **dict(HY, lr=0.0))
    assert torch.equal(p.cpu(), torch.from_numpy(t["p"])) and not torch.equal(m.cpu(), torch.from_numpy(m0))


@pytest.mark.parametrize("ci,dt", [(1, "f16"), (2, "f16"), (3, "bf16"), (4, "bf16"), (4, "f16")])
def test_adam_full_size(ci, dt):
    """Configs 2-5 at full workspace size in the launch the benchmark times; the oracle checks
    sampled chunks (elements are independent), and the copy property covers every element."""
    cfg = CONFIGS[ci]
    n = cfg.adam_n
    say(f"[adam] full size {cfg.name} n={n} dt={dt}")
    d = dev()
    p = device_normal((n,), 0.02, "f32", seed=cfg.seed, device=d)
    g = device_normal((n,), 1e-3, dt, seed=cfg.seed + 100, device=d)
    m = torch.zeros(n, dtype=torch.float32, device=d)
    v = torch.zeros(n, dtype=torch.float32, device=d)
    p_lp = torch.empty(n, dtype=g.dtype, device=d)
    rng = np.random.default_rng(cfg.seed)
    starts = np.unique(np.concatenate([[0, n - 4099], rng.integers(0, n - 4099, size=30)]))
    for step in (1, 2):
        before = [(s, p[s:s + 4099].cpu().numpy(), m[s:s + 4099].cpu().numpy(), v[s:s + 4099].cpu().numpy(),
                   from_torch(g[s:s + 4099], dt)) for s in starts]
        L.lsq_adam_step(p, m, v, g, p_lp, step=step, **HY)
        for s, hp, hm, hv, hg in before:
            rp, rm, rv = oracle.adam_step(hp, hm, hv, hg, dt, step=step, **HY)
            _check(p[s:s + 4099], m[s:s + 4099], v[s:s + 4099], rp, rm, rv, hm, decode(hg, dt))
        assert torch.equal(p_lp, p.to(p_lp.dtype))
        assert torch.isfinite(p).all() and (v >= 0).all()
