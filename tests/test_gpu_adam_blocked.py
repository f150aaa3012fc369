"""GPU parity: Adam on the blocked optimizer state through the C-ABI.

The layout is pinned by numpy (state viewed as [blocks, 3, 8192]); the step is compared with the CPU
oracle at the Adam tolerances and must equal lsq_adam_step on the same inputs bit for bit (same
arithmetic, other addresses).
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2110_05722_amd as L
from tests._util import dev, say
from tests.test_gpu_adam import _check
from workloads import ADAM_HYPER as HY
from workloads import CONFIGS, adam_tensors, decode, to_torch

pytestmark = pytest.mark.gpu
BLK = L.binding.LSQ_ADAM_BLOCK

SIZES = [1, 7, 8, 2049, BLK - 1, BLK, BLK + 1, 3 * BLK, 1000003, 1 << 20]


def _blocked_view(state, n):
    nb = -(-n // BLK)
    assert state.numel() == nb * 3 * BLK == L.lsq_adam_state_bytes(n) // 4
    return state.cpu().numpy().reshape(nb, 3, BLK)


@pytest.mark.parametrize("n", SIZES)
def test_pack_layout_and_round_trip(n):
    say(f"[adam-blocked] layout n={n}")
    d = dev()
    r = np.random.default_rng(n)
    p, m, v = (r.standard_normal(n).astype(np.float32) for _ in range(3))
    state = L.lsq_adam_state_pack(*(torch.from_numpy(a).to(d) for a in (p, m, v)))
    s = _blocked_view(state, n)
    pad = s.shape[0] * BLK - n
    for k, a in enumerate((p, m, v)):
        assert np.array_equal(s[:, k, :].reshape(-1), np.concatenate([a, np.zeros(pad, np.float32)]))
    p2, m2, v2 = L.lsq_adam_state_unpack(state, n)
    assert np.array_equal(p2.cpu().numpy(), p) and np.array_equal(m2.cpu().numpy(), m) and np.array_equal(v2.cpu().numpy(), v)
    # a fresh optimizer: moments absent -> zeros; partial unpack leaves the rest alone
    fresh = _blocked_view(L.lsq_adam_state_pack(torch.from_numpy(p).to(d)), n)
    assert not fresh[:, 1:, :].any() and np.array_equal(fresh[:, 0, :].reshape(-1)[:n], p)
    only_p, none_m, none_v = L.lsq_adam_state_unpack(state, n, want=("p",))
    assert none_m is None and none_v is None and np.array_equal(only_p.cpu().numpy(), p)


@pytest.mark.parametrize("g_dt,lp_dt", [("f16", "f16"), ("bf16", "bf16"), ("f32", "f16"), ("f16", None)])
@pytest.mark.parametrize("n", SIZES)
def test_blocked_steps_match_oracle_and_flat_entry_point(n, g_dt, lp_dt):
    say(f"[adam-blocked] n={n} g={g_dt} p_lp={lp_dt}")
    d = dev()
    t = adam_tensors(CONFIGS[0], g_dt, n=n)
    p, m, v = (torch.from_numpy(t[k].copy()).to(d) for k in ("p", "m", "v"))
    state = L.lsq_adam_state_pack(p, m, v)
    hp, hm, hv = t["p"].copy(), t["m"].copy(), t["v"].copy()
    lpt = None if lp_dt is None else (torch.float16 if lp_dt == "f16" else torch.bfloat16)
    p_lp = None if lpt is None else torch.empty(n, dtype=lpt, device=d)
    q_lp = None if lpt is None else torch.empty(n, dtype=lpt, device=d)
    for step in range(1, 4):
        g_host = adam_tensors(CONFIGS[0], g_dt, n=n, stream=60 + step)["g"]
        g = to_torch(g_host, g_dt, d)
        L.lsq_adam_step_blocked(state, g, p_lp, step=step, **HY)
        L.lsq_adam_step(p, m, v, g, q_lp, step=step, **HY)
        bp, bm, bv = L.lsq_adam_state_unpack(state, n)
        assert torch.equal(bp, p) and torch.equal(bm, m) and torch.equal(bv, v)
        if p_lp is not None:
            assert torch.equal(p_lp, q_lp) and torch.equal(p_lp, bp.to(lpt))
        rp, rm, rv = oracle.adam_step(hp, hm, hv, g_host, g_dt, step=step, **HY)
        _check(bp, bm, bv, rp, rm, rv, hm, decode(g_host, g_dt))
        hp, hm, hv = bp.cpu().numpy(), bm.cpu().numpy(), bv.cpu().numpy()
    # the padding of the last block is never touched by a step
    s = _blocked_view(state, n)
    pad = s.shape[0] * BLK - n
    if pad:
        assert not s.reshape(-1, 3, BLK)[-1, :, BLK - pad:].any()


def test_blocked_flags():
    say("[adam-blocked] weight decay / AdamW / no bias correction / grad scale")
    d, n = dev(), 100003
    t = adam_tensors(CONFIGS[0], "f16", n=n)
    rng = np.random.default_rng(3)
    m0 = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    v0 = ((rng.random(n) * 0.9 + 0.1) * 1e-6).astype(np.float32)
    g = to_torch(t["g"], "f16", d)
    for kw in (dict(weight_decay=0.01, adamw=False, inv_grad_scale=1 / 128),
               dict(weight_decay=0.01, adamw=True, bias_correction=False)):
        state = L.lsq_adam_state_pack(*(torch.from_numpy(a.copy()).to(d) for a in (t["p"], m0, v0)))
        L.lsq_adam_step_blocked(state, g, None, step=5, **HY, **kw)
        p, m, v = L.lsq_adam_state_unpack(state, n)
        rp, rm, rv = oracle.adam_step(t["p"], m0, v0, t["g"], "f16", step=5, **HY, **kw)
        wd_term = 0.01 * np.abs(t["p"].astype(np.float64)) if not kw.get("adamw", False) else 0.0
        _check(p, m, v, rp, rm, rv, m0, decode(t["g"], "f16") * kw.get("inv_grad_scale", 1.0), extra=wd_term)


@pytest.mark.parametrize("ci,dt", [(2, "f16"), (4, "f16"), (4, "bf16")])
def test_blocked_full_size(ci, dt):
    """Transformer-big and GPT-2-large workspaces at full size, the launch the benchmark times: the
    oracle checks sampled chunks, and every element must equal lsq_adam_step's result bit for bit."""
    from workloads import device_normal, from_torch
    cfg = CONFIGS[ci]
    n = cfg.adam_n
    say(f"[adam-blocked] full size {cfg.name} n={n} dt={dt}")
    d = dev()
    p = device_normal((n,), 0.02, "f32", seed=cfg.seed, device=d)
    g = device_normal((n,), 1e-3, dt, seed=cfg.seed + 100, device=d)
    m = torch.zeros(n, dtype=torch.float32, device=d)
    v = torch.zeros(n, dtype=torch.float32, device=d)
    state = L.lsq_adam_state_pack(p)
    p_lp = torch.empty(n, dtype=g.dtype, device=d)
    q_lp = torch.empty(n, dtype=g.dtype, device=d)
    rng = np.random.default_rng(cfg.seed)
    starts = np.unique(np.concatenate([[0, n - 4099], rng.integers(0, n - 4099, size=20)]))
    out = torch.empty(n, dtype=torch.float32, device=d)
    for step in (1, 2):
        before = [(s, p[s:s + 4099].cpu().numpy(), m[s:s + 4099].cpu().numpy(), v[s:s + 4099].cpu().numpy(),
                   from_torch(g[s:s + 4099], dt)) for s in starts]
        L.lsq_adam_step_blocked(state, g, p_lp, step=step, **HY)
        L.lsq_adam_step(p, m, v, g, q_lp, step=step, **HY)
        assert torch.equal(p_lp, q_lp)
        for k, ref in enumerate((p, m, v)):
            L.lsq_adam_state_unpack(state, n, **{"pmv"[k]: out}, want=())
            assert torch.equal(out, ref), "pmv"[k]
        for s, hp, hm, hv, hg in before:
            rp, rm, rv = oracle.adam_step(hp, hm, hv, hg, dt, step=step, **HY)
            _check(p[s:s + 4099], m[s:s + 4099], v[s:s + 4099], rp, rm, rv, hm, decode(hg, dt))


# ---- the general blocked trainer state: SGD ([p | buf]) and the low-precision-parameter Adam ([m | v])
@pytest.mark.parametrize("arrays", [1, 2, 3])
@pytest.mark.parametrize("n", [1, 9, BLK - 3, BLK, 2 * BLK + 5])
def test_trainer_state_layout(n, arrays):
    say(f"[trainer-state] n={n} arrays={arrays}")
    d = dev()
    r = np.random.default_rng(n + arrays)
    host = [r.standard_normal(n).astype(np.float32) for _ in range(arrays)]
    state = L.lsq_trainer_state_pack([torch.from_numpy(a).to(d) for a in host])
    nb = -(-n // BLK)
    assert state.numel() == nb * arrays * BLK == L.lsq_trainer_state_bytes(n, arrays) // 4
    s = state.cpu().numpy().reshape(nb, arrays, BLK)
    for k, a in enumerate(host):
        assert np.array_equal(s[:, k, :].reshape(-1), np.concatenate([a, np.zeros(nb * BLK - n, np.float32)]))
    back = L.lsq_trainer_state_unpack(state, n, arrays)
    for a, b in zip(host, back):
        assert np.array_equal(b.cpu().numpy(), a)


@pytest.mark.parametrize("kw", [dict(momentum=0.0), dict(momentum=0.9), dict(momentum=0.9, nesterov=True),
                                dict(momentum=0.5, weight_decay=0.01, inv_grad_scale=0.25)])
@pytest.mark.parametrize("g_dt,lp_dt", [("f16", "f16"), ("bf16", "bf16"), ("f32", None)])
@pytest.mark.parametrize("n", [3, BLK + 1, 1000003])
def test_sgd_blocked_equals_flat_entry_point(n, g_dt, lp_dt, kw):
    """lsq_sgd_step is checked against the oracle in test_gpu_trainers.py; the blocked form must equal it bit for bit."""
    say(f"[sgd-blocked] n={n} g={g_dt} p_lp={lp_dt} {kw}")
    d = dev()
    t = adam_tensors(CONFIGS[0], g_dt, n=n)
    p = torch.from_numpy(t["p"].copy()).to(d)
    buf = torch.zeros(n, dtype=torch.float32, device=d)
    state = L.lsq_trainer_state_pack([p, None])
    lpt = None if lp_dt is None else (torch.float16 if lp_dt == "f16" else torch.bfloat16)
    a_lp = None if lpt is None else torch.empty(n, dtype=lpt, device=d)
    b_lp = None if lpt is None else torch.empty(n, dtype=lpt, device=d)
    for step in range(3):
        g = to_torch(adam_tensors(CONFIGS[0], g_dt, n=n, stream=70 + step)["g"], g_dt, d)
        L.lsq_sgd_step(p, buf if kw.get("momentum", 0.0) else None, g, a_lp, lr=0.1, **kw)
        L.lsq_sgd_step_blocked(state, g, b_lp, lr=0.1, **kw)
        sp, sb = L.lsq_trainer_state_unpack(state, n, 2)
        assert torch.equal(sp, p) and torch.equal(sb, buf)
        if a_lp is not None:
            assert torch.equal(a_lp, b_lp)


@pytest.mark.parametrize("dt", ["f16", "bf16"])
@pytest.mark.parametrize("n", [5, BLK - 1, 1000003])
def test_adam_lp_blocked_equals_flat_entry_point(n, dt):
    say(f"[adam_lp-blocked] n={n} dt={dt}")
    from workloads import encode
    d = dev()
    t = adam_tensors(CONFIGS[0], dt, n=n)
    p = to_torch(encode(t["p"], dt), dt, d)
    q = p.clone()
    m = torch.zeros(n, dtype=torch.float32, device=d)
    v = torch.zeros(n, dtype=torch.float32, device=d)
    state = L.lsq_trainer_state_pack([m, v])
    for step in range(1, 4):
        g = to_torch(adam_tensors(CONFIGS[0], dt, n=n, stream=60 + step)["g"], dt, d)
        L.lsq_adam_step_lp(p, m, v, g, step=step, **HY)
        L.lsq_adam_step_lp_blocked(q, state, g, step=step, **HY)
        sm, sv = L.lsq_trainer_state_unpack(state, n, 2)
        assert torch.equal(q, p) and torch.equal(sm, m) and torch.equal(sv, v)
