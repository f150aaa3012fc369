"""GPU parity on seeded random shapes: every draw picks sizes that land in some bucket, tail or
fallback of the dispatch (row lengths with and without a factor of 8, ragged row counts, random
masks, dropout on and off, random storage type) and checks the C-ABI result against the CPU oracle
with the tolerances of the fixed-shape tests.  Sizes stay small so the oracle takes milliseconds."""
import numpy as np
import pytest
import torch

import oracle
import paper_2110_05722_amd as L
from tests._util import assert_close_f32, assert_close_store, dev, say, to_np64
from workloads import ADAM_HYPER as HY
from workloads import IGNORE_INDEX, decode, encode, from_torch, to_torch

pytestmark = pytest.mark.gpu
DTS = ["f16", "bf16", "f32"]


def _pick_len(r, hi):
    """A row length: small, a bucket edge +-1, or anything up to hi."""
    kind = r.integers(0, 4)
    if kind == 0:
        return int(r.integers(1, 40))
    if kind == 1:
        edge = int(r.choice([8, 16, 32, 64, 128, 256, 512, 1024, 1536, 2048]))
        return max(1, min(hi, edge + int(r.integers(-1, 2)) * int(r.choice([1, 8]))))
    if kind == 2:
        return int(r.integers(1, hi // 8 + 1)) * 8
    return int(r.integers(1, hi + 1))


@pytest.mark.parametrize("seed", range(24))
def test_softmax_random(seed):
    r = np.random.default_rng(1000 + seed)
    dt = DTS[seed % 3]
    Lk = _pick_len(r, 2300)
    Lq = int(r.choice([Lk, max(1, Lk - int(r.integers(0, 5))), int(r.integers(1, 9))]))
    B, N = int(r.integers(1, 4)), int(r.integers(1, 4))
    Lq = min(Lq, max(1, 60000 // (B * N * Lk)))
    causal = bool(r.integers(0, 2))
    p = float(r.choice([0.0, 0.1, 0.5]))
    use_k, use_q = bool(r.integers(0, 2)), bool(r.integers(0, 2))
    klen = r.integers(0, Lk + 2, size=B).astype(np.int32) if use_k else None
    qlen = r.integers(0, Lq + 2, size=B).astype(np.int32) if use_q else None
    say(f"[random softmax {seed}] B={B} N={N} Lq={Lq} Lk={Lk} causal={causal} p={p} klen={use_k} qlen={use_q} dt={dt}")
    d = dev()
    xs = encode(r.standard_normal((B, N, Lq, Lk), dtype=np.float32) * 2, dt)
    dys = encode(r.standard_normal((B, N, Lq, Lk), dtype=np.float32), dt)
    kl = None if klen is None else torch.from_numpy(klen).to(d)
    ql = None if qlen is None else torch.from_numpy(qlen).to(d)
    y, yd = L.lsq_softmax_varlen_fwd(to_torch(xs, dt, d), kl, ql, causal, 0.3, p, 99, seed)
    ry, ryd = oracle.softmax_fwd(xs, klen, causal, 0.3, dt, p, 99, seed, query_len=qlen)
    assert_close_store(y, ry, dt, "y", f32_floor=1e-7)
    assert not from_torch(y, dt).reshape(ry.shape)[ry == 0.0].view(np.uint16 if dt != "f32" else np.uint32).any()
    if p > 0:
        assert_close_store(yd, ryd, dt, "y_drop", f32_floor=1e-7)
        big = ry > (1e-3 if dt != "f32" else 1e-30)
        assert np.array_equal(to_np64(yd, dt).reshape(ry.shape)[big] == 0, ryd[big] == 0)
    dx = L.lsq_softmax_varlen_bwd(to_torch(dys, dt, d), y, kl, ql, causal, 0.3, p, 99, seed)
    rdx = oracle.softmax_bwd(dys, from_torch(y, dt).reshape(ry.shape), klen, causal, 0.3, dt, p, 99, seed, query_len=qlen)
    assert_close_store(dx, rdx, dt, "dx", f32_floor=1e-6)


@pytest.mark.parametrize("seed", range(24))
def test_layer_ops_random(seed):
    r = np.random.default_rng(2000 + seed)
    dt = DTS[seed % 3]
    hidden = _pick_len(r, 2100) if seed % 4 else int(r.integers(1, 30)) * 8 + int(r.integers(0, 2)) * 4096
    rows = int(r.integers(1, max(2, 40000 // hidden)))
    p = float(r.choice([0.0, 0.1, 0.3]))
    say(f"[random layer {seed}] rows={rows} hidden={hidden} p={p} dt={dt}")
    d = dev()
    f = lambda *shape, s=1.0, m=0.0: encode((r.standard_normal(shape) * s + m).astype(np.float32), dt)
    t = dict(x=f(rows, hidden), res=f(rows, hidden), dy=f(rows, hidden), bias=f(hidden, s=0.1),
             gamma=f(hidden, s=0.1, m=1.0), beta=f(hidden, s=0.1))
    g = {k: to_torch(v, dt, d) for k, v in t.items()}
    # LayerNorm
    y, mean, rstd = L.lsq_layernorm_fwd(g["x"], g["gamma"], g["beta"])
    ry, rmean, rrstd = oracle.layernorm_fwd(t["x"], t["gamma"], t["beta"], 1e-5, dt)
    rsmax = float(np.max(rrstd))
    assert_close_store(y, ry, dt, "ln y", f32_floor=1e-6 * (1 + rsmax))
    assert_close_f32(rstd, rrstd, "rstd", rel=2e-5 if hidden < 4 else 1e-5)
    dx, dgm, dbt = L.lsq_layernorm_bwd(g["dy"], g["x"], g["gamma"], mean, rstd, dres_in=g["res"])
    rdx, rdg, rdb = oracle.layernorm_bwd(t["dy"], t["x"], t["gamma"], 1e-5, dt, dres_in=t["res"])
    assert_close_store(dx, rdx, dt, "ln dx", f32_floor=4e-6 * (1 + rsmax) ** 2)
    assert_close_f32(dgm, rdg, "dgamma", floor=4e-6 * np.sqrt(rows) * 8 * (1 + rsmax))
    assert_close_f32(dbt, rdb, "dbeta", floor=4e-6 * np.sqrt(rows) * 8)
    # bias + dropout + residual
    out = L.lsq_bias_dropout_residual_fwd(g["x"], g["bias"], g["res"], p, 7, seed)
    assert_close_store(out, oracle.bias_dropout_residual_fwd(t["x"], t["bias"], t["res"], p, 7, seed, dt), dt, "bdr out")
    bdx, dbias = L.lsq_bias_dropout_residual_bwd(g["dy"], p, 7, seed)
    rbdx, rdbias = oracle.bias_dropout_residual_bwd(t["dy"], p, 7, seed, dt)
    assert_close_store(bdx, rbdx, dt, "bdr dx")
    assert np.array_equal(to_np64(bdx, dt).reshape(rbdx.shape) == 0, rbdx == 0)
    assert_close_f32(dbias, rdbias, "dbias", floor=4e-6 * np.sqrt(rows) * 8)
    # FFN activation
    act = ["relu", "gelu", "gelu_tanh"][seed % 3]
    a = L.lsq_bias_act_dropout_fwd(g["x"], g["bias"], act, p, 7, seed)
    assert_close_store(a, oracle.bias_act_dropout_fwd(t["x"], t["bias"], act, p, 7, seed, dt), dt, "act out", f32_floor=2e-6)
    adx, adb = L.lsq_bias_act_dropout_bwd(g["dy"], g["x"], g["bias"], act, p, 7, seed)
    radx, radb = oracle.bias_act_dropout_bwd(t["dy"], t["x"], t["bias"], act, p, 7, seed, dt)
    assert_close_store(adx, radx, dt, "act dx", f32_floor=4e-6)
    assert_close_f32(adb, radb, "act dbias", floor=4e-6 * np.sqrt(rows) * 8, rel=2e-5)


@pytest.mark.parametrize("seed", range(12))
def test_criterion_and_trainers_random(seed):
    r = np.random.default_rng(3000 + seed)
    dt = DTS[seed % 3]
    V = int(r.choice([int(r.integers(2, 50)), int(r.integers(50, 3000)), int(r.integers(1, 700)) * 8, 8192 + int(r.integers(-3, 4))]))
    T = int(r.integers(1, max(2, 60000 // V)))
    alpha = float(r.choice([0.0, 0.1, 0.3]))
    say(f"[random criterion {seed}] tokens={T} vocab={V} alpha={alpha} dt={dt}")
    d = dev()
    ls = encode(r.standard_normal((T, V), dtype=np.float32) * 3, dt)
    tg = r.integers(0, V, size=T).astype(np.int32)
    tg[r.random(T) < 0.2] = IGNORE_INDEX
    logits, target = to_torch(ls, dt, d), torch.from_numpy(tg).to(d)
    loss, nll, lse, sums = L.lsq_ls_xent_fwd(logits, target, alpha, IGNORE_INDEX)
    rloss, rnll, rlse, rsums = oracle.ls_xent_fwd(ls, tg, alpha, IGNORE_INDEX, dt)
    assert_close_f32(lse, rlse, "lse", floor=2e-6)
    assert_close_f32(loss, rloss, "loss", floor=4e-6)
    assert_close_f32(nll, rnll, "nll", floor=4e-6)
    assert_close_f32(sums, rsums, "sums", floor=1e-5 * max(1, T))
    dl = L.lsq_ls_xent_bwd(logits, lse, target, alpha, IGNORE_INDEX, 0.5)
    rdl = oracle.ls_xent_bwd(ls, tg, alpha, IGNORE_INDEX, 0.5, dt)
    assert_close_store(dl, rdl, dt, "dlogits", f32_floor=1e-6)
    floss, fnll, flse, fsums, fdl = L.lsq_ls_xent_fwd_bwd(logits, target, alpha, IGNORE_INDEX, 0.5)   # both in one pass
    assert_close_f32(flse, rlse, "one-pass lse", floor=2e-6)
    assert_close_f32(floss, rloss, "one-pass loss", floor=4e-6)
    assert_close_f32(fnll, rnll, "one-pass nll", floor=4e-6)
    assert_close_f32(fsums, rsums, "one-pass sums", floor=1e-5 * max(1, T))
    assert_close_store(fdl, rdl, dt, "one-pass dlogits", f32_floor=1e-6)
    # Adam, both layouts, on a random length
    n = int(r.choice([int(r.integers(1, 64)), int(r.integers(64, 20000)), 8192 * int(r.integers(1, 4)) + int(r.integers(-2, 3))]))
    hp = (r.standard_normal(n) * 0.02).astype(np.float32)
    hm = (r.standard_normal(n) * 1e-3).astype(np.float32)
    hv = ((r.random(n) * 0.9 + 0.1) * 1e-6).astype(np.float32)
    hg = encode((r.standard_normal(n) * 1e-3).astype(np.float32), dt)
    p, m, v = (torch.from_numpy(a.copy()).to(d) for a in (hp, hm, hv))
    state = L.lsq_adam_state_pack(p, m, v)
    g = to_torch(hg, dt, d)
    L.lsq_adam_step(p, m, v, g, None, step=3, **HY)
    L.lsq_adam_step_blocked(state, g, None, step=3, **HY)
    bp, bm, bv = L.lsq_adam_state_unpack(state, n)
    assert torch.equal(bp, p) and torch.equal(bm, m) and torch.equal(bv, v)
    rp, rm, rv = oracle.adam_step(hp, hm, hv, hg, dt, step=3, **HY)
    assert_close_f32(p, rp, "p", rel=1e-6, floor=1e-9)
    assert_close_f32(v, rv, "v", rel=1e-6, floor=1e-30)
    floor_m = 2.0 ** -23 * (HY["beta1"] * np.abs(hm.astype(np.float64)) + (1 - HY["beta1"]) * np.abs(decode(hg, dt)))
    assert_close_f32(m, rm, "m", rel=1e-6, floor=floor_m)


@pytest.mark.parametrize("seed", range(12))
def test_embedding_random(seed):
    """Token counts on both sides of the switch from counted ranks to the radix sort, vocabularies that take one,
    two or three radix passes, id distributions from all-distinct to a few ids only, random padding."""
    r = np.random.default_rng(5000 + seed)
    dt = DTS[seed % 3]
    B = int(r.integers(1, 40))
    Ln = int(r.choice([int(r.integers(1, 64)), int(r.integers(64, 700)), int(r.integers(700, 1200))]))
    Ln = max(1, min(Ln, 36000 // B))
    if seed % 3 == 1:                                        # beyond 16384 tokens: the radix-sorted order
        B, Ln = int(r.integers(30, 40)), int(r.integers(560, 900))
    H = int(r.choice([8, 16, 24, 64, 13]))
    V = int(r.choice([int(r.integers(3, 250)), int(r.integers(300, 60000)), int(r.integers(66000, 90000))]))
    p = float(r.choice([0.0, 0.1]))
    pad = 1
    say(f"[random embedding {seed}] B={B} L={Ln} ({B * Ln} tokens) hidden={H} vocab={V} p={p} dt={dt}")
    d = dev()
    spread = int(r.choice([3, 50, V]))                       # how many different ids the batch draws from
    tok = (r.integers(0, min(spread, V - 2), size=(B, Ln)) + 2).astype(np.int32)
    tok[r.random((B, Ln)) < float(r.choice([0.0, 0.3, 0.9]))] = pad
    embs = encode(r.standard_normal((V, H), dtype=np.float32), dt)
    poss = encode(r.standard_normal((Ln, H), dtype=np.float32) * 0.5, dt)
    dys = encode(r.standard_normal((B * Ln, H), dtype=np.float32), dt)
    scale = float(np.sqrt(H))
    tokens = torch.from_numpy(tok).to(d)
    out = L.lsq_embedding_fwd(tokens, to_torch(embs, dt, d), to_torch(poss, dt, d), pad, scale, p, 9, seed)
    assert_close_store(out, oracle.embedding_fwd(tok, embs, poss, pad, scale, p, 9, seed, dt), dt, "out", f32_floor=1e-5)
    d0 = encode(r.standard_normal((V, H), dtype=np.float32) * 0.1, dt)
    p0 = encode(r.standard_normal((Ln, H), dtype=np.float32) * 0.1, dt)
    demb, dpos = to_torch(d0, dt, d), to_torch(p0, dt, d)
    L.lsq_embedding_bwd(demb, dpos, to_torch(dys, dt, d), tokens, pad, scale, p, 9, seed)
    inc_e, inc_p = oracle.embedding_bwd(dys, tok, V, pad, scale, p, 9, seed, dt)
    # a frequent id sums thousands of rows: the fp32 floor follows the square root of the longest segment
    longest = max(1, int(np.bincount(tok.reshape(-1)[tok.reshape(-1) != pad], minlength=1).max())) if (tok != pad).any() else 1
    assert_close_store(demb, decode(d0, dt) + inc_e, dt, "demb", f32_floor=2e-6 * scale * np.sqrt(longest) * 8)
    assert_close_store(dpos, decode(p0, dt) + inc_p, dt, "dpos", f32_floor=1e-5 * np.sqrt(B))
