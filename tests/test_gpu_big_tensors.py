"""GPU parity on tensors of more than 2^31 elements (more than 4 GiB in fp16): the sizes one GPU with 288 GB holds for a
long batch.  Element indices, Philox pack counters and row offsets then no longer fit 32 bits.  Inputs are drawn on
the device; the oracle gets copies of the rows around the 2^31-element mark and of the last rows, with the flat
element index of their first element (the dropout contract counts packs over the whole tensor)."""
import gc

import numpy as np
import pytest
import torch

import oracle
import paper_2110_05722_amd as L
from tests._util import assert_close_f32, assert_close_store, dev, say, to_np64
from workloads import device_normal, from_torch

pytestmark = pytest.mark.gpu

DT = "f16"
MARK = 1 << 31


def _free():
    gc.collect()
    torch.cuda.empty_cache()


def _np(t, lo, hi):
    """rows lo..hi of a [rows, hidden] device tensor as the stored bit patterns (what the oracle takes)."""
    return from_torch(t[lo:hi].contiguous(), DT)


def _row_windows(rows, hidden):
    """a few rows at the start, around the 2^31-th element, and at the end"""
    mid = MARK // hidden
    return [(0, 3), (mid - 2, mid + 3), (rows - 3, rows)]


def test_layer_operators_beyond_2_31_elements():
    d = dev()
    rows, hidden = 2_100_003, 1024                       # 2.15e9 elements, a ragged last workgroup
    assert rows * hidden > MARK
    say(f"[big] layer operators on {rows} x {hidden} ({rows * hidden / 2**30:.2f} Gi elements)")
    x = device_normal((rows, hidden), 1.0, DT, 11, d)
    res = device_normal((rows, hidden), 1.0, DT, 12, d)
    gamma = device_normal((hidden,), 0.1, DT, 13, d, mean=1.0)
    beta = device_normal((hidden,), 0.1, DT, 14, d)
    p, seed, offset = 0.1, 77, 5

    y, mean, rstd = L.lsq_layernorm_fwd(x, gamma, beta, 1e-5)
    for lo, hi in _row_windows(rows, hidden):
        ry, rmean, rrstd = oracle.layernorm_fwd(_np(x, lo, hi), from_torch(gamma, DT), from_torch(beta, DT), 1e-5, DT)
        assert_close_store(y[lo:hi], ry, DT, f"layernorm y rows {lo}..{hi}")
        assert_close_f32(mean[lo:hi], rmean, "mean", floor=2e-7)
        assert_close_f32(rstd[lo:hi], rrstd, "rstd", floor=1e-6)

    out = L.lsq_bias_dropout_residual_fwd(x, gamma, res, p, seed, offset)          # gamma serves as the bias
    for lo, hi in _row_windows(rows, hidden):
        r = oracle.bias_dropout_residual_fwd(_np(x, lo, hi), from_torch(gamma, DT), _np(res, lo, hi), p, seed, offset, DT,
                                             e0=lo * hidden)
        assert_close_store(out[lo:hi], r, DT, f"bias+dropout+residual rows {lo}..{hi}")
    del out, res
    _free()

    dy = y                                                                       # any tensor of the shape serves as dy
    dx, dbias = L.lsq_bias_dropout_residual_bwd(dy, p, seed, offset)
    for lo, hi in _row_windows(rows, hidden):
        rdx, _ = oracle.bias_dropout_residual_bwd(_np(dy, lo, hi), p, seed, offset, DT, e0=lo * hidden)
        assert_close_store(dx[lo:hi], rdx, DT, f"bias+dropout+residual dx rows {lo}..{hi}")
    # the column sums over all rows: against the same sum taken by torch in float64 from the stored dx
    # (each stored element is within half an fp16 ulp of the fp32 value that was summed)
    ref = torch.zeros(hidden, dtype=torch.float64, device=d)
    for s in range(0, rows, 1 << 18):
        ref += dx[s:s + (1 << 18)].double().sum(0)
    assert_close_f32(dbias, ref.cpu().numpy(), "dbias", rel=1e-4, floor=2.0 ** -11 * 4 * np.sqrt(rows) + 1e-6 * rows)
    del dbias, ref
    _free()

    dxl, dgamma, dbeta = L.lsq_layernorm_bwd(dy, x, gamma, mean, rstd, dx=dx)
    for lo, hi in _row_windows(rows, hidden):
        rdx, _, _ = oracle.layernorm_bwd(_np(dy, lo, hi), _np(x, lo, hi), from_torch(gamma, DT), 1e-5, DT)
        assert_close_store(dxl[lo:hi], rdx, DT, f"layernorm dx rows {lo}..{hi}")
    refb = torch.zeros(hidden, dtype=torch.float64, device=d)
    refg = torch.zeros(hidden, dtype=torch.float64, device=d)
    for s in range(0, rows, 1 << 18):
        e = min(rows, s + (1 << 18))
        g64 = dy[s:e].double()
        refb += g64.sum(0)
        refg += (g64 * (x[s:e].double() - mean[s:e, None].double()) * rstd[s:e, None].double()).sum(0)
    assert_close_f32(dbeta, refb.cpu().numpy(), "dbeta", rel=1e-5, floor=4e-6 * np.sqrt(rows) * 8)
    assert_close_f32(dgamma, refg.cpu().numpy(), "dgamma", rel=1e-5, floor=4e-6 * np.sqrt(rows) * 8 * 4)


def test_softmax_beyond_2_31_elements():
    d = dev()
    B, N, Lq, Lk = 33, 16, 2048, 2048                    # 2.21e9 elements
    n = B * N * Lq * Lk
    assert n > MARK
    say(f"[big] softmax on {B} x {N} x {Lq} x {Lk} ({n / 2**30:.2f} Gi elements), key padding, attention dropout")
    x = device_normal((B, N, Lq, Lk), 1.0, DT, 21, d)
    kl_np = np.random.default_rng(5).integers(1, Lk + 1, size=B).astype(np.int32)
    kl_np[-1] = Lk - 5
    kl = torch.from_numpy(kl_np).to(d)
    p, seed, offset, scale = 0.1, 3, 9, 0.125
    y, yd = L.lsq_softmax_fwd(x, kl, False, scale, p, seed, offset)
    dy = x                                                # any tensor of the shape
    dx = L.lsq_softmax_bwd(dy, y, kl, False, scale, p, seed, offset)
    mid_row = MARK // Lk                                  # the row that holds element 2^31
    for first in (0, mid_row - 2, B * N * Lq - 4):
        b, rem = divmod(first, N * Lq)
        h, q0 = divmod(rem, Lq)
        q1 = min(Lq, q0 + 4)
        sl = (slice(b, b + 1), slice(h, h + 1), slice(q0, q1))
        e0 = first * Lk
        xs = from_torch(x[sl].contiguous(), DT)
        ry, ryd = oracle.softmax_fwd(xs, kl_np[b:b + 1], False, scale, DT, p, seed, offset, e0=e0)
        assert_close_store(y[sl], ry, DT, f"y rows from {first}", f32_floor=1e-7)
        assert_close_store(yd[sl], ryd, DT, f"y_drop rows from {first}", f32_floor=1e-7)
        assert np.array_equal(to_np64(yd[sl].contiguous(), DT) == 0, ryd == 0)
        rdx = oracle.softmax_bwd(from_torch(dy[sl].contiguous(), DT), from_torch(y[sl].contiguous(), DT), kl_np[b:b + 1],
                                 False, scale, DT, p, seed, offset, e0=e0)
        assert_close_store(dx[sl], rdx, DT, f"dx rows from {first}", f32_floor=1e-7)


def test_criterion_beyond_2_31_logits():
    d = dev()
    tokens, vocab = 66_000, 32768 + 8                     # 2.16e9 logits; rows start off the 128-byte grid
    assert tokens * vocab > MARK
    say(f"[big] criterion on {tokens} x {vocab} ({tokens * vocab / 2**30:.2f} Gi logits)")
    logits = device_normal((tokens, vocab), 2.0, DT, 31, d)
    tg_np = np.random.default_rng(6).integers(0, vocab, size=tokens).astype(np.int32)
    tg_np[::7] = -100
    tg_np[-1] = vocab - 1
    target = torch.from_numpy(tg_np).to(d)
    alpha, scale = 0.1, 0.5
    loss, nll, lse, sums = L.lsq_ls_xent_fwd(logits, target, alpha, -100, want_sums=True)
    dlogits = L.lsq_ls_xent_bwd(logits, lse, target, alpha, -100, scale)
    mid = MARK // vocab
    for lo, hi in ((0, 3), (mid - 2, mid + 3), (tokens - 3, tokens)):
        lg = from_torch(logits[lo:hi].contiguous(), DT)
        rl, rn, rlse, _ = oracle.ls_xent_fwd(lg, tg_np[lo:hi], alpha, -100, DT)
        assert_close_f32(loss[lo:hi], rl, f"loss {lo}..{hi}", floor=2e-6)
        assert_close_f32(nll[lo:hi], rn, "nll", floor=2e-6)
        assert_close_f32(lse[lo:hi], rlse, "lse", floor=1e-6)
        rd = oracle.ls_xent_bwd(lg, tg_np[lo:hi], alpha, -100, scale, DT)
        assert_close_store(dlogits[lo:hi], rd, DT, f"dlogits {lo}..{hi}")
    live = tg_np != -100
    assert float(sums[2]) == float(live.sum())
    assert_close_f32(sums[0:1], np.array([loss.double().sum().item()]), "sum of losses", rel=1e-6)
    del dlogits
    _free()
    # the one-pass criterion in place over the logits
    keep = {lo: from_torch(logits[lo:hi].contiguous(), DT) for lo, hi in ((0, 3), (mid - 2, mid + 3), (tokens - 3, tokens))}
    loss2, nll2, lse2, _, dl2 = L.lsq_ls_xent_fwd_bwd(logits, target, alpha, -100, scale, want_sums=False, dlogits=logits)
    for lo, hi in ((0, 3), (mid - 2, mid + 3), (tokens - 3, tokens)):
        rd = oracle.ls_xent_bwd(keep[lo], tg_np[lo:hi], alpha, -100, scale, DT)
        assert_close_store(dl2[lo:hi], rd, DT, f"one-pass dlogits {lo}..{hi}")
    assert torch.allclose(lse2, lse, rtol=1e-5, atol=1e-6) and torch.allclose(loss2, loss, rtol=1e-5, atol=2e-6)


def test_adam_beyond_2_31_parameters():
    d = dev()
    n = MARK + 4099
    say(f"[big] Adam on {n} parameters ({28 * n / 1e9:.0f} GB)")
    p = device_normal((n,), 0.02, "f32", 41, d)
    g = device_normal((n,), 1e-3, DT, 42, d)
    m = torch.zeros(n, dtype=torch.float32, device=d)
    v = torch.zeros(n, dtype=torch.float32, device=d)
    p_lp = torch.empty(n, dtype=torch.float16, device=d)
    spans = [(0, 4096), (MARK - 2048, MARK + 2048), (n - 4099, n)]
    before = {lo: (p[lo:hi].cpu().numpy().copy(), from_torch(g[lo:hi].contiguous(), DT)) for lo, hi in spans}
    hyper = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, step=1, weight_decay=0.01, adamw=True)
    L.lsq_adam_step(p, m, v, g, p_lp, **hyper)
    for lo, hi in spans:
        p0, g0 = before[lo]
        z = np.zeros(hi - lo, dtype=np.float32)
        rp, rm, rv = oracle.adam_step(p0, z, z.copy(), g0, DT, hyper["lr"], hyper["beta1"], hyper["beta2"], hyper["eps"], 1,
                                      weight_decay=0.01, adamw=True)[:3]
        assert_close_f32(p[lo:hi], rp, f"p {lo}..{hi}", rel=1e-6, floor=1e-9)
        assert_close_f32(v[lo:hi], rv, "v", rel=1e-6, floor=1e-20)
        assert_close_f32(m[lo:hi], rm, "m", rel=1e-6, floor=2.0 ** -23 * 1e-3)
        assert torch.equal(p_lp[lo:hi], p[lo:hi].to(torch.float16))
