"""One pre-LN Transformer encoder layer, forward and backward, built from the entry points of this
library (every non-GEMM step) and torch.matmul (the GEMMs), against the same layer written with plain
PyTorch operators in float64 and differentiated by autograd.  The three dropout masks of the reference
come from the CPU oracle's generator, so the check covers what no single-operator test can: that the
operators compose (layouts, mask regeneration in backward, the residual-gradient path, bias gradients).
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2110_05722_amd as L
from tests._util import dev, say

pytestmark = pytest.mark.gpu


def _close(name, got, ref, rel, floor):
    """fp32 storage: element by element.  bf16 storage (floor None): relative L2 error, because a
    rounding of a pre-activation near 0 flips a ReLU gate or a dropout-scaled term and changes single
    elements completely, while the tensor as a whole stays within the accumulated storage rounding."""
    got, ref = got.double().cpu().numpy().reshape(-1), ref.double().cpu().numpy().reshape(-1)
    if floor is None:
        e = np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-30)
        assert e <= rel, f"{name}: relative L2 error {e:.3e}"
        return
    err = np.abs(got - ref)
    tol = rel * np.abs(ref) + floor * max(1.0, float(np.abs(ref).max()))
    assert np.all(err <= tol), f"{name}: worst {err.max():.3e} (ref max {np.abs(ref).max():.3e})"


@pytest.mark.parametrize("tdt,rel,floor", [(torch.float32, 2e-4, 2e-5), (torch.bfloat16, 8e-2, None), (torch.float16, 6e-3, None)])
@pytest.mark.parametrize("act", ["relu", "gelu"])
def test_encoder_layer_forward_backward(act, tdt, rel, floor):
    B, Ln, H, N, F = 3, 24, 64, 4, 256
    D, T = H // N, B * Ln
    p_res, p_attn, p_act = 0.1, 0.1, 0.2
    seed = 777
    say(f"[layer] pre-LN encoder layer B={B} L={Ln} H={H} heads={N} ffn={F} act={act} storage={tdt}")
    d = dev()
    gen = torch.Generator(device="cpu").manual_seed(5)
    rn = lambda *s, std=1.0, mean=0.0: (torch.randn(*s, generator=gen) * std + mean).to(tdt).to(d)
    x = rn(T, H)
    W = dict(g1=rn(H, std=0.1, mean=1.0), b1=rn(H, std=0.1), Wqkv=rn(3 * H, H, std=H ** -0.5), bqkv=rn(3 * H, std=0.1),
             Wo=rn(H, H, std=H ** -0.5), bo=rn(H, std=0.1), g2=rn(H, std=0.1, mean=1.0), b2=rn(H, std=0.1),
             W1=rn(F, H, std=H ** -0.5), bf1=rn(F, std=0.1), W2=rn(H, F, std=F ** -0.5), bf2=rn(H, std=0.1))
    w_out = rn(T, H)                                             # d loss / d out
    key_len = torch.tensor([Ln, Ln - 7, 5], dtype=torch.int32, device=d)
    scale = D ** -0.5
    mm = lambda a, b: torch.matmul(a.float(), b.float()).to(tdt)  # the GEMMs: fp32 accumulate, stored like everything else

    # ------------------------------------------------------------------ this library
    y1, mean1, rstd1 = L.lsq_layernorm_fwd(x, W["g1"], W["b1"])
    qkv = mm(y1, W["Wqkv"].t())
    q, k, v = L.lsq_split_heads_fwd(qkv, W["bqkv"], B, Ln, N, D, 3)
    s = mm(q, k.transpose(-1, -2))
    pr, prd = L.lsq_softmax_fwd(s, key_len, False, scale, p_attn, seed, 1)
    ctx = mm(prd, v)
    c = L.lsq_merge_heads_fwd(ctx)
    o = mm(c, W["Wo"].t())
    h, y2, mean2, rstd2 = L.lsq_bdr_layernorm_fwd(o, W["bo"], x, W["g2"], W["b2"], p_res, seed, 2)
    f1 = mm(y2, W["W1"].t())
    a = L.lsq_bias_act_dropout_fwd(f1, W["bf1"], act, p_act, seed, 3)
    f2 = mm(a, W["W2"].t())
    out = L.lsq_bias_dropout_residual_fwd(f2, W["bf2"], h, p_res, seed, 4)

    df2, dbf2 = L.lsq_bias_dropout_residual_bwd(w_out, p_res, seed, 4)
    da, dW2 = mm(df2, W["W2"]), mm(df2.t(), a)
    df1, dbf1 = L.lsq_bias_act_dropout_bwd(da, f1, W["bf1"], act, p_act, seed, 3)
    dy2, dW1 = mm(df1, W["W1"]), mm(df1.t(), y2)
    dh, do, dg2, db2, dbo = L.lsq_bdr_layernorm_bwd(dy2, h, W["g2"], mean2, rstd2, p_res, seed, 2, dres_in=w_out)
    dc, dWo = mm(do, W["Wo"]), mm(do.t(), c)
    dctx = L.lsq_merge_heads_bwd(dc, B, Ln, N, D)
    dprd, dv = mm(dctx, v.transpose(-1, -2)), mm(prd.transpose(-1, -2), dctx)
    ds = L.lsq_softmax_bwd(dprd, pr, key_len, False, scale, p_attn, seed, 1)
    dq, dk = mm(ds, k), mm(ds.transpose(-1, -2), q)
    dqkv, dbqkv = L.lsq_split_heads_bwd([dq, dk, dv], B, Ln, N, D)
    dy1, dWqkv = mm(dqkv, W["Wqkv"]), mm(dqkv.t(), y1)
    dx, dg1, db1 = L.lsq_layernorm_bwd(dy1, x, W["g1"], mean1, rstd1, dres_in=dh)

    # ------------------------------------------------------------------ plain PyTorch, float64, autograd
    mask = lambda n, p, off: torch.from_numpy(oracle.dropout_mask(n, p, seed, off).astype(np.float64)).to(d) / (1.0 - np.float32(p).astype(np.float64))
    R = {k_: t.double().detach().clone().requires_grad_(True) for k_, t in W.items()}
    xr = x.double().detach().clone().requires_grad_(True)
    ln = lambda z, g, b: (z - z.mean(-1, keepdim=True)) / torch.sqrt(z.var(-1, unbiased=False, keepdim=True) + 1e-5) * g + b
    r_y1 = ln(xr, R["g1"], R["b1"])
    r_qkv = (r_y1 @ R["Wqkv"].t() + R["bqkv"]).view(B, Ln, 3, N, D).permute(2, 0, 3, 1, 4)
    r_q, r_k, r_v = r_qkv[0], r_qkv[1], r_qkv[2]
    r_s = (r_q @ r_k.transpose(-1, -2)) * scale
    allowed = (torch.arange(Ln, device=d)[None, :] < key_len[:, None])[:, None, None, :]
    r_p = torch.softmax(r_s.masked_fill(~allowed, float("-inf")), dim=-1)
    r_pd = r_p * mask(B * N * Ln * Ln, p_attn, 1).view(B, N, Ln, Ln)
    r_c = (r_pd @ r_v).permute(0, 2, 1, 3).reshape(T, H)
    r_h = xr + (r_c @ R["Wo"].t() + R["bo"]) * mask(T * H, p_res, 2).view(T, H)
    r_y2 = ln(r_h, R["g2"], R["b2"])
    z1 = r_y2 @ R["W1"].t() + R["bf1"]
    r_a = (torch.relu(z1) if act == "relu" else torch.nn.functional.gelu(z1)) * mask(T * F, p_act, 3).view(T, F)
    r_out = r_h + (r_a @ R["W2"].t() + R["bf2"]) * mask(T * H, p_res, 4).view(T, H)
    (r_out * w_out.double()).sum().backward()

    _close("out", out, r_out.detach(), rel, floor)
    _close("dx", dx, xr.grad, rel, floor)
    for name, got in (("g1", dg1), ("b1", db1), ("Wqkv", dWqkv), ("bqkv", dbqkv), ("Wo", dWo), ("bo", dbo), ("g2", dg2),
                      ("b2", db2), ("W1", dW1), ("bf1", dbf1), ("W2", dW2), ("bf2", dbf2)):
        _close("d" + name, got, R[name].grad, rel, floor)


@pytest.mark.parametrize("kind", ["decoder-self-causal", "cross"])
def test_decoder_attention_blocks(kind):
    """The two attention blocks a decoder adds: causal self-attention with target padding, and
    cross-attention whose keys come from a source of another length (q_len != k_len, key padding by
    source lengths, separate Q and KV projections).  fp32 storage, float64 autograd reference."""
    B, Lq, H, N = 3, 13, 64, 4
    Lk = Lq if kind != "cross" else 21
    D, Tq, Tk = H // N, B * Lq, B * Lk
    p_attn, p_res, seed = 0.1, 0.1, 4242
    causal = kind != "cross"
    say(f"[layer] {kind} attention block B={B} Lq={Lq} Lk={Lk} H={H} heads={N}")
    d = dev()
    gen = torch.Generator(device="cpu").manual_seed(11)
    rn = lambda *s, std=1.0, mean=0.0: (torch.randn(*s, generator=gen) * std + mean).to(d)
    x = rn(Tq, H)
    mem = x if kind != "cross" else rn(Tk, H)            # encoder output for cross-attention
    W = dict(g=rn(H, std=0.1, mean=1.0), b=rn(H, std=0.1), Wq=rn(H, H, std=H ** -0.5), bq=rn(H, std=0.1),
             Wkv=rn(2 * H, H, std=H ** -0.5), bkv=rn(2 * H, std=0.1), Wo=rn(H, H, std=H ** -0.5), bo=rn(H, std=0.1))
    w_out = rn(Tq, H)
    key_len = torch.tensor([Lk, Lk - 4, 2], dtype=torch.int32, device=d)
    scale = D ** -0.5
    mm = torch.matmul

    # ---- this library (Q from the normalised decoder state, K and V from `src`)
    y, mean, rstd = L.lsq_layernorm_fwd(x, W["g"], W["b"])
    src = y if kind != "cross" else mem
    (q,) = L.lsq_split_heads_fwd(mm(y, W["Wq"].t()), W["bq"], B, Lq, N, D, 1)
    k, v = L.lsq_split_heads_fwd(mm(src, W["Wkv"].t()), W["bkv"], B, Lk, N, D, 2)
    pr, prd = L.lsq_softmax_fwd(mm(q, k.transpose(-1, -2)), key_len, causal, scale, p_attn, seed, 1)
    c = L.lsq_merge_heads_fwd(mm(prd, v))
    out = L.lsq_bias_dropout_residual_fwd(mm(c, W["Wo"].t()), W["bo"], x, p_res, seed, 2)

    do, dbo = L.lsq_bias_dropout_residual_bwd(w_out, p_res, seed, 2)
    dc, dWo = mm(do, W["Wo"]), mm(do.t(), c)
    dctx = L.lsq_merge_heads_bwd(dc, B, Lq, N, D)
    dprd, dv = mm(dctx, v.transpose(-1, -2)), mm(prd.transpose(-1, -2), dctx)
    ds = L.lsq_softmax_bwd(dprd, pr, key_len, causal, scale, p_attn, seed, 1)
    dq, dk = mm(ds, k), mm(ds.transpose(-1, -2), q)
    dqp, dbq = L.lsq_split_heads_bwd([dq], B, Lq, N, D)
    dkvp, dbkv = L.lsq_split_heads_bwd([dk, dv], B, Lk, N, D)
    dWq, dWkv = mm(dqp.t(), y), mm(dkvp.t(), src)
    dy = mm(dqp, W["Wq"])
    dmem = mm(dkvp, W["Wkv"])
    if kind != "cross":
        dy = dy + dmem                                    # K and V also come from y
    dx, dg, db = L.lsq_layernorm_bwd(dy, x, W["g"], mean, rstd, dres_in=w_out)

    # ---- float64 autograd
    mask = lambda n, p, off: torch.from_numpy(oracle.dropout_mask(n, p, seed, off).astype(np.float64)).to(d) / (1.0 - np.float32(p).astype(np.float64))
    R = {k_: t.double().detach().clone().requires_grad_(True) for k_, t in W.items()}
    xr = x.double().detach().clone().requires_grad_(True)
    mr = mem.double().detach().clone().requires_grad_(True)
    ln = lambda z, g, b: (z - z.mean(-1, keepdim=True)) / torch.sqrt(z.var(-1, unbiased=False, keepdim=True) + 1e-5) * g + b
    ry = ln(xr, R["g"], R["b"])
    rsrc = ry if kind != "cross" else mr
    rq = (ry @ R["Wq"].t() + R["bq"]).view(B, Lq, N, D).permute(0, 2, 1, 3)
    rkv = (rsrc @ R["Wkv"].t() + R["bkv"]).view(B, Lk, 2, N, D).permute(2, 0, 3, 1, 4)
    rs = (rq @ rkv[0].transpose(-1, -2)) * scale
    allowed = (torch.arange(Lk, device=d)[None, :] < key_len[:, None])[:, None, None, :].expand(B, N, Lq, Lk).clone()
    if causal:
        allowed &= (torch.arange(Lk, device=d)[None, :] <= torch.arange(Lq, device=d)[:, None])[None, None]
    rp = torch.softmax(rs.masked_fill(~allowed, float("-inf")), dim=-1)
    rp = torch.where(allowed.any(-1, keepdim=True), rp, torch.zeros_like(rp))          # an empty set gives a zero row
    rc = ((rp * mask(B * N * Lq * Lk, p_attn, 1).view(B, N, Lq, Lk)) @ rkv[1]).permute(0, 2, 1, 3).reshape(Tq, H)
    rout = xr + (rc @ R["Wo"].t() + R["bo"]) * mask(Tq * H, p_res, 2).view(Tq, H)
    (rout * w_out.double()).sum().backward()

    _close("out", out, rout.detach(), 2e-4, 2e-5)
    _close("dx", dx, xr.grad, 2e-4, 2e-5)
    if kind == "cross":
        _close("dmem", dmem, mr.grad, 2e-4, 2e-5)
    for name, got in (("g", dg), ("b", db), ("Wq", dWq), ("bq", dbq), ("Wkv", dWkv), ("bkv", dbkv), ("Wo", dWo), ("bo", dbo)):
        _close("d" + name, got, R[name].grad, 2e-4, 2e-5)
