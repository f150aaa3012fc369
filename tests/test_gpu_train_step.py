"""Three whole training steps of a small tied-embedding language model: embedding, a pre-LN feed-forward block,
the final LayerNorm, the output projection onto the embedding table, the label-smoothed criterion (forward and
backward in one pass), every backward operator down to the embedding gradient, and the mixed-precision Adam
step over ONE flat workspace (blocked optimizer state, low-precision gradients in, low-precision parameters
out, loss scaling) — every non-GEMM step from this library, the GEMMs from torch.matmul.  The reference is the
same model in float64 PyTorch under autograd with a float64 Adam; its dropout masks come from the CPU oracle's
generator.  What no single-operator test can show: that the ends of the path compose — the gradient of the tied
table is the sum of the projection's and the embedding's, the flat gradient / parameter layout round-trips
through the trainer, the loss scale cancels, and the parameters after several steps agree.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2110_05722_amd as L
from tests._util import dev, say

pytestmark = pytest.mark.gpu

PAD, IGN = 1, -100
HY = dict(lr=2e-3, beta1=0.9, beta2=0.98, eps=1e-6)


def _rel_l2(a, b):
    a, b = a.double().cpu().numpy().reshape(-1), b.double().cpu().numpy().reshape(-1)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-30))


@pytest.mark.parametrize("tdt,grad_tol,step_tol", [(torch.float32, 3e-4, 3e-4), (torch.float16, 1e-2, 4e-2),
                                                   (torch.bfloat16, 6e-2, 2e-1)])
def test_three_training_steps(tdt, grad_tol, step_tol):
    B, Ln, H, F, V = 4, 19, 64, 128, 203
    T = B * Ln
    p_emb, p_act, p_res, alpha, seed = 0.1, 0.1, 0.1, 0.1, 99
    loss_scale = 1.0 if tdt == torch.float32 else 64.0
    say(f"[train step] B={B} L={Ln} H={H} ffn={F} vocab={V} storage={tdt} loss scale {loss_scale}")
    d = dev()
    gen = torch.Generator(device="cpu").manual_seed(21)
    shapes = dict(E=(V, H), P=(Ln, H), g1=(H,), bt1=(H,), W1=(F, H), b1=(F,), W2=(H, F), b2=(H,), gf=(H,), bf=(H,))
    std = dict(E=H ** -0.5, P=0.1, g1=0.1, bt1=0.1, W1=H ** -0.5, b1=0.1, W2=F ** -0.5, b2=0.1, gf=0.1, bf=0.1)
    off, n = {}, 0
    for k, s in shapes.items():
        off[k] = n
        n += int(np.prod(s))                                   # every size is a multiple of 8: views stay 16-byte aligned
    p0 = torch.empty(n)
    for k, s in shapes.items():
        t = torch.randn(*s, generator=gen) * std[k] + (1.0 if k in ("g1", "gf") else 0.0)
        p0[off[k]:off[k] + t.numel()] = t.reshape(-1)
    p0 = p0.to(tdt).float()                                    # the master copy starts at storable values
    tok = torch.randint(2, V, (B, Ln), generator=gen).to(torch.int32)
    tok[:, :3] = torch.tensor([5, 7, 5], dtype=torch.int32)    # repeated ids: their embedding gradients add up
    lens = [Ln, Ln - 6, 11, 2]
    for b, ln_ in enumerate(lens):
        tok[b, ln_:] = PAD
    tgt = torch.randint(0, V, (B, Ln), generator=gen).to(torch.int32)
    tgt[tok == PAD] = IGN
    ntok = int((tgt != IGN).sum())
    tokens, target = tok.to(d), tgt.reshape(-1).to(d)
    mm = lambda a, b: torch.matmul(a.float(), b.float()).to(tdt)
    view = lambda flat, k: flat[off[k]:off[k] + int(np.prod(shapes[k]))].view(*shapes[k])

    # ------------------------------------------------------------------ this library
    state = L.lsq_adam_state_pack(p0.to(d))                    # [p | m | v] blocks, m = v = 0
    w = p0.to(tdt).to(d)                                       # flat compute copy of the parameters
    g = torch.zeros(n, dtype=tdt, device=d)                    # flat gradient, same layout
    W = {k: view(w, k) for k in shapes}
    G = {k: view(g, k) for k in shapes}
    grads_first_step = None
    losses = []
    for step in range(1, 4):
        o = 10 * step
        h0 = L.lsq_embedding_fwd(tokens, W["E"], W["P"], PAD, float(np.sqrt(H)), p_emb, seed, o)
        y1, mean1, rstd1 = L.lsq_layernorm_fwd(h0, W["g1"], W["bt1"])
        f1 = mm(y1, W["W1"].t())
        a = L.lsq_bias_act_dropout_fwd(f1, W["b1"], "gelu", p_act, seed, o + 1)
        f2 = mm(a, W["W2"].t())
        h1, y2, mean2, rstd2 = L.lsq_bdr_layernorm_fwd(f2, W["b2"], h0, W["gf"], W["bf"], p_res, seed, o + 2)
        logits = mm(y2, W["E"].t())
        loss, _, _, sums, dlogits = L.lsq_ls_xent_fwd_bwd(logits, target, alpha, IGN, loss_scale / ntok)
        losses.append(sums[0].item() / ntok)

        dy2 = mm(dlogits, W["E"])
        G["E"].copy_(mm(dlogits.t(), y2))                      # the projection's share of the tied table's gradient
        dh1, df2, dgf, dbf, db2 = L.lsq_bdr_layernorm_bwd(dy2, h1, W["gf"], mean2, rstd2, p_res, seed, o + 2)
        da = mm(df2, W["W2"])
        G["W2"].copy_(mm(df2.t(), a))
        df1, db1 = L.lsq_bias_act_dropout_bwd(da, f1, W["b1"], "gelu", p_act, seed, o + 1)
        dy1 = mm(df1, W["W1"])
        G["W1"].copy_(mm(df1.t(), y1))
        dh0, dg1, dbt1 = L.lsq_layernorm_bwd(dy1, h0, W["g1"], mean1, rstd1, dres_in=dh1)
        G["P"].zero_()
        L.lsq_embedding_bwd(G["E"], G["P"], dh0, tokens, PAD, float(np.sqrt(H)), p_emb, seed, o)   # adds the embedding's share
        for k, t in (("g1", dg1), ("bt1", dbt1), ("b1", db1), ("b2", db2), ("gf", dgf), ("bf", dbf)):
            G[k].copy_(t)
        if step == 1:
            grads_first_step = g.float() / loss_scale
        if tdt == torch.float32:
            L.lsq_adam_step_blocked(state, g, None, step=step, inv_grad_scale=1.0 / loss_scale, **HY)
            L.lsq_adam_state_unpack(state, n, p=w, want=("p",))
        else:
            L.lsq_adam_step_blocked(state, g, w, step=step, inv_grad_scale=1.0 / loss_scale, **HY)   # w = round(p)
    p_lib, m_lib, v_lib = L.lsq_adam_state_unpack(state, n)
    if tdt != torch.float32:
        assert torch.equal(w, p_lib.to(tdt))                   # the low-precision copy is the rounded master copy

    # ------------------------------------------------------------------ float64 PyTorch, autograd, float64 Adam
    p = p0.double().to(d)
    m, v = torch.zeros_like(p), torch.zeros_like(p)
    mask = lambda cnt, pr, o_: torch.from_numpy(oracle.dropout_mask(cnt, pr, seed, o_).astype(np.float64)).to(d) / (1.0 - np.float32(pr).astype(np.float64))
    ln = lambda z, g_, b_: (z - z.mean(-1, keepdim=True)) / torch.sqrt(z.var(-1, unbiased=False, keepdim=True) + 1e-5) * g_ + b_
    real = (tokens.reshape(-1) != PAD).double()[:, None]
    pos_idx = torch.arange(T, device=d) % Ln
    live = target != IGN
    ref_losses, ref_grads_first = [], None
    for step in range(1, 4):
        o = 10 * step
        q = p.detach().clone().requires_grad_(True)
        R = {k: view(q, k) for k in shapes}
        h0 = (np.sqrt(np.float32(H)).astype(np.float64) * R["E"][tokens.reshape(-1).long()] + R["P"][pos_idx]) * real * mask(T * H, p_emb, o).view(T, H)
        z1 = ln(h0, R["g1"], R["bt1"]) @ R["W1"].t() + R["b1"]
        a = torch.nn.functional.gelu(z1) * mask(T * F, p_act, o + 1).view(T, F)
        h1 = h0 + (a @ R["W2"].t() + R["b2"]) * mask(T * H, p_res, o + 2).view(T, H)
        lg = ln(h1, R["gf"], R["bf"]) @ R["E"].t()
        lsm = torch.log_softmax(lg[live], dim=-1)
        per_tok = -(1 - alpha) * lsm.gather(1, target[live].long()[:, None])[:, 0] - alpha / V * lsm.sum(-1)
        total = per_tok.sum() / ntok
        total.backward()
        ref_losses.append(total.item())
        gr = q.grad
        if step == 1:
            ref_grads_first = gr.clone()
        m = HY["beta1"] * m + (1 - HY["beta1"]) * gr
        v = HY["beta2"] * v + (1 - HY["beta2"]) * gr * gr
        c1, c2 = 1 - HY["beta1"] ** step, 1 - HY["beta2"] ** step
        p = p - HY["lr"] * (m / c1) / (torch.sqrt(v / c2) + HY["eps"])

    # ------------------------------------------------------------------ comparison
    for a_, b_ in zip(losses, ref_losses):
        assert abs(a_ - b_) <= (2e-5 if tdt == torch.float32 else 2e-2) * abs(b_), (losses, ref_losses)
    for k in shapes:                                            # the first step's gradients, parameter by parameter
        e = _rel_l2(view(grads_first_step, k), view(ref_grads_first, k))
        assert e <= grad_tol, f"gradient of {k}: relative L2 error {e:.3e}"
    moved = (p - p0.double().to(d))
    e = _rel_l2(p_lib.double() - p0.double().to(d), moved)
    assert e <= step_tol, f"parameter movement after 3 steps: relative L2 error {e:.3e}"
    print(f"    losses {losses} | movement error {e:.2e}")
