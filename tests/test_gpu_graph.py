"""The entry points enqueue kernels only (no allocation, no memset, no synchronisation), so a caller may
capture them into a HIP graph.  Each replay is checked against the eager result, with eager work and
synchronisations between the replays."""
import pytest
import torch

import paper_2110_05722_amd as L
from tests._util import dev, say
from workloads import ADAM_HYPER as HY
from workloads import CONFIGS, IGNORE_INDEX, attention_tensors, criterion_tensors, layer_tensors, to_torch

pytestmark = pytest.mark.gpu


def test_layer_ops_replay_under_a_hip_graph():
    say("[graph] capture + 4 replays of the layer operators, criterion and Adam")
    d, dt, cfg = dev(), "f16", CONFIGS[0]
    t = layer_tensors(cfg, dt, rows=1024, hidden=1024)
    x, gamma, beta, bias, res, dy = (to_torch(t[k], dt, d) for k in ("x", "gamma", "beta", "bias", "residual", "dy"))
    a = attention_tensors(cfg, dt)
    sx, sdy, kl = to_torch(a["x"], dt, d), to_torch(a["dy"], dt, d), torch.from_numpy(a["key_len"]).to(d)
    c = criterion_tensors(cfg, dt)
    logits, target = to_torch(c["logits"], dt, d), torch.from_numpy(c["target"]).to(d)
    n = 1 << 18
    g = torch.randn(n, device=d).mul_(1e-3).to(torch.float16)

    # every output and workspace pre-allocated: the captured region allocates nothing
    rows, hidden = x.shape
    y, mean, rstd = torch.empty_like(x), torch.empty(rows, device=d), torch.empty(rows, device=d)
    out, dx, bdx = torch.empty_like(x), torch.empty_like(x), torch.empty_like(x)
    dgamma, dbeta, dbias = (torch.empty(hidden, device=d) for _ in range(3))
    ws = torch.empty(max(L.lsq_workspace_bytes(0, rows, hidden), L.lsq_workspace_bytes(1, rows, hidden)), dtype=torch.uint8, device=d)
    sy, syd, sdx = torch.empty_like(sx), torch.empty_like(sx), torch.empty_like(sx)
    T = logits.shape[0]
    loss, nll, lse = (torch.empty(T, device=d) for _ in range(3))
    sums = torch.empty(3, device=d)
    dlogits = torch.empty_like(logits)
    p0 = torch.randn(n, device=d).mul_(0.02)
    p, m, v, p_lp = p0.clone(), torch.zeros(n, device=d), torch.zeros(n, device=d), torch.empty(n, dtype=torch.float16, device=d)

    def run():
        L.lsq_layernorm_fwd(x, gamma, beta, 1e-5, y=y, mean=mean, rstd=rstd)
        L.lsq_bias_dropout_residual_fwd(y, bias, res, 0.1, 7, 3, out=out)
        L.lsq_softmax_fwd(sx, kl, True, 0.125, 0.1, 7, 4, y=sy, y_drop=syd)
        L.lsq_ls_xent_fwd(logits, target, 0.1, IGNORE_INDEX, loss=loss, nll=nll, lse=lse, sums=sums)
        L.lsq_ls_xent_bwd(logits, lse, target, 0.1, IGNORE_INDEX, 1.0, dlogits=dlogits)
        L.lsq_softmax_bwd(sdy, sy, kl, True, 0.125, 0.1, 7, 4, dx=sdx)
        L.lsq_bias_dropout_residual_bwd(dy, 0.1, 7, 3, dx=bdx, dbias=dbias, workspace=ws)
        L.lsq_layernorm_bwd(bdx, x, gamma, mean, rstd, dx=dx, dgamma=dgamma, dbeta=dbeta, workspace=ws)
        L.lsq_adam_step(p, m, v, g, p_lp, step=1, **HY)

    outputs = (y, mean, rstd, out, sy, syd, loss, nll, lse, sums, dlogits, sdx, bdx, dbias, dx, dgamma, dbeta, p, m, v, p_lp)

    def reset_state():
        p.copy_(p0); m.zero_(); v.zero_()

    reset_state()
    run()
    torch.cuda.synchronize()
    want = [o.clone() for o in outputs]

    reset_state()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    for replay in range(4):
        for o in outputs[:-4]:
            o.fill_(float("nan")) if o.is_floating_point() else o.zero_()
        reset_state()
        torch.cuda.synchronize()
        (x.float() @ x.float().t()).sum().item()          # unrelated eager work between replays
        graph.replay()
        torch.cuda.synchronize()
        for i, (o, w) in enumerate(zip(outputs, want)):
            assert torch.equal(o, w), f"replay {replay}: output {i} differs from the eager run"


def test_newer_entry_points_replay_under_a_hip_graph():
    say("[graph] capture + 3 replays: padding removal, fused boundary, query-length and unaligned softmax, blocked "
        "trainers, one-pass criterion, embedding backward")
    d = dev()
    B, Ln, H, N = 6, 37, 256, 4                       # 37 keys: the LDS-staged softmax path
    T = B * Ln
    g0 = torch.Generator(device="cpu").manual_seed(3)
    rn = lambda *s: torch.randn(*s, generator=g0).to(torch.float16).to(d)
    x, res, dy, bias, gamma, beta = rn(T, H), rn(T, H), rn(T, H), rn(H), rn(H), rn(H)
    lens = torch.tensor([37, 5, 0, 20, 37, 1], dtype=torch.int32, device=d)
    total = int(lens.sum().item())
    sx, sdy = rn(B, N, Ln, Ln), rn(B, N, Ln, Ln)
    n = 3 * 8192 + 77
    p0 = torch.randn(n, generator=g0).mul_(0.02).to(d)
    gr = torch.randn(n, generator=g0).mul_(1e-3).to(torch.float16).to(d)
    state0 = L.lsq_adam_state_pack(p0)
    sgd0 = L.lsq_trainer_state_pack([p0, None])

    offsets = torch.empty(B + 1, dtype=torch.int32, device=d)
    packed = torch.empty((total, H), dtype=torch.float16, device=d)
    padded = torch.empty((B, Ln, H), dtype=torch.float16, device=d)
    h, y, dh, dxp = (torch.empty_like(x) for _ in range(4))
    mean, rstd = torch.empty(T, device=d), torch.empty(T, device=d)
    dgm, dbt, dbi = (torch.empty(H, device=d) for _ in range(3))
    ws = torch.empty(L.lsq_workspace_bytes(5, T, H), dtype=torch.uint8, device=d)
    sy, syd, sdx = (torch.empty_like(sx) for _ in range(3))
    state, sgd, p_lp = state0.clone(), sgd0.clone(), torch.empty(n, dtype=torch.float16, device=d)
    V = 1003                                          # odd vocabulary: ragged first / last pack of every row
    logits = rn(T, V)
    target = torch.randint(0, V, (T,), generator=g0).to(torch.int32).to(d)
    target[::5] = -100
    xl, xn, xe, xs = torch.empty(T, device=d), torch.empty(T, device=d), torch.empty(T, device=d), torch.empty(3, device=d)
    dlog = torch.empty_like(logits)
    tokens = torch.randint(0, 50, (B, Ln), generator=g0).to(torch.int32).to(d)
    demb0, dpos0 = rn(50, H), rn(Ln, H)
    demb, dpos = demb0.clone(), dpos0.clone()
    ews = torch.empty(L.lsq_workspace_bytes(4, T, H), dtype=torch.uint8, device=d)

    wx, wdy, wg, wb = rn(5, 8200), rn(5, 8200), rn(8200), rn(8200)      # rows wider than 8192: the 1024-lane bucket
    wy, wdx, wmean, wrstd = torch.empty_like(wx), torch.empty_like(wx), torch.empty(5, device=d), torch.empty(5, device=d)
    wdg, wdb = torch.empty(8200, device=d), torch.empty(8200, device=d)
    wws = torch.empty(L.lsq_workspace_bytes(0, 5, 8200), dtype=torch.uint8, device=d)

    def run():
        L.lsq_layernorm_fwd(wx, wg, wb, y=wy, mean=wmean, rstd=wrstd)
        L.lsq_layernorm_bwd(wdy, wx, wg, wmean, wrstd, dx=wdx, dgamma=wdg, dbeta=wdb, workspace=wws)
        L.lsq_ls_xent_fwd_bwd(logits, target, 0.1, -100, 0.25, loss=xl, nll=xn, lse=xe, sums=xs, dlogits=dlog)
        L.lsq_embedding_bwd(demb, dpos, dy, tokens, 1, 2.0, 0.1, 9, 3, workspace=ews)
        L.lsq_pad_offsets(lens, B, Ln, offsets=offsets)
        L.lsq_pad_remove(x.view(B, Ln, H), offsets, total, packed=packed)
        L.lsq_pad_restore(packed, offsets, B, Ln, padded=padded)
        L.lsq_bdr_layernorm_fwd(x, bias, res, gamma, beta, 0.1, 9, 1, h=h, y=y, mean=mean, rstd=rstd)
        L.lsq_bdr_layernorm_bwd(dy, h, gamma, mean, rstd, 0.1, 9, 1, dres_in=res, dh=dh, dx=dxp, dgamma=dgm, dbeta=dbt,
                                dbias=dbi, workspace=ws)
        L.lsq_softmax_varlen_fwd(sx, lens, lens, True, 0.2, 0.1, 9, 2, y=sy, y_drop=syd)
        L.lsq_softmax_varlen_bwd(sdy, sy, lens, lens, True, 0.2, 0.1, 9, 2, dx=sdx)
        L.lsq_adam_step_blocked(state, gr, p_lp, step=2, **HY)
        L.lsq_sgd_step_blocked(sgd, gr, None, lr=0.1, momentum=0.9)

    outputs = (wy, wdx, wmean, wrstd, wdg, wdb, offsets, packed, padded, h, y, mean, rstd, dh, dxp, dgm, dbt, dbi, sy, syd, sdx, xl, xn, xe, xs, dlog,
               demb, dpos, state, sgd, p_lp)

    def reset_state():
        state.copy_(state0); sgd.copy_(sgd0); demb.copy_(demb0); dpos.copy_(dpos0)

    reset_state()
    run()
    torch.cuda.synchronize()
    want = [o.clone() for o in outputs]
    reset_state()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    for replay in range(3):
        for o in outputs[:-5]:
            o.fill_(float("nan")) if o.is_floating_point() else o.fill_(-7)
        reset_state()
        torch.cuda.synchronize()
        (x.float() @ x.float().t()).sum().item()
        graph.replay()
        torch.cuda.synchronize()
        for i, (o, w) in enumerate(zip(outputs, want)):
            assert torch.equal(o, w), f"replay {replay}: output {i} differs from the eager run"
