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
