#!/usr/bin/env python3
"""Benchmark of the fused non-GEMM training kernels on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config gpt2-large] [--dtype f16]

A "step" is one pass of the whole hot path over one synthetic batch of the chosen
configuration: layernorm fwd, softmax fwd, bias+dropout+residual fwd, criterion
fwd, criterion bwd, bias+dropout+residual bwd, softmax bwd, layernorm bwd and one
Adam step over the flat workspace, each through the C-ABI, inputs resident in HBM.
The Adam leg runs on the blocked optimizer state by default (lsq_adam_step_blocked:
same arithmetic and bytes as lsq_adam_step, the trainer's private p, m, v interleaved
in 8 Ki-element blocks); the same step with lsq_adam_step on three separate arrays is
timed right after it and reported under "same_step_other_adam_layout".
The layer-sized tensors (tens of MiB) rotate through enough buffer sets that
neither L2 nor the 256 MB Infinity Cache can serve them ("cold" numbers).

Prints ONE JSON line: whole-step throughput in algorithmic GB/s, the roofline
entry of the dominant kernel (Adam), a per-operator table (us, GB/s, fraction of
the 8 TB/s HBM peak), the per-layer non-GEMM roll-up, and the CPU oracle timed on
a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
COLD_FOOTPRINT = 768 << 20       # rotate layer tensors over at least this many bytes


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="gpt2-large")
    ap.add_argument("--dtype", default="f16", choices=["f16", "bf16"])
    ap.add_argument("--op-reps", type=int, default=40, help="back-to-back launches per operator in the per-op table")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--warm", action="store_true", help="do not rotate buffers (cache-warm numbers)")
    ap.add_argument("--no-graph", action="store_true", help="time the per-op table with eager launches")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run a plain 1 GiB -> 1 GiB elementwise copy three times (counter calibration under rocprofv3 --pmc)")
    ap.add_argument("--adam-state", default="blocked", choices=["blocked", "flat"],
                    help="trainer leg of the step: lsq_adam_step_blocked on the blocked optimizer state (default), or "
                         "lsq_adam_step on three separate fp32 arrays; the other one is timed too and reported beside it")
    ap.add_argument("--skip-ops", default="", help="comma-separated operators left out of the per-op table "
                    "(profiling runs: rows that reuse a kernel at another size would blur its per-kernel average)")
    ap.add_argument("--ops", default="", help="comma-separated subset of operators (tuning runs; the default is all nine)")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the JSON line: tables of operator time over tensor sizes (tokens x hidden, sequence "
                         "length, vocabulary, parameter count), the way the paper evaluates its kernels one by one")
    return ap.parse_args()


def sweep(args):
    """Per-operator time and fraction of the HBM peak (algorithmic bytes) over sizes, fp16 or bf16 storage, cold
    buffers, launches replayed from a HIP graph.  Prints markdown tables; not part of the JSON contract."""
    import torch

    import paper_2110_05722_amd as L
    from workloads import ADAM_HYPER, device_normal, torch_dtype

    L.load()
    dev, dt, tdt = torch.device("cuda:0"), args.dtype, torch_dtype(args.dtype)
    torch.cuda.set_device(dev)

    def timed(fn, nbytes):
        reps = max(3, min(40, int(1e10 // max(nbytes, 1)) + 3))
        for i in range(3):
            fn(i)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for i in range(reps):
                fn(i)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        graph.replay()
        torch.cuda.synchronize()
        a.record()
        graph.replay()
        b.record()
        torch.cuda.synchronize()
        us = a.elapsed_time(b) * 1e3 / reps
        return f"{us:.1f} us ({nbytes / us / 1e3 / HBM_PEAK_GBS:.2f})"

    def nsets(per_set):
        return int(max(1, min(8, COLD_FOOTPRINT // max(per_set, 1) + 1)))

    print(f"storage {dt}; every cell: time per launch (fraction of the {HBM_PEAK_GBS / 1000:.0f} TB/s HBM peak on algorithmic bytes)\n")
    print("| tokens x hidden | layernorm fwd | layernorm bwd | bias+dropout+residual fwd | bwd (+dbias) | fused boundary fwd | fused boundary bwd |")
    print("|---|---|---|---|---|---|---|")
    for T in (2048, 8192, 32768):
        for H in (512, 1024, 1280, 2048, 4096, 8192, 12288):
            E = T * H
            k = nsets(12 * E)
            bufs = [{n: device_normal((T, H), 1.0, dt, 7 * i + j, dev) for j, n in enumerate(("x", "res", "dy"))} for i in range(k)]
            outs = [{n: torch.empty((T, H), dtype=tdt, device=dev) for n in ("y", "h", "dx", "dh")} for _ in range(k)]
            gamma, beta, bias = (device_normal((H,), 1.0, dt, 90 + j, dev) for j in range(3))
            mean, rstd = torch.zeros(T, device=dev), torch.ones(T, device=dev)
            dg, db, dbi = (torch.empty(H, device=dev) for _ in range(3))
            ws = torch.empty(max(L.lsq_workspace_bytes(5, T, H), 16), dtype=torch.uint8, device=dev)
            cells = [
                timed(lambda i: L.lsq_layernorm_fwd(bufs[i % k]["x"], gamma, beta, y=outs[i % k]["y"], mean=mean, rstd=rstd), 4 * E + 8 * T),
                timed(lambda i: L.lsq_layernorm_bwd(bufs[i % k]["dy"], bufs[i % k]["x"], gamma, mean, rstd, dx=outs[i % k]["dx"],
                                                    dgamma=dg, dbeta=db, workspace=ws), 6 * E + 8 * T),
                timed(lambda i: L.lsq_bias_dropout_residual_fwd(bufs[i % k]["x"], bias, bufs[i % k]["res"], 0.1, 1, i, out=outs[i % k]["h"]), 6 * E),
                timed(lambda i: L.lsq_bias_dropout_residual_bwd(bufs[i % k]["dy"], 0.1, 1, i, dx=outs[i % k]["dx"], dbias=dbi, workspace=ws), 4 * E),
                timed(lambda i: L.lsq_bdr_layernorm_fwd(bufs[i % k]["x"], bias, bufs[i % k]["res"], gamma, beta, 0.1, 1, i, h=outs[i % k]["h"],
                                                        y=outs[i % k]["y"], mean=mean, rstd=rstd), 8 * E + 8 * T),
                timed(lambda i: L.lsq_bdr_layernorm_bwd(bufs[i % k]["dy"], bufs[i % k]["x"], gamma, mean, rstd, 0.1, 1, i, dres_in=bufs[i % k]["res"],
                                                        dh=outs[i % k]["dh"], dx=outs[i % k]["dx"], dgamma=dg, dbeta=db, dbias=dbi, workspace=ws),
                      10 * E + 8 * T),
            ]
            print(f"| {T} x {H} | " + " | ".join(cells) + " |", flush=True)
            del bufs, outs

    print("\n| batch*heads x length (keys = queries) | softmax fwd | softmax bwd | causal fwd | causal bwd | fwd with attention dropout |")
    print("|---|---|---|---|---|---|")
    for Ln in (64, 128, 256, 512, 1024, 2048, 4096):
        BN = max(1, (1 << 27) // (Ln * Ln))
        B, N = max(1, BN // 16), min(16, BN)
        Es = B * N * Ln * Ln
        k = nsets(8 * Es)
        xs = [device_normal((B, N, Ln, Ln), 1.0, dt, 300 + i, dev) for i in range(k)]
        ys = [torch.empty_like(xs[0]) for _ in range(k)]
        yd = [torch.empty_like(xs[0]) for _ in range(k)]
        causal_frac = (Ln + 1) / (2 * Ln)
        cells = [
            timed(lambda i: L.lsq_softmax_fwd(xs[i % k], None, False, 0.125, y=ys[i % k]), 4 * Es),
            timed(lambda i: L.lsq_softmax_bwd(xs[i % k], ys[i % k], None, False, 0.125, dx=yd[i % k]), 6 * Es),
            timed(lambda i: L.lsq_softmax_fwd(xs[i % k], None, True, 0.125, y=ys[i % k]), int(2 * Es * causal_frac) + 2 * Es),
            timed(lambda i: L.lsq_softmax_bwd(xs[i % k], ys[i % k], None, True, 0.125, dx=yd[i % k]), int(4 * Es * causal_frac) + 2 * Es),
            timed(lambda i: L.lsq_softmax_fwd(xs[i % k], None, False, 0.125, 0.1, 3, i, y=ys[i % k], y_drop=yd[i % k]), 6 * Es),
        ]
        print(f"| {B * N} x {Ln} | " + " | ".join(cells) + " |", flush=True)
        del xs, ys, yd

    print("\n| tokens x vocabulary | criterion fwd | criterion bwd | fwd + bwd in one pass |")
    print("|---|---|---|---|")
    for V in (1000, 8000, 32768, 50257, 128256):
        T = max(64, (1 << 28) // V)
        logits = device_normal((T, V), 2.0, dt, 500, dev)
        dlog = torch.empty_like(logits)
        target = torch.randint(0, V, (T,), device=dev, dtype=torch.int32)
        loss, nll, lse, sums = torch.empty(T, device=dev), torch.empty(T, device=dev), torch.empty(T, device=dev), torch.empty(3, device=dev)
        cells = [
            timed(lambda i: L.lsq_ls_xent_fwd(logits, target, 0.1, -100, loss=loss, nll=nll, lse=lse, sums=sums), 2 * T * V),
            timed(lambda i: L.lsq_ls_xent_bwd(logits, lse, target, 0.1, -100, 1.0 / T, dlogits=dlog), 4 * T * V),
            timed(lambda i: L.lsq_ls_xent_fwd_bwd(logits, target, 0.1, -100, 1.0 / T, loss=loss, nll=nll, lse=lse, sums=sums, dlogits=dlog), 4 * T * V),
        ]
        print(f"| {T} x {V} | " + " | ".join(cells) + " |", flush=True)
        del logits, dlog

    print("\n| parameters | Adam, blocked state | Adam, separate arrays | SGD with momentum, blocked |")
    print("|---|---|---|---|")
    for n in (1 << 20, 1 << 24, 100_000_000, 774_000_000):
        p = device_normal((n,), 0.02, "f32", 700, dev)
        m, v = torch.zeros_like(p), torch.zeros_like(p)
        g = device_normal((n,), 1e-3, dt, 701, dev)
        p_lp = torch.empty(n, dtype=tdt, device=dev)
        state = L.lsq_adam_state_pack(p)
        sgd = L.lsq_trainer_state_pack([p, None])
        cells = [
            timed(lambda i: L.lsq_adam_step_blocked(state, g, p_lp, step=i + 1, **ADAM_HYPER), 28 * n),
            timed(lambda i: L.lsq_adam_step(p, m, v, g, p_lp, step=i + 1, **ADAM_HYPER), 28 * n),
            timed(lambda i: L.lsq_sgd_step_blocked(sgd, g, p_lp, lr=1e-3, momentum=0.9), 20 * n),
        ]
        print(f"| {n} | " + " | ".join(cells) + " |", flush=True)
        del p, m, v, g, p_lp, state, sgd


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the path has no collective: every operator is per row or per element). "
              f"--gpus {args.gpus} is not supported.", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2110_05722_amd as L
    from workloads import ADAM_HYPER, CONFIGS, IGNORE_INDEX, device_normal, torch_dtype

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; there is no CPU path to time.", file=sys.stderr)
        sys.exit(2)
    if args.sweep:
        sweep(args)
        return
    L.load()
    cfg = next(c for c in CONFIGS if c.name == args.config)
    dt = args.dtype
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    tdt = torch_dtype(dt)
    T, H, V, n = cfg.tokens, cfg.hidden, cfg.vocab, cfg.adam_n
    B, N, Lq = cfg.batch, cfg.heads, cfg.max_len
    E = T * H
    Es = B * N * Lq * Lq
    scale = 1.0 / float(np.sqrt(H / N))

    # ------------------------------------------------------------------ inputs
    layer_bytes = 6 * E * 2
    sets = 1 if args.warm else max(2, -(-COLD_FOOTPRINT // layer_bytes))
    seed = cfg.seed * 1000
    layer = []
    for s in range(sets):
        layer.append(dict(
            x=device_normal((T, H), 1.0, dt, seed + 10 * s + 1, dev),
            res=device_normal((T, H), 1.0, dt, seed + 10 * s + 2, dev),
            dy=device_normal((T, H), 1.0, dt, seed + 10 * s + 3, dev),
            out=torch.empty((T, H), dtype=tdt, device=dev),
            y=torch.empty((T, H), dtype=tdt, device=dev),
            dx=torch.empty((T, H), dtype=tdt, device=dev),
            mean=torch.empty(T, dtype=torch.float32, device=dev),
            rstd=torch.empty(T, dtype=torch.float32, device=dev),
        ))
    gamma = device_normal((H,), 0.1, dt, seed + 5, dev, mean=1.0)
    beta = device_normal((H,), 0.1, dt, seed + 6, dev)
    bias = device_normal((H,), 0.1, dt, seed + 7, dev)
    dgamma = torch.empty(H, dtype=torch.float32, device=dev)
    dbeta = torch.empty(H, dtype=torch.float32, device=dev)
    dbias = torch.empty(H, dtype=torch.float32, device=dev)
    ws = torch.empty(max(L.lsq_workspace_bytes(0, T, H), L.lsq_workspace_bytes(1, T, H), 16), dtype=torch.uint8, device=dev)

    soft_sets = 1 if args.warm else max(2, -(-COLD_FOOTPRINT // (4 * Es * 2)))
    soft = []
    rng = np.random.Generator(np.random.PCG64([cfg.seed, 99]))
    from workloads import sentence_lengths
    key_len = None if cfg.lengths == "full" else torch.from_numpy(sentence_lengths(cfg, rng)).to(dev)
    for s in range(soft_sets):
        soft.append(dict(
            x=device_normal((B, N, Lq, Lq), 1.0, dt, seed + 100 + s, dev),
            dy=device_normal((B, N, Lq, Lq), 1.0, dt, seed + 200 + s, dev),
            y=torch.empty((B, N, Lq, Lq), dtype=tdt, device=dev),
            yd=torch.empty((B, N, Lq, Lq), dtype=tdt, device=dev) if cfg.p_attn > 0 else None,
            dx=torch.empty((B, N, Lq, Lq), dtype=tdt, device=dev),
        ))
    allowed = _allowed_elements(cfg, None if key_len is None else key_len.cpu().numpy())

    logits = device_normal((T, V), cfg.logit_std, dt, seed + 300, dev)
    dlogits = torch.empty((T, V), dtype=tdt, device=dev)
    tgt = rng.integers(0, V, size=T).astype(np.int32)
    if cfg.active_frac < 1.0:
        tgt[rng.random(T) >= cfg.active_frac] = IGNORE_INDEX
    elif key_len is not None:
        pad = (np.arange(Lq)[None, :] >= key_len.cpu().numpy()[:, None]).reshape(-1)
        tgt[pad] = IGNORE_INDEX
    t_active = int((tgt != IGNORE_INDEX).sum())
    target = torch.from_numpy(tgt).to(dev)
    loss = torch.empty(T, dtype=torch.float32, device=dev)
    lse = torch.empty(T, dtype=torch.float32, device=dev)
    nll = torch.empty(T, dtype=torch.float32, device=dev)
    sums = torch.empty(3, dtype=torch.float32, device=dev)

    p = device_normal((n,), 0.02, "f32", seed + 400, dev)
    g = device_normal((n,), 1e-3, dt, seed + 401, dev)
    m = torch.zeros(n, dtype=torch.float32, device=dev)
    v = torch.zeros(n, dtype=torch.float32, device=dev)
    p_lp = torch.empty(n, dtype=tdt, device=dev)

    pr, pa, ps = cfg.p_residual, cfg.p_attn, cfg.philox_seed
    causal = cfg.causal
    state = dict(step=0)

    # --------------------------------------------------------------- operators
    def op_ln_fwd(i):
        a = layer[i % sets]
        L.lsq_layernorm_fwd(a["x"], gamma, beta, 1e-5, y=a["y"], mean=a["mean"], rstd=a["rstd"])

    def op_ln_bwd(i):
        a = layer[i % sets]
        L.lsq_layernorm_bwd(a["dy"], a["x"], gamma, a["mean"], a["rstd"], dx=a["dx"], dgamma=dgamma, dbeta=dbeta,
                            workspace=ws)

    def op_bdr_fwd(i):
        a = layer[i % sets]
        L.lsq_bias_dropout_residual_fwd(a["x"], bias, a["res"], pr, ps, i, out=a["out"])

    def op_bdr_bwd(i):
        a = layer[i % sets]
        L.lsq_bias_dropout_residual_bwd(a["dy"], pr, ps, i, dx=a["dx"], dbias=dbias, workspace=ws)

    def op_sm_fwd(i):
        a = soft[i % soft_sets]
        L.lsq_softmax_fwd(a["x"], key_len, causal, scale, pa, ps, 1000 + i, y=a["y"], y_drop=a["yd"])

    def op_sm_bwd(i):
        a = soft[i % soft_sets]
        L.lsq_softmax_bwd(a["dy"], a["y"], key_len, causal, scale, pa, ps, 1000 + i, dx=a["dx"])

    def op_xent_fwd(i):
        L.lsq_ls_xent_fwd(logits, target, cfg.alpha, IGNORE_INDEX, loss=loss, nll=nll, lse=lse, sums=sums)

    def op_xent_bwd(i):
        L.lsq_ls_xent_bwd(logits, lse, target, cfg.alpha, IGNORE_INDEX, 1.0 / max(t_active, 1), dlogits=dlogits)

    def op_xent_fwd_bwd(i):      # forward and backward in one pass over the logits
        L.lsq_ls_xent_fwd_bwd(logits, target, cfg.alpha, IGNORE_INDEX, 1.0 / max(t_active, 1), loss=loss, nll=nll, lse=lse,
                              sums=sums, dlogits=dlogits)

    def op_adam(i):
        state["step"] += 1
        L.lsq_adam_step(p, m, v, g, p_lp, step=state["step"], **ADAM_HYPER)

    # ---- rows beyond the nine (bias+activation+dropout of the FFN, trainer variants): per-op table only
    F = 4 * H
    EF = T * F
    act = "relu" if cfg.name.startswith("transformer") or cfg.name == "tiny" else ("gelu" if cfg.name == "bert-large" else "gelu_tanh")
    ffn_sets = 1 if args.warm else max(2, -(-COLD_FOOTPRINT // (4 * EF * 2)))
    ffn = []
    if not args.ops or any(o.startswith("bias_act") for o in args.ops.split(",")):
        for s_ in range(ffn_sets):
            ffn.append(dict(x=device_normal((T, F), 1.0, dt, seed + 500 + s_, dev),
                            dy=device_normal((T, F), 1.0, dt, seed + 600 + s_, dev),
                            out=torch.empty((T, F), dtype=tdt, device=dev), dx=torch.empty((T, F), dtype=tdt, device=dev)))
    fbias = device_normal((F,), 0.1, dt, seed + 8, dev)
    fdbias = torch.empty(F, dtype=torch.float32, device=dev)
    fws = torch.empty(max(L.lsq_workspace_bytes(2, T, F), 16), dtype=torch.uint8, device=dev)

    def op_bad_fwd(i):
        a = ffn[i % ffn_sets]
        L.lsq_bias_act_dropout_fwd(a["x"], fbias, act, pa, ps, 2000 + i, out=a["out"])

    def op_bad_bwd(i):
        a = ffn[i % ffn_sets]
        L.lsq_bias_act_dropout_bwd(a["dy"], a["x"], fbias, act, pa, ps, 2000 + i, dx=a["dx"], dbias=fdbias, workspace=fws)

    D = H // N
    head_sets = 1 if args.warm else max(2, -(-COLD_FOOTPRINT // (12 * E * 2)))
    heads_buf = []
    if not args.ops or any("heads" in o for o in args.ops.split(",")):
        for s_ in range(head_sets):
            heads_buf.append(dict(qkv=device_normal((T, 3 * H), 1.0, dt, seed + 700 + s_, dev),
                                  q=[torch.empty((B, N, Lq, D), dtype=tdt, device=dev) for _ in range(3)],
                                  dqkv=torch.empty((T, 3 * H), dtype=tdt, device=dev),
                                  merged=torch.empty((T, H), dtype=tdt, device=dev)))
    qkv_bias = device_normal((3 * H,), 0.1, dt, seed + 9, dev)
    qkv_dbias = torch.empty(3 * H, dtype=torch.float32, device=dev)
    hws = torch.empty(max(L.lsq_workspace_bytes(3, T, 3 * H), 16), dtype=torch.uint8, device=dev)

    def op_split_fwd(i):
        a = heads_buf[i % head_sets]
        L.lsq_split_heads_fwd(a["qkv"], qkv_bias, B, Lq, N, D, 3, outs=a["q"])

    def op_split_bwd(i):
        a = heads_buf[i % head_sets]
        L.lsq_split_heads_bwd(a["q"], B, Lq, N, D, din=a["dqkv"], dbias=qkv_dbias, workspace=hws)

    def op_merge_fwd(i):
        a = heads_buf[i % head_sets]
        L.lsq_merge_heads_fwd(a["q"][0], out=a["merged"])

    # token ids with a 1/rank frequency law over the vocabulary (the most frequent id takes ~9 % of the positions)
    w_ = 1.0 / np.arange(1, V - 1, dtype=np.float64)
    zipf = (rng.choice(V - 2, size=(B, Lq), p=w_ / w_.sum()) + 2).astype(np.int32)
    if key_len is not None:
        zipf[np.arange(Lq)[None, :] >= key_len.cpu().numpy()[:, None]] = 1
    emb_tokens = torch.from_numpy(zipf).to(dev)
    n_unique = int(np.unique(zipf[zipf != 1]).size)
    emb_tab = demb_tab = None
    if not args.ops or any("embedding" in o for o in args.ops.split(",")):
        emb_tab = device_normal((V, H), 1.0, dt, seed + 800, dev)
        demb_tab = torch.zeros((V, H), dtype=tdt, device=dev)
    pos_tab = device_normal((Lq, H), 0.5, dt, seed + 801, dev)
    dpos_tab = torch.zeros((Lq, H), dtype=tdt, device=dev)
    ews = torch.empty(max(L.lsq_workspace_bytes(4, T, H), 16), dtype=torch.uint8, device=dev)

    def op_emb_fwd(i):
        a = layer[i % sets]
        L.lsq_embedding_fwd(emb_tokens, emb_tab, pos_tab, 1, float(np.sqrt(H)), pr, ps, 3000 + i, out=a["out"])

    def op_emb_bwd(i):
        a = layer[i % sets]
        L.lsq_embedding_bwd(demb_tab, dpos_tab, a["dy"], emb_tokens, 1, float(np.sqrt(H)), pr, ps, 3000 + i, workspace=ews)

    # the sub-layer boundary in one pass: bias+dropout+residual and the next LayerNorm, forward and backward
    fws3 = torch.empty(max(L.lsq_workspace_bytes(5, T, H), 16), dtype=torch.uint8, device=dev)

    def op_bdr_ln_fwd(i):
        a = layer[i % sets]
        L.lsq_bdr_layernorm_fwd(a["x"], bias, a["res"], gamma, beta, pr, ps, i, 1e-5, h=a["out"], y=a["y"], mean=a["mean"],
                                rstd=a["rstd"])

    def op_ln_bwd_dres(i):       # LayerNorm backward with the residual gradient added: what the fused backward replaces
        a = layer[i % sets]
        L.lsq_layernorm_bwd(a["dy"], a["x"], gamma, a["mean"], a["rstd"], dres_in=a["res"], dx=a["dx"], dgamma=dgamma,
                            dbeta=dbeta, workspace=ws)

    def op_bdr_ln_bwd(i):
        a = layer[i % sets]
        L.lsq_bdr_layernorm_bwd(a["dy"], a["x"], gamma, a["mean"], a["rstd"], pr, ps, i, dres_in=a["res"], dh=a["dx"],
                                dx=a["out"], dgamma=dgamma, dbeta=dbeta, dbias=dbias, workspace=fws3)

    # padding removal: the layer tensors of the batch packed to sum(len) rows and back; the softmax with
    # query lengths (self-attention: query_len == key_len); LayerNorm on the packed rows
    lens_np = np.full(B, Lq, dtype=np.int64) if key_len is None else np.clip(key_len.cpu().numpy(), 0, Lq).astype(np.int64)
    T_real = int(lens_np.sum())
    pad_off = L.lsq_pad_offsets(key_len, B, Lq)
    allowed_q = _allowed_elements(cfg, lens_np, lens_np)

    def op_pad_remove(i):
        a = layer[i % sets]
        L.lsq_pad_remove(a["x"].view(B, Lq, H), pad_off, T, packed=a["out"])

    def op_pad_restore(i):
        a = layer[i % sets]
        L.lsq_pad_restore(a["x"][:T_real], pad_off, B, Lq, padded=a["out"].view(B, Lq, H))

    def op_ln_fwd_packed(i):
        a = layer[i % sets]
        L.lsq_layernorm_fwd(a["x"][:T_real], gamma, beta, 1e-5, y=a["y"][:T_real], mean=a["mean"][:T_real],
                            rstd=a["rstd"][:T_real])

    def op_smv_fwd(i):
        a = soft[i % soft_sets]
        L.lsq_softmax_varlen_fwd(a["x"], key_len, key_len, causal, scale, pa, ps, 1000 + i, y=a["y"], y_drop=a["yd"])

    def op_smv_bwd(i):
        a = soft[i % soft_sets]
        L.lsq_softmax_varlen_bwd(a["dy"], a["y"], key_len, key_len, causal, scale, pa, ps, 1000 + i, dx=a["dx"])

    # the same Adam step on the blocked optimizer state (p, m, v interleaved in 8 Ki-element blocks)
    state_blocked = None
    if not args.ops or "adam_step_blocked" in args.ops.split(",") or args.adam_state == "blocked":
        state_blocked = L.lsq_adam_state_pack(p, m, v)

    def op_adam_blocked(i):
        state["step"] += 1
        L.lsq_adam_step_blocked(state_blocked, g, p_lp, step=state["step"], **ADAM_HYPER)

    def op_adam_lp(i):
        state["step"] += 1
        L.lsq_adam_step_lp(p_lp, m, v, g, step=state["step"], **ADAM_HYPER)

    state_lp = state_sgd = None
    if not args.ops or "adam_step_lp_blocked" in args.ops.split(","):
        state_lp = L.lsq_trainer_state_pack([m, v])
    if not args.ops or "sgd_step_blocked" in args.ops.split(","):
        state_sgd = L.lsq_trainer_state_pack([p, m])

    def op_adam_lp_blocked(i):
        state["step"] += 1
        L.lsq_adam_step_lp_blocked(p_lp, state_lp, g, step=state["step"], **ADAM_HYPER)

    def op_sgd_blocked(i):
        L.lsq_sgd_step_blocked(state_sgd, g, p_lp, lr=1e-3, momentum=0.9)

    def op_sgd(i):
        L.lsq_sgd_step(p, m, g, p_lp, lr=1e-3, momentum=0.9)      # m doubles as the momentum buffer here

    # algorithmic bytes per launch: what the method must move, counted per element / row / parameter
    bts = {
        "layernorm_fwd": 4 * E + 8 * T + 4 * H,
        "layernorm_bwd": 6 * E + 8 * T + 2 * H + 8 * H,
        "bias_dropout_residual_fwd": 6 * E + 2 * H,
        "bias_dropout_residual_bwd": 4 * E + 4 * H,
        "softmax_fwd": 2 * allowed + 2 * Es + (2 * Es if pa > 0 else 0),
        "softmax_bwd": 4 * allowed + 2 * Es,
        "ls_xent_fwd": 2 * t_active * V + 16 * T,
        "ls_xent_bwd": 2 * t_active * V + 2 * T * V + 8 * T,
        "ls_xent_fwd_bwd": 2 * t_active * V + 2 * T * V + 16 * T,
        "adam_step": 28 * n,
        "bias_act_dropout_fwd": 4 * EF + 2 * F, "bias_act_dropout_bwd": 6 * EF + 6 * F,
        "adam_step_lp": 22 * n, "sgd_step": 20 * n, "adam_step_blocked": 28 * n,
        "adam_step_lp_blocked": 22 * n, "sgd_step_blocked": 20 * n,
        "embedding_fwd": 4 * E + 4 * T, "embedding_bwd": 2 * E + 4 * n_unique * H + 4 * Lq * H + 4 * T,
        "split_heads_fwd": 12 * E + 6 * H, "split_heads_bwd": 12 * E + 12 * H, "merge_heads_fwd": 4 * E,
        "layernorm_bwd_dres": 8 * E + 8 * T + 2 * H + 8 * H,
        "bdr_layernorm_fwd": 8 * E + 8 * T + 6 * H, "bdr_layernorm_bwd": 10 * E + 8 * T + 2 * H + 12 * H,
        "pad_remove": 4 * T_real * H + 4 * B, "pad_restore": 2 * T_real * H + 2 * E + 4 * B,
        "layernorm_fwd_packed": 4 * T_real * H + 8 * T_real + 4 * H,
        "softmax_varlen_fwd": 2 * allowed_q + 2 * Es + (2 * Es if pa > 0 else 0),
        "softmax_varlen_bwd": 4 * allowed_q + 2 * Es,
    }
    ops = [
        ("layernorm_fwd", op_ln_fwd), ("softmax_fwd", op_sm_fwd), ("bias_dropout_residual_fwd", op_bdr_fwd),
        ("ls_xent_fwd", op_xent_fwd), ("ls_xent_bwd", op_xent_bwd), ("bias_dropout_residual_bwd", op_bdr_bwd),
        ("softmax_bwd", op_sm_bwd), ("layernorm_bwd", op_ln_bwd),
    ]
    # the trainer leg: same arithmetic and bytes either way, the layout of the private fp32 state differs
    adam_main = ("adam_step_blocked", op_adam_blocked) if args.adam_state == "blocked" else ("adam_step", op_adam)
    adam_other = ("adam_step", op_adam) if args.adam_state == "blocked" else ("adam_step_blocked", op_adam_blocked)
    ops.append(adam_main)

    all_nine = list(ops)
    extra = [adam_other, ("ls_xent_fwd_bwd", op_xent_fwd_bwd), ("bias_act_dropout_fwd", op_bad_fwd), ("bias_act_dropout_bwd", op_bad_bwd),
             ("embedding_fwd", op_emb_fwd), ("embedding_bwd", op_emb_bwd),
             ("split_heads_fwd", op_split_fwd), ("split_heads_bwd", op_split_bwd), ("merge_heads_fwd", op_merge_fwd),
             ("layernorm_bwd_dres", op_ln_bwd_dres), ("bdr_layernorm_fwd", op_bdr_ln_fwd), ("bdr_layernorm_bwd", op_bdr_ln_bwd),
             ("pad_remove", op_pad_remove), ("pad_restore", op_pad_restore), ("layernorm_fwd_packed", op_ln_fwd_packed),
             ("softmax_varlen_fwd", op_smv_fwd), ("softmax_varlen_bwd", op_smv_bwd),
             ("adam_step_lp", op_adam_lp), ("adam_step_lp_blocked", op_adam_lp_blocked),
             ("sgd_step", op_sgd), ("sgd_step_blocked", op_sgd_blocked)]
    if args.skip_ops:
        drop = set(args.skip_ops.split(","))
        extra = [o for o in extra if o[0] not in drop]
    if args.ops:
        keep = set(args.ops.split(","))
        ops = [o for o in ops if o[0] in keep]
        extra = [o for o in extra if o[0] in keep]
        if not ops and not extra:
            sys.exit("bench.py: --ops matched nothing")

    def one_step(i):
        for _, f in ops:
            f(i)

    # ---------------------------------------------------------- timed region
    def time_steps(op_list):
        """W warm-up steps, then K timed steps; events bracket the trainer launch inside the timed region."""
        for i in range(args.warmup):
            for _, f in op_list:
                f(i)
        torch.cuda.synchronize()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
        t0 = time.perf_counter()
        for i in range(args.steps):
            for name, f in op_list:
                if name.startswith("adam_step"):
                    ev[i][0].record()
                    f(args.warmup + i)
                    ev[i][1].record()
                else:
                    f(args.warmup + i)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        has_adam = any(nm.startswith("adam_step") for nm, _ in op_list)
        return (t1 - t0) * 1e3 / args.steps, (float(np.mean([a.elapsed_time(b) for a, b in ev])) if has_adam else float("nan"))

    ms_per_step, adam_ms = time_steps(ops)
    names = [o[0] for o in ops]
    step_bytes = sum(bts[k] for k in names)
    if not names:
        ms_per_step, step_bytes = float("nan"), 0
    value = step_bytes / (ms_per_step * 1e-3) / 1e9
    other = None
    if not args.ops:      # the same step with the other trainer layout, for the record
        ms_o, adam_ms_o = time_steps(ops[:-1] + [adam_other])
        other = {"entry_point": "lsq_" + adam_other[0], "value": round(step_bytes / (ms_o * 1e-3) / 1e9, 1),
                 "ms_per_step": round(ms_o, 4), "adam_avg_launch_ms": round(adam_ms_o, 4),
                 "adam_frac_of_peak": round(bts["adam_step"] / (adam_ms_o * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}

    one_pass = None
    if not args.ops:      # and with the criterion's forward and backward replaced by the one-pass entry point
        swapped = [o for o in ops if o[0] not in ("ls_xent_fwd", "ls_xent_bwd")]
        swapped.insert(3, ("ls_xent_fwd_bwd", op_xent_fwd_bwd))
        ms_f, _ = time_steps(swapped)
        one_pass = {"entry_point": "lsq_ls_xent_fwd_bwd", "ms_per_step": round(ms_f, 4),
                    "note": "same outputs; 2 B/elem fewer algorithmic bytes, so only the time is comparable"}

    # ------------------------------------------- per-operator table (cold, back to back)
    # `reps` launches of one operator are captured into a HIP graph and the graph is replayed
    # between two events: what is timed is the GPU running the kernels back to back, not the
    # Python interpreter issuing them (a ctypes call costs more than a 10 us kernel).
    table = {}
    timing = "eager" if args.no_graph else "hipgraph"
    for name, f in ops + extra:
        reps = max(3, min(args.op_reps, int(2e10 // max(bts[name], 1)) + 3))
        for i in range(3):
            f(i)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        graph = None
        if not args.no_graph:
            try:
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph):
                    for i in range(reps):
                        f(3 + i)
                graph.replay()
                torch.cuda.synchronize()
            except Exception as e:  # capture is an optimisation of the measurement, not of the product
                print(f"bench.py: graph capture failed for {name} ({e}); timing eagerly", file=sys.stderr)
                graph, timing = None, "eager"
        a.record()
        if graph is not None:
            graph.replay()
        else:
            for i in range(reps):
                f(3 + i)
        b.record()
        torch.cuda.synchronize()
        us = a.elapsed_time(b) * 1e3 / reps
        gbs = bts[name] / (us * 1e-6) / 1e9
        table[name] = {"us": round(us, 2), "GBps": round(gbs, 1), "frac_of_peak": round(gbs / HBM_PEAK_GBS, 4),
                       "bytes": int(bts[name]), "launches": reps}
    next_table = {k: table.pop(k) for k, _ in extra if k in table}
    for k, _ in all_nine:
        table.setdefault(k, {"us": float("nan")})
    enc = 2 * table["layernorm_fwd"]["us"] + 2 * table["bias_dropout_residual_fwd"]["us"] + table["softmax_fwd"]["us"] \
        + 2 * table["layernorm_bwd"]["us"] + 2 * table["bias_dropout_residual_bwd"]["us"] + table["softmax_bwd"]["us"]
    dec = 3 * (table["layernorm_fwd"]["us"] + table["bias_dropout_residual_fwd"]["us"] + table["layernorm_bwd"]["us"]
               + table["bias_dropout_residual_bwd"]["us"]) + 2 * (table["softmax_fwd"]["us"] + table["softmax_bwd"]["us"])

    fused_layer = None
    need = ("bdr_layernorm_fwd", "bdr_layernorm_bwd", "layernorm_bwd_dres")
    if all(k in next_table for k in need) and not np.isnan(enc):
        # a pre-LN layer as it really runs: the LayerNorm backward also adds the gradient of the residual
        # branch (dres_in), which the plain layernorm_bwd row above leaves out.  "separate" = four entry
        # points per sub-layer boundary, "fused" = lsq_bdr_layernorm_fwd/bwd.
        sm = table["softmax_fwd"]["us"] + table["softmax_bwd"]["us"]
        sep = table["layernorm_fwd"]["us"] + table["bias_dropout_residual_fwd"]["us"] \
            + next_table["layernorm_bwd_dres"]["us"] + table["bias_dropout_residual_bwd"]["us"]
        fus = next_table["bdr_layernorm_fwd"]["us"] + next_table["bdr_layernorm_bwd"]["us"]
        fused_layer = {"separate": {"encoder_layer_fwd_bwd_nongemm": round(2 * sep + sm, 1),
                                    "decoder_layer_fwd_bwd_nongemm": round(3 * sep + 2 * sm, 1)},
                       "fused": {"encoder_layer_fwd_bwd_nongemm": round(2 * fus + sm, 1),
                                 "decoder_layer_fwd_bwd_nongemm": round(3 * fus + 2 * sm, 1)}}

    if args.calibrate:
        # known traffic for scaling FETCH_SIZE / WRITE_SIZE: reads 2^30 bytes, writes 2^30 bytes per launch
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    achieved = bts["adam_step"] / (adam_ms * 1e-3) / 1e9
    roofline = {"kernel": "adam_kernel (" + ("blocked optimizer state" if args.adam_state == "blocked" else "separate p, m, v arrays") + ")",
                "entry_point": "lsq_" + adam_main[0], "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": _traffic(cfg.name, dt, args.adam_state),
                "bytes_per_launch": int(bts["adam_step"]), "avg_launch_ms": round(adam_ms, 4)}

    out = {
        "metric": "achieved HBM GB/s over one pass of the fused non-GEMM training kernels "
                  "(per-op GB/s, % of peak and us per layer in 'ops' / 'layer_us')",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "storage_dtype": dt, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {B}x{Lq} tokens, hidden {H}, heads {N}, vocab {V}, Adam n={n}, "
                               f"{'causal' if causal else 'key-padding'} softmax, storage {dt}",
                   "buffers": "warm" if args.warm else f"cold (layer tensors rotate over {sets} sets, softmax over {soft_sets})"},
        "roofline": roofline,
        "same_step_other_adam_layout": other,
        "ops": table, "ops_timing": timing,
        "ops_next": dict(next_table, note=f"rows beyond the nine: FFN bias+{act}+dropout(p={pa}) on [{T}, {F}], the paper's "
                                          "low-precision-parameter Adam (22 B/param), SGD with momentum (20 B/param), Adam on the blocked "
                                          "optimizer state (p, m, v interleaved in 8 Ki-element blocks; same 28 B/param), bias+dropout+residual fused "
                                          "with the LayerNorm that follows it (8 B/elem forward, 10 B/elem backward with dres), "
                                          f"QKV bias + head split on [{T}, {3 * H}] and its backward, head merge, embedding of {T} Zipf-"
                                          f"distributed tokens ({n_unique} distinct ids) into [{T}, {H}] and its backward; padding removal "
                                          f"({T_real} real rows of {T}): pack, unpack, LayerNorm on the packed rows, softmax "
                                          "with query lengths (rows of padded queries neither read nor computed)"),
        "layer_us": {"encoder_layer_fwd_bwd_nongemm": round(enc, 1), "decoder_layer_fwd_bwd_nongemm": round(dec, 1)},
        "layer_us_with_residual_gradient": fused_layer,
        "same_step_one_pass_criterion": one_pass,
        "criterion_us": ({"separate": round(table["ls_xent_fwd"]["us"] + table["ls_xent_bwd"]["us"], 1),
                          "one_pass": round(next_table["ls_xent_fwd_bwd"]["us"], 1)}
                         if "ls_xent_fwd" in table and "ls_xent_bwd" in table and "ls_xent_fwd_bwd" in next_table else None),
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, dt)
    else:
        out["cpu_baseline"] = None
    print(json.dumps(out))


def _allowed_elements(cfg, key_len, query_len=None):
    """Number of (row, key) pairs inside the allowed set: what a masked softmax must read."""
    B, N, L = cfg.batch, cfg.heads, cfg.max_len
    kl = np.full(B, L) if key_len is None else np.clip(key_len, 0, L)
    ql = np.full(B, L) if query_len is None else np.clip(query_len, 0, L)
    total = 0
    for b in range(B):
        i = np.arange(int(ql[b]))
        if cfg.causal:
            total += int(np.minimum(i + 1, kl[b]).sum()) * N
        else:
            total += int(kl[b]) * len(i) * N
    return total


def _traffic(cfg_name, dt, adam_state="blocked"):
    """HBM bytes per Adam launch as measured by rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE, scaled by the
    copy-kernel calibration): read from the committed profile summary of this workload, if there is one."""
    path = os.path.join(ROOT, "profiles", f"adam_kernel_{cfg_name}_{dt}_pmc.txt")
    try:
        for line in open(path):
            if line.startswith(f"traffic_bytes_per_launch_{adam_state}:"):
                return int(float(line.split(":", 1)[1].strip()))
    except OSError:
        pass
    return None


def cpu_baseline(cfg, dt):
    """The CPU oracle as it stands, timed on a bounded sample of the same workload on the host cores."""
    import oracle
    from workloads import ADAM_HYPER, IGNORE_INDEX, encode

    rng = np.random.Generator(np.random.PCG64([cfg.seed, 555]))
    H, V, L, N = cfg.hidden, cfg.vocab, cfg.max_len, cfg.heads
    rows = min(cfg.tokens, 8192)
    sb = max(1, min(cfg.batch, 64_000_000 // (N * L * L)))
    xt = min(cfg.tokens, 200_000_000 // V)
    an = min(cfg.adam_n, 128_000_000)
    f = lambda shape, s=1.0: encode(rng.standard_normal(shape, dtype=np.float32) * np.float32(s), dt)
    x, res, dy = f((rows, H)), f((rows, H)), f((rows, H))
    gamma, beta, bias = f((H,)), f((H,)), f((H,))
    sx, sdy = f((sb, N, L, L)), f((sb, N, L, L))
    logits = f((xt, V), cfg.logit_std)
    tgt = rng.integers(0, V, size=xt).astype(np.int32)
    p = rng.standard_normal(an, dtype=np.float32) * np.float32(0.02)
    g = f((an,), 1e-3)
    z = np.zeros(an, np.float32)
    oracle.lib()
    E, Es = rows * H, sb * N * L * L

    def one_pass():
        oracle.layernorm_fwd(x, gamma, beta, 1e-5, dt)
        oracle.layernorm_bwd(dy, x, gamma, 1e-5, dt)
        oracle.bias_dropout_residual_fwd(x, bias, res, cfg.p_residual, 1, 0, dt)
        oracle.bias_dropout_residual_bwd(dy, cfg.p_residual, 1, 0, dt)
        y, _ = oracle.softmax_fwd(sx, None, cfg.causal, 0.125, dt, cfg.p_attn, 1, 0)
        oracle.softmax_bwd(sdy, encode(y, dt), None, cfg.causal, 0.125, dt, cfg.p_attn, 1, 0)
        oracle.ls_xent_fwd(logits, tgt, cfg.alpha, IGNORE_INDEX, dt)
        oracle.ls_xent_bwd(logits, tgt, cfg.alpha, IGNORE_INDEX, 1.0, dt)
        oracle.adam_step(p, z, z, g, dt, step=1, **ADAM_HYPER)

    # repeat the sample until about 10 s of CPU work have been timed (at most 30 passes)
    passes = 0
    t0 = time.perf_counter()
    while True:
        one_pass()
        passes += 1
        t1 = time.perf_counter()
        if t1 - t0 >= 10.0 or passes >= 30:
            break
    half = 0.5 if cfg.causal else 1.0
    nbytes = (4 * E + 6 * E + 6 * E + 4 * E) + (2 * half + 2 + (2 if cfg.p_attn > 0 else 0)) * Es \
        + (4 * half + 2) * Es + 2 * xt * V + 4 * xt * V + 28 * an
    return {"value": round(passes * nbytes / (t1 - t0) / 1e9, 3), "unit": "GB/s", "cores": oracle.num_threads(),
            "kind": "oracle", "seconds": round(t1 - t0, 2),
            "sample": f"{passes} passes of all nine operators on {rows} of {cfg.tokens} tokens (layer ops), "
                      f"{sb} of {cfg.batch} batches (softmax), {xt} tokens (criterion), {an} of {cfg.adam_n} parameters "
                      f"(Adam); same algorithmic byte counts as the GPU line"}


if __name__ == "__main__":
    main()
