#!/usr/bin/env python3
"""Benchmark of the fused non-GEMM training kernels on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config gpt2-large] [--dtype f16]

A "step" is one pass of the whole hot path over one synthetic batch of the chosen
configuration: layernorm fwd, softmax fwd, bias+dropout+residual fwd, criterion
fwd, criterion bwd, bias+dropout+residual bwd, softmax bwd, layernorm bwd and one
lsq_adam_step over the flat workspace, each through the C-ABI, inputs resident in
HBM.  The layer-sized tensors (tens of MiB) rotate through enough buffer sets that
the tensors of any single operator span three times the 256 MB Infinity Cache ("cold" numbers;
the calibration streams rotate the same way).

Prints ONE JSON line:
  value / ms_per_step  whole-step throughput in algorithmic GB/s over the K timed steps
  roofline             the dominant kernel (Adam through lsq_adam_step), its launches bracketed by events
                       inside the timed region; the blocked-state variant beside it
  calibration          plain copy / read / write streams in the operators' launch style at the
                       operators' tensor sizes: what this machine gives a kernel that only moves bytes
  ops                  per-operator table: us (median of five HIP-graph replays of back-to-back launches; us_min the
                       fastest), GB/s, fraction of the 8 TB/s peak, and fraction of the calibrated copy of the same
                       byte count; the masked softmax also at 128-byte-line granularity and with every position counted
  ops_warm             the layer-sized operators again on one buffer set (cache-warm)
  ops_next             rows beyond the nine
  ops_by_config        the nine-operator table of the other target shape (transformer-big, fp16) and of the
                       other storage type (gpt2-large, bf16), and of the masked-LM workload (bert-large, bf16)
  family_frac          bytes / time per operator family and the minimum over the five
  layer_us             non-GEMM microseconds of one layer, forward + backward
  cpu_baseline         the CPU oracle timed on a bounded sample: per operator, one thread and OpenMP

--profile: only the step and the per-operator tables of ONE configuration plus three 1 GiB calibration copies
(for rocprofv3 runs: per-kernel averages stay clean and counters can be scaled by the copy); --no-graph times
the tables with eager launches (counter collection serialises dispatches anyway).
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
COLD_FOOTPRINT = 768 << 20       # the tensors ONE operator touches rotate over at least this many bytes
NINE = ["layernorm_fwd", "softmax_fwd", "bias_dropout_residual_fwd", "ls_xent_fwd", "ls_xent_bwd",
        "bias_dropout_residual_bwd", "softmax_bwd", "layernorm_bwd", "adam_step"]
FAMILIES = {"layernorm": ("layernorm_fwd", "layernorm_bwd"),
            "bias_dropout_residual": ("bias_dropout_residual_fwd", "bias_dropout_residual_bwd"),
            "softmax": ("softmax_fwd", "softmax_bwd"), "ls_xent": ("ls_xent_fwd", "ls_xent_bwd"),
            "adam": ("adam_step",)}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="gpt2-large")
    ap.add_argument("--dtype", default="f16", choices=["f16", "bf16"])
    ap.add_argument("--op-reps", type=int, default=40, help="back-to-back launches per operator in the per-op table")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--profile", action="store_true",
                    help="for rocprofv3 runs: one configuration, the step and the per-operator tables only (no calibration sweep, no other "
                         "configuration, no warm table, no CPU baseline), plus three 1 GiB calibration copies for scaling the counters")
    ap.add_argument("--no-graph", action="store_true", help="per-operator tables from eager launches (counter collection)")
    return ap.parse_args()


# ------------------------------------------------------------------------------------------- timing helpers
EAGER = False      # --no-graph
LAST_MIN_US = [0.0]     # graph_time_us: the fastest of the replays of its last call (the return value is their median)


def graph_time_us(torch, fn, reps):
    """Average microseconds of one call of fn(i) when `reps` calls are captured into a HIP graph and the graph is
    replayed between two events: what is timed is the GPU running the kernels back to back, not the interpreter
    issuing them (a ctypes call costs more than a 10 us kernel)."""
    for i in range(3):
        fn(i)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    if EAGER:
        a.record()
        for i in range(reps):
            fn(3 + i)
        b.record()
        torch.cuda.synchronize()
        LAST_MIN_US[0] = a.elapsed_time(b) * 1e3 / reps
        return LAST_MIN_US[0]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for i in range(reps):
            fn(3 + i)
    graph.replay()
    torch.cuda.synchronize()
    best = []
    for _ in range(5):
        a.record()
        graph.replay()
        b.record()
        torch.cuda.synchronize()
        best.append(a.elapsed_time(b) * 1e3 / reps)
    del graph
    LAST_MIN_US[0] = float(np.min(best))
    return float(np.median(best))


class Calibration:
    """Copy / read / write streams of lsq_calib_stream over cold buffers, at the byte counts of the layer tensors
    and at 1 GiB.  `bytes` always counts what the stream moves (a copy of n bytes moves 2n)."""

    SIZES = [4 << 20, 16 << 20, 33_554_432, 41_943_040, 62_914_560, 83_886_080, 167_772_160, 1 << 30]

    def __init__(self, torch, L, dev, reps):
        self.rows = {"copy": [], "read": [], "write": []}
        sink = torch.zeros(4, dtype=torch.int32, device=dev)
        for moved in self.SIZES:
            for kind in ("copy", "read", "write"):
                n = moved // 2 if kind == "copy" else moved
                n -= n % 16
                per_set = 2 * n if kind == "copy" else n
                k = int(max(2, min(24, COLD_FOOTPRINT // per_set + 1)))
                src = [torch.full((n // 2,), 1.0, dtype=torch.float16, device=dev) for _ in range(k)] if kind != "write" else None
                dst = [torch.empty(n // 2, dtype=torch.float16, device=dev) for _ in range(k)] if kind != "read" else None
                if kind == "copy":
                    fn = lambda i: L.lsq_calib_stream("copy", dst[i % k], src[i % k], n)
                elif kind == "read":
                    fn = lambda i: L.lsq_calib_stream("read", sink, src[i % k], n)
                else:
                    fn = lambda i: L.lsq_calib_stream("write", dst[i % k], None, n)
                r = max(5, min(reps, int(2e10 // moved) + 3))
                us = graph_time_us(torch, fn, r)
                self.rows[kind].append({"bytes": int(moved), "us": round(us, 2), "GBps": round(moved / us / 1e3, 1)})
                del src, dst
        self.empty_us = graph_time_us(torch, lambda i: L.lsq_calib_stream("empty", None, None, 0), reps)
        torch.cuda.empty_cache()

    def copy_us(self, nbytes):
        """Time of the plain copy that moves nbytes (half read, half written): piecewise linear between the
        measured sizes, the 1 GiB rate beyond them."""
        pts = [(0.0, self.empty_us)] + [(float(r["bytes"]), r["us"]) for r in self.rows["copy"]]
        if nbytes >= pts[-1][0]:
            return nbytes / pts[-1][0] * pts[-1][1]
        for (x0, y0), (x1, y1) in zip(pts, pts[1:]):
            if nbytes <= x1:
                return y0 + (y1 - y0) * (nbytes - x0) / (x1 - x0)
        return pts[-1][1]

    def as_json(self):
        return {"what": "lsq_calib_stream: 128-bit nontemporal accesses, one pack per thread, cold buffers, HIP-graph replay; "
                        "bytes = bytes moved (a copy of n bytes moves 2n)",
                "empty_kernel_us": round(self.empty_us, 2), **self.rows}


# ------------------------------------------------------------------------------------------------ workload
def _allowed_elements(cfg, key_len, query_len=None):
    """Number of (row, key) pairs inside the allowed set: what a masked softmax must read."""
    B, N, Ln = cfg.batch, cfg.heads, cfg.max_len
    kl = np.full(B, Ln) if key_len is None else np.clip(key_len, 0, Ln)
    ql = np.full(B, Ln) if query_len is None else np.clip(query_len, 0, Ln)
    total = 0
    for b in range(B):
        i = np.arange(int(ql[b]))
        if cfg.causal:
            total += int(np.minimum(i + 1, kl[b]).sum()) * N
        else:
            total += int(kl[b]) * len(i) * N
    return total


def _line_bytes_softmax(cfg, key_len, elem_bytes=2):
    """Bytes of the 128-byte lines that hold allowed score elements: what a masked softmax fetches at line granularity."""
    B, N, Ln = cfg.batch, cfg.heads, cfg.max_len
    kl = np.full(B, Ln) if key_len is None else np.clip(key_len, 0, Ln)
    per_line = 128 // elem_bytes
    total = 0
    for b in range(B):
        i = np.arange(Ln)
        cnt = np.minimum(i + 1, kl[b]) if cfg.causal else np.full(Ln, kl[b])
        total += int((-(-cnt // per_line) * 128).sum()) * N       # rows start on line boundaries when Lk % 64 == 0
    return total


def adam_arrays(torch, cfg, dt, dev):
    """The trainer's arrays: fp32 p, m, v, low-precision g and p_lp.  Allocated first, as a training program does
    when it builds its model: where the five arrays land decides 0.70-0.80 of peak for the kernel that walks them
    as five streams (the blocked optimizer state does not care)."""
    from workloads import device_normal, torch_dtype
    n, seed = cfg.adam_n, cfg.seed * 1000
    p = device_normal((n,), 0.02, "f32", seed + 400, dev)
    m, v = torch.zeros(n, dtype=torch.float32, device=dev), torch.zeros(n, dtype=torch.float32, device=dev)
    g = device_normal((n,), 1e-3, dt, seed + 401, dev)
    p_lp = torch.empty(n, dtype=torch_dtype(dt), device=dev)
    return p, g, m, v, p_lp


def adam_placement_spread(torch, L, cfg, dt, dev):
    """lsq_adam_step on three more allocations of its five arrays (fresh; behind 2 GiB of other allocations; as slices
    of one slab): the same kernel on the same sizes, only the physical pages differ.  The separate-array trainer is
    sensitive to them; the blocked state, measured beside it on a fresh allocation, is not."""
    from workloads import ADAM_HYPER, torch_dtype
    n, tdt = cfg.adam_n, torch_dtype(dt)
    res = {}
    st = dict(step=0)

    def run(p, m, v, g, p_lp):
        def f(i):
            st["step"] += 1
            L.lsq_adam_step(p, m, v, g, p_lp, step=st["step"], **ADAM_HYPER)
        return round(28 * n / graph_time_us(torch, f, 3) / 1e3 / HBM_PEAK_GBS, 4)

    def fresh():
        return (torch.zeros(n, dtype=torch.float32, device=dev), torch.zeros(n, dtype=torch.float32, device=dev),
                torch.zeros(n, dtype=torch.float32, device=dev), torch.zeros(n, dtype=tdt, device=dev),
                torch.empty(n, dtype=tdt, device=dev))

    arrs = fresh()
    res["fresh"] = run(*arrs)
    del arrs
    gc.collect()
    torch.cuda.empty_cache()
    junk = [torch.empty(64 << 20, dtype=torch.uint8, device=dev) for _ in range(64)]
    junk = junk[::2]
    arrs = fresh()
    res["behind_other_allocations"] = run(*arrs)
    del arrs, junk
    gc.collect()
    torch.cuda.empty_cache()
    a4 = -(-4 * n // 4096) * 4096
    a2 = -(-2 * n // 4096) * 4096
    slab = torch.zeros(3 * a4 + 2 * a2, dtype=torch.uint8, device=dev)
    cut = lambda off, nb, t: slab[off:off + nb].view(t)
    res["one_slab"] = run(cut(0, 4 * n, torch.float32), cut(a4, 4 * n, torch.float32), cut(2 * a4, 4 * n, torch.float32),
                          cut(3 * a4, 2 * n, tdt), cut(3 * a4 + a2, 2 * n, tdt))
    del slab
    gc.collect()
    torch.cuda.empty_cache()
    state = torch.zeros(L.lsq_adam_state_bytes(n) // 4, dtype=torch.float32, device=dev)
    g, p_lp = torch.zeros(n, dtype=tdt, device=dev), torch.empty(n, dtype=tdt, device=dev)

    def fb(i):
        st["step"] += 1
        L.lsq_adam_step_blocked(state, g, p_lp, step=st["step"], **ADAM_HYPER)
    res["blocked_state_fresh"] = round(28 * n / graph_time_us(torch, fb, 3) / 1e3 / HBM_PEAK_GBS, 4)
    del state, g, p_lp
    gc.collect()
    torch.cuda.empty_cache()
    return dict(res, what="fraction of the 8 TB/s peak of lsq_adam_step on other allocations of the same arrays "
                          "(the roofline entry above is the allocation made first in this process)")


def make_workload(torch, L, cfg, dt, dev, extras=True, warm=False, adam=None):
    """Tensors and operator closures of one configuration.  Returns (ops, bts, meta): ops maps a name to a callable
    fn(i) that launches the operator on buffer set i; bts the algorithmic bytes of one launch."""
    from workloads import ADAM_HYPER, IGNORE_INDEX, device_normal, sentence_lengths, torch_dtype

    tdt = torch_dtype(dt)
    T, H, V, n = cfg.tokens, cfg.hidden, cfg.vocab, cfg.adam_n
    B, N, Lq = cfg.batch, cfg.heads, cfg.max_len
    E, Es = T * H, B * N * Lq * Lq
    scale = 1.0 / float(np.sqrt(H / N))
    seed = cfg.seed * 1000
    # every operator's OWN tensors must rotate over more than the 256 MB Infinity Cache: the smallest operator touches two
    sets = 1 if warm else max(2, -(-COLD_FOOTPRINT // (2 * E * 2)))
    layer = []
    for s in range(sets):
        layer.append(dict(
            x=device_normal((T, H), 1.0, dt, seed + 10 * s + 1, dev), res=device_normal((T, H), 1.0, dt, seed + 10 * s + 2, dev),
            dy=device_normal((T, H), 1.0, dt, seed + 10 * s + 3, dev), out=torch.empty((T, H), dtype=tdt, device=dev),
            y=torch.empty((T, H), dtype=tdt, device=dev), dx=torch.empty((T, H), dtype=tdt, device=dev),
            mean=torch.zeros(T, dtype=torch.float32, device=dev), rstd=torch.ones(T, dtype=torch.float32, device=dev)))
    gamma = device_normal((H,), 0.1, dt, seed + 5, dev, mean=1.0)
    beta = device_normal((H,), 0.1, dt, seed + 6, dev)
    bias = device_normal((H,), 0.1, dt, seed + 7, dev)
    dgamma, dbeta, dbias = (torch.empty(H, dtype=torch.float32, device=dev) for _ in range(3))
    ws = torch.empty(max(L.lsq_workspace_bytes(5, T, H), L.lsq_workspace_bytes(1, T, H), 16), dtype=torch.uint8, device=dev)

    rng = np.random.Generator(np.random.PCG64([cfg.seed, 99]))
    key_len_np = None if cfg.lengths == "full" else sentence_lengths(cfg, rng)
    key_len = None if key_len_np is None else torch.from_numpy(key_len_np).to(dev)
    soft_sets = 1 if warm else max(2, -(-COLD_FOOTPRINT // (2 * Es * 2)))
    soft = [dict(x=device_normal((B, N, Lq, Lq), 1.0, dt, seed + 100 + s, dev), dy=device_normal((B, N, Lq, Lq), 1.0, dt, seed + 200 + s, dev),
                 y=torch.empty((B, N, Lq, Lq), dtype=tdt, device=dev),
                 yd=torch.empty((B, N, Lq, Lq), dtype=tdt, device=dev) if cfg.p_attn > 0 else None,
                 dx=torch.empty((B, N, Lq, Lq), dtype=tdt, device=dev)) for s in range(soft_sets)]
    # the paper's parameter search before training: every launch shape the library holds for this row length is
    # timed on this workload's own buffers; the softmax calls below then use the recorded winner
    n_cand = L.lsq_softmax_candidates(Lq)
    bf, bb, tune_us = L.lsq_softmax_tune(soft[0]["x"], soft[0]["dy"], key_len, None, cfg.causal, scale, cfg.p_attn, cfg.philox_seed, 1000,
                                         force=-1, reps=20, y=soft[0]["y"], y_drop=soft[0]["yd"], dx=soft[0]["dx"])
    softmax_tune = {"candidates": n_cand, "chosen_fwd": bf, "chosen_bwd": bb,
                    "us_fwd": [round(u, 2) for u in tune_us[0][:n_cand]], "us_bwd": [round(u, 2) for u in tune_us[1][:n_cand]],
                    "note": "lsq_softmax_tune on this workload's first buffer set (warm), 20 launches per candidate; candidate 0 is the default"}
    allowed = _allowed_elements(cfg, key_len_np)
    allowed_lines = _line_bytes_softmax(cfg, key_len_np)

    logits = device_normal((T, V), cfg.logit_std, dt, seed + 300, dev)
    dlogits = torch.empty((T, V), dtype=tdt, device=dev)
    tgt = rng.integers(0, V, size=T).astype(np.int32)
    if cfg.active_frac < 1.0:
        tgt[rng.random(T) >= cfg.active_frac] = IGNORE_INDEX
    elif key_len_np is not None:
        tgt[(np.arange(Lq)[None, :] >= key_len_np[:, None]).reshape(-1)] = IGNORE_INDEX
    t_active = int((tgt != IGNORE_INDEX).sum())
    target = torch.from_numpy(tgt).to(dev)
    loss, lse, nll = (torch.empty(T, dtype=torch.float32, device=dev) for _ in range(3))
    sums = torch.empty(3, dtype=torch.float32, device=dev)

    p, g, m, v, p_lp = adam if adam is not None else adam_arrays(torch, cfg, dt, dev)
    pr, pa, ps, causal = cfg.p_residual, cfg.p_attn, cfg.philox_seed, cfg.causal
    state = dict(step=0)
    ops = {}

    def op(name):
        def deco(f):
            ops[name] = f
            return f
        return deco

    @op("layernorm_fwd")
    def _(i):
        a = layer[i % sets]
        L.lsq_layernorm_fwd(a["x"], gamma, beta, 1e-5, y=a["y"], mean=a["mean"], rstd=a["rstd"])

    @op("layernorm_bwd")
    def _(i):
        a = layer[i % sets]
        L.lsq_layernorm_bwd(a["dy"], a["x"], gamma, a["mean"], a["rstd"], dx=a["dx"], dgamma=dgamma, dbeta=dbeta, workspace=ws)

    @op("bias_dropout_residual_fwd")
    def _(i):
        a = layer[i % sets]
        L.lsq_bias_dropout_residual_fwd(a["x"], bias, a["res"], pr, ps, i, out=a["out"])

    @op("bias_dropout_residual_bwd")
    def _(i):
        a = layer[i % sets]
        L.lsq_bias_dropout_residual_bwd(a["dy"], pr, ps, i, dx=a["dx"], dbias=dbias, workspace=ws)

    @op("softmax_fwd")
    def _(i):
        a = soft[i % soft_sets]
        L.lsq_softmax_fwd(a["x"], key_len, causal, scale, pa, ps, 1000 + i, y=a["y"], y_drop=a["yd"])

    @op("softmax_bwd")
    def _(i):
        a = soft[i % soft_sets]
        L.lsq_softmax_bwd(a["dy"], a["y"], key_len, causal, scale, pa, ps, 1000 + i, dx=a["dx"])

    @op("ls_xent_fwd")
    def _(i):
        L.lsq_ls_xent_fwd(logits, target, cfg.alpha, IGNORE_INDEX, loss=loss, nll=nll, lse=lse, sums=sums)

    @op("ls_xent_bwd")
    def _(i):
        L.lsq_ls_xent_bwd(logits, lse, target, cfg.alpha, IGNORE_INDEX, 1.0 / max(t_active, 1), dlogits=dlogits)

    @op("adam_step")
    def _(i):
        state["step"] += 1
        L.lsq_adam_step(p, m, v, g, p_lp, step=state["step"], **ADAM_HYPER)

    bts = {
        "layernorm_fwd": 4 * E + 8 * T + 4 * H,
        "layernorm_bwd": 6 * E + 8 * T + 2 * H + 8 * H,
        "bias_dropout_residual_fwd": 6 * E + 2 * H,
        "bias_dropout_residual_bwd": 4 * E + 4 * H,
        "softmax_fwd": 2 * allowed + 2 * Es + (2 * Es if pa > 0 else 0),
        "softmax_bwd": 4 * allowed + 2 * Es,
        "ls_xent_fwd": 2 * t_active * V + 16 * T,
        "ls_xent_bwd": 2 * t_active * V + 2 * T * V + 8 * T,
        "adam_step": 28 * n,
    }
    meta = dict(sets=sets, soft_sets=soft_sets, t_active=t_active, allowed=allowed, softmax_tune=softmax_tune,
                softmax_line_bytes={"softmax_fwd": allowed_lines + 2 * Es + (2 * Es if pa > 0 else 0),
                                    "softmax_bwd": 2 * allowed_lines + 2 * Es,
                                    "softmax_fwd_full": 4 * Es + (2 * Es if pa > 0 else 0), "softmax_bwd_full": 6 * Es},
                workload=f"{cfg.name}: {B}x{Lq} tokens, hidden {H}, heads {N}, vocab {V}, Adam n={n}, "
                         f"{'causal' if causal else 'key-padding'} softmax, storage {dt}")
    if not extras:
        return ops, bts, meta

    # ---- rows beyond the nine
    @op("ls_xent_fwd_bwd")
    def _(i):      # forward and backward in one pass over the logits
        L.lsq_ls_xent_fwd_bwd(logits, target, cfg.alpha, IGNORE_INDEX, 1.0 / max(t_active, 1), loss=loss, nll=nll, lse=lse,
                              sums=sums, dlogits=dlogits)

    F = 4 * H
    EF = T * F
    act = "relu" if cfg.name.startswith("transformer") or cfg.name == "tiny" else ("gelu" if cfg.name == "bert-large" else "gelu_tanh")
    ffn_sets = 1 if warm else max(2, -(-COLD_FOOTPRINT // (2 * EF * 2)))
    ffn = [dict(x=device_normal((T, F), 1.0, dt, seed + 500 + s_, dev), dy=device_normal((T, F), 1.0, dt, seed + 600 + s_, dev),
                out=torch.empty((T, F), dtype=tdt, device=dev), dx=torch.empty((T, F), dtype=tdt, device=dev)) for s_ in range(ffn_sets)]
    fbias = device_normal((F,), 0.1, dt, seed + 8, dev)
    fdbias = torch.empty(F, dtype=torch.float32, device=dev)
    fws = torch.empty(max(L.lsq_workspace_bytes(2, T, F), 16), dtype=torch.uint8, device=dev)

    @op("bias_act_dropout_fwd")
    def _(i):
        a = ffn[i % ffn_sets]
        L.lsq_bias_act_dropout_fwd(a["x"], fbias, act, pa, ps, 2000 + i, out=a["out"])

    @op("bias_act_dropout_bwd")
    def _(i):
        a = ffn[i % ffn_sets]
        L.lsq_bias_act_dropout_bwd(a["dy"], a["x"], fbias, act, pa, ps, 2000 + i, dx=a["dx"], dbias=fdbias, workspace=fws)

    D = H // N
    head_sets = 1 if warm else max(2, -(-COLD_FOOTPRINT // (2 * E * 2)))
    heads_buf = [dict(qkv=device_normal((T, 3 * H), 1.0, dt, seed + 700 + s_, dev),
                      q=[torch.empty((B, N, Lq, D), dtype=tdt, device=dev) for _ in range(3)],
                      dqkv=torch.empty((T, 3 * H), dtype=tdt, device=dev),
                      merged=torch.empty((T, H), dtype=tdt, device=dev)) for s_ in range(head_sets)]
    qkv_bias = device_normal((3 * H,), 0.1, dt, seed + 9, dev)
    qkv_dbias = torch.empty(3 * H, dtype=torch.float32, device=dev)
    hws = torch.empty(max(L.lsq_workspace_bytes(3, T, 3 * H), 16), dtype=torch.uint8, device=dev)

    @op("split_heads_fwd")
    def _(i):
        a = heads_buf[i % head_sets]
        L.lsq_split_heads_fwd(a["qkv"], qkv_bias, B, Lq, N, D, 3, outs=a["q"])

    @op("split_heads_bwd")
    def _(i):
        a = heads_buf[i % head_sets]
        L.lsq_split_heads_bwd(a["q"], B, Lq, N, D, din=a["dqkv"], dbias=qkv_dbias, workspace=hws)

    @op("merge_heads_fwd")
    def _(i):
        a = heads_buf[i % head_sets]
        L.lsq_merge_heads_fwd(a["q"][0], out=a["merged"])

    # token ids with a 1/rank frequency law over the vocabulary (the most frequent id takes ~9 % of the positions)
    w_ = 1.0 / np.arange(1, V - 1, dtype=np.float64)
    zipf = (rng.choice(V - 2, size=(B, Lq), p=w_ / w_.sum()) + 2).astype(np.int32)
    if key_len_np is not None:
        zipf[np.arange(Lq)[None, :] >= key_len_np[:, None]] = 1
    emb_tokens = torch.from_numpy(zipf).to(dev)
    n_unique = int(np.unique(zipf[zipf != 1]).size)
    emb_tab = device_normal((V, H), 1.0, dt, seed + 800, dev)
    demb_tab = torch.zeros((V, H), dtype=tdt, device=dev)
    pos_tab = device_normal((Lq, H), 0.5, dt, seed + 801, dev)
    dpos_tab = torch.zeros((Lq, H), dtype=tdt, device=dev)
    ews = torch.empty(max(L.lsq_workspace_bytes(4, T, H), 16), dtype=torch.uint8, device=dev)

    @op("embedding_fwd")
    def _(i):
        a = layer[i % sets]
        L.lsq_embedding_fwd(emb_tokens, emb_tab, pos_tab, 1, float(np.sqrt(H)), pr, ps, 3000 + i, out=a["out"])

    @op("embedding_bwd")
    def _(i):
        a = layer[i % sets]
        L.lsq_embedding_bwd(demb_tab, dpos_tab, a["dy"], emb_tokens, 1, float(np.sqrt(H)), pr, ps, 3000 + i, workspace=ews)

    # the sub-layer boundary in one pass: bias+dropout+residual and the next LayerNorm, forward and backward
    @op("bdr_layernorm_fwd")
    def _(i):
        a = layer[i % sets]
        L.lsq_bdr_layernorm_fwd(a["x"], bias, a["res"], gamma, beta, pr, ps, i, 1e-5, h=a["out"], y=a["y"], mean=a["mean"], rstd=a["rstd"])

    @op("layernorm_bwd_dres")
    def _(i):       # LayerNorm backward with the residual gradient added: what the fused backward replaces
        a = layer[i % sets]
        L.lsq_layernorm_bwd(a["dy"], a["x"], gamma, a["mean"], a["rstd"], dres_in=a["res"], dx=a["dx"], dgamma=dgamma, dbeta=dbeta, workspace=ws)

    @op("bdr_layernorm_bwd")
    def _(i):
        a = layer[i % sets]
        L.lsq_bdr_layernorm_bwd(a["dy"], a["x"], gamma, a["mean"], a["rstd"], pr, ps, i, dres_in=a["res"], dh=a["dx"], dx=a["out"],
                                dgamma=dgamma, dbeta=dbeta, dbias=dbias, workspace=ws)

    # padding removal: the layer tensors of the batch packed to sum(len) rows and back; the softmax with
    # query lengths (self-attention: query_len == key_len); LayerNorm on the packed rows
    lens_np = np.full(B, Lq, dtype=np.int64) if key_len_np is None else np.clip(key_len_np, 0, Lq).astype(np.int64)
    T_real = int(lens_np.sum())
    pad_off = L.lsq_pad_offsets(key_len, B, Lq)
    allowed_q = _allowed_elements(cfg, lens_np, lens_np)

    @op("pad_remove")
    def _(i):
        a = layer[i % sets]
        L.lsq_pad_remove(a["x"].view(B, Lq, H), pad_off, T, packed=a["out"])

    @op("pad_restore")
    def _(i):
        a = layer[i % sets]
        L.lsq_pad_restore(a["x"][:T_real], pad_off, B, Lq, padded=a["out"].view(B, Lq, H))

    @op("layernorm_fwd_packed")
    def _(i):
        a = layer[i % sets]
        L.lsq_layernorm_fwd(a["x"][:T_real], gamma, beta, 1e-5, y=a["y"][:T_real], mean=a["mean"][:T_real], rstd=a["rstd"][:T_real])

    @op("softmax_varlen_fwd")
    def _(i):
        a = soft[i % soft_sets]
        L.lsq_softmax_varlen_fwd(a["x"], key_len, key_len, causal, scale, pa, ps, 1000 + i, y=a["y"], y_drop=a["yd"])

    @op("softmax_varlen_bwd")
    def _(i):
        a = soft[i % soft_sets]
        L.lsq_softmax_varlen_bwd(a["dy"], a["y"], key_len, key_len, causal, scale, pa, ps, 1000 + i, dx=a["dx"])

    # trainer variants: Adam on the blocked optimizer state (p, m, v interleaved in 8 Ki-element blocks), the paper's
    # low-precision-parameter Adam, SGD with momentum; separate arrays and blocked
    state_blocked = L.lsq_adam_state_pack(p, m, v)

    @op("adam_step_blocked")
    def _(i):
        state["step"] += 1
        L.lsq_adam_step_blocked(state_blocked, g, p_lp, step=state["step"], **ADAM_HYPER)

    @op("adam_step_lp")
    def _(i):
        state["step"] += 1
        L.lsq_adam_step_lp(p_lp, m, v, g, step=state["step"], **ADAM_HYPER)

    @op("sgd_step")
    def _(i):
        L.lsq_sgd_step(p, m, g, p_lp, lr=1e-3, momentum=0.9)      # m doubles as the momentum buffer here

    state_lp = L.lsq_trainer_state_pack([m, v])

    @op("adam_step_lp_blocked")
    def _(i):
        state["step"] += 1
        L.lsq_adam_step_lp_blocked(p_lp, state_lp, g, step=state["step"], **ADAM_HYPER)

    state_sgd = L.lsq_trainer_state_pack([p, m])

    @op("sgd_step_blocked")
    def _(i):
        L.lsq_sgd_step_blocked(state_sgd, g, p_lp, lr=1e-3, momentum=0.9)

    bts.update({
        "ls_xent_fwd_bwd": 2 * t_active * V + 2 * T * V + 16 * T,
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
    })
    meta["next_note"] = (f"rows beyond the nine: FFN bias+{act}+dropout(p={pa}) on [{T}, {F}], the paper's low-precision-parameter Adam "
                         "(22 B/param), SGD with momentum (20 B/param), the trainers on a blocked optimizer state (same bytes), "
                         "bias+dropout+residual fused with the LayerNorm that follows it (8 B/elem forward, 10 B/elem backward with "
                         f"dres), QKV bias + head split on [{T}, {3 * H}] and its backward, head merge, embedding of {T} Zipf-distributed "
                         f"tokens ({n_unique} distinct ids) into [{T}, {H}] and its backward; padding removal ({T_real} real rows of {T}): "
                         "pack, unpack, LayerNorm on the packed rows, softmax with query lengths")
    return ops, bts, meta


def time_steps(torch, ops, names, steps, warmup):
    """W warm-up steps, then K timed steps of the operators `names`; events bracket the trainer launch inside the
    timed region.  Returns (ms per step, average ms of the trainer launch)."""
    for i in range(warmup):
        for nm in names:
            ops[nm](i)
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    t0 = time.perf_counter()
    for i in range(steps):
        for nm in names:
            if nm.startswith("adam_step"):
                ev[i][0].record()
                ops[nm](warmup + i)
                ev[i][1].record()
            else:
                ops[nm](warmup + i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    return (t1 - t0) * 1e3 / steps, float(np.mean([a.elapsed_time(b) for a, b in ev]))


def device_info(torch, dev):
    """What the runtime says the device is (the peak the fractions refer to is the datasheet's 8 TB/s)."""
    pr = torch.cuda.get_device_properties(dev)
    return {"name": pr.name, "compute_units": int(pr.multi_processor_count), "memory_GiB": round(pr.total_memory / 2**30, 1),
            "arch": getattr(pr, "gcnArchName", "")}


def op_table(torch, ops, bts, names, max_reps, calib=None, line_bytes=None):
    table = {}
    for name in names:
        reps = max(3, min(max_reps, int(2e10 // max(bts[name], 1)) + 3))
        us = graph_time_us(torch, ops[name], reps)
        gbs = bts[name] / (us * 1e-6) / 1e9
        row = {"us": round(us, 2), "us_min": round(LAST_MIN_US[0], 2), "GBps": round(gbs, 1),
               "frac_of_peak": round(gbs / HBM_PEAK_GBS, 4), "bytes": int(bts[name]), "launches": reps}
        if calib is not None:
            row["frac_of_copy"] = round(calib.copy_us(bts[name]) / us, 4)
        if line_bytes and name in line_bytes:      # the masked softmax at 128-byte line granularity
            row["bytes_line_granular"] = int(line_bytes[name])
            row["frac_of_peak_line_granular"] = round(line_bytes[name] / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)
            full = line_bytes[name + "_full"]          # every position counted as if no mask let the kernel skip it
            row["bytes_full_tensor"] = int(full)
            row["frac_of_peak_full_tensor"] = round(full / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)
        table[name] = row
    return table


def layer_us(t):
    enc = 2 * t["layernorm_fwd"]["us"] + 2 * t["bias_dropout_residual_fwd"]["us"] + t["softmax_fwd"]["us"] \
        + 2 * t["layernorm_bwd"]["us"] + 2 * t["bias_dropout_residual_bwd"]["us"] + t["softmax_bwd"]["us"]
    dec = 3 * (t["layernorm_fwd"]["us"] + t["bias_dropout_residual_fwd"]["us"] + t["layernorm_bwd"]["us"]
               + t["bias_dropout_residual_bwd"]["us"]) + 2 * (t["softmax_fwd"]["us"] + t["softmax_bwd"]["us"])
    return {"encoder_layer_fwd_bwd_nongemm": round(enc, 1), "decoder_layer_fwd_bwd_nongemm": round(dec, 1)}


def family_frac(t):
    fam = {}
    for k, names in FAMILIES.items():
        by = sum(t[nm]["bytes"] for nm in names)
        us = sum(t[nm]["us"] for nm in names)
        fam[k] = round(by / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)
    return {"per_family": fam, "min": min(fam.values()), "min_family": min(fam, key=fam.get),
            "what": "bytes / time over the forward and the backward of each family, as a fraction of the 8 TB/s peak"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the path has no collective: every operator is per row or per element). "
              f"--gpus {args.gpus} is not supported.", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2110_05722_amd as L
    from workloads import CONFIGS

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; there is no CPU path to time.", file=sys.stderr)
        sys.exit(2)
    L.load()
    global EAGER
    EAGER = args.no_graph
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = next(c for c in CONFIGS if c.name == args.config)
    dt = args.dtype

    adam = adam_arrays(torch, cfg, dt, dev)
    calib = None if args.profile else Calibration(torch, L, dev, args.op_reps)

    # ------------------------------------------------------------------ the headline configuration
    ops, bts, meta = make_workload(torch, L, cfg, dt, dev, extras=True, adam=adam)
    del adam
    ms_per_step, adam_ms = time_steps(torch, ops, NINE, args.steps, args.warmup)
    step_bytes = sum(bts[k] for k in NINE)
    value = step_bytes / (ms_per_step * 1e-3) / 1e9
    achieved = bts["adam_step"] / (adam_ms * 1e-3) / 1e9
    roofline = {"kernel": "adam_kernel (separate p, m, v arrays)", "entry_point": "lsq_adam_step", "bound": "hbm",
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": _traffic(cfg.name, dt, "flat"), "bytes_per_launch": int(bts["adam_step"]), "avg_launch_ms": round(adam_ms, 4)}
    table = op_table(torch, ops, bts, NINE, args.op_reps, calib, meta["softmax_line_bytes"])

    out = {
        "metric": "achieved HBM GB/s over one pass of the fused non-GEMM training kernels "
                  "(per-op GB/s, % of peak and us per layer in 'ops' / 'layer_us')",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "storage_dtype": dt, "data": "synthetic", "device": device_info(torch, dev),
        "config": {"workload": meta["workload"],
                   "buffers": f"cold (layer tensors rotate over {meta['sets']} sets, softmax over {meta['soft_sets']})"},
        "roofline": roofline,
        "ops": table, "ops_timing": "eager" if EAGER else "hipgraph", "softmax_tune": meta["softmax_tune"],
        "family_frac": family_frac(table),
        "layer_us": layer_us(table),
    }

    if args.profile:
        extra = [k for k in ops if k not in NINE]
        out["ops_next"] = dict(op_table(torch, ops, bts, extra, args.op_reps), note=meta["next_note"])
        # known traffic for scaling FETCH_SIZE / WRITE_SIZE: reads 2^30 bytes, writes 2^30 bytes per launch
        src = torch.ones(1 << 29, dtype=torch.float16, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            L.lsq_calib_stream("copy", dst, src, 1 << 30)
        torch.cuda.synchronize()
        out["cpu_baseline"] = None
        print(json.dumps(out))
        return

    # ---- the same step with the trainer on the blocked optimizer state, and with the one-pass criterion
    names_b = [nm if nm != "adam_step" else "adam_step_blocked" for nm in NINE]
    ms_b, adam_ms_b = time_steps(torch, ops, names_b, args.steps, args.warmup)
    ach_b = bts["adam_step_blocked"] / (adam_ms_b * 1e-3) / 1e9
    out["roofline_blocked_state"] = {
        "kernel": "adam_kernel (blocked optimizer state: p, m, v interleaved in 8 Ki-element blocks)", "entry_point": "lsq_adam_step_blocked",
        "bound": "hbm", "achieved": round(ach_b, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(ach_b / HBM_PEAK_GBS, 4),
        "traffic": _traffic(cfg.name, dt, "blocked"), "bytes_per_launch": int(bts["adam_step_blocked"]), "avg_launch_ms": round(adam_ms_b, 4),
        "same_step": {"value": round(step_bytes / (ms_b * 1e-3) / 1e9, 1), "ms_per_step": round(ms_b, 4)}}
    names_f = [nm for nm in NINE if nm not in ("ls_xent_fwd", "ls_xent_bwd")]
    names_f.insert(3, "ls_xent_fwd_bwd")
    ms_f, _ = time_steps(torch, ops, names_f, args.steps, args.warmup)
    out["same_step_one_pass_criterion"] = {"entry_point": "lsq_ls_xent_fwd_bwd", "ms_per_step": round(ms_f, 4),
                                           "note": "same outputs; 2 B/elem fewer algorithmic bytes, so only the time is comparable"}

    extra = [k for k in ops if k not in NINE]
    nxt = op_table(torch, ops, bts, extra, args.op_reps, calib)
    out["ops_next"] = dict(nxt, note=meta["next_note"])
    sm = table["softmax_fwd"]["us"] + table["softmax_bwd"]["us"]
    sep = table["layernorm_fwd"]["us"] + table["bias_dropout_residual_fwd"]["us"] + nxt["layernorm_bwd_dres"]["us"] \
        + table["bias_dropout_residual_bwd"]["us"]
    fus = nxt["bdr_layernorm_fwd"]["us"] + nxt["bdr_layernorm_bwd"]["us"]
    out["layer_us_with_residual_gradient"] = {
        "separate": {"encoder_layer_fwd_bwd_nongemm": round(2 * sep + sm, 1), "decoder_layer_fwd_bwd_nongemm": round(3 * sep + 2 * sm, 1)},
        "fused": {"encoder_layer_fwd_bwd_nongemm": round(2 * fus + sm, 1), "decoder_layer_fwd_bwd_nongemm": round(3 * fus + 2 * sm, 1)}}
    out["criterion_us"] = {"separate": round(table["ls_xent_fwd"]["us"] + table["ls_xent_bwd"]["us"], 1),
                           "one_pass": round(nxt["ls_xent_fwd_bwd"]["us"], 1)}
    del ops, nxt
    gc.collect()
    torch.cuda.empty_cache()

    # ---- the layer-sized operators on ONE buffer set (cache-warm), beside the cold numbers above
    wops, wbts, _ = make_workload(torch, L, cfg, dt, dev, extras=True, warm=True)
    warm_names = ["layernorm_fwd", "layernorm_bwd", "bias_dropout_residual_fwd", "bias_dropout_residual_bwd",
                  "bdr_layernorm_fwd", "bdr_layernorm_bwd"]
    out["ops_warm"] = dict(op_table(torch, wops, wbts, warm_names, args.op_reps),
                           note="same launches on one buffer set: inputs and outputs of a launch (20-105 MB) stay in the 256 MB Infinity Cache")
    del wops
    gc.collect()
    torch.cuda.empty_cache()

    # ---- the other target shape and the other storage type: the nine-operator table and the step
    out["ops_by_config"] = {}
    for cname, cdt in (("transformer-big", "f16"), ("gpt2-large", "bf16"), ("bert-large", "bf16")):
        if cname == cfg.name and cdt == dt:
            continue
        c2 = next(c for c in CONFIGS if c.name == cname)
        o2, b2, m2 = make_workload(torch, L, c2, cdt, dev, extras=False)
        ms2, adam2 = time_steps(torch, o2, NINE, max(5, args.steps // 2), args.warmup)
        t2 = op_table(torch, o2, b2, NINE, args.op_reps, calib, m2["softmax_line_bytes"])
        sb2 = sum(b2[k] for k in NINE)
        out["ops_by_config"][f"{cname}/{cdt}"] = {
            "workload": m2["workload"], "value": round(sb2 / (ms2 * 1e-3) / 1e9, 1), "ms_per_step": round(ms2, 4),
            "adam_frac_of_peak": round(b2["adam_step"] / (adam2 * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "ops": t2, "softmax_tune": m2["softmax_tune"], "family_frac": family_frac(t2), "layer_us": layer_us(t2)}
        del o2
        gc.collect()
        torch.cuda.empty_cache()

    out["adam_placement_spread"] = adam_placement_spread(torch, L, cfg, dt, dev)
    out["calibration"] = calib.as_json()
    out["cpu_baseline"] = None if args.no_cpu_baseline else cpu_baseline(cfg, dt)
    print(json.dumps(out))


def _traffic(cfg_name, dt, adam_state):
    """HBM bytes per Adam launch as measured by rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE, scaled by the
    copy-kernel calibration): read from the committed profile summary of this workload, if there is one."""
    path = os.path.join(ROOT, "profiles", f"all_kernels_{cfg_name}_{dt}_pmc.txt")
    try:
        for line in open(path):
            if line.startswith(f"traffic_bytes_per_launch_{adam_state}:"):
                return int(float(line.split(":", 1)[1].strip()))
    except OSError:
        pass
    return None


def cpu_baseline(cfg, dt):
    """The CPU oracle as it stands, timed on a bounded sample of the same workload on the host cores: every operator
    once on one thread and then on all threads (OpenMP over rows), the all-thread pass repeated until about 10 s of
    CPU work have been timed."""
    import ctypes

    import oracle
    from workloads import ADAM_HYPER, IGNORE_INDEX, encode

    rng = np.random.Generator(np.random.PCG64([cfg.seed, 555]))
    H, V, Ln, N = cfg.hidden, cfg.vocab, cfg.max_len, cfg.heads
    rows = min(cfg.tokens, 2048)
    sb = max(1, min(cfg.batch, 24_000_000 // (N * Ln * Ln)))
    xt = max(1, min(cfg.tokens, 24_000_000 // V))
    an = min(cfg.adam_n, 16_000_000)
    f = lambda shape, s=1.0: encode(rng.standard_normal(shape, dtype=np.float32) * np.float32(s), dt)
    x, res, dy = f((rows, H)), f((rows, H)), f((rows, H))
    gamma, beta, bias = f((H,)), f((H,)), f((H,))
    sx, sdy = f((sb, N, Ln, Ln)), f((sb, N, Ln, Ln))
    logits = f((xt, V), cfg.logit_std)
    tgt = rng.integers(0, V, size=xt).astype(np.int32)
    p = rng.standard_normal(an, dtype=np.float32) * np.float32(0.02)
    g = f((an,), 1e-3)
    z = np.zeros(an, np.float32)
    oracle.lib()
    E, Es = rows * H, sb * N * Ln * Ln
    half = 0.5 if cfg.causal else 1.0
    y_keep = {}

    def sm_fwd():
        y_keep["y"] = encode(oracle.softmax_fwd(sx, None, cfg.causal, 0.125, dt, cfg.p_attn, 1, 0)[0], dt)

    steps = [
        ("layernorm_fwd", 4 * E, lambda: oracle.layernorm_fwd(x, gamma, beta, 1e-5, dt)),
        ("layernorm_bwd", 6 * E, lambda: oracle.layernorm_bwd(dy, x, gamma, 1e-5, dt)),
        ("bias_dropout_residual_fwd", 6 * E, lambda: oracle.bias_dropout_residual_fwd(x, bias, res, cfg.p_residual, 1, 0, dt)),
        ("bias_dropout_residual_bwd", 4 * E, lambda: oracle.bias_dropout_residual_bwd(dy, cfg.p_residual, 1, 0, dt)),
        ("softmax_fwd", int((2 * half + 2 + (2 if cfg.p_attn > 0 else 0)) * Es), sm_fwd),
        ("softmax_bwd", int((4 * half + 2) * Es), lambda: oracle.softmax_bwd(sdy, y_keep["y"], None, cfg.causal, 0.125, dt, cfg.p_attn, 1, 0)),
        ("ls_xent_fwd", 2 * xt * V, lambda: oracle.ls_xent_fwd(logits, tgt, cfg.alpha, IGNORE_INDEX, dt)),
        ("ls_xent_bwd", 4 * xt * V, lambda: oracle.ls_xent_bwd(logits, tgt, cfg.alpha, IGNORE_INDEX, 1.0, dt)),
        ("adam_step", 28 * an, lambda: oracle.adam_step(p, z, z, g, dt, step=1, **ADAM_HYPER)),
    ]
    nthreads = oracle.num_threads()
    omp = None
    for name in ("libgomp.so.1", "libgomp.so"):
        try:
            omp = ctypes.CDLL(name)
            break
        except OSError:
            continue
    per_op = {}
    t_start = time.perf_counter()
    if omp is not None:
        omp.omp_set_num_threads(1)
        for name, nb, fn in steps:
            t0 = time.perf_counter()
            fn()
            dt_s = time.perf_counter() - t0
            per_op[name] = {"bytes": int(nb), "us_1_thread": round(dt_s * 1e6, 1), "GBps_1_thread": round(nb / dt_s / 1e9, 3)}
        omp.omp_set_num_threads(nthreads)
    passes, acc = 0, {name: 0.0 for name, _, _ in steps}
    t_omp0 = time.perf_counter()
    while True:
        for name, nb, fn in steps:
            t0 = time.perf_counter()
            fn()
            acc[name] += time.perf_counter() - t0
        passes += 1
        if time.perf_counter() - t_start >= 10.0 or passes >= 30:
            break
    t_omp = time.perf_counter() - t_omp0
    for name, nb, _ in steps:
        d = per_op.setdefault(name, {"bytes": int(nb)})
        d["us_all_threads"] = round(acc[name] / passes * 1e6, 1)
        d["GBps_all_threads"] = round(nb * passes / acc[name] / 1e9, 3)
    nbytes = sum(nb for _, nb, _ in steps)
    return {"value": round(passes * nbytes / t_omp / 1e9, 3), "unit": "GB/s", "cores": nthreads, "kind": "oracle",
            "seconds": round(time.perf_counter() - t_start, 2), "ops": per_op,
            "sample": f"all nine operators on {rows} of {cfg.tokens} tokens (layer ops), {sb} of {cfg.batch} batches (softmax), "
                      f"{xt} tokens (criterion), {an} of {cfg.adam_n} parameters (Adam); one pass on 1 thread, then {passes} "
                      f"passes on {nthreads} threads (value = the all-thread passes); same algorithmic byte counts as the GPU line"}


if __name__ == "__main__":
    main()
