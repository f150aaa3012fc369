"""ctypes binding of include/lsq.h.  Argument marshalling only.

Every wrapper takes torch tensors that already live on the GPU, passes their
device pointers, the sizes and the current HIP stream to the C entry point of
the same name, and returns the output tensors.  Optional `out=`-style arguments
let a caller (the benchmark) reuse buffers so that a call allocates nothing.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liblsq.so")
_lib = None

LSQ_F16, LSQ_BF16, LSQ_F32 = 0, 1, 2
LSQ_OP_LAYERNORM_BWD, LSQ_OP_BIAS_DROPOUT_RESIDUAL_BWD, LSQ_OP_BIAS_ACT_DROPOUT_BWD = 0, 1, 2
LSQ_OP_SPLIT_HEADS_BWD = 3
LSQ_OP_EMBEDDING_BWD = 4
LSQ_OP_BDR_LAYERNORM_BWD = 5
LSQ_ACT = {"relu": 0, "gelu": 1, "gelu_tanh": 2}
_DT = {torch.float16: LSQ_F16, torch.bfloat16: LSQ_BF16, torch.float32: LSQ_F32}

EXPORTS = [
    "lsq_workspace_bytes", "lsq_status_string", "lsq_layernorm_fwd", "lsq_layernorm_bwd", "lsq_layernorm_bwd_noalloc",
    "lsq_bias_dropout_residual_fwd", "lsq_bias_dropout_residual_bwd", "lsq_softmax_fwd", "lsq_softmax_bwd",
    "lsq_ls_xent_fwd", "lsq_ls_xent_bwd", "lsq_ls_xent_fwd_bwd", "lsq_adam_step",
    "lsq_bias_act_dropout_fwd", "lsq_bias_act_dropout_bwd", "lsq_adam_step_lp", "lsq_sgd_step",
    "lsq_split_heads_fwd", "lsq_split_heads_bwd", "lsq_merge_heads_fwd", "lsq_merge_heads_bwd",
    "lsq_embedding_fwd", "lsq_embedding_bwd",
    "lsq_bdr_layernorm_fwd", "lsq_bdr_layernorm_bwd",
    "lsq_adam_state_bytes", "lsq_adam_state_pack", "lsq_adam_state_unpack", "lsq_adam_step_blocked",
    "lsq_trainer_state_bytes", "lsq_trainer_state_pack", "lsq_trainer_state_unpack", "lsq_sgd_step_blocked",
    "lsq_adam_step_lp_blocked",
    "lsq_pad_offsets", "lsq_pad_remove", "lsq_pad_restore", "lsq_softmax_varlen_fwd", "lsq_softmax_varlen_bwd",
    "lsq_calib_stream", "lsq_softmax_candidates", "lsq_softmax_tune",
]


class LsqError(RuntimeError):
    pass


def lib_path() -> str:
    return _LIB_PATH


def load():
    """Load liblsq.so (built by `python -m paper_2110_05722_amd.build`).  Raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise LsqError(f"{_LIB_PATH} is missing: build it with `python -m paper_2110_05722_amd.build` "
                       "(there is no fallback path)")
    lib = C.CDLL(_LIB_PATH)
    vp, i32, i64, u64, f32, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_float, C.c_size_t
    sig = {
        "lsq_workspace_bytes": (sz, [i32, i64, i32]),
        "lsq_status_string": (C.c_char_p, [C.c_int]),
        "lsq_layernorm_fwd": (C.c_int, [vp, vp, vp, vp, vp, vp, i64, i32, f32, C.c_int, vp]),
        "lsq_layernorm_bwd": (C.c_int, [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, i64, i32, C.c_int, vp]),
        "lsq_layernorm_bwd_noalloc": (C.c_int, [vp, vp, vp, vp, vp, vp, vp, vp, vp, i64, i32, C.c_int, vp]),
        "lsq_calib_stream": (C.c_int, [i32, vp, vp, i64, vp]),
        "lsq_softmax_candidates": (i32, [i32]),
        "lsq_softmax_tune": (C.c_int, [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, f32, f32, u64, u64,
                                       C.c_int, i32, i32, vp]),
        "lsq_bias_dropout_residual_fwd": (C.c_int, [vp, vp, vp, vp, i64, i32, f32, u64, u64, C.c_int, vp]),
        "lsq_bias_dropout_residual_bwd": (C.c_int, [vp, vp, vp, i64, i32, f32, u64, u64, vp, sz, C.c_int, vp]),
        "lsq_softmax_fwd": (C.c_int, [vp, vp, vp, vp, i32, i32, i32, i32, i32, f32, f32, u64, u64, C.c_int, vp]),
        "lsq_softmax_bwd": (C.c_int, [vp, vp, vp, vp, i32, i32, i32, i32, i32, f32, f32, u64, u64, C.c_int, vp]),
        "lsq_ls_xent_fwd": (C.c_int, [vp, vp, vp, vp, vp, vp, i64, i32, f32, i32, C.c_int, vp]),
        "lsq_ls_xent_bwd": (C.c_int, [vp, vp, vp, vp, i64, i32, f32, i32, f32, C.c_int, vp]),
        "lsq_ls_xent_fwd_bwd": (C.c_int, [vp, vp, vp, vp, vp, vp, vp, i64, i32, f32, i32, f32, C.c_int, vp]),
        "lsq_adam_step": (C.c_int, [vp, vp, vp, vp, vp, i64, f32, f32, f32, f32, f32, i32, i32, i32, f32,
                                    C.c_int, C.c_int, vp]),
        "lsq_bias_act_dropout_fwd": (C.c_int, [vp, vp, vp, i64, i32, i32, f32, u64, u64, C.c_int, vp]),
        "lsq_bias_act_dropout_bwd": (C.c_int, [vp, vp, vp, vp, vp, i64, i32, i32, f32, u64, u64, vp, sz, C.c_int, vp]),
        "lsq_adam_step_lp": (C.c_int, [vp, vp, vp, vp, i64, f32, f32, f32, f32, f32, i32, i32, i32, f32, C.c_int, vp]),
        "lsq_sgd_step": (C.c_int, [vp, vp, vp, vp, i64, f32, f32, f32, i32, f32, C.c_int, C.c_int, vp]),
        "lsq_split_heads_fwd": (C.c_int, [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, C.c_int, vp]),
        "lsq_split_heads_bwd": (C.c_int, [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, vp, sz, C.c_int, vp]),
        "lsq_merge_heads_fwd": (C.c_int, [vp, vp, i32, i32, i32, i32, C.c_int, vp]),
        "lsq_merge_heads_bwd": (C.c_int, [vp, vp, i32, i32, i32, i32, C.c_int, vp]),
        "lsq_embedding_fwd": (C.c_int, [vp, vp, vp, vp, i32, i32, i32, i32, i32, f32, f32, u64, u64, C.c_int, vp]),
        "lsq_embedding_bwd": (C.c_int, [vp, vp, vp, vp, i32, i32, i32, i32, i32, f32, f32, u64, u64, vp, sz, C.c_int, vp]),
        "lsq_bdr_layernorm_fwd": (C.c_int, [vp, vp, vp, vp, vp, vp, vp, vp, vp, i64, i32, f32, u64, u64, f32, C.c_int, vp]),
        "lsq_bdr_layernorm_bwd": (C.c_int, [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, i64, i32, f32, u64, u64,
                                             C.c_int, vp]),
        "lsq_adam_state_bytes": (sz, [i64]),
        "lsq_adam_state_pack": (C.c_int, [vp, vp, vp, vp, i64, vp]),
        "lsq_adam_state_unpack": (C.c_int, [vp, vp, vp, vp, i64, vp]),
        "lsq_adam_step_blocked": (C.c_int, [vp, vp, vp, i64, f32, f32, f32, f32, f32, i32, i32, i32, f32, C.c_int, C.c_int, vp]),
        "lsq_trainer_state_bytes": (sz, [i64, i32]),
        "lsq_trainer_state_pack": (C.c_int, [vp, vp, vp, vp, i64, i32, vp]),
        "lsq_trainer_state_unpack": (C.c_int, [vp, vp, vp, vp, i64, i32, vp]),
        "lsq_sgd_step_blocked": (C.c_int, [vp, vp, vp, i64, f32, f32, f32, i32, f32, C.c_int, C.c_int, vp]),
        "lsq_adam_step_lp_blocked": (C.c_int, [vp, vp, vp, i64, f32, f32, f32, f32, f32, i32, i32, i32, f32, C.c_int, vp]),
        "lsq_pad_offsets": (C.c_int, [vp, vp, i32, i32, vp]),
        "lsq_pad_remove": (C.c_int, [vp, vp, vp, i32, i32, i32, i64, C.c_int, vp]),
        "lsq_pad_restore": (C.c_int, [vp, vp, vp, i32, i32, i32, i64, C.c_int, vp]),
        "lsq_softmax_varlen_fwd": (C.c_int, [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, f32, f32, u64, u64, C.c_int, vp]),
        "lsq_softmax_varlen_bwd": (C.c_int, [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, f32, f32, u64, u64, C.c_int, vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


def lsq_status_string(code: int) -> str:
    return load().lsq_status_string(code).decode()


def lsq_workspace_bytes(op: int, rows: int, cols: int) -> int:
    return int(load().lsq_workspace_bytes(op, rows, cols))


def _check(code: int, name: str):
    if code != 0:
        raise LsqError(f"{name} failed: {lsq_status_string(code)}")


def _ptr(t):
    if t is None:
        return None
    if not t.is_cuda:
        raise LsqError("tensors must live on the GPU (there is no CPU path)")
    if not t.is_contiguous():
        raise LsqError("tensors must be contiguous")
    return C.c_void_p(t.data_ptr())


def _dt(t) -> int:
    try:
        return _DT[t.dtype]
    except KeyError:
        raise LsqError(f"unsupported dtype {t.dtype}") from None


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _need(name: str, t, numel: int, dtype=None):
    """The library takes bare pointers: a tensor shorter than what the kernel will touch is refused here."""
    if t is None:
        return
    if t.numel() < numel:
        raise LsqError(f"{name} holds {t.numel()} elements, the call needs {numel}")
    if dtype is not None and t.dtype != dtype:
        raise LsqError(f"{name} is {t.dtype}, expected {dtype}")


def _workspace(nbytes: int, like, ws):
    if ws is not None:
        return ws
    return torch.empty(max(nbytes, 16), dtype=torch.uint8, device=like.device)


# ---------------------------------------------------------------------------
def lsq_layernorm_fwd(x, gamma, beta, eps: float = 1e-5, y=None, mean=None, rstd=None):
    """x: [rows, hidden] -> (y, mean[rows] fp32, rstd[rows] fp32)."""
    rows, hidden = x.shape
    y = torch.empty_like(x) if y is None else y
    mean = torch.empty(rows, dtype=torch.float32, device=x.device) if mean is None else mean
    rstd = torch.empty(rows, dtype=torch.float32, device=x.device) if rstd is None else rstd
    _need("y", y, rows * hidden, x.dtype); _need("gamma", gamma, hidden, x.dtype); _need("beta", beta, hidden, x.dtype)
    _need("mean", mean, rows, torch.float32); _need("rstd", rstd, rows, torch.float32)
    _check(load().lsq_layernorm_fwd(_ptr(y), _ptr(mean), _ptr(rstd), _ptr(x), _ptr(gamma), _ptr(beta), rows, hidden,
                                    eps, _dt(x), _stream()), "lsq_layernorm_fwd")
    return y, mean, rstd


def lsq_layernorm_bwd(dy, x, gamma, mean, rstd, dres_in=None, dx=None, dgamma=None, dbeta=None, workspace=None):
    """-> (dx, dgamma[hidden] fp32, dbeta[hidden] fp32)."""
    rows, hidden = x.shape
    dx = torch.empty_like(x) if dx is None else dx
    dgamma = torch.empty(hidden, dtype=torch.float32, device=x.device) if dgamma is None else dgamma
    dbeta = torch.empty(hidden, dtype=torch.float32, device=x.device) if dbeta is None else dbeta
    ws = _workspace(lsq_workspace_bytes(LSQ_OP_LAYERNORM_BWD, rows, hidden), x, workspace)
    for name, t in (("dy", dy), ("dx", dx), ("dres_in", dres_in)):
        _need(name, t, rows * hidden, x.dtype)
    _need("gamma", gamma, hidden, x.dtype)
    for name, t, k in (("mean", mean, rows), ("rstd", rstd, rows), ("dgamma", dgamma, hidden), ("dbeta", dbeta, hidden)):
        _need(name, t, k, torch.float32)
    _check(load().lsq_layernorm_bwd(_ptr(dx), _ptr(dgamma), _ptr(dbeta), _ptr(dy), _ptr(x), _ptr(gamma), _ptr(mean),
                                    _ptr(rstd), _ptr(dres_in), _ptr(ws), ws.numel() * ws.element_size(), rows, hidden,
                                    _dt(x), _stream()), "lsq_layernorm_bwd")
    return dx, dgamma, dbeta


def lsq_layernorm_bwd_noalloc(dy, x, gamma, mean, rstd, dx, dgamma, dbeta, dres_in=None):
    """LayerNorm backward into caller-supplied outputs, scratch held by the library: the call allocates nothing."""
    rows, hidden = x.shape
    for name, t in (("dy", dy), ("dx", dx), ("dres_in", dres_in)):
        _need(name, t, rows * hidden, x.dtype)
    _need("gamma", gamma, hidden, x.dtype)
    for name, t, k in (("mean", mean, rows), ("rstd", rstd, rows), ("dgamma", dgamma, hidden), ("dbeta", dbeta, hidden)):
        _need(name, t, k, torch.float32)
    _check(load().lsq_layernorm_bwd_noalloc(_ptr(dx), _ptr(dgamma), _ptr(dbeta), _ptr(dy), _ptr(x), _ptr(gamma), _ptr(mean),
                                            _ptr(rstd), _ptr(dres_in), rows, hidden, _dt(x), _stream()),
           "lsq_layernorm_bwd_noalloc")
    return dx, dgamma, dbeta


def lsq_bias_dropout_residual_fwd(x, bias, residual, p: float, seed: int, offset: int, out=None):
    rows, hidden = x.shape
    out = torch.empty_like(x) if out is None else out
    _need("out", out, rows * hidden, x.dtype); _need("residual", residual, rows * hidden, x.dtype)
    _need("bias", bias, hidden, x.dtype)
    _check(load().lsq_bias_dropout_residual_fwd(_ptr(out), _ptr(x), _ptr(bias), _ptr(residual), rows, hidden, p, seed,
                                                offset, _dt(x), _stream()), "lsq_bias_dropout_residual_fwd")
    return out


def lsq_bias_dropout_residual_bwd(dy, p: float, seed: int, offset: int, want_dbias: bool = True, dx=None, dbias=None,
                                  workspace=None):
    """-> (dx, dbias[hidden] fp32 or None)."""
    rows, hidden = dy.shape
    dx = torch.empty_like(dy) if dx is None else dx
    if want_dbias and dbias is None:
        dbias = torch.empty(hidden, dtype=torch.float32, device=dy.device)
    ws = _workspace(lsq_workspace_bytes(LSQ_OP_BIAS_DROPOUT_RESIDUAL_BWD, rows, hidden), dy, workspace)
    _need("dx", dx, rows * hidden, dy.dtype); _need("dbias", dbias, hidden, torch.float32)
    _check(load().lsq_bias_dropout_residual_bwd(_ptr(dx), _ptr(dbias) if want_dbias else None, _ptr(dy), rows, hidden,
                                                p, seed, offset, _ptr(ws), ws.numel() * ws.element_size(), _dt(dy),
                                                _stream()), "lsq_bias_dropout_residual_bwd")
    return dx, (dbias if want_dbias else None)


def lsq_softmax_fwd(x, key_len=None, causal: bool = False, scale: float = 1.0, p_attn: float = 0.0, seed: int = 0,
                    offset: int = 0, y=None, y_drop=None):
    """x: [batch, heads, q_len, k_len]; key_len: int32[batch] or None -> (y, y_drop or None)."""
    B, N, Lq, Lk = x.shape
    y = torch.empty_like(x) if y is None else y
    if p_attn > 0 and y_drop is None:
        y_drop = torch.empty_like(x)
    _need("y", y, x.numel(), x.dtype); _need("y_drop", y_drop, x.numel(), x.dtype)
    _need("key_len", key_len, B, torch.int32)
    _check(load().lsq_softmax_fwd(_ptr(y), _ptr(y_drop) if p_attn > 0 else None, _ptr(x), _ptr(key_len), B, N, Lq, Lk,
                                  int(causal), scale, p_attn, seed, offset, _dt(x), _stream()), "lsq_softmax_fwd")
    return y, (y_drop if p_attn > 0 else None)


def lsq_softmax_bwd(dy, y, key_len=None, causal: bool = False, scale: float = 1.0, p_attn: float = 0.0, seed: int = 0,
                    offset: int = 0, dx=None):
    B, N, Lq, Lk = y.shape
    dx = torch.empty_like(y) if dx is None else dx
    _need("dx", dx, y.numel(), y.dtype); _need("dy", dy, y.numel(), y.dtype); _need("key_len", key_len, B, torch.int32)
    _check(load().lsq_softmax_bwd(_ptr(dx), _ptr(dy), _ptr(y), _ptr(key_len), B, N, Lq, Lk, int(causal), scale, p_attn,
                                  seed, offset, _dt(y), _stream()), "lsq_softmax_bwd")
    return dx


def lsq_ls_xent_fwd(logits, target, alpha: float, ignore_index: int = -100, want_sums: bool = True,
                    want_nll: bool = True, loss=None, nll=None, lse=None, sums=None):
    """logits: [tokens, vocab]; target: int32[tokens] -> (loss[tokens], nll[tokens] or None, lse[tokens],
    sums[3] or None), all fp32."""
    T, V = logits.shape
    loss = torch.empty(T, dtype=torch.float32, device=logits.device) if loss is None else loss
    lse = torch.empty(T, dtype=torch.float32, device=logits.device) if lse is None else lse
    if want_nll and nll is None:
        nll = torch.empty(T, dtype=torch.float32, device=logits.device)
    if want_sums and sums is None:
        sums = torch.empty(3, dtype=torch.float32, device=logits.device)
    _need("target", target, T, torch.int32)
    for name, t, k in (("loss", loss, T), ("nll", nll, T), ("lse", lse, T), ("sums", sums, 3)):
        _need(name, t, k, torch.float32)
    _check(load().lsq_ls_xent_fwd(_ptr(loss), _ptr(nll) if want_nll else None, _ptr(lse),
                                  _ptr(sums) if want_sums else None, _ptr(logits), _ptr(target), T, V, alpha,
                                  ignore_index, _dt(logits), _stream()), "lsq_ls_xent_fwd")
    return loss, (nll if want_nll else None), lse, (sums if want_sums else None)


def lsq_ls_xent_bwd(logits, lse, target, alpha: float, ignore_index: int = -100, grad_scale: float = 1.0,
                    dlogits=None):
    T, V = logits.shape
    dlogits = torch.empty_like(logits) if dlogits is None else dlogits
    _need("target", target, T, torch.int32); _need("lse", lse, T, torch.float32)
    _need("dlogits", dlogits, T * V, logits.dtype)
    _check(load().lsq_ls_xent_bwd(_ptr(dlogits), _ptr(logits), _ptr(lse), _ptr(target), T, V, alpha, ignore_index,
                                  grad_scale, _dt(logits), _stream()), "lsq_ls_xent_bwd")
    return dlogits


def lsq_ls_xent_fwd_bwd(logits, target, alpha: float, ignore_index: int = -100, grad_scale: float = 1.0,
                        want_sums: bool = True, want_nll: bool = True, loss=None, nll=None, lse=None, sums=None,
                        dlogits=None):
    """Forward and backward in one pass -> (loss, nll or None, lse, sums or None, dlogits).  dlogits may be
    `logits` itself (in place)."""
    T, V = logits.shape
    loss = torch.empty(T, dtype=torch.float32, device=logits.device) if loss is None else loss
    lse = torch.empty(T, dtype=torch.float32, device=logits.device) if lse is None else lse
    if want_nll and nll is None:
        nll = torch.empty(T, dtype=torch.float32, device=logits.device)
    if want_sums and sums is None:
        sums = torch.empty(3, dtype=torch.float32, device=logits.device)
    dlogits = torch.empty_like(logits) if dlogits is None else dlogits
    _need("target", target, T, torch.int32)
    for name, t, k in (("loss", loss, T), ("nll", nll, T), ("lse", lse, T), ("sums", sums, 3)):
        _need(name, t, k, torch.float32)
    _need("dlogits", dlogits, T * V, logits.dtype)
    _check(load().lsq_ls_xent_fwd_bwd(_ptr(loss), _ptr(nll) if want_nll else None, _ptr(lse),
                                      _ptr(sums) if want_sums else None, _ptr(dlogits), _ptr(logits), _ptr(target), T, V,
                                      alpha, ignore_index, grad_scale, _dt(logits), _stream()), "lsq_ls_xent_fwd_bwd")
    return loss, (nll if want_nll else None), lse, (sums if want_sums else None), dlogits


def lsq_adam_step(p, m, v, g, p_lp=None, *, lr: float, beta1: float, beta2: float, eps: float, step: int,
                  weight_decay: float = 0.0, adamw: bool = False, bias_correction: bool = True,
                  inv_grad_scale: float = 1.0):
    """In place on fp32 p, m, v (flat); g low precision (or fp32); p_lp optional low-precision copy out."""
    for t in (p, m, v):
        if t.dtype != torch.float32:
            raise LsqError("p, m, v must be fp32")
    n = p.numel()
    _need("m", m, n); _need("v", v, n); _need("g", g, n); _need("p_lp", p_lp, n)
    _check(load().lsq_adam_step(_ptr(p), _ptr(m), _ptr(v), _ptr(g), _ptr(p_lp), n, lr, beta1, beta2, eps, weight_decay,
                                step, int(adamw), int(bias_correction), inv_grad_scale, _dt(g),
                                _dt(p_lp) if p_lp is not None else LSQ_F16, _stream()), "lsq_adam_step")
    return p, m, v, p_lp


def lsq_bias_act_dropout_fwd(x, bias, act: str, p: float, seed: int, offset: int, out=None):
    """out = Dropout_p(act(x + bias)); act in {"relu", "gelu", "gelu_tanh"}."""
    rows, hidden = x.shape
    out = torch.empty_like(x) if out is None else out
    _need("out", out, rows * hidden, x.dtype); _need("bias", bias, hidden, x.dtype)
    _check(load().lsq_bias_act_dropout_fwd(_ptr(out), _ptr(x), _ptr(bias), rows, hidden, LSQ_ACT[act], p, seed, offset,
                                           _dt(x), _stream()), "lsq_bias_act_dropout_fwd")
    return out


def lsq_bias_act_dropout_bwd(dy, x, bias, act: str, p: float, seed: int, offset: int, want_dbias: bool = True, dx=None,
                             dbias=None, workspace=None):
    """-> (dx, dbias[hidden] fp32 or None)."""
    rows, hidden = x.shape
    dx = torch.empty_like(x) if dx is None else dx
    if want_dbias and dbias is None:
        dbias = torch.empty(hidden, dtype=torch.float32, device=x.device)
    ws = _workspace(lsq_workspace_bytes(LSQ_OP_BIAS_ACT_DROPOUT_BWD, rows, hidden), x, workspace)
    _need("dy", dy, rows * hidden, x.dtype); _need("dx", dx, rows * hidden, x.dtype)
    _need("bias", bias, hidden, x.dtype); _need("dbias", dbias, hidden, torch.float32)
    _check(load().lsq_bias_act_dropout_bwd(_ptr(dx), _ptr(dbias) if want_dbias else None, _ptr(dy), _ptr(x), _ptr(bias),
                                           rows, hidden, LSQ_ACT[act], p, seed, offset, _ptr(ws),
                                           ws.numel() * ws.element_size(), _dt(x), _stream()), "lsq_bias_act_dropout_bwd")
    return dx, (dbias if want_dbias else None)


def lsq_adam_step_lp(p_lp, m, v, g, *, lr: float, beta1: float, beta2: float, eps: float, step: int,
                     weight_decay: float = 0.0, adamw: bool = False, bias_correction: bool = True,
                     inv_grad_scale: float = 1.0):
    """In place on the low-precision p_lp and fp32 m, v (flat); g in the same low precision."""
    if g.dtype != p_lp.dtype:
        raise LsqError("g and p_lp must share one low-precision dtype")
    _need("m", m, p_lp.numel(), torch.float32); _need("v", v, p_lp.numel(), torch.float32); _need("g", g, p_lp.numel())
    _check(load().lsq_adam_step_lp(_ptr(p_lp), _ptr(m), _ptr(v), _ptr(g), p_lp.numel(), lr, beta1, beta2, eps,
                                   weight_decay, step, int(adamw), int(bias_correction), inv_grad_scale, _dt(p_lp),
                                   _stream()), "lsq_adam_step_lp")
    return p_lp, m, v


def lsq_sgd_step(p, momentum_buf, g, p_lp=None, *, lr: float, momentum: float = 0.0, weight_decay: float = 0.0,
                 nesterov: bool = False, inv_grad_scale: float = 1.0):
    """In place on fp32 p (and momentum_buf if momentum > 0); p_lp optional low-precision copy out."""
    if p.dtype != torch.float32:
        raise LsqError("p must be fp32")
    _need("momentum_buf", momentum_buf, p.numel(), torch.float32); _need("g", g, p.numel()); _need("p_lp", p_lp, p.numel())
    _check(load().lsq_sgd_step(_ptr(p), _ptr(momentum_buf), _ptr(g), _ptr(p_lp), p.numel(), lr, momentum, weight_decay,
                               int(nesterov), inv_grad_scale, _dt(g), _dt(p_lp) if p_lp is not None else LSQ_F16,
                               _stream()), "lsq_sgd_step")
    return p, momentum_buf, p_lp


def lsq_split_heads_fwd(x, bias, batch: int, length: int, heads: int, head_dim: int, parts: int, outs=None):
    """x: [batch*len, parts*heads*head_dim] (+ bias) -> list of `parts` tensors [batch, heads, len, head_dim]."""
    if outs is None:
        outs = [torch.empty((batch, heads, length, head_dim), dtype=x.dtype, device=x.device) for _ in range(parts)]
    hidden = heads * head_dim
    _need("x", x, batch * length * parts * hidden); _need("bias", bias, parts * hidden, x.dtype)
    if len(outs) < parts:
        raise LsqError(f"{parts} parts need {parts} output tensors")
    for o in outs[:parts]:
        _need("out", o, batch * length * hidden, x.dtype)
    ptrs = [_ptr(o) for o in outs[:parts]] + [None] * (3 - parts)
    _check(load().lsq_split_heads_fwd(ptrs[0], ptrs[1], ptrs[2], _ptr(x), _ptr(bias), batch, length, heads, head_dim,
                                      parts, _dt(x), _stream()), "lsq_split_heads_fwd")
    return outs


def lsq_split_heads_bwd(grads, batch: int, length: int, heads: int, head_dim: int, want_dbias: bool = True, din=None,
                        dbias=None, workspace=None):
    """grads: list of `parts` tensors [batch, heads, len, head_dim] -> (din [batch*len, parts*hidden], dbias or None)."""
    parts = len(grads)
    cols = parts * heads * head_dim
    g0 = grads[0]
    din = torch.empty((batch * length, cols), dtype=g0.dtype, device=g0.device) if din is None else din
    if want_dbias and dbias is None:
        dbias = torch.empty(cols, dtype=torch.float32, device=g0.device)
    ws = _workspace(lsq_workspace_bytes(LSQ_OP_SPLIT_HEADS_BWD, batch * length, cols), g0, workspace)
    if not 1 <= parts <= 3:
        raise LsqError("1 to 3 parts")
    for g in grads:
        _need("grad", g, batch * length * heads * head_dim, g0.dtype)
    _need("din", din, batch * length * cols, g0.dtype); _need("dbias", dbias, cols, torch.float32)
    ptrs = [_ptr(g) for g in grads] + [None] * (3 - parts)
    _check(load().lsq_split_heads_bwd(_ptr(din), _ptr(dbias) if want_dbias else None, ptrs[0], ptrs[1], ptrs[2], batch,
                                      length, heads, head_dim, parts, _ptr(ws), ws.numel() * ws.element_size(), _dt(g0),
                                      _stream()), "lsq_split_heads_bwd")
    return din, (dbias if want_dbias else None)


def lsq_merge_heads_fwd(x, out=None):
    """x: [batch, heads, len, head_dim] -> [batch*len, heads*head_dim]."""
    B, N, Ln, D = x.shape
    out = torch.empty((B * Ln, N * D), dtype=x.dtype, device=x.device) if out is None else out
    _need("out", out, x.numel(), x.dtype)
    _check(load().lsq_merge_heads_fwd(_ptr(out), _ptr(x), B, Ln, N, D, _dt(x), _stream()), "lsq_merge_heads_fwd")
    return out


def lsq_merge_heads_bwd(dy, batch: int, length: int, heads: int, head_dim: int, dx=None):
    """dy: [batch*len, heads*head_dim] -> [batch, heads, len, head_dim]."""
    dx = torch.empty((batch, heads, length, head_dim), dtype=dy.dtype, device=dy.device) if dx is None else dx
    _need("dy", dy, batch * heads * length * head_dim); _need("dx", dx, batch * heads * length * head_dim, dy.dtype)
    _check(load().lsq_merge_heads_bwd(_ptr(dx), _ptr(dy), batch, length, heads, head_dim, _dt(dy), _stream()),
           "lsq_merge_heads_bwd")
    return dx


def lsq_embedding_fwd(tokens, emb, pos, pad_idx: int, scale: float, p: float, seed: int, offset: int, out=None):
    """tokens: int32 [batch, len]; emb: [vocab, hidden]; pos: [>= len, hidden] -> out [batch*len, hidden]."""
    if tokens.dtype != torch.int32:
        raise LsqError("tokens must be int32")
    B, Ln = tokens.shape
    V, H = emb.shape
    out = torch.empty((B * Ln, H), dtype=emb.dtype, device=emb.device) if out is None else out
    _need("out", out, B * Ln * H, emb.dtype); _need("pos", pos, Ln * H, emb.dtype)
    if pos.shape[-1] != H:
        raise LsqError("pos must be [>= len, hidden]")
    _check(load().lsq_embedding_fwd(_ptr(out), _ptr(tokens), _ptr(emb), _ptr(pos), B, Ln, H, V, pad_idx, scale, p, seed,
                                    offset, _dt(emb), _stream()), "lsq_embedding_fwd")
    return out


def lsq_embedding_bwd(demb, dpos, dy, tokens, pad_idx: int, scale: float, p: float, seed: int, offset: int,
                      workspace=None):
    """Accumulates into demb [vocab, hidden] and (if not None) dpos [len, hidden]."""
    if tokens.dtype != torch.int32:
        raise LsqError("tokens must be int32")
    B, Ln = tokens.shape
    V, H = demb.shape
    ws = _workspace(lsq_workspace_bytes(LSQ_OP_EMBEDDING_BWD, B * Ln, H), dy, workspace)
    _need("dy", dy, B * Ln * H, demb.dtype); _need("dpos", dpos, Ln * H, demb.dtype)
    _check(load().lsq_embedding_bwd(_ptr(demb), _ptr(dpos), _ptr(dy), _ptr(tokens), B, Ln, H, V, pad_idx, scale, p, seed,
                                    offset, _ptr(ws), ws.numel() * ws.element_size(), _dt(demb), _stream()),
           "lsq_embedding_bwd")
    return demb, dpos


def lsq_bdr_layernorm_fwd(x, bias, residual, gamma, beta, p: float, seed: int, offset: int, eps: float = 1e-5,
                          h=None, y=None, mean=None, rstd=None):
    """h = residual + Dropout(x + bias); y = LayerNorm(h), one pass -> (h, y, mean, rstd)."""
    rows, hidden = x.shape
    h = torch.empty_like(x) if h is None else h
    y = torch.empty_like(x) if y is None else y
    mean = torch.empty(rows, dtype=torch.float32, device=x.device) if mean is None else mean
    rstd = torch.empty(rows, dtype=torch.float32, device=x.device) if rstd is None else rstd
    for name, t in (("h", h), ("y", y), ("residual", residual)):
        _need(name, t, rows * hidden, x.dtype)
    for name, t in (("bias", bias), ("gamma", gamma), ("beta", beta)):
        _need(name, t, hidden, x.dtype)
    _need("mean", mean, rows, torch.float32); _need("rstd", rstd, rows, torch.float32)
    _check(load().lsq_bdr_layernorm_fwd(_ptr(h), _ptr(y), _ptr(mean), _ptr(rstd), _ptr(x), _ptr(bias), _ptr(residual),
                                        _ptr(gamma), _ptr(beta), rows, hidden, p, seed, offset, eps, _dt(x), _stream()),
           "lsq_bdr_layernorm_fwd")
    return h, y, mean, rstd


def lsq_bdr_layernorm_bwd(dy, h, gamma, mean, rstd, p: float, seed: int, offset: int, dres_in=None, dh=None, dx=None,
                          dgamma=None, dbeta=None, dbias=None, workspace=None):
    """Backward of lsq_bdr_layernorm_fwd -> (dh, dx, dgamma, dbeta, dbias)."""
    rows, hidden = h.shape
    dh = torch.empty_like(h) if dh is None else dh
    dx = torch.empty_like(h) if dx is None else dx
    mk = lambda t: torch.empty(hidden, dtype=torch.float32, device=h.device) if t is None else t
    dgamma, dbeta, dbias = mk(dgamma), mk(dbeta), mk(dbias)
    ws = _workspace(lsq_workspace_bytes(LSQ_OP_BDR_LAYERNORM_BWD, rows, hidden), h, workspace)
    for name, t in (("dy", dy), ("dh", dh), ("dx", dx), ("dres_in", dres_in)):
        _need(name, t, rows * hidden, h.dtype)
    _need("gamma", gamma, hidden, h.dtype)
    for name, t, k in (("mean", mean, rows), ("rstd", rstd, rows), ("dgamma", dgamma, hidden), ("dbeta", dbeta, hidden),
                       ("dbias", dbias, hidden)):
        _need(name, t, k, torch.float32)
    _check(load().lsq_bdr_layernorm_bwd(_ptr(dh), _ptr(dx), _ptr(dgamma), _ptr(dbeta), _ptr(dbias), _ptr(dy), _ptr(h),
                                        _ptr(gamma), _ptr(mean), _ptr(rstd), _ptr(dres_in), _ptr(ws),
                                        ws.numel() * ws.element_size(), rows, hidden, p, seed, offset, _dt(h), _stream()),
           "lsq_bdr_layernorm_bwd")
    return dh, dx, dgamma, dbeta, dbias


LSQ_ADAM_BLOCK = 8192


def lsq_adam_state_bytes(n: int) -> int:
    return int(load().lsq_adam_state_bytes(n))


def lsq_adam_state_pack(p, m=None, v=None, state=None):
    """fp32 p (and m, v; None = zeros) -> blocked optimizer state (fp32, lsq_adam_state_bytes(n) bytes)."""
    n = p.numel()
    need = lsq_adam_state_bytes(n) // 4
    state = torch.empty(need, dtype=torch.float32, device=p.device) if state is None else state
    _need("state", state, need, torch.float32); _need("p", p, n, torch.float32)
    _need("m", m, n, torch.float32); _need("v", v, n, torch.float32)
    _check(load().lsq_adam_state_pack(_ptr(state), _ptr(p), _ptr(m), _ptr(v), n, _stream()), "lsq_adam_state_pack")
    return state


def lsq_adam_state_unpack(state, n: int, p=None, m=None, v=None, want=("p", "m", "v")):
    """Blocked optimizer state -> (p, m, v) fp32[n]; entries not in `want` (and not passed) come back as None."""
    dev = state.device
    p = torch.empty(n, dtype=torch.float32, device=dev) if p is None and "p" in want else p
    m = torch.empty(n, dtype=torch.float32, device=dev) if m is None and "m" in want else m
    v = torch.empty(n, dtype=torch.float32, device=dev) if v is None and "v" in want else v
    _need("state", state, lsq_adam_state_bytes(n) // 4, torch.float32)
    for name, t in (("p", p), ("m", m), ("v", v)):
        _need(name, t, n, torch.float32)
    _check(load().lsq_adam_state_unpack(_ptr(p), _ptr(m), _ptr(v), _ptr(state), n, _stream()), "lsq_adam_state_unpack")
    return p, m, v


def lsq_adam_step_blocked(state, g, p_lp=None, *, lr: float, beta1: float, beta2: float, eps: float, step: int,
                          weight_decay: float = 0.0, adamw: bool = False, bias_correction: bool = True,
                          inv_grad_scale: float = 1.0):
    """lsq_adam_step on the blocked state (in place); g [n] low precision or fp32; p_lp optional copy out."""
    n = g.numel()
    _need("state", state, lsq_adam_state_bytes(n) // 4, torch.float32); _need("p_lp", p_lp, n)
    _check(load().lsq_adam_step_blocked(_ptr(state), _ptr(g), _ptr(p_lp), n, lr, beta1, beta2, eps, weight_decay, step,
                                        int(adamw), int(bias_correction), inv_grad_scale, _dt(g),
                                        _dt(p_lp) if p_lp is not None else LSQ_F16, _stream()), "lsq_adam_step_blocked")
    return state, p_lp


def lsq_trainer_state_bytes(n: int, arrays: int) -> int:
    return int(load().lsq_trainer_state_bytes(n, arrays))


def lsq_trainer_state_pack(arrays_in, state=None):
    """List of 1..3 fp32 tensors [n] (entries after the first may be None = zeros) -> blocked state."""
    k = len(arrays_in)
    a0 = arrays_in[0]
    n = a0.numel()
    need = lsq_trainer_state_bytes(n, k) // 4
    state = torch.empty(need, dtype=torch.float32, device=a0.device) if state is None else state
    _need("state", state, need, torch.float32)
    for t in arrays_in:
        _need("array", t, n, torch.float32)
    ptrs = [_ptr(t) for t in arrays_in] + [None] * (3 - k)
    _check(load().lsq_trainer_state_pack(_ptr(state), ptrs[0], ptrs[1], ptrs[2], n, k, _stream()), "lsq_trainer_state_pack")
    return state


def lsq_trainer_state_unpack(state, n: int, arrays: int):
    """Blocked state -> list of `arrays` fp32 tensors [n]."""
    _need("state", state, lsq_trainer_state_bytes(n, arrays) // 4, torch.float32)
    outs = [torch.empty(n, dtype=torch.float32, device=state.device) for _ in range(arrays)]
    ptrs = [_ptr(t) for t in outs] + [None] * (3 - arrays)
    _check(load().lsq_trainer_state_unpack(ptrs[0], ptrs[1], ptrs[2], _ptr(state), n, arrays, _stream()),
           "lsq_trainer_state_unpack")
    return outs


def lsq_sgd_step_blocked(state, g, p_lp=None, *, lr: float, momentum: float = 0.0, weight_decay: float = 0.0,
                         nesterov: bool = False, inv_grad_scale: float = 1.0):
    """lsq_sgd_step on the [p | momentum buffer] blocked state (in place)."""
    n = g.numel()
    _need("state", state, lsq_trainer_state_bytes(n, 2) // 4, torch.float32); _need("p_lp", p_lp, n)
    _check(load().lsq_sgd_step_blocked(_ptr(state), _ptr(g), _ptr(p_lp), n, lr, momentum, weight_decay, int(nesterov),
                                       inv_grad_scale, _dt(g), _dt(p_lp) if p_lp is not None else LSQ_F16, _stream()),
           "lsq_sgd_step_blocked")
    return state, p_lp


def lsq_adam_step_lp_blocked(p_lp, state, g, *, lr: float, beta1: float, beta2: float, eps: float, step: int,
                             weight_decay: float = 0.0, adamw: bool = False, bias_correction: bool = True,
                             inv_grad_scale: float = 1.0):
    """lsq_adam_step_lp with the moments in the [m | v] blocked state (p_lp and the state in place)."""
    if g.dtype != p_lp.dtype:
        raise LsqError("g and p_lp must share one low-precision dtype")
    n = p_lp.numel()
    _need("state", state, lsq_trainer_state_bytes(n, 2) // 4, torch.float32); _need("g", g, n)
    _check(load().lsq_adam_step_lp_blocked(_ptr(p_lp), _ptr(state), _ptr(g), n, lr, beta1, beta2, eps, weight_decay, step,
                                           int(adamw), int(bias_correction), inv_grad_scale, _dt(p_lp), _stream()),
           "lsq_adam_step_lp_blocked")
    return p_lp, state


def lsq_pad_offsets(key_len, batch: int, max_len: int, offsets=None):
    """key_len: int32[batch] (or None: all full) -> offsets int32[batch+1] on the device."""
    if offsets is None:
        dev = key_len.device if key_len is not None else torch.device("cuda", torch.cuda.current_device())
        offsets = torch.empty(batch + 1, dtype=torch.int32, device=dev)
    _need("key_len", key_len, batch, torch.int32); _need("offsets", offsets, batch + 1, torch.int32)
    _check(load().lsq_pad_offsets(_ptr(offsets), _ptr(key_len), batch, max_len, _stream()), "lsq_pad_offsets")
    return offsets


def lsq_pad_remove(padded, offsets, packed_rows: int, packed=None):
    """padded: [batch, max_len, hidden] -> packed [packed_rows, hidden] (rows from sum(len) on are not written)."""
    B, L, H = padded.shape
    packed = torch.empty((packed_rows, H), dtype=padded.dtype, device=padded.device) if packed is None else packed
    _need("offsets", offsets, B + 1, torch.int32)
    if packed.dim() != 2 or packed.shape[1] != H or packed.dtype != padded.dtype:
        raise LsqError("packed must be [rows, hidden] of the padded tensor's dtype")
    _check(load().lsq_pad_remove(_ptr(packed) if packed.numel() else None, _ptr(padded) if padded.numel() else None,
                                 _ptr(offsets), B, L, H, packed.shape[0], _dt(padded), _stream()), "lsq_pad_remove")
    return packed


def lsq_pad_restore(packed, offsets, batch: int, max_len: int, padded=None):
    """packed: [rows, hidden] -> padded [batch, max_len, hidden], zeros on the padding."""
    H = packed.shape[1]
    padded = torch.empty((batch, max_len, H), dtype=packed.dtype, device=packed.device) if padded is None else padded
    _need("offsets", offsets, batch + 1, torch.int32); _need("padded", padded, batch * max_len * H, packed.dtype)
    _check(load().lsq_pad_restore(_ptr(padded) if padded.numel() else None, _ptr(packed) if packed.numel() else None,
                                  _ptr(offsets), batch, max_len, H, packed.shape[0], _dt(packed), _stream()),
           "lsq_pad_restore")
    return padded


def lsq_softmax_varlen_fwd(x, key_len=None, query_len=None, causal: bool = False, scale: float = 1.0,
                           p_attn: float = 0.0, seed: int = 0, offset: int = 0, y=None, y_drop=None):
    """lsq_softmax_fwd with query_len: int32[batch]; rows of padded queries are not read and come out as zeros."""
    B, N, Lq, Lk = x.shape
    y = torch.empty_like(x) if y is None else y
    if p_attn > 0 and y_drop is None:
        y_drop = torch.empty_like(x)
    _need("y", y, x.numel(), x.dtype); _need("y_drop", y_drop, x.numel(), x.dtype)
    _need("key_len", key_len, B, torch.int32); _need("query_len", query_len, B, torch.int32)
    _check(load().lsq_softmax_varlen_fwd(_ptr(y), _ptr(y_drop) if p_attn > 0 else None, _ptr(x), _ptr(key_len),
                                         _ptr(query_len), B, N, Lq, Lk, int(causal), scale, p_attn, seed, offset,
                                         _dt(x), _stream()), "lsq_softmax_varlen_fwd")
    return y, (y_drop if p_attn > 0 else None)


def lsq_softmax_varlen_bwd(dy, y, key_len=None, query_len=None, causal: bool = False, scale: float = 1.0,
                           p_attn: float = 0.0, seed: int = 0, offset: int = 0, dx=None):
    B, N, Lq, Lk = y.shape
    dx = torch.empty_like(y) if dx is None else dx
    _need("dx", dx, y.numel(), y.dtype); _need("dy", dy, y.numel(), y.dtype)
    _need("key_len", key_len, B, torch.int32); _need("query_len", query_len, B, torch.int32)
    _check(load().lsq_softmax_varlen_bwd(_ptr(dx), _ptr(dy), _ptr(y), _ptr(key_len), _ptr(query_len), B, N, Lq, Lk,
                                         int(causal), scale, p_attn, seed, offset, _dt(y), _stream()),
           "lsq_softmax_varlen_bwd")
    return dx


def lsq_calib_stream(kind: str, dst, src=None, nbytes: int = 0):
    """A plain memory stream (measurement aid): kind = "copy" | "read" | "write" | "empty"."""
    k = {"copy": 0, "read": 1, "write": 2, "empty": 3}[kind]
    _check(load().lsq_calib_stream(k, _ptr(dst), _ptr(src), nbytes, _stream()), "lsq_calib_stream")


def lsq_softmax_candidates(k_len: int) -> int:
    return int(load().lsq_softmax_candidates(k_len))


def lsq_softmax_tune(x, dy, key_len=None, query_len=None, causal: bool = False, scale: float = 1.0, p_attn: float = 0.0,
                     seed: int = 0, offset: int = 0, force: int = -1, reps: int = 20, y=None, y_drop=None, dx=None):
    """Search (force = -1), set (force >= 0) or forget (force = -2) the launch shape of the softmax for problems like
    this one -> (best_fwd, best_bwd, us[2][4])."""
    B, N, Lq, Lk = x.shape
    y = torch.empty_like(x) if y is None else y
    dx = torch.empty_like(x) if dx is None else dx
    if p_attn > 0 and y_drop is None:
        y_drop = torch.empty_like(x)
    bf, bb = C.c_int32(0), C.c_int32(0)
    us = (C.c_float * 8)()
    _check(load().lsq_softmax_tune(C.byref(bf), C.byref(bb), us, _ptr(y), _ptr(y_drop) if p_attn > 0 else None, _ptr(dx), _ptr(x),
                                   _ptr(dy), _ptr(key_len), _ptr(query_len), B, N, Lq, Lk, int(causal), scale, p_attn, seed, offset,
                                   _dt(x), force, reps, _stream()), "lsq_softmax_tune")
    return bf.value, bb.value, [[us[d * 4 + c] for c in range(4)] for d in range(2)]
