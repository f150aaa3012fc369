"""CPU oracle — TEST INFRASTRUCTURE, not the product.

numpy-facing wrapper around `lsq_oracle.c` (plain C, double precision).  Only
`tests/`, `__graft_entry__.smoke()` and the `cpu_baseline` leg of `bench.py` may
import this package; the HIP library and its Python binding never do.

Low-precision inputs are passed in their storage representation (uint16 bit
patterns for "f16"/"bf16", float32 arrays for "f32"); every output is float64,
unrounded.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lsq_oracle.c")
_LIB = os.path.join(_HERE, "liblsq_oracle.so")
_DT = {"f16": 0, "bf16": 1, "f32": 2}
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP over rows).  Returns the library path.

    LSQ_ORACLE_SRC (the mutation test of the pins sets it, nothing else does) names another C
    source to compile and load instead: an oracle with a planted mistake."""
    src, lib_path = _SRC, _LIB
    alt = os.environ.get("LSQ_ORACLE_SRC")
    if alt:
        src, lib_path, force = alt, alt + ".so", True
    if force or not os.path.exists(lib_path) or os.path.getmtime(lib_path) < os.path.getmtime(src):
        cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
               "-o", lib_path, src, "-lm"]
        subprocess.run(cmd, check=True)
    return lib_path


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _stored(a, dt):
    want = np.float32 if dt == "f32" else np.uint16
    a = np.ascontiguousarray(a)
    if a.dtype != want:
        raise TypeError(f"storage array for {dt} must be {want}, got {a.dtype}")
    return a


def _i32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def num_threads() -> int:
    """Threads the OpenMP loops will use (what the CPU baseline reports as cores)."""
    n = os.environ.get("OMP_NUM_THREADS")
    if n:
        return int(n.split(",")[0])
    return len(os.sched_getaffinity(0))


# ------------------------------------------------------------------ dropout
def philox4x32_10(ctr, key) -> np.ndarray:
    c = (C.c_uint32 * 4)(*[int(v) & 0xFFFFFFFF for v in ctr])
    k = (C.c_uint32 * 2)(*[int(v) & 0xFFFFFFFF for v in key])
    o = (C.c_uint32 * 4)()
    lib().lsqo_philox4x32_10(c, k, o)
    return np.array(list(o), dtype=np.uint32)


def dropout_mask(n: int, p: float, seed: int, offset: int, e0: int = 0) -> np.ndarray:
    keep = np.empty(n, dtype=np.uint8)
    lib().lsqo_dropout_mask(_p(keep), C.c_uint64(e0), C.c_int64(n), C.c_double(float(np.float32(p))),
                            C.c_uint64(seed), C.c_uint64(offset))
    return keep


# ---------------------------------------------------------------- layernorm
def layernorm_fwd(x, gamma, beta, eps: float, dt: str):
    x, gamma, beta = _stored(x, dt), _stored(gamma, dt), _stored(beta, dt)
    rows, hidden = x.shape
    y = np.empty((rows, hidden)); mean = np.empty(rows); rstd = np.empty(rows)
    lib().lsqo_layernorm_fwd(_p(y), _p(mean), _p(rstd), _p(x), _p(gamma), _p(beta), C.c_int64(rows),
                             C.c_int32(hidden), C.c_double(float(np.float32(eps))), C.c_int(_DT[dt]))
    return y, mean, rstd


def layernorm_bwd(dy, x, gamma, eps: float, dt: str, dres_in=None):
    dy, x, gamma = _stored(dy, dt), _stored(x, dt), _stored(gamma, dt)
    if dres_in is not None:
        dres_in = _stored(dres_in, dt)
    rows, hidden = x.shape
    dx = np.empty((rows, hidden)); dgamma = np.empty(hidden); dbeta = np.empty(hidden)
    lib().lsqo_layernorm_bwd(_p(dx), _p(dgamma), _p(dbeta), _p(dy), _p(x), _p(gamma), _p(dres_in),
                             C.c_int64(rows), C.c_int32(hidden), C.c_double(float(np.float32(eps))),
                             C.c_int(_DT[dt]))
    return dx, dgamma, dbeta


def layernorm_bwd_rearranged(dy, x, gamma, eps: float, dt: str):
    dy, x, gamma = _stored(dy, dt), _stored(x, dt), _stored(gamma, dt)
    rows, hidden = x.shape
    dx = np.empty((rows, hidden))
    lib().lsqo_layernorm_bwd_rearranged(_p(dx), _p(dy), _p(x), _p(gamma), C.c_int64(rows),
                                        C.c_int32(hidden), C.c_double(float(np.float32(eps))),
                                        C.c_int(_DT[dt]))
    return dx


# ------------------------------------------------- bias + dropout + residual
def bias_dropout_residual_fwd(x, bias, residual, p: float, seed: int, offset: int, dt: str, e0: int = 0):
    x, residual = _stored(x, dt), _stored(residual, dt)
    if bias is not None:
        bias = _stored(bias, dt)
    rows, hidden = x.shape
    out = np.empty((rows, hidden))
    lib().lsqo_bias_dropout_residual_fwd(_p(out), _p(x), _p(bias), _p(residual), C.c_int64(rows),
                                         C.c_int32(hidden), C.c_double(float(np.float32(p))),
                                         C.c_uint64(seed), C.c_uint64(offset), C.c_uint64(e0),
                                         C.c_int(_DT[dt]))
    return out


def bias_dropout_residual_bwd(dy, p: float, seed: int, offset: int, dt: str, e0: int = 0):
    dy = _stored(dy, dt)
    rows, hidden = dy.shape
    dx = np.empty((rows, hidden)); dbias = np.empty(hidden)
    lib().lsqo_bias_dropout_residual_bwd(_p(dx), _p(dbias), _p(dy), C.c_int64(rows), C.c_int32(hidden),
                                         C.c_double(float(np.float32(p))), C.c_uint64(seed),
                                         C.c_uint64(offset), C.c_uint64(e0), C.c_int(_DT[dt]))
    return dx, dbias


# ------------------------------------------------------------------ softmax
def softmax_fwd(x, key_len, causal: bool, scale: float, dt: str, p: float = 0.0, seed: int = 0,
                offset: int = 0, e0: int = 0, query_len=None):
    x = _stored(x, dt)
    B, N, Lq, Lk = x.shape
    key_len = _i32(key_len)
    query_len = _i32(query_len)
    y = np.empty(x.shape)
    yd = np.empty(x.shape) if p > 0 else None
    lib().lsqo_softmax_varlen_fwd(_p(y), _p(yd), _p(x), _p(key_len), _p(query_len), C.c_int32(B), C.c_int32(N), C.c_int32(Lq),
                           C.c_int32(Lk), C.c_int32(int(causal)), C.c_double(float(np.float32(scale))),
                           C.c_double(float(np.float32(p))), C.c_uint64(seed), C.c_uint64(offset),
                           C.c_uint64(e0), C.c_int(_DT[dt]))
    return y, yd


def softmax_bwd(dy, y, key_len, causal: bool, scale: float, dt: str, p: float = 0.0, seed: int = 0,
                offset: int = 0, e0: int = 0, query_len=None):
    dy, y = _stored(dy, dt), _stored(y, dt)
    B, N, Lq, Lk = y.shape
    key_len = _i32(key_len)
    query_len = _i32(query_len)
    dx = np.empty(y.shape)
    lib().lsqo_softmax_varlen_bwd(_p(dx), _p(dy), _p(y), _p(key_len), _p(query_len), C.c_int32(B), C.c_int32(N), C.c_int32(Lq),
                           C.c_int32(Lk), C.c_int32(int(causal)), C.c_double(float(np.float32(scale))),
                           C.c_double(float(np.float32(p))), C.c_uint64(seed), C.c_uint64(offset),
                           C.c_uint64(e0), C.c_int(_DT[dt]))
    return dx


# ---------------------------------------------------------------- criterion
def ls_xent_fwd(logits, target, alpha: float, ignore_index: int, dt: str):
    logits = _stored(logits, dt)
    target = _i32(target)
    T, V = logits.shape
    loss = np.empty(T); nll = np.empty(T); lse = np.empty(T); sums = np.empty(3)
    lib().lsqo_ls_xent_fwd(_p(loss), _p(nll), _p(lse), _p(sums), _p(logits), _p(target), C.c_int64(T),
                           C.c_int32(V), C.c_double(float(np.float32(alpha))), C.c_int32(ignore_index),
                           C.c_int(_DT[dt]))
    return loss, nll, lse, sums


def ls_xent_bwd(logits, target, alpha: float, ignore_index: int, grad_scale: float, dt: str):
    logits = _stored(logits, dt)
    target = _i32(target)
    T, V = logits.shape
    d = np.empty((T, V))
    lib().lsqo_ls_xent_bwd(_p(d), _p(logits), _p(target), C.c_int64(T), C.c_int32(V),
                           C.c_double(float(np.float32(alpha))), C.c_int32(ignore_index),
                           C.c_double(float(np.float32(grad_scale))), C.c_int(_DT[dt]))
    return d


# --------------------------------------------------------------------- adam
def adam_step(p, m, v, g, g_dt: str, lr, beta1, beta2, eps, step: int, weight_decay=0.0, adamw=False,
              bias_correction=True, inv_grad_scale=1.0):
    p = np.ascontiguousarray(p, dtype=np.float32)
    m = np.ascontiguousarray(m, dtype=np.float32)
    v = np.ascontiguousarray(v, dtype=np.float32)
    g = _stored(g, g_dt)
    n = p.size
    po = np.empty(n); mo = np.empty(n); vo = np.empty(n)
    f = lambda s: C.c_double(float(np.float32(s)))
    lib().lsqo_adam_step(_p(po), _p(mo), _p(vo), _p(p), _p(m), _p(v), _p(g), C.c_int64(n), f(lr), f(beta1),
                         f(beta2), f(eps), f(weight_decay), C.c_int32(step), C.c_int32(int(adamw)),
                         C.c_int32(int(bias_correction)), f(inv_grad_scale), C.c_int(_DT[g_dt]))
    return po, mo, vo


# ------------------------------------------------ bias + activation + dropout
ACT = {"relu": 0, "gelu": 1, "gelu_tanh": 2}


def bias_act_dropout_fwd(x, bias, act: str, p: float, seed: int, offset: int, dt: str, e0: int = 0):
    x = _stored(x, dt)
    if bias is not None:
        bias = _stored(bias, dt)
    rows, hidden = x.shape
    out = np.empty((rows, hidden))
    lib().lsqo_bias_act_dropout_fwd(_p(out), _p(x), _p(bias), C.c_int64(rows), C.c_int32(hidden), C.c_int32(ACT[act]),
                                    C.c_double(float(np.float32(p))), C.c_uint64(seed), C.c_uint64(offset),
                                    C.c_uint64(e0), C.c_int(_DT[dt]))
    return out


def bias_act_dropout_bwd(dy, x, bias, act: str, p: float, seed: int, offset: int, dt: str, e0: int = 0):
    dy, x = _stored(dy, dt), _stored(x, dt)
    if bias is not None:
        bias = _stored(bias, dt)
    rows, hidden = x.shape
    dx = np.empty((rows, hidden)); dbias = np.empty(hidden)
    lib().lsqo_bias_act_dropout_bwd(_p(dx), _p(dbias), _p(dy), _p(x), _p(bias), C.c_int64(rows), C.c_int32(hidden),
                                    C.c_int32(ACT[act]), C.c_double(float(np.float32(p))), C.c_uint64(seed),
                                    C.c_uint64(offset), C.c_uint64(e0), C.c_int(_DT[dt]))
    return dx, dbias


# ------------------------------------------------------------ trainer variants
def adam_step_lp(p_lp, m, v, g, dt: str, lr, beta1, beta2, eps, step: int, weight_decay=0.0, adamw=False,
                 bias_correction=True, inv_grad_scale=1.0):
    p_lp = _stored(p_lp, dt)
    g = _stored(g, dt)
    m = np.ascontiguousarray(m, dtype=np.float32)
    v = np.ascontiguousarray(v, dtype=np.float32)
    n = p_lp.size
    po = np.empty(n); mo = np.empty(n); vo = np.empty(n)
    f = lambda s: C.c_double(float(np.float32(s)))
    lib().lsqo_adam_step_lp(_p(po), _p(mo), _p(vo), _p(p_lp), _p(m), _p(v), _p(g), C.c_int64(n), f(lr), f(beta1),
                            f(beta2), f(eps), f(weight_decay), C.c_int32(step), C.c_int32(int(adamw)),
                            C.c_int32(int(bias_correction)), f(inv_grad_scale), C.c_int(_DT[dt]))
    return po, mo, vo


def sgd_step(p, buf, g, g_dt: str, lr, momentum=0.0, weight_decay=0.0, nesterov=False, inv_grad_scale=1.0):
    p = np.ascontiguousarray(p, dtype=np.float32)
    g = _stored(g, g_dt)
    n = p.size
    po = np.empty(n)
    bo = np.empty(n) if momentum != 0.0 else None
    if momentum != 0.0:
        buf = np.ascontiguousarray(buf, dtype=np.float32)
    f = lambda s: C.c_double(float(np.float32(s)))
    lib().lsqo_sgd_step(_p(po), _p(bo), _p(p), _p(buf) if momentum != 0.0 else None, _p(g), C.c_int64(n), f(lr),
                        f(momentum), f(weight_decay), C.c_int32(int(nesterov)), f(inv_grad_scale), C.c_int(_DT[g_dt]))
    return po, bo


# ---------------------------------------------------------- head split / merge
def split_heads_fwd(x, bias, batch: int, length: int, heads: int, head_dim: int, parts: int, dt: str):
    """x: [batch*len, parts*heads*head_dim] (+bias) -> `parts` arrays [batch, heads, len, head_dim]."""
    x = _stored(x, dt)
    if bias is not None:
        bias = _stored(bias, dt)
    outs = [np.empty((batch, heads, length, head_dim)) for _ in range(parts)]
    ptrs = [_p(o) for o in outs] + [None] * (3 - parts)
    lib().lsqo_split_heads_fwd(ptrs[0], ptrs[1], ptrs[2], _p(x), _p(bias), C.c_int32(batch), C.c_int32(length),
                               C.c_int32(heads), C.c_int32(head_dim), C.c_int32(parts), C.c_int(_DT[dt]))
    return outs


def split_heads_bwd(grads, batch: int, length: int, heads: int, head_dim: int, dt: str, want_dbias: bool = True):
    """grads: list of `parts` arrays [batch, heads, len, head_dim] -> (din [batch*len, parts*hidden], dbias)."""
    parts = len(grads)
    grads = [_stored(g, dt) for g in grads]
    hidden = heads * head_dim
    din = np.empty((batch * length, parts * hidden))
    dbias = np.empty(parts * hidden) if want_dbias else None
    ptrs = [_p(g) for g in grads] + [None] * (3 - parts)
    lib().lsqo_split_heads_bwd(_p(din), _p(dbias), ptrs[0], ptrs[1], ptrs[2], C.c_int32(batch), C.c_int32(length),
                               C.c_int32(heads), C.c_int32(head_dim), C.c_int32(parts), C.c_int(_DT[dt]))
    return din, dbias


# ------------------------------------------------------------------ embedding
def embedding_fwd(tokens, emb, pos, pad_idx: int, scale: float, p: float, seed: int, offset: int, dt: str, e0: int = 0):
    """tokens: int32 [batch, len]; emb: [vocab, hidden]; pos: [>=len, hidden] -> out [batch*len, hidden]."""
    tokens = _i32(tokens)
    emb, pos = _stored(emb, dt), _stored(pos, dt)
    B, Ln = tokens.shape
    V, H = emb.shape
    out = np.empty((B * Ln, H))
    lib().lsqo_embedding_fwd(_p(out), _p(tokens), _p(emb), _p(pos), C.c_int32(B), C.c_int32(Ln), C.c_int32(H),
                             C.c_int32(V), C.c_int32(pad_idx), C.c_double(float(np.float32(scale))),
                             C.c_double(float(np.float32(p))), C.c_uint64(seed), C.c_uint64(offset), C.c_uint64(e0),
                             C.c_int(_DT[dt]))
    return out


def embedding_bwd(dy, tokens, vocab: int, pad_idx: int, scale: float, p: float, seed: int, offset: int, dt: str,
                  want_dpos: bool = True, e0: int = 0):
    """-> (increment of dE [vocab, hidden], increment of dP [len, hidden] or None), float64."""
    tokens = _i32(tokens)
    dy = _stored(dy, dt)
    B, Ln = tokens.shape
    H = dy.shape[-1]
    demb = np.empty((vocab, H))
    dpos = np.empty((Ln, H)) if want_dpos else None
    lib().lsqo_embedding_bwd(_p(demb), _p(dpos), _p(dy), _p(tokens), C.c_int32(B), C.c_int32(Ln), C.c_int32(H),
                             C.c_int32(vocab), C.c_int32(pad_idx), C.c_double(float(np.float32(scale))),
                             C.c_double(float(np.float32(p))), C.c_uint64(seed), C.c_uint64(offset), C.c_uint64(e0),
                             C.c_int(_DT[dt]))
    return demb, dpos


# ------------------------------------------------------------ padding removal
def pad_offsets(key_len, max_len: int) -> np.ndarray:
    """int32[batch+1]: first packed row of every sentence, then the total."""
    key_len = _i32(key_len)
    off = np.empty(len(key_len) + 1, dtype=np.int32)
    lib().lsqo_pad_offsets(_p(off), _p(key_len), C.c_int32(len(key_len)), C.c_int32(max_len))
    return off


def pad_remove(padded, key_len, dt: str) -> np.ndarray:
    """padded [batch, max_len, hidden] -> packed [sum(len), hidden]."""
    padded = _stored(padded, dt)
    B, L, H = padded.shape
    key_len = _i32(key_len)
    total = int(pad_offsets(key_len, L)[-1])
    packed = np.empty((total, H))
    lib().lsqo_pad_remove(_p(packed), _p(padded), _p(key_len), C.c_int32(B), C.c_int32(L), C.c_int32(H),
                          C.c_int(_DT[dt]))
    return packed


def pad_restore(packed, key_len, max_len: int, dt: str) -> np.ndarray:
    """packed [sum(len), hidden] -> padded [batch, max_len, hidden], zeros on the padding."""
    packed = _stored(packed, dt)
    key_len = _i32(key_len)
    H = packed.shape[1]
    padded = np.empty((len(key_len), max_len, H))
    lib().lsqo_pad_restore(_p(padded), _p(packed), _p(key_len), C.c_int32(len(key_len)), C.c_int32(max_len),
                           C.c_int32(H), C.c_int(_DT[dt]))
    return padded
