"""Seeded synthetic inputs shaped like the paper's workloads.

This module serves BOTH the CPU oracle's tests and the HIP path's tests and
benchmark.  It holds storage-format helpers (fp16 / bf16 bit patterns) and random
input recipes only: none of the operators' arithmetic lives here.

The five configurations mirror the shapes the paper trains on (Sec. VI:
Transformer-base / Transformer-big on WMT14 En-De, BERT-large on GLUE-MRPC,
GPT-2-large on WikiText).  The datasets themselves are not used: every operator
on the path is data-oblivious apart from sentence lengths, targets and the mask
pattern, so N(0, s) activations with a realistic length mix stand in for them.
"N(0, s)" means standard deviation s.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np

LP_BYTES = {"f16": 2, "bf16": 2, "f32": 4}
DTYPE_CODE = {"f16": 0, "bf16": 1, "f32": 2}  # lsq_dtype in include/lsq.h


# --------------------------------------------------------------------------- #
# storage formats: numpy has no bfloat16, so low-precision tensors travel as
# uint16 bit patterns ("bits"); fp32 tensors travel as np.float32.
# --------------------------------------------------------------------------- #
def encode(a, dt: str) -> np.ndarray:
    """Round a float array to storage type `dt` (nearest even) and return the
    stored representation: uint16 bit patterns for f16/bf16, float32 for f32."""
    a = np.asarray(a)
    if dt == "f32":
        return np.ascontiguousarray(a, dtype=np.float32)
    if dt == "f16":
        return np.ascontiguousarray(a.astype(np.float16)).view(np.uint16)
    if dt == "bf16":
        b = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
        lsb = (b >> 16) & 1
        r = ((b + 0x7FFF + lsb) >> 16).astype(np.uint16)
        return r
    raise ValueError(dt)


def decode(bits, dt: str) -> np.ndarray:
    """Stored representation -> float64, exactly."""
    if dt == "f32":
        return np.asarray(bits, dtype=np.float32).astype(np.float64)
    bits = np.asarray(bits)
    if dt == "f16":
        return bits.view(np.float16).astype(np.float64)
    if dt == "bf16":
        return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    raise ValueError(dt)


def to_torch(stored: np.ndarray, dt: str, device="cpu"):
    """Stored representation -> torch tensor of the matching dtype (bit copy)."""
    import torch

    if dt == "f32":
        return torch.from_numpy(np.ascontiguousarray(stored)).to(device)
    t = torch.from_numpy(np.ascontiguousarray(stored).view(np.int16)).to(device)
    return t.view(torch.float16 if dt == "f16" else torch.bfloat16)


def from_torch(t, dt: str) -> np.ndarray:
    """torch tensor (any device) -> stored representation on the host (bit copy)."""
    import torch

    t = t.detach().contiguous().cpu()
    if dt == "f32":
        return t.numpy()
    return t.view(torch.int16).numpy().view(np.uint16)


def torch_dtype(dt: str):
    import torch

    return {"f16": torch.float16, "bf16": torch.bfloat16, "f32": torch.float32}[dt]


# --------------------------------------------------------------------------- #
# configurations
# --------------------------------------------------------------------------- #
@dataclass(frozen=True)
class Config:
    name: str
    seed: int
    dtypes: tuple          # storage types the configuration is run in
    batch: int
    max_len: int
    hidden: int
    heads: int
    vocab: int
    adam_n: int
    p_residual: float      # dropout on the residual branch
    p_attn: float          # dropout on attention probabilities (0 = off)
    alpha: float           # label smoothing
    logit_std: float
    lengths: str           # "uniform16" | "lognormal" | "full"
    len_median: float = 0.0
    causal: bool = False
    active_frac: float = 1.0   # fraction of positions that carry a target
    philox_seed: int = 1234
    extra: dict = field(default_factory=dict)

    @property
    def tokens(self) -> int:
        return self.batch * self.max_len


CONFIGS = [
    Config("tiny", 0, ("f16",), 8, 64, 512, 8, 8000, 1 << 20, 0.1, 0.0, 0.1, 2.0, "uniform16"),
    Config("transformer-base", 1, ("f16",), 128, 32, 512, 8, 32768, 61_000_000, 0.1, 0.0, 0.1,
           2.0, "lognormal", 22.0),
    Config("transformer-big", 2, ("f16",), 64, 128, 1024, 16, 32768, 210_000_000, 0.3, 0.1, 0.1,
           2.0, "lognormal", 60.0),
    Config("bert-large", 3, ("bf16", "f16"), 16, 512, 1024, 16, 30522, 335_000_000, 0.1, 0.0, 0.0,
           2.0, "full", active_frac=0.15),
    Config("gpt2-large", 4, ("bf16", "f16"), 8, 1024, 1280, 20, 50257, 774_000_000, 0.1, 0.0, 0.1,
           3.0, "full", causal=True),
]

ADAM_HYPER = dict(lr=1e-3, beta1=0.9, beta2=0.98, eps=1e-8)
IGNORE_INDEX = -100
LOGNORMAL_SIGMA = 0.5  # the configurations give median and maximum only


def rng_for(cfg: Config, stream: int = 0) -> np.random.Generator:
    """Independent PCG64 stream per (config seed, purpose)."""
    return np.random.Generator(np.random.PCG64([cfg.seed, stream]))


def sentence_lengths(cfg: Config, rng: np.random.Generator) -> np.ndarray:
    """int32[batch] sentence lengths in [1, max_len] following the config's mix."""
    B, L = cfg.batch, cfg.max_len
    if cfg.lengths == "full":
        return np.full(B, L, dtype=np.int32)
    if cfg.lengths == "uniform16":
        return rng.integers(16, L + 1, size=B).astype(np.int32)
    if cfg.lengths == "lognormal":
        raw = rng.lognormal(mean=math.log(cfg.len_median), sigma=LOGNORMAL_SIGMA, size=B)
        return np.clip(np.rint(raw), 1, L).astype(np.int32)
    raise ValueError(cfg.lengths)


def normal(rng: np.random.Generator, shape, std=1.0, mean=0.0) -> np.ndarray:
    return (rng.standard_normal(shape, dtype=np.float32) * np.float32(std) + np.float32(mean))


def layer_tensors(cfg: Config, dt: str, rows: int | None = None, hidden: int | None = None,
                  stream: int = 1) -> dict:
    """Activations for LayerNorm and bias+dropout+residual: x, residual, dy ~ N(0,1);
    gamma ~ N(1,0.1); beta, bias ~ N(0,0.1).  All in storage type `dt`."""
    rng = rng_for(cfg, stream)
    T = cfg.tokens if rows is None else rows
    H = cfg.hidden if hidden is None else hidden
    return dict(
        x=encode(normal(rng, (T, H)), dt),
        residual=encode(normal(rng, (T, H)), dt),
        dy=encode(normal(rng, (T, H)), dt),
        gamma=encode(normal(rng, (H,), 0.1, 1.0), dt),
        beta=encode(normal(rng, (H,), 0.1), dt),
        bias=encode(normal(rng, (H,), 0.1), dt),
    )


def attention_tensors(cfg: Config, dt: str, batch: int | None = None, heads: int | None = None,
                      q_len: int | None = None, k_len: int | None = None, stream: int = 2) -> dict:
    """Attention scores x and upstream gradient dy ~ N(0,1), plus key lengths."""
    rng = rng_for(cfg, stream)
    B = cfg.batch if batch is None else batch
    N = cfg.heads if heads is None else heads
    Lq = cfg.max_len if q_len is None else q_len
    Lk = cfg.max_len if k_len is None else k_len
    if B == cfg.batch and Lk == cfg.max_len:
        key_len = sentence_lengths(cfg, rng)
    else:
        key_len = rng.integers(1, Lk + 1, size=B).astype(np.int32)
    return dict(
        x=encode(normal(rng, (B, N, Lq, Lk)), dt),
        dy=encode(normal(rng, (B, N, Lq, Lk)), dt),
        key_len=key_len,
    )


def criterion_tensors(cfg: Config, dt: str, tokens: int | None = None, vocab: int | None = None,
                      stream: int = 3) -> dict:
    """Decoder-output logits ~ N(0, logit_std) and int32 targets; padded positions
    (beyond the sentence length) and, for masked-LM configs, the inactive positions
    carry IGNORE_INDEX."""
    rng = rng_for(cfg, stream)
    T = cfg.tokens if tokens is None else tokens
    V = cfg.vocab if vocab is None else vocab
    logits = encode(normal(rng, (T, V), cfg.logit_std), dt)
    target = rng.integers(0, V, size=T).astype(np.int32)
    if T == cfg.tokens:
        lens = sentence_lengths(cfg, rng)
        pos = np.arange(cfg.max_len)[None, :]
        pad = (pos >= lens[:, None]).reshape(-1)
        target[pad] = IGNORE_INDEX
    if cfg.active_frac < 1.0:
        inactive = rng.random(T) >= cfg.active_frac
        target[inactive] = IGNORE_INDEX
    return dict(logits=logits, target=target)


def adam_tensors(cfg: Config, g_dt: str, n: int | None = None, stream: int = 4) -> dict:
    """Flat workspace: fp32 master p ~ N(0,0.02), gradient g ~ N(0,1e-3) in `g_dt`,
    moments m = v = 0 (state before step 1)."""
    rng = rng_for(cfg, stream)
    n = cfg.adam_n if n is None else n
    return dict(
        p=normal(rng, (n,), 0.02),
        g=encode(normal(rng, (n,), 1e-3), g_dt),
        m=np.zeros(n, dtype=np.float32),
        v=np.zeros(n, dtype=np.float32),
    )


def device_normal(shape, std: float, dt: str, seed: int, device="cuda", mean: float = 0.0):
    """Full-size tensors for the benchmark and the full-size parity tests, drawn on
    the device (host generation of 10^9 normals would dominate the run).  Seeded;
    the oracle receives copies of whatever rows it checks."""
    import torch

    g = torch.Generator(device=device)
    g.manual_seed(seed)
    numel = int(np.prod(shape))
    out = torch.empty(shape, dtype=torch_dtype(dt), device=device)
    flat = out.view(-1)
    chunk = 1 << 26
    for s in range(0, numel, chunk):
        e = min(numel, s + chunk)
        t = torch.randn(e - s, generator=g, device=device, dtype=torch.float32)
        if std != 1.0:
            t.mul_(std)
        if mean != 0.0:
            t.add_(mean)
        flat[s:e] = t.to(out.dtype)
    return out
