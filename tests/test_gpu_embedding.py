"""GPU parity: embedding forward / backward through the C-ABI against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2110_05722_amd as L
from tests._util import LP_TOL, assert_close_store, dev, say
from workloads import decode, encode, from_torch, to_torch

pytestmark = pytest.mark.gpu
PAD = 1

# (batch, len, vocab, hidden, p)
CASES = [(8, 64, 8000, 512, 0.1), (128, 32, 32768, 512, 0.1), (16, 128, 4096, 1024, 0.3), (4, 512, 30522, 1024, 0.1),
         (2, 1024, 50257, 1280, 0.1), (3, 50, 97, 768, 0.0), (5, 7, 11, 8, 0.25), (2, 9, 13, 257, 0.2), (1, 1, 3, 64, 0.1),
         (4, 300, 5, 64, 0.1),
         (40, 520, 1000, 64, 0.1),      # beyond 16384 tokens: the radix-sorted order, two passes
         (36, 512, 100, 16, 0.1), (9, 2048, 70001, 16, 0.1),      # one pass (ids below 256) and three (above 65535)
         (550, 2000, 3000, 8, 0.1),     # 1.1 M tokens: the radix passes with the stand-alone offset scan
         (1, 70000, 500, 8, 0.1),       # one sentence longer than 65535 positions
         (4, 4096, 50257, 8, 0.0)]      # exactly 16384 tokens: the last size whose ranks are counted, 64 one-tile spans


def _tokens(B, Ln, V, rng):
    # Zipf-like ids so that some tokens repeat hundreds of times, the tail of each sentence padded
    tok = np.minimum((rng.pareto(1.1, size=(B, Ln)) * 3).astype(np.int64) + 2, V - 1).astype(np.int32)
    lens = rng.integers(max(1, Ln // 2), Ln + 1, size=B)
    tok[np.arange(Ln)[None, :] >= lens[:, None]] = PAD
    if B * Ln > 4:
        tok.reshape(-1)[3] = V            # out of range -> padding
        tok.reshape(-1)[2] = V - 1
    return tok


@pytest.mark.parametrize("dt", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("B,Ln,V,H,p", CASES)
def test_embedding_fwd_bwd(B, Ln, V, H, p, dt):
    if dt == "f32" and (B * Ln * H > 1 << 21 or V * H > 1 << 23):
        pytest.skip("fp32 storage is exercised on the small shapes only")
    say(f"[embedding] B={B} L={Ln} V={V} H={H} p={p} dt={dt}")
    d = dev()
    rng = np.random.default_rng(B * 7 + Ln + V)
    tok = _tokens(B, Ln, V, rng)
    embs = encode(rng.standard_normal((V, H), dtype=np.float32), dt)
    poss = encode(rng.standard_normal((Ln, H), dtype=np.float32) * 0.5, dt)
    dys = encode(rng.standard_normal((B * Ln, H), dtype=np.float32), dt)
    scale, seed, offset = float(np.sqrt(H)), 31, Ln
    tokens = torch.from_numpy(tok).to(d)
    emb, pos, dy = to_torch(embs, dt, d), to_torch(poss, dt, d), to_torch(dys, dt, d)
    out = L.lsq_embedding_fwd(tokens, emb, pos, PAD, scale, p, seed, offset)
    ref = oracle.embedding_fwd(tok, embs, poss, PAD, scale, p, seed, offset, dt)
    # values reach |scale * 4|: the relative (one ulp) branch of the tolerance is the one that binds
    assert_close_store(out, ref, dt, "out", f32_floor=1e-5)
    assert np.array_equal(decode(from_torch(out, dt), dt).reshape(ref.shape) == 0, ref == 0)

    # backward accumulates into existing gradients
    d0 = encode(rng.standard_normal((V, H), dtype=np.float32) * 0.1, dt)
    p0 = encode(rng.standard_normal((Ln, H), dtype=np.float32) * 0.1, dt)
    demb, dpos = to_torch(d0, dt, d), to_torch(p0, dt, d)
    L.lsq_embedding_bwd(demb, dpos, dy, tokens, PAD, scale, p, seed, offset)
    inc_e, inc_p = oracle.embedding_bwd(dys, tok, V, PAD, scale, p, seed, offset, dt)
    # a frequent token sums hundreds of rows of size scale*|dy|: widen the absolute term by the row's own magnitude
    assert_close_store(demb, decode(d0, dt) + inc_e, dt, "demb", f32_floor=1e-4 * scale)
    assert_close_store(dpos, decode(p0, dt) + inc_p, dt, "dpos", f32_floor=1e-4)
    # untouched rows keep their bits (padding row, ids that do not occur)
    flat = tok.reshape(-1)
    used = np.unique(flat[(flat != PAD) & (flat >= 0) & (flat < V)])
    unused = np.setdiff1d(np.arange(V), used)
    assert np.array_equal(from_torch(demb, dt)[unused], d0[unused])
    # run-to-run bit reproducibility (no atomics), and dpos is optional
    demb2 = to_torch(d0, dt, d)
    L.lsq_embedding_bwd(demb2, None, dy, tokens, PAD, scale, p, seed, offset)
    assert torch.equal(demb, demb2)


@pytest.mark.parametrize("kind", ["all padding", "one id everywhere", "all distinct"])
def test_embedding_bwd_degenerate_batches(kind):
    """Batches at the ends of the id distribution: nothing to accumulate, one segment that spans every window of the
    sorted order, and no repeated id at all."""
    say(f"[embedding] degenerate batch: {kind}")
    d, dt = dev(), "f16"
    B, Ln, V, H = 7, 41, 400, 64                   # 287 tokens: a ragged last rank tile and a ragged last window
    rng = np.random.default_rng(17)
    if kind == "all padding":
        tok = np.full((B, Ln), PAD, np.int32)
    elif kind == "one id everywhere":
        tok = np.full((B, Ln), 9, np.int32)
    else:
        tok = (rng.permutation(V - 2)[:B * Ln] + 2).astype(np.int32).reshape(B, Ln)
    dys = encode(rng.standard_normal((B * Ln, H), dtype=np.float32), dt)
    d0 = encode(rng.standard_normal((V, H), dtype=np.float32) * 0.1, dt)
    p0 = encode(rng.standard_normal((Ln, H), dtype=np.float32) * 0.1, dt)
    demb, dpos = to_torch(d0, dt, d), to_torch(p0, dt, d)
    L.lsq_embedding_bwd(demb, dpos, to_torch(dys, dt, d), torch.from_numpy(tok).to(d), PAD, 8.0, 0.1, 5, 2)
    inc_e, inc_p = oracle.embedding_bwd(dys, tok, V, PAD, 8.0, 0.1, 5, 2, dt)
    assert_close_store(demb, decode(d0, dt) + inc_e, dt, "demb", f32_floor=1e-3)
    assert_close_store(dpos, decode(p0, dt) + inc_p, dt, "dpos", f32_floor=1e-4)
    if kind == "all padding":
        assert np.array_equal(from_torch(demb, dt), d0) and np.array_equal(from_torch(dpos, dt), p0)
