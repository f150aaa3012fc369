"""Pins for the oracle's embedding layer (Sec. IV-A): numpy fancy indexing and np.add.at are the
independent statements of the gather and of the scatter-add."""
import numpy as np
import pytest

import oracle
from workloads import decode, encode

PAD = 1


def _case(B, L, V, H, dt, seed=0):
    r = np.random.default_rng(seed)
    tok = r.integers(0, V, size=(B, L)).astype(np.int32)
    tok[0, -2:] = PAD
    tok[-1, 0] = tok[0, 0]                      # at least one repeated id
    if B > 1:
        tok[1, 1] = V                           # out of range: treated as padding
    emb = encode(r.standard_normal((V, H)), dt)
    pos = encode(r.standard_normal((L, H)) * 0.5, dt)
    return tok, emb, pos, r


@pytest.mark.parametrize("dt", ["f32", "f16", "bf16"])
def test_fwd_is_gather_scale_add(dt):
    B, L, V, H = 3, 7, 11, 16
    tok, emb, pos, _ = _case(B, L, V, H, dt)
    out = oracle.embedding_fwd(tok, emb, pos, PAD, 4.0, 0.0, 1, 0, dt)
    E, P = decode(emb, dt), decode(pos, dt)
    flat = tok.reshape(-1)
    valid = (flat != PAD) & (flat >= 0) & (flat < V)
    ref = np.where(valid[:, None], 4.0 * E[np.clip(flat, 0, V - 1)] + P[np.arange(B * L) % L], 0.0)
    assert np.array_equal(out, ref)
    # dropout = the pinned mask over the flat [T, H] index
    p, seed, off = 0.3, 9, 2
    outd = oracle.embedding_fwd(tok, emb, pos, PAD, 4.0, p, seed, off, dt)
    keep = oracle.dropout_mask(B * L * H, p, seed, off).reshape(B * L, H)
    assert np.allclose(outd, keep * ref / (1 - np.float64(np.float32(p))), rtol=1e-15)


def test_bwd_is_scatter_add():
    B, L, V, H = 4, 6, 9, 8
    tok, _, _, r = _case(B, L, V, H, "f32", seed=3)
    dy = r.standard_normal((B * L, H)).astype(np.float32)
    p, seed, off, scale = 0.25, 5, 1, 3.0
    demb, dpos = oracle.embedding_bwd(dy, tok, V, PAD, scale, p, seed, off, "f32")
    keep = oracle.dropout_mask(B * L * H, p, seed, off).reshape(B * L, H)
    g = keep * dy.astype(np.float64) / (1 - np.float64(np.float32(p)))
    flat = tok.reshape(-1)
    valid = (flat != PAD) & (flat >= 0) & (flat < V)
    ref = np.zeros((V, H)); np.add.at(ref, flat[valid], scale * g[valid])
    refp = np.zeros((L, H)); np.add.at(refp, (np.arange(B * L) % L)[valid], g[valid])
    assert np.allclose(demb, ref, rtol=1e-13, atol=1e-15) and np.allclose(dpos, refp, rtol=1e-13, atol=1e-15)
    assert np.all(demb[PAD] == 0)                      # padding receives no gradient
    unused = np.setdiff1d(np.arange(V), flat[valid])
    assert np.all(demb[unused] == 0)
    # adjointness: <fwd(E, P), dy> is linear in (E, P) with gradient (demb, dpos) when the mask is frozen
    emb = r.standard_normal((V, H)).astype(np.float32)
    pos = r.standard_normal((L, H)).astype(np.float32)
    out = oracle.embedding_fwd(tok, emb, pos, PAD, scale, p, seed, off, "f32")
    lhs = float((out * dy).sum())
    rhs = float((emb.astype(np.float64) * demb).sum() + (pos.astype(np.float64) * dpos).sum())
    assert lhs == pytest.approx(rhs, rel=1e-12)
    d2, none = oracle.embedding_bwd(dy, tok, V, PAD, scale, p, seed, off, "f32", want_dpos=False)
    assert none is None and np.array_equal(d2, demb)
