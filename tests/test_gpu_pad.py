"""GPU parity: padding removal and the query-length softmax through the C-ABI against the CPU oracle.

Moves and offsets are index work: bit-exact.  The softmax keeps its storage tolerance on the real
rows and must give exact zeros on the rows of padded queries.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2110_05722_amd as L
from tests._util import assert_close_store, dev, say
from workloads import CONFIGS, decode, encode, from_torch, rng_for, sentence_lengths, to_torch

pytestmark = pytest.mark.gpu


def _lens(case, B, Lmax, r):
    if case == "uniform":
        return r.integers(0, Lmax + 1, size=B).astype(np.int32)
    if case == "full":
        return np.full(B, Lmax, dtype=np.int32)
    if case == "empty":
        return np.zeros(B, dtype=np.int32)
    if case == "wild":            # out-of-range lengths are clamped to [0, max_len]
        return r.integers(-3, Lmax + 4, size=B).astype(np.int32)
    raise ValueError(case)


@pytest.mark.parametrize("B,Lmax", [(1, 1), (4, 8), (64, 128), (300, 17), (1000, 3)])
@pytest.mark.parametrize("case", ["uniform", "full", "empty", "wild"])
def test_offsets(B, Lmax, case):
    say(f"[pad] offsets B={B} L={Lmax} {case}")
    r = np.random.default_rng(B + Lmax)
    lens = _lens(case, B, Lmax, r)
    off = L.lsq_pad_offsets(torch.from_numpy(lens).to(dev()), B, Lmax)
    assert np.array_equal(off.cpu().numpy(), oracle.pad_offsets(lens, Lmax))
    full = L.lsq_pad_offsets(None, B, Lmax)
    assert np.array_equal(full.cpu().numpy(), np.arange(B + 1, dtype=np.int32) * Lmax)


# (batch, max_len, hidden): several column tiles, ragged row tails, a scalar-path hidden size
SHAPES = [(8, 64, 512), (64, 128, 1024), (128, 32, 512), (3, 50, 768), (5, 33, 1280), (2, 7, 257), (1, 1, 8),
          (7, 9, 4), (16, 512, 1024)]


@pytest.mark.parametrize("dt", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("B,Lmax,H", SHAPES)
@pytest.mark.parametrize("case", ["uniform", "full", "empty", "wild"])
def test_remove_and_restore(B, Lmax, H, case, dt):
    if (dt == "f32" or case != "uniform") and B * Lmax * H > 1 << 21:
        pytest.skip("the large shapes run once, in 16-bit storage with mixed lengths")
    say(f"[pad] B={B} L={Lmax} H={H} {case} dt={dt}")
    d = dev()
    r = np.random.default_rng(B * 100 + Lmax + H)
    lens = _lens(case, B, Lmax, r)
    xs = encode(r.standard_normal((B, Lmax, H), dtype=np.float32), dt)
    x = to_torch(xs, dt, d)
    off = L.lsq_pad_offsets(torch.from_numpy(lens).to(d), B, Lmax)
    ref = oracle.pad_remove(xs, lens, dt)
    total = ref.shape[0]
    # capacity = the padded row count (what a caller that does not know sum(len) passes); the tail is untouched
    sentinel = to_torch(encode(np.full((B * Lmax, H), 7.0, dtype=np.float32), dt), dt, d)
    packed = L.lsq_pad_remove(x, off, B * Lmax, packed=sentinel.clone())
    got = decode(from_torch(packed, dt), dt).reshape(B * Lmax, H)
    assert np.array_equal(got[:total], ref)
    assert np.all(got[total:] == 7.0)
    # exact capacity
    packed2 = L.lsq_pad_remove(x, off, total)
    assert packed2.shape[0] == total
    if total:
        assert torch.equal(packed2, packed[:total])
    # restore: every element written, zeros on the padding
    back = L.lsq_pad_restore(packed2, off, B, Lmax, padded=to_torch(xs, dt, d).clone().fill_(3.0))
    rb = oracle.pad_restore(from_torch(packed2, dt).reshape(total, H), lens, Lmax, dt)
    assert np.array_equal(decode(from_torch(back, dt), dt).reshape(rb.shape), rb)
    # too small a capacity: rows beyond it are skipped, nothing is written outside
    if total > 1:
        cap = total // 2
        small = L.lsq_pad_remove(x, off, cap)
        assert torch.equal(small, packed[:cap])


@pytest.mark.parametrize("name", ["transformer-base", "transformer-big"])
def test_workload_lengths_round_trip(name):
    cfg = next(c for c in CONFIGS if c.name == name)
    say(f"[pad] workload {name}")
    d = dev()
    lens = sentence_lengths(cfg, rng_for(cfg, 0))
    B, Lmax, H = cfg.batch, cfg.max_len, cfg.hidden
    x = torch.randn((B, Lmax, H), device=d).to(torch.float16)
    off = L.lsq_pad_offsets(torch.from_numpy(lens).to(d), B, Lmax)
    total = int(lens.sum())
    assert int(off[-1].item()) == total
    packed = L.lsq_pad_remove(x, off, total)
    mask = torch.arange(Lmax, device=d)[None, :] < torch.from_numpy(lens).to(d)[:, None]
    assert torch.equal(packed, x[mask])
    back = L.lsq_pad_restore(packed, off, B, Lmax)
    assert torch.equal(back, torch.where(mask[:, :, None], x, torch.zeros_like(x)))


@pytest.mark.parametrize("dt", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("B,N,Lq,Lk,causal,p", [(8, 8, 64, 64, False, 0.0), (8, 8, 64, 64, True, 0.1),
                                                 (4, 2, 128, 128, False, 0.1), (3, 2, 50, 50, True, 0.0),
                                                 (2, 2, 33, 40, False, 0.1), (2, 1, 16, 2056, False, 0.0)])
def test_softmax_with_query_lengths(B, N, Lq, Lk, causal, p, dt):
    say(f"[pad] softmax B={B} N={N} Lq={Lq} Lk={Lk} causal={causal} p={p} dt={dt}")
    d = dev()
    r = np.random.default_rng(B * 10 + Lq)
    klen = r.integers(0, Lk + 1, size=B).astype(np.int32)
    qlen = r.integers(0, Lq + 1, size=B).astype(np.int32)
    qlen[0] = Lq
    xs = encode(r.standard_normal((B, N, Lq, Lk), dtype=np.float32), dt)
    x = to_torch(xs, dt, d)
    kl, ql = torch.from_numpy(klen).to(d), torch.from_numpy(qlen).to(d)
    y, yd = L.lsq_softmax_varlen_fwd(x, kl, ql, causal, 0.125, p, 1234, 5)
    ry, ryd = oracle.softmax_fwd(xs, klen, causal, 0.125, dt, p, 1234, 5, query_len=qlen)
    assert_close_store(y, ry, dt, "y")
    gy = decode(from_torch(y, dt), dt).reshape(ry.shape)
    for b in range(B):
        assert not gy[b, :, qlen[b]:].any()
    if p > 0:
        assert_close_store(yd, ryd, dt, "y_drop")
        assert np.array_equal(decode(from_torch(yd, dt), dt).reshape(ry.shape)[ry > 1e-3] == 0, ryd[ry > 1e-3] == 0)
    # backward from the stored forward output
    ys = from_torch(y, dt).reshape(ry.shape)
    dys = encode(r.standard_normal((B, N, Lq, Lk), dtype=np.float32), dt)
    dx = L.lsq_softmax_varlen_bwd(to_torch(dys, dt, d), y, kl, ql, causal, 0.125, p, 1234, 5)
    rdx = oracle.softmax_bwd(dys, ys, klen, causal, 0.125, dt, p, 1234, 5, query_len=qlen)
    assert_close_store(dx, rdx, dt, "dx")
    gdx = from_torch(dx, dt).reshape(ry.shape)
    for b in range(B):
        assert not gdx[b, :, qlen[b]:].any()           # +0 bit patterns, not -0
    # without query lengths the entry points are the plain ones
    y0, _ = L.lsq_softmax_varlen_fwd(x, kl, None, causal, 0.125, 0.0)
    y1, _ = L.lsq_softmax_fwd(x, kl, causal, 0.125, 0.0)
    assert torch.equal(y0, y1)
