"""Pins for the oracle's padding removal and for the query-length form of the softmax.

Independent statements: numpy boolean-mask indexing for the packing, numpy cumsum for the offsets,
and a numpy softmax written out per row for the padded-query rule.
"""
import numpy as np
import pytest

import oracle
from workloads import decode, encode


def _mask(lens, L):
    return np.arange(L)[None, :] < np.clip(lens, 0, L)[:, None]          # [B, L] True on real positions


@pytest.mark.parametrize("lens,L", [([3, 0, 5, 1], 5), ([7], 7), ([0, 0], 4), ([9, -2, 4], 6)])
def test_offsets_are_the_exclusive_cumsum_of_clamped_lengths(lens, L):
    off = oracle.pad_offsets(lens, L)
    c = np.clip(np.array(lens), 0, L)
    assert off.dtype == np.int32
    assert np.array_equal(off, np.concatenate([[0], np.cumsum(c)]))


@pytest.mark.parametrize("dt", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("lens,L,H", [([3, 0, 5, 1], 5, 8), ([7, 2], 7, 3), ([0, 0], 4, 16), ([9, -2, 4], 6, 5)])
def test_remove_is_boolean_mask_indexing_and_restore_is_its_zero_filled_inverse(lens, L, H, dt):
    r = np.random.default_rng(len(lens) * 10 + L)
    lens = np.array(lens)
    x = encode(r.standard_normal((len(lens), L, H)), dt)
    m = _mask(lens, L)
    packed = oracle.pad_remove(x, lens, dt)
    assert np.array_equal(packed, decode(x, dt)[m])
    back = oracle.pad_restore(encode(packed, dt), lens, L, dt)
    ref = np.where(m[:, :, None], decode(x, dt), 0.0)
    assert np.array_equal(back, ref)
    # restore is the adjoint of remove: <remove(x), g> == <x, restore(g)>
    g = encode(r.standard_normal(packed.shape), dt)
    lhs = float((packed * decode(g, dt)).sum())
    rhs = float((decode(x, dt) * oracle.pad_restore(g, lens, L, dt)).sum())
    assert lhs == pytest.approx(rhs, rel=1e-12, abs=1e-12)


@pytest.mark.parametrize("causal", [False, True])
def test_softmax_padded_query_rows_are_zero_and_the_rest_is_unchanged(causal):
    r = np.random.default_rng(5)
    B, N, Lq, Lk = 3, 2, 6, 6
    x = r.standard_normal((B, N, Lq, Lk)).astype(np.float32)
    klen = np.array([6, 3, 0])
    qlen = np.array([4, 6, 2])
    y, _ = oracle.softmax_fwd(x, klen, causal, 0.5, "f32", query_len=qlen)
    y0, _ = oracle.softmax_fwd(x, klen, causal, 0.5, "f32")
    # independent statement, row by row
    for b in range(B):
        for i in range(Lq):
            ok = np.arange(Lk) < klen[b]
            if causal:
                ok &= np.arange(Lk) <= i
            if i >= qlen[b]:
                ok[:] = False
            ref = np.zeros(Lk)
            if ok.any():
                e = np.exp(0.5 * x[b, 0, i, ok].astype(np.float64) - (0.5 * x[b, 0, i, ok].astype(np.float64)).max())
                ref[ok] = e / e.sum()
            assert np.allclose(y[b, 0, i], ref, rtol=1e-14, atol=0)
            if i >= qlen[b]:
                assert not y[b, :, i].any()
            else:
                assert np.array_equal(y[b, :, i], y0[b, :, i])
    dy = r.standard_normal(x.shape).astype(np.float32)
    dx = oracle.softmax_bwd(dy, y.astype(np.float32), klen, causal, 0.5, "f32", query_len=qlen)
    dx0 = oracle.softmax_bwd(dy, y.astype(np.float32), klen, causal, 0.5, "f32")
    for b in range(B):
        assert not dx[b, :, qlen[b]:].any()
        assert np.array_equal(dx[b, :, :qlen[b]], dx0[b, :, :qlen[b]])
