"""Pins for the oracle's head split / merge: numpy's reshape + transpose is the independent statement."""
import numpy as np
import pytest

import oracle
from workloads import decode, encode


@pytest.mark.parametrize("dt", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("B,L,N,D,parts", [(2, 5, 3, 8, 3), (1, 7, 2, 4, 1), (3, 4, 4, 16, 2), (2, 3, 1, 5, 3)])
def test_split_is_reshape_transpose_plus_bias(B, L, N, D, parts, dt):
    r = np.random.default_rng(B * 100 + L)
    H = N * D
    x = encode(r.standard_normal((B * L, parts * H)), dt)
    bias = encode(r.standard_normal(parts * H) * 0.1, dt)
    outs = oracle.split_heads_fwd(x, bias, B, L, N, D, parts, dt)
    z = decode(x, dt) + decode(bias, dt)
    ref = z.reshape(B, L, parts, N, D).transpose(2, 0, 3, 1, 4)      # [parts, B, N, L, D]
    for k in range(parts):
        assert np.array_equal(outs[k], ref[k])
    nb = oracle.split_heads_fwd(x, None, B, L, N, D, parts, dt)
    ref0 = decode(x, dt).reshape(B, L, parts, N, D).transpose(2, 0, 3, 1, 4)
    for k in range(parts):
        assert np.array_equal(nb[k], ref0[k])


@pytest.mark.parametrize("B,L,N,D,parts", [(2, 5, 3, 8, 3), (1, 7, 2, 4, 1), (3, 4, 4, 16, 2)])
def test_bwd_is_the_inverse_permutation_and_column_sums(B, L, N, D, parts):
    r = np.random.default_rng(7)
    grads = [r.standard_normal((B, N, L, D)).astype(np.float32) for _ in range(parts)]
    din, dbias = oracle.split_heads_bwd(grads, B, L, N, D, "f32")
    ref = np.stack([g.astype(np.float64) for g in grads]).transpose(1, 3, 0, 2, 4).reshape(B * L, parts * N * D)
    assert np.array_equal(din, ref)
    assert np.allclose(dbias, ref.sum(0), rtol=1e-14, atol=1e-15)
    # round trip: split(merge(g)) == g
    back = oracle.split_heads_fwd(din.astype(np.float32), None, B, L, N, D, parts, "f32")
    for k in range(parts):
        assert np.array_equal(back[k], grads[k].astype(np.float64))
    # <split(x), g> == <x, split_bwd(g)>  (adjointness of forward and backward)
    x = r.standard_normal((B * L, parts * N * D)).astype(np.float32)
    fwd = oracle.split_heads_fwd(x, None, B, L, N, D, parts, "f32")
    lhs = sum(float((f * g).sum()) for f, g in zip(fwd, grads))
    assert lhs == pytest.approx(float((x.astype(np.float64) * din).sum()), rel=1e-12)
