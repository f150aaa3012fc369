"""Pins for the oracle's label-smoothed cross-entropy (Sec. IV-A, criterion layer)."""
import numpy as np
import pytest

import oracle
from workloads import decode, encode

IGN = -100


def _rand(shape, seed, std=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * std


def _logq(h):
    m = h.max(-1, keepdims=True)
    return h - m - np.log(np.exp(h - m).sum(-1, keepdims=True))


@pytest.mark.parametrize("dt", ["f32", "f16", "bf16"])
def test_alpha_zero_is_minus_log_q_target(dt):
    T, V = 9, 37
    h = encode(_rand((T, V), 0, 2.0), dt)
    k = np.random.default_rng(1).integers(0, V, T).astype(np.int32)
    loss, nll, lse, sums = oracle.ls_xent_fwd(h, k, 0.0, IGN, dt)
    lq = _logq(decode(h, dt))
    exp = -lq[np.arange(T), k]
    assert np.allclose(loss, exp, rtol=1e-12, atol=1e-14)
    assert np.allclose(nll, exp, rtol=1e-12, atol=1e-14)
    assert np.allclose(sums, [exp.sum(), exp.sum(), T], rtol=1e-12)


def test_closed_form_and_special_cases():
    T, V, alpha = 6, 50, 0.1
    h32 = _rand((T, V), 2, 2.0).astype(np.float32)
    k = np.random.default_rng(3).integers(0, V, T).astype(np.int32)
    loss, nll, lse, _ = oracle.ls_xent_fwd(h32, k, alpha, IGN, "f32")
    h = h32.astype(np.float64)
    a = np.float64(np.float32(alpha))
    ref_lse = np.log(np.exp(h - h.max(1, keepdims=True)).sum(1)) + h.max(1)
    assert np.allclose(lse, ref_lse, rtol=1e-13)
    # closed form: lse - (1-a) h_k - (a/V) sum h
    cf = ref_lse - (1 - a) * h[np.arange(T), k] - a / V * h.sum(1)
    assert np.allclose(loss, cf, rtol=1e-12)
    # alpha = 1 -> lse - mean(h)
    l1, _, _, _ = oracle.ls_xent_fwd(h32, k, 1.0, IGN, "f32")
    assert np.allclose(l1, ref_lse - h.mean(1), rtol=1e-12)
    # all-equal logits -> log V for any alpha and any target
    c = np.full((3, V), -1.25, np.float32)
    for al in (0.0, 0.1, 0.7):
        lc, _, _, _ = oracle.ls_xent_fwd(c, np.array([0, 7, V - 1], np.int32), al, IGN, "f32")
        assert np.allclose(lc, np.log(V), rtol=1e-13)
    # V = 2, alpha = 0 -> softplus(h_other - h_target)
    h2 = np.array([[0.5, -1.5], [2.0, 3.0]], np.float32)
    l2, _, _, _ = oracle.ls_xent_fwd(h2, np.array([0, 0], np.int32), 0.0, IGN, "f32")
    assert np.allclose(l2, [np.log1p(np.exp(-2.0)), np.log1p(np.exp(1.0))], rtol=1e-13)
    # Gibbs: cross-entropy >= entropy of the smoothed target distribution
    ent = -((1 - a + a / V) * np.log(1 - a + a / V) + (V - 1) * (a / V) * np.log(a / V))
    assert np.all(loss >= ent - 1e-12)
    # shift invariance (exactly representable shift on a coarse grid)
    hg = (np.round(h32 * 16) / 16).astype(np.float32)
    la, _, _, _ = oracle.ls_xent_fwd(hg, k, alpha, IGN, "f32")
    lb, _, _, _ = oracle.ls_xent_fwd(hg + np.float32(8.0), k, alpha, IGN, "f32")
    assert np.allclose(la, lb, rtol=1e-12)


def test_bruteforce_tiny_vocab():
    h = np.array([[1.0, -0.5, 0.25, 2.0, 0.0]], np.float32)
    k, alpha = 3, 0.25
    e = np.exp(h[0].astype(np.float64)); q = e / e.sum()
    p = np.full(5, alpha / 5); p[k] += 1 - alpha
    exp = -sum(p[i] * np.log(q[i]) for i in range(5))
    loss, nll, _, _ = oracle.ls_xent_fwd(h, np.array([k], np.int32), alpha, IGN, "f32")
    assert loss[0] == pytest.approx(exp, rel=1e-13)
    assert nll[0] == pytest.approx(-np.log(q[k]), rel=1e-13)
    d = oracle.ls_xent_bwd(h, np.array([k], np.int32), alpha, IGN, 1.0, "f32")
    assert np.allclose(d[0], q - p, rtol=1e-12, atol=1e-15)


def test_ignored_tokens():
    T, V = 5, 11
    h = _rand((T, V), 4).astype(np.float32)
    k = np.array([3, IGN, 11, -1, 0], np.int32)  # ignore_index, out of range high and low
    loss, nll, lse, sums = oracle.ls_xent_fwd(h, k, 0.1, IGN, "f32")
    assert np.all(loss[1:4] == 0) and np.all(nll[1:4] == 0) and np.all(lse[1:4] == 0) and np.all(lse[[0, 4]] != 0)
    assert sums[2] == 2 and sums[0] == pytest.approx(loss[0] + loss[4], rel=1e-14)
    d = oracle.ls_xent_bwd(h, k, 0.1, IGN, 1.0, "f32")
    assert np.all(d[1:4] == 0) and np.all(d[0] != 0)


@pytest.mark.parametrize("alpha", [0.0, 0.1])
def test_bwd_matches_finite_differences_of_literal_fwd(alpha):
    T, V = 3, 16
    h = (np.round(_rand((T, V), 5, 2.0) * 32) / 32).astype(np.float32)
    k = np.array([2, 15, 0], np.int32)
    gs = 0.5
    d = oracle.ls_xent_bwd(h, k, alpha, IGN, gs, "f32")

    def total(hh):
        return gs * float(oracle.ls_xent_fwd(hh, k, alpha, IGN, "f32")[0].sum())

    eps = 2.0 ** -10
    for (t, i) in [(0, 2), (0, 5), (1, 15), (2, 0), (2, 9), (1, 0)]:
        hp, hm = h.copy(), h.copy()
        hp[t, i] += eps; hm[t, i] -= eps
        assert (total(hp) - total(hm)) / (2 * eps) == pytest.approx(d[t, i], rel=1e-5, abs=1e-8)


def test_bwd_invariants():
    T, V, alpha = 7, 64, 0.1
    h = _rand((T, V), 6, 3.0).astype(np.float32)
    k = np.random.default_rng(7).integers(0, V, T).astype(np.int32)
    d = oracle.ls_xent_bwd(h, k, alpha, IGN, 1.0, "f32")
    a = np.float64(np.float32(alpha))
    assert np.allclose(d.sum(1), 0, atol=1e-13)
    assert np.all(d[np.arange(T), k] < 0)
    off = np.ones((T, V), bool); off[np.arange(T), k] = False
    assert np.all(d[off] > -a / V)
    # alpha = 0 -> q - onehot
    d0 = oracle.ls_xent_bwd(h, k, 0.0, IGN, 1.0, "f32")
    q = np.exp(_logq(h.astype(np.float64)))
    q[np.arange(T), k] -= 1
    assert np.allclose(d0, q, rtol=1e-11, atol=1e-15)
    # grad_scale is linear
    d2 = oracle.ls_xent_bwd(h, k, alpha, IGN, 4.0, "f32")
    assert np.allclose(d2, 4 * d, rtol=1e-15)
