"""GPU parity of the softmax's launch-shape candidates and of the run-time search (paper Sec. IV-B, Softmax: several
templates, the best found by a search before training).  Every candidate of every row-length bucket is forced in turn
and must match the CPU oracle like the default does; then the search itself is run and its record checked."""
import numpy as np
import pytest
import torch

import oracle
import paper_2110_05722_amd as L
from tests._util import assert_close_store, dev, say, to_np64
from workloads import CONFIGS, attention_tensors, from_torch, to_torch

pytestmark = pytest.mark.gpu

# (batch, heads, q_len, k_len): one row length per bucket that has a choice, rows enough for several workgroups
# (so that candidates with two rows per lane group are not folded to one) and a ragged last workgroup
SHAPES = [(70, 4, 37, 8), (36, 4, 37, 16), (20, 4, 37, 32), (12, 4, 37, 64), (6, 4, 37, 128), (3, 4, 37, 256), (2, 4, 37, 512),
          (1, 4, 37, 1024), (700, 4, 40, 128)]


def _run_and_check(t, dt, kl_np, causal, p, tag):
    d = dev()
    scale, seed, offset = 0.125, 99, 5
    x, dy = to_torch(t["x"], dt, d), to_torch(t["dy"], dt, d)
    kl = None if kl_np is None else torch.from_numpy(kl_np).to(d)
    y, yd = L.lsq_softmax_fwd(x, kl, causal, scale, p, seed, offset)
    ry, ryd = oracle.softmax_fwd(t["x"], kl_np, causal, scale, dt, p, seed, offset)
    assert_close_store(y, ry, dt, tag + " y", f32_floor=1e-7)
    masked = ry == 0.0
    assert not from_torch(y, dt).reshape(ry.shape)[masked].view(np.uint16 if dt != "f32" else np.uint32).any()
    if p > 0:
        assert_close_store(yd, ryd, dt, tag + " y_drop", f32_floor=1e-7)
        assert np.array_equal(to_np64(yd, dt) == 0, ryd == 0)
    dx = L.lsq_softmax_bwd(dy, y, kl, causal, scale, p, seed, offset)
    rdx = oracle.softmax_bwd(t["dy"], from_torch(y, dt), kl_np, causal, scale, dt, p, seed, offset)
    assert_close_store(dx, rdx, dt, tag + " dx", f32_floor=1e-7)
    assert not from_torch(dx, dt).reshape(ry.shape)[masked].view(np.uint16 if dt != "f32" else np.uint32).any()


@pytest.mark.parametrize("dt", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("B,N,Lq,Lk", SHAPES)
def test_every_candidate_matches_the_oracle(B, N, Lq, Lk, dt):
    if dt == "f32" and B > 100:
        pytest.skip("fp32 storage is exercised on the small shapes only")
    ncand = L.lsq_softmax_candidates(Lk)
    assert 1 <= ncand <= 4
    t = attention_tensors(CONFIGS[0], dt, batch=B, heads=N, q_len=Lq, k_len=Lk, stream=700 + Lk)
    x = to_torch(t["x"], dt, dev())
    dy = to_torch(t["dy"], dt, dev())
    try:
        for mask, p in (("pad", 0.1), ("pad+causal", 0.0), ("none", 0.0), ("causal", 0.1)):
            kl_np = t["key_len"] if "pad" in mask else None
            kl = None if kl_np is None else torch.from_numpy(kl_np).to(dev())
            for c in range(ncand):
                say(f"[softmax_tune] B={B} N={N} Lq={Lq} Lk={Lk} mask={mask} p={p} dt={dt} candidate {c} of {ncand}")
                bf, bb, _ = L.lsq_softmax_tune(x, dy, kl, None, "causal" in mask, 0.125, p, force=c)
                assert (bf, bb) == (c, c)
                _run_and_check(t, dt, kl_np, "causal" in mask, p, f"candidate {c}")
    finally:
        for mask, p in (("pad", 0.1), ("pad+causal", 0.0), ("none", 0.0), ("causal", 0.1)):
            kl = torch.from_numpy(t["key_len"]).to(dev()) if "pad" in mask else None
            L.lsq_softmax_tune(x, dy, kl, None, "causal" in mask, 0.125, p, force=-2)


def test_search_records_a_valid_choice_and_results_stay_right():
    say("[softmax_tune] search on the transformer-big attention shape (8 of 64 batches)")
    dt, d = "f16", dev()
    B, N, Lq, Lk = 8, 16, 128, 128
    t = attention_tensors(CONFIGS[2], dt, batch=B, heads=N, q_len=Lq, k_len=Lk, stream=811)
    x, dy = to_torch(t["x"], dt, d), to_torch(t["dy"], dt, d)
    kl = torch.from_numpy(t["key_len"]).to(d)
    try:
        bf, bb, us = L.lsq_softmax_tune(x, dy, kl, None, False, 0.125, 0.1, seed=99, offset=5, force=-1, reps=10)
        n = L.lsq_softmax_candidates(Lk)
        assert 0 <= bf < n and 0 <= bb < n
        for dirn in range(2):
            assert all(u > 0 for u in us[dirn][:n]) and all(u == -1 for u in us[dirn][n:])
            assert us[dirn][(bf, bb)[dirn]] == min(us[dirn][:n])
        say(f"[softmax_tune] chosen fwd {bf} bwd {bb}; us per launch {us}")
        _run_and_check(t, dt, t["key_len"], False, 0.1, "after the search")
    finally:
        L.lsq_softmax_tune(x, dy, kl, None, False, 0.125, 0.1, force=-2)
    # a row length with one shape only: nothing to search, nothing launched
    assert L.lsq_softmax_candidates(2048) == 1 and L.lsq_softmax_candidates(100) == 1
    x2 = torch.zeros((1, 1, 2, 2048), dtype=torch.float16, device=d)
    assert L.lsq_softmax_tune(x2, x2, force=-1)[:2] == (0, 0)
    with pytest.raises(L.LsqError, match="INVALID_ARG"):
        L.lsq_softmax_tune(x, dy, kl, None, False, 0.125, 0.1, force=7)
