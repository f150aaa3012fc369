"""Host threads sharing the library on one GPU: the three pieces of host-side state the library keeps (the raised LDS
limit of the widest LayerNorm backward, the per-device address of the no-alloc entry point's scratch array, the table
of recorded softmax launch shapes) are set up and read under concurrent calls from several threads, each on its own
stream.  Every result must equal the bits of the same call made alone: for the softmax, whose recorded launch shape
another thread keeps changing meanwhile, the bits of one of its candidates."""
import threading

import numpy as np
import pytest
import torch

import paper_2110_05722_amd as L
from tests._util import dev, say
from workloads import encode, to_torch

pytestmark = pytest.mark.gpu

ROUNDS = 12


def _ln_inputs(rows, hidden, seed, d):
    r = np.random.default_rng(seed)
    f = lambda *shape, s=1.0, m=0.0: to_torch(encode((r.standard_normal(shape) * s + m).astype(np.float32), "f16"), "f16", d)
    x, gamma, beta, dy = f(rows, hidden), f(hidden, s=0.1, m=1.0), f(hidden, s=0.1), f(rows, hidden)
    _, mean, rstd = L.lsq_layernorm_fwd(x, gamma, beta, 1e-5)
    return dy, x, gamma, mean, rstd


def test_concurrent_host_threads_give_the_single_thread_bits():
    d = dev()
    say("[threads] four host threads: wide LayerNorm backward, no-alloc LayerNorm backward, softmax, softmax shape records")
    wide = _ln_inputs(48, 16384, 1, d)          # the 1024-thread kernel whose LDS limit is raised on first use
    noal = _ln_inputs(600, 1024, 2, d)
    wide_ref = L.lsq_layernorm_bwd(*wide)
    noal_ref = L.lsq_layernorm_bwd(*noal)

    B, N, Lq, Lk = 6, 4, 96, 128
    g = torch.Generator(device="cpu").manual_seed(3)
    x = (torch.randn(B, N, Lq, Lk, generator=g) * 2).to(torch.float16).to(d)
    dy = torch.randn(B, N, Lq, Lk, generator=g).to(torch.float16).to(d)
    kl = torch.tensor([128, 1, 77, 64, 100, 9], dtype=torch.int32, device=d)
    ncand = L.lsq_softmax_candidates(Lk)
    sm_refs = []
    try:
        for c in range(ncand):
            L.lsq_softmax_tune(x, dy, kl, None, False, 0.125, 0.1, force=c)
            y, yd = L.lsq_softmax_fwd(x, kl, False, 0.125, 0.1, 11, 3)
            sm_refs.append((y, yd))
        y0 = sm_refs[0][0]
        bw_refs = []
        for c in range(ncand):                  # backward of ONE stored y under every candidate
            L.lsq_softmax_tune(x, dy, kl, None, False, 0.125, 0.1, force=c)
            bw_refs.append(L.lsq_softmax_bwd(dy, y0, kl, False, 0.125, 0.1, 11, 3))
    finally:
        L.lsq_softmax_tune(x, dy, kl, None, False, 0.125, 0.1, force=-2)
    torch.cuda.synchronize()

    errors = []
    start = threading.Barrier(4)

    def guarded(fn):
        def run():
            try:
                torch.cuda.set_device(d)
                start.wait(timeout=60)
                with torch.cuda.stream(torch.cuda.Stream(device=d)):
                    fn()
                    torch.cuda.current_stream().synchronize()
            except Exception as e:          # noqa: BLE001 - reported by the main thread
                errors.append(repr(e))
        return run

    def t_wide():
        for i in range(ROUNDS):
            out = L.lsq_layernorm_bwd(*wide)
            torch.cuda.current_stream().synchronize()
            if not all(torch.equal(a, b) for a, b in zip(out, wide_ref)):
                errors.append(f"wide LayerNorm backward differs in round {i}")

    def t_noalloc():
        rows, hidden = noal[1].shape
        dx, dg, db = torch.empty_like(noal[1]), torch.empty(hidden, device=d), torch.empty(hidden, device=d)
        for i in range(ROUNDS):
            L.lsq_layernorm_bwd_noalloc(*noal, dx, dg, db)
            torch.cuda.current_stream().synchronize()
            if not all(torch.equal(a, b) for a, b in zip((dx, dg, db), noal_ref)):
                errors.append(f"no-alloc LayerNorm backward differs in round {i}")

    def t_softmax():
        for i in range(ROUNDS):
            y, yd = L.lsq_softmax_fwd(x, kl, False, 0.125, 0.1, 11, 3)
            dx = L.lsq_softmax_bwd(dy, y0, kl, False, 0.125, 0.1, 11, 3)
            torch.cuda.current_stream().synchronize()
            if not any(torch.equal(y, r[0]) and torch.equal(yd, r[1]) for r in sm_refs):
                errors.append(f"softmax forward equals none of its candidates in round {i}")
            if not any(torch.equal(dx, r) for r in bw_refs):
                errors.append(f"softmax backward equals none of its candidates in round {i}")

    def t_records():
        for i in range(ROUNDS * 4):
            L.lsq_softmax_tune(x, dy, kl, None, False, 0.125, 0.1, force=i % ncand)
        L.lsq_softmax_tune(x, dy, kl, None, False, 0.125, 0.1, force=-2)

    threads = [threading.Thread(target=guarded(f)) for f in (t_wide, t_noalloc, t_softmax, t_records)]
    try:
        for t in threads:
            t.start()
        for t in threads:
            t.join(timeout=120)
        assert not any(t.is_alive() for t in threads), "a host thread did not finish"
    finally:
        torch.cuda.synchronize()
        L.lsq_softmax_tune(x, dy, kl, None, False, 0.125, 0.1, force=-2)
    assert not errors, errors
    # and afterwards the default is back
    y, yd = L.lsq_softmax_fwd(x, kl, False, 0.125, 0.1, 11, 3)
    assert torch.equal(y, sm_refs[0][0]) and torch.equal(yd, sm_refs[0][1])
