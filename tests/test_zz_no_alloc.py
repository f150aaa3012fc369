"""GPU test of the entry point that allocates nothing: lsq_layernorm_bwd_noalloc keeps the partial rows of its
column sums in a device array the library holds, and must give the bits of lsq_layernorm_bwd (same kernels)
and match the oracle, on two calls in a row, the second one smaller than the first (stale partial rows of the
first call stay in the array behind the second call's)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2110_05722_amd as L
from tests._util import assert_close_f32, assert_close_store, dev, say
from workloads import encode, to_torch

pytestmark = pytest.mark.gpu


def _case(rows, hidden, dt, seed):
    r = np.random.default_rng(seed)
    f = lambda *shape, s=1.0, m=0.0: encode((r.standard_normal(shape) * s + m).astype(np.float32), dt)
    return dict(x=f(rows, hidden), gamma=f(hidden, s=0.1, m=1.0), beta=f(hidden, s=0.1), dy=f(rows, hidden),
                dres=f(rows, hidden))


@pytest.mark.parametrize("dt", ["f16", "bf16"])
def test_two_calls_in_a_row_second_smaller(dt):
    d = dev()
    # the first call fills all 256 partial rows of the widest row the array takes; the second uses a
    # corner of the same memory (fewer, shorter partial rows), the third a shape off the register buckets
    for rows, hidden, with_res in ((4096, 4096, True), (200, 768, False), (37, 260, True)):
        say(f"[layernorm_bwd_noalloc] rows={rows} hidden={hidden} dres={with_res} dt={dt}")
        t = _case(rows, hidden, dt, rows + hidden)
        g = {k: to_torch(v, dt, d) for k, v in t.items()}
        _, mean, rstd = L.lsq_layernorm_fwd(g["x"], g["gamma"], g["beta"], 1e-5)
        dres = g["dres"] if with_res else None
        dx_ref, dg_ref, db_ref = L.lsq_layernorm_bwd(g["dy"], g["x"], g["gamma"], mean, rstd, dres_in=dres)
        dx, dg, db = torch.empty_like(g["x"]), torch.empty(hidden, device=d), torch.empty(hidden, device=d)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        L.lsq_layernorm_bwd_noalloc(g["dy"], g["x"], g["gamma"], mean, rstd, dx, dg, db, dres_in=dres)
        assert torch.cuda.memory_allocated() == before            # nothing came from torch's allocator either
        torch.cuda.synchronize()
        assert torch.equal(dx, dx_ref) and torch.equal(dg, dg_ref) and torch.equal(db, db_ref)
        rdx, rdg, rdb = oracle.layernorm_bwd(t["dy"], t["x"], t["gamma"], 1e-5, dt, dres_in=t["dres"] if with_res else None)
        rstd_max = float(rstd.max())
        assert_close_store(dx, rdx, dt, "dx")
        assert_close_f32(dg, rdg, "dgamma", floor=4e-6 * np.sqrt(rows) * 8 * (1 + rstd_max))
        assert_close_f32(db, rdb, "dbeta", floor=4e-6 * np.sqrt(rows) * 8)


def test_limit_and_empty():
    d = dev()
    say("[layernorm_bwd_noalloc] beyond the limit, empty batch")
    hidden = 8192                                   # 256 partial rows x 2 x 8192 x 4 B = 16 MiB > 8 MiB
    x = torch.zeros((4096, hidden), dtype=torch.float16, device=d)
    v = torch.ones(hidden, dtype=torch.float16, device=d)
    s = torch.ones(4096, device=d)
    o = torch.empty(hidden, device=d)
    with pytest.raises(L.LsqError, match="WORKSPACE_TOO_SMALL"):
        L.lsq_layernorm_bwd_noalloc(x, x, v, s, s, torch.empty_like(x), o, o.clone())
    z = torch.zeros((0, 64), dtype=torch.float16, device=d)
    dg, db = torch.ones(64, device=d), torch.ones(64, device=d)
    L.lsq_layernorm_bwd_noalloc(z, z, torch.ones(64, dtype=torch.float16, device=d), s[:0], s[:0], z.clone(), dg, db)
    torch.cuda.synchronize()
    assert not dg.any() and not db.any()
