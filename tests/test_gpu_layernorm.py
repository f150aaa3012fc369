"""GPU parity: LayerNorm forward / backward through the C-ABI against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2110_05722_amd as L
from tests._util import assert_close_f32, assert_close_store, dev, say
from workloads import CONFIGS, layer_tensors, to_torch

pytestmark = pytest.mark.gpu
EPS = 1e-5

# (rows, hidden): the shapes of the five workload configurations first, then every shape bucket, ragged tails and the generic path
SHAPES = [
    (512, 512), (4096, 512), (8192, 1024), (8192, 1280),
    (4096, 256), (1000, 768), (37, 64), (5, 8), (129, 128), (3, 1536), (67, 2048),
    (9, 4096), (5, 8192), (1, 1024), (7, 257), (33, 50), (3, 16384), (2, 1),
    (11, 5120), (6, 6144), (5, 4104),         # 256 lanes x 3 packs: ragged, exact, first past 256 x 2
    (300, 12288), (11, 8200), (7, 16392),     # the 1024-lane row bucket (up to 16384), ragged inside it, and beyond it
    (13, 2051), (6, 20001), (5, 20480),       # rows off the pack grid: one wave per row up to 2048 columns, a workgroup per row beyond; whole packs beyond 16384
]


def _case(rows, hidden, dt, seed=0):
    cfg = CONFIGS[seed % len(CONFIGS)]
    return layer_tensors(cfg, dt, rows=rows, hidden=hidden, stream=100 + rows % 97 + hidden)


@pytest.mark.parametrize("dt", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("rows,hidden", SHAPES)
def test_layernorm_fwd_bwd(rows, hidden, dt):
    if dt == "f32" and rows * hidden > 1 << 21:
        pytest.skip("fp32 storage is exercised on the small shapes only")
    say(f"[layernorm] rows={rows} hidden={hidden} dt={dt}")
    t = _case(rows, hidden, dt)
    d = dev()
    x, gamma, beta, dy, res = (to_torch(t[k], dt, d) for k in ("x", "gamma", "beta", "dy", "residual"))
    y, mean, rstd = L.lsq_layernorm_fwd(x, gamma, beta, EPS)
    ry, rmean, rrstd = oracle.layernorm_fwd(t["x"], t["gamma"], t["beta"], EPS, dt)
    assert_close_store(y, ry, dt, "y")
    # mean: |x| ~ 1, a sum of `hidden` terms carries about sqrt(hidden) * 2^-24 absolute error before the division
    assert_close_f32(mean, rmean, "mean", floor=2e-7)
    assert_close_f32(rstd, rrstd, "rstd")

    for with_res in (False, True):
        dx, dgamma, dbeta = L.lsq_layernorm_bwd(dy, x, gamma, mean, rstd, dres_in=res if with_res else None)
        rdx, rdg, rdb = oracle.layernorm_bwd(t["dy"], t["x"], t["gamma"], EPS, dt,
                                             dres_in=t["residual"] if with_res else None)
        # dx = rstd * (difference of O(|g|) terms): the fp32 rounding floor scales with rstd, which is
        # 1/sqrt(eps) = 316 for a zero-variance row (hidden == 1)
        assert_close_store(dx, rdx, dt, f"dx(res={with_res})", f32_floor=1e-6 * max(1.0, float(rrstd.max())))
        floor = 1e-6 * np.sqrt(rows) * 4
        assert_close_f32(dgamma, rdg, "dgamma", floor=floor)
        assert_close_f32(dbeta, rdb, "dbeta", floor=floor)


def test_layernorm_special_rows():
    say("[layernorm] constant rows / large offset")
    d = dev()
    H = 1024
    x = torch.full((4, H), 3.25, dtype=torch.float16, device=d)
    x[1] = 1000.0                       # |mean| >> sigma: the one-pass variance would cancel here
    x[2, ::2] = 1000.0; x[2, 1::2] = 1001.0
    x[3] = torch.linspace(-2, 2, H, device=d).to(torch.float16)
    gamma = torch.ones(H, dtype=torch.float16, device=d)
    beta = torch.full((H,), 0.5, dtype=torch.float16, device=d)
    y, mean, rstd = L.lsq_layernorm_fwd(x, gamma, beta, EPS)
    xs = x.cpu().numpy().view(np.uint16)
    ry, rmean, rrstd = oracle.layernorm_fwd(xs, gamma.cpu().numpy().view(np.uint16),
                                            beta.cpu().numpy().view(np.uint16), EPS, "f16")
    assert_close_store(y, ry, "f16", "y")
    assert torch.equal(y[0], beta) and torch.equal(y[1], beta)   # constant row -> beta exactly
    assert_close_f32(mean, rmean, "mean")
    assert_close_f32(rstd, rrstd, "rstd")


def test_layernorm_bwd_in_place_and_reproducible():
    say("[layernorm] dx aliasing dy; run-to-run bit reproducibility")
    dt, d = "f16", dev()
    t = _case(2048, 1024, dt, seed=2)
    x, gamma, beta, dy = (to_torch(t[k], dt, d) for k in ("x", "gamma", "beta", "dy"))
    _, mean, rstd = L.lsq_layernorm_fwd(x, gamma, beta, EPS)
    dx1, dg1, db1 = L.lsq_layernorm_bwd(dy, x, gamma, mean, rstd)
    dx2, dg2, db2 = L.lsq_layernorm_bwd(dy, x, gamma, mean, rstd)
    assert torch.equal(dx1, dx2) and torch.equal(dg1, dg2) and torch.equal(db1, db2)
    dyc = dy.clone()
    dx3, dg3, db3 = L.lsq_layernorm_bwd(dyc, x, gamma, mean, rstd, dx=dyc)
    assert torch.equal(dx3, dx1) and torch.equal(dg3, dg1) and torch.equal(db3, db1)


def test_layernorm_empty():
    d = dev()
    x = torch.empty((0, 64), dtype=torch.float16, device=d)
    g = torch.ones(64, dtype=torch.float16, device=d)
    y, mean, rstd = L.lsq_layernorm_fwd(x, g, g, EPS)
    dx, dg, db = L.lsq_layernorm_bwd(x, x, g, mean, rstd)
    torch.cuda.synchronize()
    assert y.numel() == 0 and dg.abs().sum().item() == 0 and db.abs().sum().item() == 0
