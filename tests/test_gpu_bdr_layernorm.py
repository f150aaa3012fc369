"""GPU parity: the fused sub-layer boundary (bias+dropout+residual + LayerNorm in one pass) through the C-ABI.

Two statements are checked: (1) the fused entry points equal the two separate entry points bit for bit on
every streamed output (the column sums only up to summation order); (2) they match the CPU oracle, which
is the composition of the two oracle operators with the intermediate rounded to its storage type.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2110_05722_amd as L
from tests._util import assert_close_f32, assert_close_store, dev, say
from workloads import decode, encode, from_torch, to_torch

pytestmark = pytest.mark.gpu

# (rows, hidden): the five workload shapes, every register bucket, ragged tails, the no-bucket fallback
SHAPES = [(512, 512), (4096, 512), (8192, 1024), (8192, 1280), (37, 64), (19, 128), (5, 256), (33, 768), (9, 1536),
          (7, 2048), (3, 4096), (2, 8192), (1, 8), (50, 257), (3, 16384), (6, 5120), (3, 6144),
          (300, 12288), (11, 8200), (7, 16392)]


def _inputs(rows, hidden, dt, seed):
    r = np.random.default_rng(seed)
    f = lambda *shape, s=1.0, m=0.0: encode((r.standard_normal(shape) * s + m).astype(np.float32), dt)
    return dict(x=f(rows, hidden), res=f(rows, hidden), bias=f(hidden, s=0.1), gamma=f(hidden, s=0.1, m=1.0),
                beta=f(hidden, s=0.1), dy=f(rows, hidden), dres=f(rows, hidden))


@pytest.mark.parametrize("dt", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("rows,hidden", SHAPES)
@pytest.mark.parametrize("p", [0.0, 0.1])
def test_fused_equals_the_two_operators_and_the_oracle(rows, hidden, p, dt):
    if dt == "f32" and rows * hidden > 1 << 21:
        pytest.skip("fp32 storage is exercised on the small shapes only")
    say(f"[bdr+ln] rows={rows} hidden={hidden} p={p} dt={dt}")
    d = dev()
    t = _inputs(rows, hidden, dt, rows * 7 + hidden)
    g = {k: to_torch(v, dt, d) for k, v in t.items()}
    seed, off = 1234, 77
    # ---- forward
    h, y, mean, rstd = L.lsq_bdr_layernorm_fwd(g["x"], g["bias"], g["res"], g["gamma"], g["beta"], p, seed, off)
    h2 = L.lsq_bias_dropout_residual_fwd(g["x"], g["bias"], g["res"], p, seed, off)
    y2, mean2, rstd2 = L.lsq_layernorm_fwd(h2, g["gamma"], g["beta"])
    assert torch.equal(h, h2) and torch.equal(y, y2) and torch.equal(mean, mean2) and torch.equal(rstd, rstd2)
    rh = oracle.bias_dropout_residual_fwd(t["x"], t["bias"], t["res"], p, seed, off, dt)
    assert_close_store(h, rh, dt, "h")
    hs = from_torch(h, dt).reshape(rows, hidden)                        # the stored h is what is normalised
    ry, rmean, rrstd = oracle.layernorm_fwd(hs, t["gamma"], t["beta"], 1e-5, dt)
    assert_close_store(y, ry, dt, "y", f32_floor=1e-6 * (1 + float(np.max(rrstd))))
    assert_close_f32(mean, rmean, "mean", floor=2e-7 * float(np.max(np.abs(decode(hs, dt))) + 1))
    assert_close_f32(rstd, rrstd, "rstd", floor=0.0)
    # without a bias
    h3, y3, _, _ = L.lsq_bdr_layernorm_fwd(g["x"], None, g["res"], g["gamma"], g["beta"], p, seed, off)
    h4 = L.lsq_bias_dropout_residual_fwd(g["x"], None, g["res"], p, seed, off)
    assert torch.equal(h3, h4) and torch.equal(y3, L.lsq_layernorm_fwd(h4, g["gamma"], g["beta"])[0])
    # ---- backward
    for dres in (g["dres"], None):
        dh, dx, dgm, dbt, dbi = L.lsq_bdr_layernorm_bwd(g["dy"], h, g["gamma"], mean, rstd, p, seed, off, dres_in=dres)
        dh2, dgm2, dbt2 = L.lsq_layernorm_bwd(g["dy"], h, g["gamma"], mean, rstd, dres_in=dres)
        dx2, dbi2 = L.lsq_bias_dropout_residual_bwd(dh2, p, seed, off)
        assert torch.equal(dh, dh2) and torch.equal(dx, dx2)
        fl = 4e-6 * np.sqrt(rows) * 4
        assert_close_f32(dgm, dgm2.cpu().numpy(), "dgamma vs two calls", floor=fl * (1 + float(np.max(rrstd))))
        assert_close_f32(dbt, dbt2.cpu().numpy(), "dbeta vs two calls", floor=fl)
        assert_close_f32(dbi, dbi2.cpu().numpy(), "dbias vs two calls", floor=fl * 2)
    rdh, rdg, rdb = oracle.layernorm_bwd(t["dy"], hs, t["gamma"], 1e-5, dt)
    assert_close_store(dh, rdh, dt, "dh", f32_floor=1e-6 * (1 + float(np.max(rrstd))) ** 2 * 4)
    rdx, rdbias = oracle.bias_dropout_residual_bwd(from_torch(dh, dt).reshape(rows, hidden), p, seed, off, dt)
    assert_close_store(dx, rdx, dt, "dx")
    assert np.array_equal(decode(from_torch(dx, dt), dt).reshape(rows, hidden) == 0, rdx == 0)     # the mask, bit for bit
    assert_close_f32(dbi, rdbias, "dbias", floor=4e-6 * np.sqrt(rows) * 8)
    assert_close_f32(dgm, rdg, "dgamma", floor=4e-6 * np.sqrt(rows) * 8 * (1 + float(np.max(rrstd))))


def test_errors_and_empty():
    say("[bdr+ln] empty batch, workspace too small")
    d = dev()
    H = 64
    z = torch.zeros((0, H), dtype=torch.float16, device=d)
    v = torch.ones(H, dtype=torch.float16, device=d)
    h, y, mean, rstd = L.lsq_bdr_layernorm_fwd(z, v, z, v, v, 0.1, 1, 0)
    assert h.shape == (0, H) and mean.numel() == 0
    dh, dx, dgm, dbt, dbi = L.lsq_bdr_layernorm_bwd(z, z, v, mean, rstd, 0.1, 1, 0)
    assert not dgm.any() and not dbt.any() and not dbi.any()
    x = torch.randn((64, H), device=d).half()
    h, y, mean, rstd = L.lsq_bdr_layernorm_fwd(x, v, x, v, v, 0.1, 1, 0)
    with pytest.raises(L.LsqError, match="WORKSPACE_TOO_SMALL"):
        L.lsq_bdr_layernorm_bwd(x, h, v, mean, rstd, 0.1, 1, 0, workspace=torch.empty(16, dtype=torch.uint8, device=d))
