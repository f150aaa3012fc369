"""GPU parity: fused bias + dropout + residual through the C-ABI against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2110_05722_amd as L
from tests._util import assert_close_f32, assert_close_store, dev, say
from workloads import CONFIGS, layer_tensors, to_torch

pytestmark = pytest.mark.gpu

SHAPES = [
    (512, 512, 0.1), (4096, 512, 0.1), (8192, 1024, 0.3), (8192, 1280, 0.1),
    (4096, 256, 0.1), (1000, 768, 0.5), (37, 64, 0.1), (5, 8, 0.25), (3, 1536, 0.1), (2, 8192, 0.1),
    (1, 1024, 0.1), (7, 257, 0.2), (33, 50, 0.1), (9, 1, 0.5), (131, 520, 0.0),
    # hidden not a multiple of 8 (the flat walk in packs): a ragged last pack, rows shorter than a pack, two trips per
    # workgroup (more than 512 x 8192 elements), column accumulators outside LDS (more than 8192 columns), no dropout
    (3, 13, 0.1), (1031, 3, 0.2), (4100, 1031, 0.1), (9, 8197, 0.1), (700, 1281, 0.0),
]


def _case(rows, hidden, dt):
    return layer_tensors(CONFIGS[0], dt, rows=rows, hidden=hidden, stream=200 + rows % 89 + hidden)


@pytest.mark.parametrize("dt", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("rows,hidden,p", SHAPES)
def test_bdr_fwd_bwd(rows, hidden, p, dt):
    if dt == "f32" and rows * hidden > 1 << 21:
        pytest.skip("fp32 storage is exercised on the small shapes only")
    say(f"[bias_dropout_residual] rows={rows} hidden={hidden} p={p} dt={dt}")
    seed, offset = 1234, rows  # a different Philox offset per case
    t = _case(rows, hidden, dt)
    d = dev()
    x, bias, res, dy = (to_torch(t[k], dt, d) for k in ("x", "bias", "residual", "dy"))
    out = L.lsq_bias_dropout_residual_fwd(x, bias, res, p, seed, offset)
    ref = oracle.bias_dropout_residual_fwd(t["x"], t["bias"], t["residual"], p, seed, offset, dt)
    assert_close_store(out, ref, dt, "out")
    out_nb = L.lsq_bias_dropout_residual_fwd(x, None, res, p, seed, offset)
    ref_nb = oracle.bias_dropout_residual_fwd(t["x"], None, t["residual"], p, seed, offset, dt)
    assert_close_store(out_nb, ref_nb, dt, "out(no bias)")

    dx, dbias = L.lsq_bias_dropout_residual_bwd(dy, p, seed, offset)
    rdx, rdb = oracle.bias_dropout_residual_bwd(t["dy"], p, seed, offset, dt)
    assert_close_store(dx, rdx, dt, "dx")
    assert_close_f32(dbias, rdb, "dbias", floor=1e-6 * np.sqrt(rows) * 4)
    dx2, none = L.lsq_bias_dropout_residual_bwd(dy, p, seed, offset, want_dbias=False)
    assert none is None and torch.equal(dx, dx2)


@pytest.mark.parametrize("rows,hidden", [(8192, 1024), (513, 520), (64, 257)])
@pytest.mark.parametrize("p", [0.1, 0.3])
def test_dropout_mask_is_bit_exact_and_shared_by_fwd_and_bwd(rows, hidden, p):
    say(f"[bias_dropout_residual] mask rows={rows} hidden={hidden} p={p}")
    d = dev()
    seed, offset = 0xDEADBEEF12345678, (1 << 33) + 5
    ones = torch.ones((rows, hidden), dtype=torch.float16, device=d)
    zeros = torch.zeros_like(ones)
    keep = oracle.dropout_mask(rows * hidden, p, seed, offset).reshape(rows, hidden)
    fwd = L.lsq_bias_dropout_residual_fwd(ones, None, zeros, p, seed, offset)
    dx, _ = L.lsq_bias_dropout_residual_bwd(ones, p, seed, offset)
    m_fwd = (fwd != 0).cpu().numpy().astype(np.uint8)
    m_bwd = (dx != 0).cpu().numpy().astype(np.uint8)
    assert np.array_equal(m_fwd, keep)
    assert np.array_equal(m_bwd, keep)
    # kept values carry exactly the nominal 1/(1-p)
    scale = torch.tensor(1.0 / (1.0 - float(np.float32(p))), dtype=torch.float32).to(torch.float16).item()
    assert torch.all((fwd == 0) | (fwd == scale))


def test_dropout_rate_below_the_16_bit_grid_keeps_everything_and_still_scales():
    """p < 2^-17 rounds to T16 = 0: every element is kept, the nominal 1/(1-p) is still applied (oracle: same)."""
    say("[bias_dropout_residual] p = 2^-18")
    dt, d, p = "f32", dev(), 2.0 ** -18
    t = _case(64, 264, dt)
    x, bias, res, dy = (to_torch(t[k], dt, d) for k in ("x", "bias", "residual", "dy"))
    out = L.lsq_bias_dropout_residual_fwd(x, bias, res, p, 5, 0)
    assert_close_store(out, oracle.bias_dropout_residual_fwd(t["x"], t["bias"], t["residual"], p, 5, 0, dt), dt, "out")
    dx, dbias = L.lsq_bias_dropout_residual_bwd(dy, p, 5, 0)
    rdx, rdb = oracle.bias_dropout_residual_bwd(t["dy"], p, 5, 0, dt)
    assert_close_store(dx, rdx, dt, "dx")
    scale = torch.tensor(1.0 / (1.0 - p), dtype=torch.float32, device=d)
    assert torch.equal(dx, dy * scale)                       # all kept, all scaled
    # the softmax takes y_drop for any p > 0
    sx = torch.randn((2, 2, 8, 16), device=d).half()
    y, yd = L.lsq_softmax_fwd(sx, None, False, 1.0, p, 5, 0)
    assert torch.allclose(yd.float(), y.float() * scale, rtol=2e-3, atol=1e-6) and bool((yd > 0).all())


def test_bdr_generic_in_place_sums_columns_before_it_overwrites_dy():
    say("[bias_dropout_residual] in place, hidden 257 (generic path)")
    dt, d = "f16", dev()
    t = _case(300, 257, dt)
    dy = to_torch(t["dy"], dt, d)
    dyc = dy.clone()
    dx, dbias = L.lsq_bias_dropout_residual_bwd(dyc, 0.25, 11, 3, dx=dyc)
    rdx, rdb = oracle.bias_dropout_residual_bwd(t["dy"], 0.25, 11, 3, dt)
    assert_close_store(dx, rdx, dt, "dx in place")
    assert_close_f32(dbias, rdb, "dbias in place", floor=4e-6 * np.sqrt(300) * 8)


def test_bdr_in_place_and_reproducible():
    say("[bias_dropout_residual] in place / reproducible")
    dt, d = "f16", dev()
    t = _case(1024, 1024, dt)
    x, bias, res, dy = (to_torch(t[k], dt, d) for k in ("x", "bias", "residual", "dy"))
    a = L.lsq_bias_dropout_residual_fwd(x, bias, res, 0.1, 7, 0)
    xc = x.clone()
    b = L.lsq_bias_dropout_residual_fwd(xc, bias, res, 0.1, 7, 0, out=xc)
    assert torch.equal(a, b)
    dx1, db1 = L.lsq_bias_dropout_residual_bwd(dy, 0.1, 7, 0)
    dyc = dy.clone()
    dx2, db2 = L.lsq_bias_dropout_residual_bwd(dyc, 0.1, 7, 0, dx=dyc)
    assert torch.equal(dx1, dx2) and torch.equal(db1, db2)


def test_bdr_empty():
    d = dev()
    x = torch.empty((0, 64), dtype=torch.float16, device=d)
    out = L.lsq_bias_dropout_residual_fwd(x, None, x, 0.1, 1, 0)
    dx, dbias = L.lsq_bias_dropout_residual_bwd(x, 0.1, 1, 0)
    torch.cuda.synchronize()
    assert out.numel() == 0 and dbias.abs().sum().item() == 0
