"""GPU parity: fused bias + activation + dropout (FFN) through the C-ABI against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2110_05722_amd as L
from tests._util import assert_close_f32, assert_close_store, dev, say
from workloads import CONFIGS, layer_tensors, to_torch

pytestmark = pytest.mark.gpu

# (rows, ffn width, p): the FFN widths of the configurations, then buckets, ragged and generic shapes
SHAPES = [(512, 2048, 0.1), (2048, 4096, 0.1), (1024, 5120, 0.1), (1000, 768, 0.3), (37, 64, 0.0), (5, 8, 0.25),
          (3, 1536, 0.1), (7, 257, 0.2), (33, 50, 0.1), (1, 4096, 0.1),
          # hidden not a multiple of 8 (the flat walk in packs): ragged last pack, two trips, accumulators outside LDS
          (3, 13, 0.1), (4100, 1031, 0.1), (9, 8197, 0.1), (300, 5124, 0.0)]


@pytest.mark.parametrize("act", ["relu", "gelu", "gelu_tanh"])
@pytest.mark.parametrize("dt", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("rows,hidden,p", SHAPES)
def test_bias_act_dropout_fwd_bwd(rows, hidden, p, dt, act):
    if dt == "f32" and rows * hidden > 1 << 21:
        pytest.skip("fp32 storage is exercised on the small shapes only")
    say(f"[bias_act_dropout] rows={rows} hidden={hidden} p={p} dt={dt} act={act}")
    seed, offset = 99, hidden
    t = layer_tensors(CONFIGS[0], dt, rows=rows, hidden=hidden, stream=500 + rows % 83 + hidden)
    d = dev()
    x, bias, dy = (to_torch(t[k], dt, d) for k in ("x", "bias", "dy"))
    out = L.lsq_bias_act_dropout_fwd(x, bias, act, p, seed, offset)
    ref = oracle.bias_act_dropout_fwd(t["x"], t["bias"], act, p, seed, offset, dt)
    assert_close_store(out, ref, dt, "out", f32_floor=2e-6)
    out_nb = L.lsq_bias_act_dropout_fwd(x, None, act, p, seed, offset)
    assert_close_store(out_nb, oracle.bias_act_dropout_fwd(t["x"], None, act, p, seed, offset, dt), dt, "out(no bias)",
                       f32_floor=2e-6)
    dx, dbias = L.lsq_bias_act_dropout_bwd(dy, x, bias, act, p, seed, offset)
    rdx, rdb = oracle.bias_act_dropout_bwd(t["dy"], t["x"], t["bias"], act, p, seed, offset, dt)
    assert_close_store(dx, rdx, dt, "dx", f32_floor=4e-6)
    assert_close_f32(dbias, rdb, "dbias", floor=1e-6 * np.sqrt(rows) * 4)
    # in place over dy, and without dbias
    dyc = dy.clone()
    dx2, none = L.lsq_bias_act_dropout_bwd(dyc, x, bias, act, p, seed, offset, want_dbias=False, dx=dyc)
    assert none is None and torch.equal(dx, dx2)


def test_bias_act_relu_kink_and_mask():
    say("[bias_act_dropout] ReLU at exactly zero; mask bit-exact")
    d = dev()
    x = torch.tensor([[-1.0, 0.0, 1.0, 0.0, 2.0, -0.0, 0.5, -3.0]], dtype=torch.float16, device=d)
    one = torch.ones_like(x)
    dx, _ = L.lsq_bias_act_dropout_bwd(one, x, None, "relu", 0.0, 1, 0)
    assert dx.cpu().tolist() == [[0, 0, 1, 0, 1, 0, 1, 0]]
    rows, hidden, p = 513, 520, 0.3
    ones = torch.ones((rows, hidden), dtype=torch.float16, device=d)
    out = L.lsq_bias_act_dropout_fwd(ones, None, "relu", p, 77, 5)
    keep = oracle.dropout_mask(rows * hidden, p, 77, 5).reshape(rows, hidden)
    assert np.array_equal((out != 0).cpu().numpy().astype(np.uint8), keep)


def test_bias_act_empty():
    d = dev()
    x = torch.empty((0, 64), dtype=torch.float16, device=d)
    out = L.lsq_bias_act_dropout_fwd(x, None, "gelu", 0.1, 1, 0)
    dx, dbias = L.lsq_bias_act_dropout_bwd(x, x, None, "gelu", 0.1, 1, 0)
    torch.cuda.synchronize()
    assert out.numel() == 0 and dbias.abs().sum().item() == 0
