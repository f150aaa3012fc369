"""GPU parity: masked attention softmax forward / backward through the C-ABI against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2110_05722_amd as L
from tests._util import assert_close_store, dev, say, to_np64
from workloads import CONFIGS, attention_tensors, device_normal, from_torch, to_torch

pytestmark = pytest.mark.gpu

# (batch, heads, q_len, k_len, mask, p_attn); mask in {"none", "pad", "causal", "pad+causal"}
CASES = [
    (8, 8, 64, 64, "pad", 0.0), (8, 8, 64, 64, "pad+causal", 0.0),            # config 1
    (128, 8, 32, 32, "pad", 0.0), (128, 8, 32, 32, "pad+causal", 0.0),        # config 2: enc self, dec self
    (64, 16, 128, 128, "pad", 0.1), (64, 16, 128, 128, "pad+causal", 0.1),    # config 3 with attention dropout
    (2, 16, 512, 512, "none", 0.0),                                           # config 4 shape (2 of 16 batches)
    (1, 20, 1024, 1024, "causal", 0.0),                                       # config 5 shape (1 of 8 batches)
    (3, 2, 5, 8, "pad", 0.25), (3, 2, 16, 16, "pad+causal", 0.25),            # 1 and 2 lanes per row
    (2, 3, 50, 50, "pad", 0.1), (2, 3, 33, 33, "pad+causal", 0.2),            # odd lengths: generic path
    (2, 2, 7, 24, "causal", 0.0), (2, 2, 24, 40, "pad+causal", 0.1),          # q_len != k_len, end-aligned
    (2, 2, 9, 256, "pad", 0.0), (2, 2, 9, 768, "pad", 0.1), (1, 2, 5, 1536, "causal", 0.0),
    (1, 2, 3, 2048, "pad", 0.1), (1, 1, 3, 4096, "pad", 0.1), (1, 1, 2, 1, "none", 0.0),
    # long rows: one workgroup per row (2048 < k_len <= 16384), and the fallback beyond
    (2, 1, 4, 2056, "pad", 0.1), (1, 2, 3, 8192, "pad+causal", 0.1), (1, 1, 2, 16384, "pad", 0.0),
    (1, 1, 2, 16392, "pad", 0.1), (2, 1, 5, 4099, "pad+causal", 0.1),
    # lengths that are not a multiple of 8: element-granular lanes (every bucket, both sides of each edge)
    (3, 2, 5, 7, "pad", 0.25), (3, 2, 9, 9, "pad+causal", 0.1), (4, 2, 17, 17, "pad", 0.1), (2, 2, 31, 33, "pad+causal", 0.0),
    (2, 2, 63, 63, "pad", 0.1), (2, 2, 65, 65, "causal", 0.1), (64, 4, 100, 100, "pad", 0.1), (2, 3, 127, 127, "pad+causal", 0.1),
    (2, 2, 20, 129, "pad", 0.0), (2, 2, 12, 255, "pad", 0.1), (2, 1, 9, 500, "pad", 0.1), (2, 1, 6, 513, "causal", 0.1),
    (1, 2, 5, 1001, "pad", 0.1), (1, 2, 4, 1025, "pad", 0.0), (1, 1, 3, 2047, "pad", 0.1), (1, 1, 3, 2049, "pad", 0.1),
    (1, 3, 1, 3, "none", 0.5),
]


@pytest.mark.parametrize("dt", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("B,N,Lq,Lk,mask,p", CASES)
def test_softmax_fwd_bwd(B, N, Lq, Lk, mask, p, dt):
    if dt == "f32" and B * N * Lq * Lk > 1 << 21:
        pytest.skip("fp32 storage is exercised on the small shapes only")
    say(f"[softmax] B={B} N={N} Lq={Lq} Lk={Lk} mask={mask} p={p} dt={dt}")
    cfg = next((c for c in CONFIGS if c.batch == B and c.max_len == Lk), CONFIGS[0])
    t = attention_tensors(cfg, dt, batch=B, heads=N, q_len=Lq, k_len=Lk, stream=300 + Lk)
    key_len = t["key_len"] if "pad" in mask else None
    causal = "causal" in mask
    scale = 1.0 / np.sqrt(64.0)
    seed, offset = 4321, Lk
    d = dev()
    x, dy = to_torch(t["x"], dt, d), to_torch(t["dy"], dt, d)
    kl = None if key_len is None else torch.from_numpy(key_len).to(d)
    y, yd = L.lsq_softmax_fwd(x, kl, causal, scale, p, seed, offset)
    ry, ryd = oracle.softmax_fwd(t["x"], key_len, causal, scale, dt, p, seed, offset)
    assert_close_store(y, ry, dt, "y", f32_floor=1e-7)
    # positions outside the allowed set are exactly +0 (bit pattern), not merely small
    masked = ry == 0.0
    ybits = from_torch(y, dt)
    assert not ybits.reshape(ry.shape)[masked].view(np.uint16 if dt != "f32" else np.uint32).any()
    if p > 0:
        assert_close_store(yd, ryd, dt, "y_drop", f32_floor=1e-7)
        # the dropped set is bit-exact
        assert np.array_equal(to_np64(yd, dt) == 0, ryd == 0)
    # backward takes the y the GPU stored, on both sides
    ystored = from_torch(y, dt)
    dx = L.lsq_softmax_bwd(dy, y, kl, causal, scale, p, seed, offset)
    rdx = oracle.softmax_bwd(t["dy"], ystored, key_len, causal, scale, dt, p, seed, offset)
    assert_close_store(dx, rdx, dt, "dx", f32_floor=1e-7)
    assert not from_torch(dx, dt).reshape(ry.shape)[masked].view(np.uint16 if dt != "f32" else np.uint32).any()
    # in place: dx over dy
    dyc = dy.clone()
    dx2 = L.lsq_softmax_bwd(dyc, y, kl, causal, scale, p, seed, offset, dx=dyc)
    assert torch.equal(dx, dx2)


@pytest.mark.parametrize("scale", [-0.125, 0.0, 3.0])
@pytest.mark.parametrize("B,N,Lq,Lk,mask,p", [(2, 2, 9, 128, "pad", 0.1), (1, 2, 5, 1024, "causal", 0.0), (2, 1, 3, 2048, "pad+causal", 0.1),
                                              (1, 1, 3, 4096, "pad", 0.1)])
def test_softmax_other_scales(B, N, Lq, Lk, mask, p, scale):
    """The scale is any float by contract: negative and zero scales (rows of whole packs up to 2048 keys take
    another kernel for them), and a large one that spreads the exponents."""
    say(f"[softmax] scale={scale} B={B} N={N} Lq={Lq} Lk={Lk} mask={mask} p={p}")
    dt = "f16"
    t = attention_tensors(CONFIGS[0], dt, batch=B, heads=N, q_len=Lq, k_len=Lk, stream=900 + Lk)
    key_len = t["key_len"] if "pad" in mask else None
    causal = "causal" in mask
    d = dev()
    x, dy = to_torch(t["x"], dt, d), to_torch(t["dy"], dt, d)
    kl = None if key_len is None else torch.from_numpy(key_len).to(d)
    y, yd = L.lsq_softmax_fwd(x, kl, causal, scale, p, 77, 5)
    ry, ryd = oracle.softmax_fwd(t["x"], key_len, causal, scale, dt, p, 77, 5)
    assert_close_store(y, ry, dt, "y", f32_floor=1e-7)
    if p > 0:
        assert_close_store(yd, ryd, dt, "y_drop", f32_floor=1e-7)
    dx = L.lsq_softmax_bwd(dy, y, kl, causal, scale, p, 77, 5)
    rdx = oracle.softmax_bwd(t["dy"], from_torch(y, dt), key_len, causal, scale, dt, p, 77, 5)
    assert_close_store(dx, rdx, dt, "dx", f32_floor=1e-7)


def test_softmax_key_len_edge_values():
    say("[softmax] key_len 0, 1, beyond k_len, negative")
    d, dt = dev(), "f16"
    t = attention_tensors(CONFIGS[0], dt, batch=4, heads=2, q_len=16, k_len=64, stream=399)
    key_len = np.array([0, 1, 100, -3], np.int32)
    x = to_torch(t["x"], dt, d)
    y, _ = L.lsq_softmax_fwd(x, torch.from_numpy(key_len).to(d), False, 1.0)
    ry, _ = oracle.softmax_fwd(t["x"], key_len, False, 1.0, dt)
    assert_close_store(y, ry, dt, "y")
    yy = y.float().cpu().numpy()
    assert (yy[0] == 0).all() and (yy[3] == 0).all() and (yy[1, :, :, 0] == 1).all() and np.isfinite(yy).all()
    assert np.allclose(yy[2].sum(-1), 1, atol=2e-3)


@pytest.mark.parametrize("dt", ["bf16", "f16"])
def test_softmax_full_size_gpt2_large(dt):
    """Config 5 at full size, the launch the benchmark times; the oracle checks two whole batches."""
    say(f"[softmax] full size [8,20,1024,1024] causal dt={dt}")
    d = dev()
    B, N, Lq = 8, 20, 1024
    x = device_normal((B, N, Lq, Lq), 1.0, dt, seed=4, device=d)
    dy = device_normal((B, N, Lq, Lq), 1.0, dt, seed=5, device=d)
    scale = 0.125
    y, _ = L.lsq_softmax_fwd(x, None, True, scale)
    dx = L.lsq_softmax_bwd(dy, y, None, True, scale)
    for b in (0, 7):
        ry, _ = oracle.softmax_fwd(from_torch(x[b:b + 1], dt), None, True, scale, dt)
        assert_close_store(y[b:b + 1], ry, dt, f"y[{b}]")
        rdx = oracle.softmax_bwd(from_torch(dy[b:b + 1], dt), from_torch(y[b:b + 1], dt), None, True, scale, dt)
        assert_close_store(dx[b:b + 1], rdx, dt, f"dx[{b}]")
    # properties over the whole tensor: rows sum to 1, the strict upper triangle is exactly zero
    s = y.float().sum(-1)
    assert torch.all((s - 1).abs() < (2e-2 if dt == "bf16" else 4e-3))
    upper = torch.triu(torch.ones(Lq, Lq, dtype=torch.bool, device=d), diagonal=1)
    assert not y[:, :, upper].any() and not dx[:, :, upper].any()


def test_softmax_full_size_transformer_big_with_dropout():
    """Config 3 at full size with attention dropout and both masks."""
    say("[softmax] full size [64,16,128,128] pad+causal p=0.1")
    d, dt = dev(), "f16"
    cfg = CONFIGS[2]
    t = attention_tensors(cfg, dt)
    x, dy = to_torch(t["x"], dt, d), to_torch(t["dy"], dt, d)
    kl = torch.from_numpy(t["key_len"]).to(d)
    y, yd = L.lsq_softmax_fwd(x, kl, True, 0.125, cfg.p_attn, cfg.philox_seed, 9)
    ry, ryd = oracle.softmax_fwd(t["x"], t["key_len"], True, 0.125, dt, cfg.p_attn, cfg.philox_seed, 9)
    assert_close_store(y, ry, dt, "y")
    assert_close_store(yd, ryd, dt, "y_drop")
    assert np.array_equal(to_np64(yd, dt) == 0, ryd == 0)
    dx = L.lsq_softmax_bwd(dy, y, kl, True, 0.125, cfg.p_attn, cfg.philox_seed, 9)
    rdx = oracle.softmax_bwd(t["dy"], from_torch(y, dt), t["key_len"], True, 0.125, dt, cfg.p_attn, cfg.philox_seed, 9)
    assert_close_store(dx, rdx, dt, "dx")
