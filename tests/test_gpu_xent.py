"""GPU parity: label-smoothed cross-entropy forward / backward through the C-ABI against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2110_05722_amd as L
from tests._util import assert_close_f32, assert_close_store, dev, say
from workloads import CONFIGS, IGNORE_INDEX, criterion_tensors, device_normal, from_torch, to_torch

pytestmark = pytest.mark.gpu

# (tokens, vocab, alpha): config 1 whole; odd vocabularies exercise every head/tail alignment
CASES = [
    (512, 8000, 0.1), (64, 32768, 0.1), (48, 30522, 0.0), (40, 50257, 0.1),
    (33, 8001, 0.1), (17, 257, 0.3), (9, 5, 0.1), (11, 8, 0.0), (7, 1, 0.5), (16, 13, 1.0), (5, 2051, 0.1),
    (10, 12345, 0.1), (9, 70001, 0.1),      # the widest 256-thread row bucket of the one-pass kernel; a row beyond its buckets
]


def _run(t, T, V, alpha, dt, grad_scale=1.0):
    d = dev()
    logits = to_torch(t["logits"], dt, d)
    target = torch.from_numpy(t["target"]).to(d)
    loss, nll, lse, sums = L.lsq_ls_xent_fwd(logits, target, alpha, IGNORE_INDEX)
    rloss, rnll, rlse, rsums = oracle.ls_xent_fwd(t["logits"], t["target"], alpha, IGNORE_INDEX, dt)
    # lse and loss are O(log V): relative tolerance plus the rounding floor of a V-term fp32 sum
    assert_close_f32(lse, rlse, "lse", floor=1e-6)
    assert_close_f32(loss, rloss, "loss", floor=2e-6)
    assert_close_f32(nll, rnll, "nll", floor=2e-6)
    assert_close_f32(sums, rsums, "sums", floor=1e-5)
    # without the nll output the sums come from a second gather of the target logits: same numbers
    loss_b, none, lse_b, sums_b = L.lsq_ls_xent_fwd(logits, target, alpha, IGNORE_INDEX, want_nll=False)
    assert none is None and torch.equal(loss, loss_b) and torch.equal(lse, lse_b)
    assert_close_f32(sums_b, rsums, "sums (gathered)", floor=1e-5)
    ign = (t["target"] == IGNORE_INDEX) | (t["target"] < 0) | (t["target"] >= V)
    assert (loss.cpu().numpy()[ign] == 0).all()
    dl = L.lsq_ls_xent_bwd(logits, lse, target, alpha, IGNORE_INDEX, grad_scale)
    rdl = oracle.ls_xent_bwd(t["logits"], t["target"], alpha, IGNORE_INDEX, grad_scale, dt)
    assert_close_store(dl, rdl, dt, "dlogits", f32_floor=1e-7)
    bits = from_torch(dl, dt)
    assert not bits[ign].view(np.uint16 if dt != "f32" else np.uint32).any()      # ignored rows: exact zeros
    # in place over the logits
    lc = logits.clone()
    dl2 = L.lsq_ls_xent_bwd(lc, lse, target, alpha, IGNORE_INDEX, grad_scale, dlogits=lc)
    assert torch.equal(dl, dl2)
    # forward and backward in one pass: the same outputs to the same tolerances, ignored rows exact zeros,
    # in place allowed
    floss, fnll, flse, fsums, fdl = L.lsq_ls_xent_fwd_bwd(logits, target, alpha, IGNORE_INDEX, grad_scale)
    assert_close_f32(flse, rlse, "one-pass lse", floor=1e-6)
    assert_close_f32(floss, rloss, "one-pass loss", floor=2e-6)
    assert_close_f32(fnll, rnll, "one-pass nll", floor=2e-6)
    assert_close_f32(fsums, rsums, "one-pass sums", floor=1e-5)
    assert_close_store(fdl, rdl, dt, "one-pass dlogits", f32_floor=1e-7)
    assert not from_torch(fdl, dt)[ign].view(np.uint16 if dt != "f32" else np.uint32).any()
    assert (floss.cpu().numpy()[ign] == 0).all() and (flse.cpu().numpy()[ign] == 0).all()
    lc = logits.clone()
    out = L.lsq_ls_xent_fwd_bwd(lc, target, alpha, IGNORE_INDEX, grad_scale, want_sums=False, want_nll=False, dlogits=lc)
    assert out[1] is None and out[3] is None
    assert torch.equal(out[4], fdl) and torch.equal(out[0], floss) and torch.equal(out[2], flse)
    # in place WITH sums: the sum of nll must come from the per-token nll (the logits are gone by then);
    # without nll the call is refused
    lc = logits.clone()
    out = L.lsq_ls_xent_fwd_bwd(lc, target, alpha, IGNORE_INDEX, grad_scale, want_sums=True, want_nll=True, dlogits=lc)
    assert torch.equal(out[3], fsums) and torch.equal(out[4], fdl)
    lc = logits.clone()
    with pytest.raises(L.LsqError, match="INVALID_ARG"):
        L.lsq_ls_xent_fwd_bwd(lc, target, alpha, IGNORE_INDEX, grad_scale, want_sums=True, want_nll=False, dlogits=lc)
    assert torch.equal(lc, logits)                                              # refused before any launch
    out = L.lsq_ls_xent_fwd_bwd(logits, target, alpha, IGNORE_INDEX, grad_scale, want_sums=True, want_nll=False)
    assert_close_f32(out[3], rsums, "one-pass sums without nll, out of place", floor=1e-5)
    return loss, lse, sums


@pytest.mark.parametrize("dt", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("T,V,alpha", CASES)
def test_ls_xent_fwd_bwd(T, V, alpha, dt):
    say(f"[ls_xent] tokens={T} vocab={V} alpha={alpha} dt={dt}")
    cfg = CONFIGS[0] if V != 50257 else CONFIGS[4]
    t = criterion_tensors(cfg, dt, tokens=T if T != cfg.tokens else None, vocab=V, stream=400 + V % 1000)
    if T >= 9:                                   # sprinkle ignored and out-of-range targets
        t["target"][1] = IGNORE_INDEX
        t["target"][4] = V
        t["target"][7] = -1
        t["target"][2] = 0
        t["target"][3] = V - 1
    _run(t, T, V, alpha, dt, grad_scale=0.5)


def test_ls_xent_alpha_zero_equals_nll_and_sums_reproducible():
    say("[ls_xent] alpha=0 -> loss == nll; sums bit-reproducible")
    dt, d = "f16", dev()
    t = criterion_tensors(CONFIGS[0], dt)
    logits = to_torch(t["logits"], dt, d)
    target = torch.from_numpy(t["target"]).to(d)
    loss, nll, lse, sums = L.lsq_ls_xent_fwd(logits, target, 0.0, IGNORE_INDEX)
    loss2, nll2, lse2, sums2 = L.lsq_ls_xent_fwd(logits, target, 0.0, IGNORE_INDEX)
    assert torch.equal(loss, loss2) and torch.equal(lse, lse2) and torch.equal(sums, sums2) and torch.equal(nll, nll2)
    assert_close_f32(loss, nll.cpu().numpy(), "loss == nll at alpha 0", floor=1e-6)
    assert abs(sums[0].item() - sums[1].item()) <= 1e-5 * abs(sums[1].item())
    assert sums[2].item() == int((t["target"] != IGNORE_INDEX).sum())


@pytest.mark.parametrize("ci,dt", [(1, "f16"), (2, "f16"), (3, "bf16"), (3, "f16"), (4, "bf16"), (4, "f16")])
def test_ls_xent_full_size(ci, dt):
    """Configs 2-5 at full size in the launch the benchmark times; the oracle checks sampled tokens
    one by one, and whole-tensor properties cover the rest."""
    cfg = CONFIGS[ci]
    T, V = cfg.tokens, cfg.vocab
    say(f"[ls_xent] full size {cfg.name} tokens={T} vocab={V} dt={dt}")
    d = dev()
    logits = device_normal((T, V), cfg.logit_std, dt, seed=cfg.seed, device=d)
    rng = np.random.Generator(np.random.PCG64([cfg.seed, 77]))
    tgt = rng.integers(0, V, size=T).astype(np.int32)
    if cfg.active_frac < 1.0:
        tgt[rng.random(T) >= cfg.active_frac] = IGNORE_INDEX
    else:
        tgt[rng.random(T) < 0.2] = IGNORE_INDEX      # padded positions
    target = torch.from_numpy(tgt).to(d)
    gs = 1.0      # fp16 gradients of size alpha/V * 1/64 would sit below half the smallest subnormal
    loss, nll, lse, sums = L.lsq_ls_xent_fwd(logits, target, cfg.alpha, IGNORE_INDEX)
    dl = L.lsq_ls_xent_bwd(logits, lse, target, cfg.alpha, IGNORE_INDEX, gs)
    rows = np.sort(rng.choice(T, size=96, replace=False))
    rows[:4] = [0, 1, T - 2, T - 1]
    rows = np.unique(rows)
    idx = torch.from_numpy(rows).to(d)
    sub = from_torch(logits[idx], dt)
    rloss, rnll, rlse, _ = oracle.ls_xent_fwd(sub, tgt[rows], cfg.alpha, IGNORE_INDEX, dt)
    assert_close_f32(lse[idx], rlse, "lse", floor=1e-6)
    assert_close_f32(loss[idx], rloss, "loss", floor=2e-6)
    assert_close_f32(nll[idx], rnll, "nll", floor=2e-6)
    rdl = oracle.ls_xent_bwd(sub, tgt[rows], cfg.alpha, IGNORE_INDEX, gs, dt)
    assert_close_store(dl[idx], rdl, dt, "dlogits")
    # properties at any size: ignored rows are all-zero; gradient rows sum to ~0; sums == sum of the vector
    ign = torch.from_numpy(tgt == IGNORE_INDEX).to(d)
    assert not dl[ign].any()
    assert (loss[ign] == 0).all()
    rs = dl[~ign].float().sum(-1).abs().max().item()
    assert rs < gs * (3e-2 if dt == "bf16" else 4e-3) + 1e-4   # + the fp16 subnormal rounding floor over V terms
    assert abs(sums[0].item() - loss.double().sum().item()) <= 1e-5 * loss.double().sum().item()
    assert abs(sums[1].item() - nll.double().sum().item()) <= 1e-5 * nll.double().sum().item()
    assert sums[2].item() == int((tgt != IGNORE_INDEX).sum())
    # the one-pass entry point at the same size: sampled rows against the oracle, the whole gradient against the
    # stand-alone backward (two roundings to the storage type apart at most), then in place over the logits
    del dl
    floss, fnll, flse, fsums, fdl = L.lsq_ls_xent_fwd_bwd(logits, target, cfg.alpha, IGNORE_INDEX, gs)
    assert_close_f32(flse[idx], rlse, "one-pass lse", floor=1e-6)
    assert_close_f32(floss[idx], rloss, "one-pass loss", floor=2e-6)
    assert_close_f32(fnll[idx], rnll, "one-pass nll", floor=2e-6)
    assert_close_store(fdl[idx], rdl, dt, "one-pass dlogits")
    assert fsums[2].item() == sums[2].item() and abs(fsums[0].item() - sums[0].item()) <= 1e-5 * sums[0].item()
    ref = L.lsq_ls_xent_bwd(logits, flse, target, cfg.alpha, IGNORE_INDEX, gs)
    ulp = 2.0 ** -7 if dt == "bf16" else 2.0 ** -10
    err = (fdl.float() - ref.float()).abs_()
    err -= ref.float().abs_().mul_(2 * ulp)
    assert err.max().item() <= (1e-7 if dt != "bf16" else 1e-6), err.max().item()
    assert not fdl[ign].any()
    del ref, err
    L.lsq_ls_xent_fwd_bwd(logits, target, cfg.alpha, IGNORE_INDEX, gs, dlogits=logits)
    assert torch.equal(logits, fdl)


def test_ls_xent_every_token_ignored():
    say("[ls_xent] a batch whose every token is ignored: zeros everywhere, count 0, nothing read")
    d, dt = dev(), "bf16"
    T, V = 37, 1003
    logits = torch.full((T, V), float("nan"), dtype=torch.bfloat16, device=d)      # must not be looked at
    target = torch.full((T,), IGNORE_INDEX, dtype=torch.int32, device=d)
    loss, nll, lse, sums = L.lsq_ls_xent_fwd(logits, target, 0.1, IGNORE_INDEX)
    dl = L.lsq_ls_xent_bwd(logits, lse, target, 0.1, IGNORE_INDEX, 1.0)
    floss, fnll, flse, fsums, fdl = L.lsq_ls_xent_fwd_bwd(logits, target, 0.1, IGNORE_INDEX, 1.0)
    for t in (loss, nll, lse, sums, dl, floss, fnll, flse, fsums, fdl):
        assert not t.float().ne(0).any()
