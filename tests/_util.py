"""Shared helpers of the GPU parity tests: tolerances and comparisons.

Tolerances (the storage type of the output decides):
  fp16 outputs : |gpu - ref| <= max(5e-3, 2^-10 |ref|)   (5e-3 absolute, or one fp16 ulp where an ulp is larger)
  bf16 outputs : |gpu - ref| <= max(2e-2, 2^-8  |ref|)
  fp32 outputs : |gpu - ref| <= 1e-5 |ref| + floor       (floor: the op's absolute rounding floor, passed in)
  Adam master  : |gpu - ref| <= 1e-6 |ref| + floor
`ref` is the oracle's UNROUNDED float64 value.
"""
import numpy as np
import torch

from workloads import decode, from_torch

LP_TOL = {"f16": (5e-3, 2.0 ** -10), "bf16": (2e-2, 2.0 ** -8)}


def dev():
    return torch.device("cuda:0")


def to_np64(t, dt):
    """device tensor in storage type dt -> float64 numpy (exact)."""
    return decode(from_torch(t, dt), dt).reshape(tuple(t.shape))


def assert_close_store(gpu, ref, dt, what="", f32_floor=1e-6):
    """gpu: tensor stored in dt; ref: float64 array."""
    g = to_np64(gpu, dt)
    ref = np.asarray(ref, dtype=np.float64).reshape(g.shape)
    assert np.isfinite(g).all(), f"{what}: non-finite values in the GPU output"
    err = np.abs(g - ref)
    if dt == "f32":
        tol = 1e-5 * np.abs(ref) + f32_floor
    else:
        a, r = LP_TOL[dt]
        tol = np.maximum(a, r * np.abs(ref))
    bad = err > tol
    if bad.any():
        i = np.unravel_index(np.argmax(err - tol), err.shape)
        raise AssertionError(f"{what}: {bad.sum()} of {bad.size} outside tolerance; worst at {i}: "
                             f"gpu={g[i]!r} ref={ref[i]!r} err={err[i]:.3e} tol={tol[i]:.3e}")
    return float(err.max())


def assert_close_f32(gpu, ref, what="", rel=1e-5, floor=0.0):
    g = gpu.detach().cpu().numpy().astype(np.float64)
    ref = np.asarray(ref, dtype=np.float64).reshape(g.shape)
    assert np.isfinite(g).all(), f"{what}: non-finite values in the GPU output"
    err = np.abs(g - ref)
    tol = rel * np.abs(ref) + floor
    bad = err > tol
    if bad.any():
        i = np.unravel_index(np.argmax(err - tol), err.shape)
        raise AssertionError(f"{what}: {bad.sum()} of {bad.size} outside tolerance; worst at {i}: "
                             f"gpu={g[i]!r} ref={ref[i]!r} err={err[i]:.3e} tol={tol[i]:.3e}")
    return float(err.max())


def say(msg):
    print(msg, flush=True)
