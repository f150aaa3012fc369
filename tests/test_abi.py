"""CPU-side checks of the boundary: the shared library loads, exports every symbol
the header declares, and rejects bad arguments on the host before any launch."""
import ctypes as C
import os
import re

import pytest

import paper_2110_05722_amd as L
from paper_2110_05722_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(L.lib_path()):
        from paper_2110_05722_amd.build import build
        build(verbose=False)
    return L.load()


def test_every_declared_symbol_is_exported(lib):
    hdr = open(os.path.join(ROOT, "include", "lsq.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(lsq_[a-z0-9_]+)\s*\(", hdr))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_status_strings_and_workspace(lib):
    names = [L.lsq_status_string(i) for i in range(6)]
    assert names == ["LSQ_OK", "LSQ_INVALID_ARG", "LSQ_UNSUPPORTED_DTYPE", "LSQ_MISALIGNED",
                     "LSQ_WORKSPACE_TOO_SMALL", "LSQ_LAUNCH_FAILED"]
    assert L.lsq_workspace_bytes(0, 0, 1024) == 0
    w = L.lsq_workspace_bytes(0, 8192, 1024)
    assert w > 0 and w % (2 * 1024 * 4) == 0
    w = L.lsq_workspace_bytes(1, 8192, 1024)
    assert w > 0 and w % (1024 * 4) == 0
    assert L.lsq_workspace_bytes(2, 8192, 4096) > 0 and L.lsq_workspace_bytes(2, 8192, 4096) % (4096 * 4) == 0
    assert L.lsq_workspace_bytes(99, 8192, 1024) == 0


A = C.c_void_p(4096)      # aligned, never dereferenced: every call below fails before a launch
U = C.c_void_p(4096 + 2)  # misaligned


def test_host_side_argument_errors(lib):
    INVALID, DTYPE, MISALIGNED, WS = 1, 2, 3, 4
    # adam: step < 1, beta out of range, bad dtype, misaligned, null
    f = lib.lsq_adam_step
    assert f(A, A, A, A, None, 8, 1e-3, .9, .98, 1e-8, 0., 0, 0, 1, 1., 0, 0, None) == INVALID
    assert f(A, A, A, A, None, 8, 1e-3, 1.0, .98, 1e-8, 0., 1, 0, 1, 1., 0, 0, None) == INVALID
    assert f(A, A, A, A, None, -1, 1e-3, .9, .98, 1e-8, 0., 1, 0, 1, 1., 0, 0, None) == INVALID
    assert f(A, A, A, A, None, 8, 1e-3, .9, .98, 1e-8, 0., 1, 0, 1, 1., 7, 0, None) == DTYPE
    assert f(A, A, A, A, A, 8, 1e-3, .9, .98, 1e-8, 0., 1, 0, 1, 1., 0, 2, None) == DTYPE
    assert f(U, A, A, A, None, 8, 1e-3, .9, .98, 1e-8, 0., 1, 0, 1, 1., 0, 0, None) == MISALIGNED
    assert f(None, A, A, A, None, 8, 1e-3, .9, .98, 1e-8, 0., 1, 0, 1, 1., 0, 0, None) == INVALID
    assert f(None, None, None, None, None, 0, 1e-3, .9, .98, 1e-8, 0., 1, 0, 1, 1., 0, 0, None) == 0
    # layernorm
    f = lib.lsq_layernorm_fwd
    assert f(A, A, A, A, A, A, 4, 0, 1e-5, 0, None) == INVALID
    assert f(A, A, A, A, A, A, 4, 8, -1.0, 0, None) == INVALID
    assert f(A, A, A, U, A, A, 4, 8, 1e-5, 0, None) == MISALIGNED
    assert f(A, A, A, A, A, A, 4, 8, 1e-5, 5, None) == DTYPE
    assert f(None, None, None, None, None, None, 0, 8, 1e-5, 0, None) == 0
    f = lib.lsq_layernorm_bwd
    assert f(A, A, A, A, A, A, A, A, None, A, 16, 64, 512, 0, None) == WS
    assert f(A, A, A, A, A, A, A, A, None, None, 0, 64, 512, 0, None) == WS
    assert f(A, None, A, A, A, A, A, A, None, A, 1 << 30, 64, 512, 0, None) == INVALID
    f = lib.lsq_layernorm_bwd_noalloc
    assert f(A, A, A, A, A, A, A, A, None, 4096, 8192, 0, None) == WS          # 16 MiB of partial rows > the 8 MiB held
    assert f(A, A, A, A, A, A, A, A, None, -1, 64, 0, None) == INVALID
    # bias + dropout + residual: p outside [0, 1)
    f = lib.lsq_bias_dropout_residual_fwd
    assert f(A, A, A, A, 4, 8, 1.0, 1, 0, 0, None) == INVALID
    assert f(A, A, A, A, 4, 8, -0.1, 1, 0, 0, None) == INVALID
    assert f(A, A, A, A, 4, 8, float("nan"), 1, 0, 0, None) == INVALID
    assert f(A, U, A, A, 4, 8, 0.1, 1, 0, 0, None) == MISALIGNED
    f = lib.lsq_bias_dropout_residual_bwd
    assert f(A, A, A, 64, 512, 0.1, 1, 0, A, 8, 0, None) == WS
    assert f(A, None, A, 64, 512, 1.5, 1, 0, None, 0, 0, None) == INVALID
    # softmax: y_drop must be given iff p_attn > 0
    f = lib.lsq_softmax_fwd
    assert f(A, None, A, None, 2, 2, 8, 8, 0, 1.0, 0.1, 1, 0, 0, None) == INVALID
    assert f(A, A, A, None, 2, 2, 8, 8, 0, 1.0, 0.0, 1, 0, 0, None) == INVALID
    assert f(A, None, A, None, -1, 2, 8, 8, 0, 1.0, 0.0, 1, 0, 0, None) == INVALID
    assert f(A, None, U, None, 2, 2, 8, 8, 0, 1.0, 0.0, 1, 0, 0, None) == MISALIGNED
    assert f(None, None, None, None, 0, 2, 8, 8, 0, 1.0, 0.0, 1, 0, 0, None) == 0
    f = lib.lsq_softmax_bwd
    assert f(A, A, None, None, 2, 2, 8, 8, 0, 1.0, 0.0, 1, 0, 0, None) == INVALID
    # criterion
    f = lib.lsq_ls_xent_fwd
    assert f(A, None, A, None, A, A, 4, 0, 0.1, -100, 0, None) == INVALID
    assert f(A, None, A, None, A, A, 4, 8, 1.5, -100, 0, None) == INVALID
    assert f(A, A, A, None, U, A, 4, 8, 0.1, -100, 0, None) == MISALIGNED
    assert f(None, None, A, None, A, A, 4, 8, 0.1, -100, 0, None) == INVALID
    f = lib.lsq_ls_xent_bwd
    assert f(A, A, None, A, 4, 8, 0.1, -100, 1.0, 0, None) == INVALID
    assert f(A, A, A, A, 4, 8, 0.1, -100, 1.0, 9, None) == DTYPE
    f = lib.lsq_ls_xent_fwd_bwd
    assert f(A, None, A, None, None, A, A, 4, 8, 0.1, -100, 1.0, 0, None) == INVALID      # no dlogits
    assert f(A, None, A, None, A, A, A, 4, 8, -0.1, -100, 1.0, 0, None) == INVALID
    assert f(A, None, A, None, U, A, A, 4, 8, 0.1, -100, 1.0, 0, None) == MISALIGNED
    assert f(A, None, A, None, A, A, A, 4, 8, 0.1, -100, 1.0, 3, None) == DTYPE
    assert f(None, None, None, None, None, None, None, 0, 8, 0.1, -100, 1.0, 0, None) == 0
    assert f(A, None, A, A, A, A, A, 4, 8, 0.1, -100, 1.0, 0, None) == INVALID        # in place + sums without nll


def test_host_side_argument_errors_of_the_next_rows(lib):
    INVALID, DTYPE, MISALIGNED, WS = 1, 2, 3, 4
    f = lib.lsq_bias_act_dropout_fwd
    assert f(A, A, A, 4, 8, 3, 0.1, 1, 0, 0, None) == INVALID          # unknown activation
    assert f(A, A, A, 4, 8, 0, 1.0, 1, 0, 0, None) == INVALID
    assert f(A, U, A, 4, 8, 0, 0.1, 1, 0, 0, None) == MISALIGNED
    assert f(None, None, None, 0, 8, 1, 0.1, 1, 0, 0, None) == 0
    f = lib.lsq_bias_act_dropout_bwd
    assert f(A, A, A, A, A, 64, 512, 1, 0.1, 1, 0, A, 8, 0, None) == WS
    assert f(A, None, A, None, A, 64, 512, 1, 0.1, 1, 0, None, 0, 0, None) == INVALID
    f = lib.lsq_adam_step_lp
    assert f(A, A, A, A, 8, 1e-3, .9, .98, 1e-8, 0., 0, 0, 1, 1., 0, None) == INVALID
    assert f(A, A, A, A, 8, 1e-3, .9, .98, 1e-8, 0., 1, 0, 1, 1., 2, None) == DTYPE   # fp32 is not "low precision"
    assert f(A, U, A, A, 8, 1e-3, .9, .98, 1e-8, 0., 1, 0, 1, 1., 0, None) == MISALIGNED
    f = lib.lsq_sgd_step
    assert f(A, None, A, None, 8, 0.1, 0.9, 0., 0, 1., 0, 0, None) == INVALID         # momentum without a buffer
    assert f(A, None, A, None, 8, 0.1, 0.0, 0., 1, 1., 0, 0, None) == INVALID         # nesterov without momentum
    assert f(A, A, A, None, 8, 0.1, -0.5, 0., 0, 1., 0, 0, None) == INVALID
    assert f(A, A, A, A, 8, 0.1, 0.9, 0., 0, 1., 0, 2, None) == DTYPE
    assert f(None, None, None, None, 0, 0.1, 0.0, 0., 0, 1., 0, 0, None) == 0


def test_host_side_argument_errors_of_padding_removal(lib):
    INVALID, DTYPE = 1, 2
    f = lib.lsq_pad_offsets
    assert f(None, A, 4, 8, None) == INVALID
    assert f(A, A, -1, 8, None) == INVALID
    assert f(A, A, 1 << 20, 1 << 20, None) == INVALID                  # batch * max_len beyond int32
    for f in (lib.lsq_pad_remove, lib.lsq_pad_restore):
        assert f(A, A, None, 4, 8, 16, 32, 0, None) == INVALID         # no offsets
        assert f(A, A, A, 4, 8, 16, -1, 0, None) == INVALID
        assert f(A, A, A, 4, 8, 16, 32, 7, None) == DTYPE
        assert f(None, None, None, 0, 8, 16, 0, 0, None) == 0          # empty batch: nothing to do
    f = lib.lsq_softmax_varlen_fwd
    assert f(A, None, A, A, A, 2, 2, 8, 8, 0, float("nan"), 0.0, 1, 0, 0, None) == INVALID
    assert f(A, None, A, A, A, 2, 2, 8, 8, 0, 1.0, 0.1, 1, 0, 0, None) == INVALID   # dropout without y_drop
    assert f(None, None, None, None, None, 0, 2, 8, 8, 0, 1.0, 0.0, 1, 0, 0, None) == 0


def test_host_side_argument_errors_of_the_blocked_adam(lib):
    INVALID, DTYPE, MISALIGNED = 1, 2, 3
    lib.lsq_adam_state_bytes.restype = C.c_size_t
    assert lib.lsq_adam_state_bytes(0) == 0 and lib.lsq_adam_state_bytes(-5) == 0
    assert lib.lsq_adam_state_bytes(1) == 3 * 8192 * 4 and lib.lsq_adam_state_bytes(8193) == 2 * 3 * 8192 * 4
    assert lib.lsq_adam_state_pack(None, A, A, A, 8, None) == INVALID
    assert lib.lsq_adam_state_pack(A, U, None, None, 8, None) == MISALIGNED
    assert lib.lsq_adam_state_unpack(A, A, A, None, 8, None) == INVALID
    assert lib.lsq_adam_state_unpack(None, None, None, None, 0, None) == 0
    f = lib.lsq_adam_step_blocked
    assert f(A, A, A, 8, 1e-3, .9, .98, 1e-8, 0., 0, 0, 1, 1., 0, 0, None) == INVALID      # step 0
    assert f(A, A, A, 8, 1e-3, 1.0, .98, 1e-8, 0., 1, 0, 1, 1., 0, 0, None) == INVALID     # beta1 = 1
    assert f(A, A, A, 8, 1e-3, .9, .98, 1e-8, 0., 1, 0, 1, 1., 5, 0, None) == DTYPE
    assert f(A, A, A, 8, 1e-3, .9, .98, 1e-8, 0., 1, 0, 1, 1., 0, 2, None) == DTYPE        # fp32 p_lp
    assert f(None, A, A, 8, 1e-3, .9, .98, 1e-8, 0., 1, 0, 1, 1., 0, 0, None) == INVALID
    assert f(None, None, None, 0, 1e-3, .9, .98, 1e-8, 0., 1, 0, 1, 1., 0, 0, None) == 0


def test_host_side_argument_errors_of_the_blocked_trainers(lib):
    INVALID, DTYPE = 1, 2
    lib.lsq_trainer_state_bytes.restype = C.c_size_t
    assert lib.lsq_trainer_state_bytes(10, 0) == 0 and lib.lsq_trainer_state_bytes(10, 4) == 0
    assert lib.lsq_trainer_state_bytes(10, 2) == 2 * 8192 * 4
    assert lib.lsq_trainer_state_pack(A, A, A, A, 8, 4, None) == INVALID
    assert lib.lsq_trainer_state_pack(A, None, A, A, 8, 2, None) == INVALID
    assert lib.lsq_trainer_state_unpack(A, A, A, A, 8, 0, None) == INVALID
    f = lib.lsq_sgd_step_blocked
    assert f(A, A, None, 8, 0.1, -0.5, 0., 0, 1., 0, 0, None) == INVALID
    assert f(A, A, None, 8, 0.1, 0.0, 0., 1, 1., 0, 0, None) == INVALID          # nesterov without momentum
    assert f(None, A, None, 8, 0.1, 0.9, 0., 0, 1., 0, 0, None) == INVALID
    assert f(A, A, A, 8, 0.1, 0.9, 0., 0, 1., 0, 2, None) == DTYPE
    f = lib.lsq_adam_step_lp_blocked
    assert f(A, A, A, 8, 1e-3, .9, .98, 1e-8, 0., 0, 0, 1, 1., 0, None) == INVALID  # step 0
    assert f(A, A, A, 8, 1e-3, .9, .98, 1e-8, 0., 1, 0, 1, 1., 2, None) == DTYPE
    assert f(A, None, A, 8, 1e-3, .9, .98, 1e-8, 0., 1, 0, 1, 1., 0, None) == INVALID


def test_binding_refuses_cpu_tensors(lib):
    import torch
    x = torch.zeros(4, 8, dtype=torch.float16)
    with pytest.raises(L.LsqError):
        L.lsq_layernorm_fwd(x, x[0], x[0])


def test_binding_refuses_operands_shorter_than_the_call_needs(lib):
    import torch
    x = torch.zeros(4, 8, dtype=torch.float16)
    with pytest.raises(L.LsqError, match="gamma holds 4 elements"):
        L.lsq_layernorm_fwd(x, x[0][:4], x[0])
    p = torch.zeros(16)
    with pytest.raises(L.LsqError, match="v holds 8 elements"):
        L.lsq_adam_step(p, p.clone(), p[:8].clone(), p.half(), None, lr=1e-3, beta1=0.9, beta2=0.98, eps=1e-8, step=1)
    with pytest.raises(L.LsqError, match="mean is torch.float16"):
        L.lsq_layernorm_fwd(x, x[0], x[0], mean=torch.zeros(4, dtype=torch.float16))
