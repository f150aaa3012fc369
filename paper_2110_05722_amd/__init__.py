"""MI355X-native fused non-GEMM Transformer training kernels (LightSeq2's hot path).

Thin Python binding over the C-ABI library `liblsq.so` (declared in
`include/lsq.h`).  PyTorch is used for device memory and streams only: every
function below marshals pointers and sizes and calls the entry point of the
same name; all arithmetic runs in the hand-written gfx950 kernels.  There is no
CPU fallback: if the library is missing, or a tensor is not on the GPU, the call
raises.
"""
from .binding import (  # noqa: F401
    LsqError,
    lib_path,
    load,
    lsq_adam_state_bytes,
    lsq_adam_state_pack,
    lsq_adam_state_unpack,
    lsq_adam_step,
    lsq_adam_step_blocked,
    lsq_adam_step_lp_blocked,
    lsq_sgd_step_blocked,
    lsq_trainer_state_bytes,
    lsq_trainer_state_pack,
    lsq_trainer_state_unpack,
    lsq_adam_step_lp,
    lsq_bdr_layernorm_bwd,
    lsq_calib_stream,
    lsq_bdr_layernorm_fwd,
    lsq_bias_act_dropout_bwd,
    lsq_bias_act_dropout_fwd,
    lsq_sgd_step,
    lsq_bias_dropout_residual_bwd,
    lsq_bias_dropout_residual_fwd,
    lsq_embedding_bwd,
    lsq_embedding_fwd,
    lsq_layernorm_bwd,
    lsq_layernorm_bwd_noalloc,
    lsq_layernorm_fwd,
    lsq_ls_xent_bwd,
    lsq_ls_xent_fwd_bwd,
    lsq_ls_xent_fwd,
    lsq_merge_heads_bwd,
    lsq_merge_heads_fwd,
    lsq_pad_offsets,
    lsq_pad_remove,
    lsq_pad_restore,
    lsq_softmax_varlen_bwd,
    lsq_softmax_varlen_fwd,
    lsq_split_heads_bwd,
    lsq_split_heads_fwd,
    lsq_softmax_bwd,
    lsq_softmax_candidates,
    lsq_softmax_tune,
    lsq_softmax_fwd,
    lsq_status_string,
    lsq_workspace_bytes,
)

__all__ = [
    "LsqError", "lib_path", "load", "lsq_adam_state_bytes", "lsq_adam_state_pack", "lsq_adam_state_unpack", "lsq_adam_step",
    "lsq_adam_step_blocked", "lsq_adam_step_lp", "lsq_adam_step_lp_blocked", "lsq_sgd_step_blocked",
    "lsq_trainer_state_bytes", "lsq_trainer_state_pack", "lsq_trainer_state_unpack", "lsq_bdr_layernorm_bwd", "lsq_bdr_layernorm_fwd", "lsq_calib_stream", "lsq_bias_act_dropout_bwd",
    "lsq_bias_act_dropout_fwd", "lsq_sgd_step", "lsq_bias_dropout_residual_bwd",
    "lsq_bias_dropout_residual_fwd", "lsq_embedding_bwd", "lsq_embedding_fwd", "lsq_layernorm_bwd", "lsq_layernorm_bwd_noalloc", "lsq_layernorm_fwd", "lsq_ls_xent_bwd",
    "lsq_ls_xent_fwd_bwd",    "lsq_ls_xent_fwd", "lsq_merge_heads_bwd", "lsq_merge_heads_fwd", "lsq_split_heads_bwd", "lsq_split_heads_fwd",
    "lsq_pad_offsets", "lsq_pad_remove", "lsq_pad_restore", "lsq_softmax_varlen_bwd", "lsq_softmax_varlen_fwd",
    "lsq_softmax_bwd", "lsq_softmax_candidates", "lsq_softmax_fwd", "lsq_softmax_tune", "lsq_status_string", "lsq_workspace_bytes",
]
