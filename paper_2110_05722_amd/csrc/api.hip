// Entry points that launch nothing: workspace sizing and status names.
#include "host.hpp"

extern "C" size_t lsq_workspace_bytes(int32_t op, int64_t rows, int32_t cols)
{
    using namespace lsq;
    if (rows <= 0 || cols <= 0) return 0;
    switch (op) {
        case LSQ_OP_LAYERNORM_BWD:
            // one [2][cols] fp32 partial row (dgamma, dbeta) per workgroup
            return static_cast<size_t>(ln_bwd_blocks(rows, cols)) * 2u * static_cast<size_t>(cols) * sizeof(float);
        case LSQ_OP_BDR_LAYERNORM_BWD:
            // one [3][cols] fp32 partial row (dgamma, dbeta, dbias) per workgroup; also enough for the
            // two separate operators that serve row lengths without a register bucket
            {
                const size_t fused = static_cast<size_t>(ln_bwd_blocks(rows, cols)) * 3u * static_cast<size_t>(cols) * sizeof(float);
                const size_t apart = lsq_workspace_bytes(LSQ_OP_BIAS_DROPOUT_RESIDUAL_BWD, rows, cols);
                return fused > apart ? fused : apart;
            }
        case LSQ_OP_BIAS_DROPOUT_RESIDUAL_BWD:
            // one [cols] fp32 partial row (dbias) per row block
            if (!bdr_bwd_is_flat(cols))
                return static_cast<size_t>(bdr_bwd_plan(rows, cols).row_blocks) * static_cast<size_t>(cols) * sizeof(float);
            return flat_workspace_bytes(rows, cols);        // one per workgroup of the flat walk
        case LSQ_OP_BIAS_ACT_DROPOUT_BWD:
            if (bad_is_flat(cols)) return flat_workspace_bytes(rows, cols);
            return static_cast<size_t>(bad_bwd_row_blocks(rows, cols)) * static_cast<size_t>(cols) * sizeof(float);
        case LSQ_OP_SPLIT_HEADS_BWD:
            // one [cols] fp32 partial row (dbias) per row block
            return static_cast<size_t>(heads_bwd_row_blocks(rows, cols)) * static_cast<size_t>(cols) * sizeof(float);
        case LSQ_OP_EMBEDDING_BWD:
            // sorted order, fp32 rows of the id segments that cross a window, rank counts
            return emb_bwd_plan(rows, cols).total();
        default:
            return 0;
    }
}

extern "C" const char* lsq_status_string(lsq_status s)
{
    switch (s) {
        case LSQ_OK: return "LSQ_OK";
        case LSQ_INVALID_ARG: return "LSQ_INVALID_ARG";
        case LSQ_UNSUPPORTED_DTYPE: return "LSQ_UNSUPPORTED_DTYPE";
        case LSQ_MISALIGNED: return "LSQ_MISALIGNED";
        case LSQ_WORKSPACE_TOO_SMALL: return "LSQ_WORKSPACE_TOO_SMALL";
        case LSQ_LAUNCH_FAILED: return "LSQ_LAUNCH_FAILED";
        default: return "LSQ_UNKNOWN_STATUS";
    }
}
