/*
 * lsq.h — C-ABI of the fused, memory-bound (non-GEMM) kernels of one Transformer
 * training step on AMD MI355X (gfx950): LayerNorm, bias+dropout+residual,
 * attention softmax, label-smoothed cross-entropy and the mixed-precision Adam
 * trainer, each forward and backward, as the LightSeq2 paper (arXiv 2110.05722)
 * states them in Sec. IV-A (computational graph optimisations), Sec. IV-B
 * (dependent reduction rewriting) and Sec. IV-C (mixed-precision trainer).
 *
 * Conventions that hold for every entry point
 *   - Every data pointer is a DEVICE pointer owned by the caller; the library
 *     allocates nothing, frees nothing and never synchronises.  It keeps no state
 *     between calls except two host-side "done once per device" notes, both
 *     guarded for concurrent host threads: the raised dynamic-LDS limit of the
 *     LayerNorm backward kernel for rows of 8193..16384 columns
 *     (hipFuncSetAttribute on its first use on a device) and the device address
 *     of the array behind lsq_layernorm_bwd_noalloc; and the launch shapes
 *     lsq_softmax_tune has recorded, if it was called.  None is a stream
 *     operation; a caller that captures such a call into a HIP graph should
 *     have made one eager call of it on that device before.  Work is
 *     enqueued on `stream` (a hipStream_t passed as void*; NULL = the null
 *     stream) and the call returns as soon as the launches are queued.
 *   - Tensors are dense, row-major, innermost dimension contiguous.  Base
 *     pointers must be 16-byte aligned (LSQ_MISALIGNED otherwise); inner
 *     dimensions are arbitrary (the paper's "arbitrary shape of inputs",
 *     Sec. III).
 *   - `dt` is the storage type of activations / gradients / parameters
 *     (LSQ_F16, LSQ_BF16, or LSQ_F32).  All arithmetic and accumulation is
 *     fp32 (Sec. IV-B, last paragraph on LayerNorm: low-precision storage,
 *     single-precision computation).  Results are rounded once, to nearest
 *     even, when stored.
 *   - Outputs must not alias inputs except where a comment says they may.
 *   - Results are bit-reproducible from run to run: no floating-point atomics.  (A launch
 *     shape recorded by lsq_softmax_tune sums a row in another order than the default: the
 *     last bit of a few softmax outputs may differ from the default's, reproducibly.)
 *   - Return value: LSQ_OK, or an error code; on error nothing was launched.
 *     Sizes of zero (rows == 0, n == 0, ...) are valid and launch nothing.
 *
 * Dropout contract (the paper fixes no generator; Sec. IV-A only names the op)
 *   Philox4x32-10 (Salmon et al., SC'11) keyed by `seed`, one call per group of
 *   8 consecutive elements: for flat element index e (row-major over the whole
 *   tensor), group g = e / 8, key = (seed_lo, seed_hi),
 *   counter = (g_lo, g_hi, offset_lo, offset_hi).  The four 32-bit output words
 *   w0..w3 are cut into eight 16-bit lanes; element e uses lane e % 8, i.e.
 *   r16 = (w[(e%8)/2] >> (16*(e%2))) & 0xFFFF.  With T16 = round(p * 65536)
 *   (host double arithmetic, clamped to [0, 65535]) the element is KEPT iff
 *   r16 >= T16, and kept values are scaled by 1/(1-p) (inverted dropout, the
 *   nominal p).  p == 0 keeps everything and draws nothing; a p > 0 so small that T16 is 0
 *   (p < 2^-17) keeps everything too and still scales by 1/(1-p).  Nothing is stored:
 *   the backward entry points regenerate the mask from (seed, offset).
 */
#ifndef LSQ_H_
#define LSQ_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LSQ_OK = 0,
    LSQ_INVALID_ARG = 1,         /* null pointer, negative size, p outside [0,1), step < 1 ... */
    LSQ_UNSUPPORTED_DTYPE = 2,
    LSQ_MISALIGNED = 3,          /* a base pointer is not 16-byte aligned */
    LSQ_WORKSPACE_TOO_SMALL = 4,
    LSQ_LAUNCH_FAILED = 5        /* the HIP runtime rejected a launch */
} lsq_status;

typedef enum { LSQ_F16 = 0, LSQ_BF16 = 1, LSQ_F32 = 2 } lsq_dtype;

/* Operators that need a caller-supplied device workspace (column reductions). */
typedef enum {
    LSQ_OP_LAYERNORM_BWD = 0,
    LSQ_OP_BIAS_DROPOUT_RESIDUAL_BWD = 1,
    LSQ_OP_BIAS_ACT_DROPOUT_BWD = 2,
    LSQ_OP_SPLIT_HEADS_BWD = 3,         /* cols = parts * heads * head_dim */
    LSQ_OP_EMBEDDING_BWD = 4,           /* rows = batch * len tokens */
    LSQ_OP_BDR_LAYERNORM_BWD = 5
} lsq_op;

/* Activations of the feed-forward block. */
typedef enum { LSQ_ACT_RELU = 0, LSQ_ACT_GELU = 1 /* erf form */, LSQ_ACT_GELU_TANH = 2 /* tanh approximation */ } lsq_act;

/* Bytes of device workspace `op` needs for a [rows, cols] problem (0 if none).
 * Contents on entry are ignored; contents on exit are unspecified. */
size_t lsq_workspace_bytes(int32_t op, int64_t rows, int32_t cols);

/* Static, human-readable name of a status code. */
const char* lsq_status_string(lsq_status s);

/* LayerNorm forward (Sec. IV-B, LayerNorm equation):
 *   y[r,i] = gamma[i] * (x[r,i] - mean[r]) * rstd[r] + beta[i],
 *   mean[r] = sum_i x[r,i] / hidden,  rstd[r] = 1/sqrt(var[r] + eps),
 *   var = biased variance (divide by hidden), as the paper's mu(x^2)-mu(x)^2
 *   form implies.  The variance is taken about the mean in a second pass over
 *   registers, so it cannot go negative.
 * x, y: [rows, hidden] dt;  gamma, beta: [hidden] dt;  mean, rstd: [rows] fp32
 * (saved for backward).  Errors: null pointers, rows < 0, hidden <= 0, eps < 0.
 * Speed: rows of up to 16384 columns, hidden a multiple of 8, stay in registers (one
 * pass over memory, forward and backward); any other hidden takes a generic path that
 * re-reads the row from cache and takes about twice the time. */
lsq_status lsq_layernorm_fwd(void* y, float* mean, float* rstd,
                             const void* x, const void* gamma, const void* beta,
                             int64_t rows, int32_t hidden, float eps,
                             lsq_dtype dt, void* stream);

/* LayerNorm backward (Sec. IV-B, the gradient equation after "the final gradient"):
 *   xhat = (x - mean) * rstd,  g_i = gamma_i * dy_i,
 *   dx_i = rstd * (g_i - (sum_j g_j + xhat_i * sum_j g_j xhat_j) / hidden) [+ dres_in_i]
 *   dgamma_i = sum_rows dy_i * xhat_i,   dbeta_i = sum_rows dy_i
 * (dgamma/dbeta are the standard parameter gradients; the paper prints only dx).
 * dy, x, dx: [rows, hidden] dt;  gamma: [hidden] dt;  mean, rstd: [rows] fp32 as
 * written by the forward;  dgamma, dbeta: [hidden] fp32, overwritten;
 * dres_in: nullable [rows, hidden] dt, added into dx (gradient arriving over the
 * residual branch of a pre-LayerNorm block).  dx may alias dy or dres_in.
 * workspace: >= lsq_workspace_bytes(LSQ_OP_LAYERNORM_BWD, rows, hidden) bytes. */
lsq_status lsq_layernorm_bwd(void* dx, float* dgamma, float* dbeta,
                             const void* dy, const void* x, const void* gamma,
                             const float* mean, const float* rstd, const void* dres_in,
                             void* workspace, size_t workspace_bytes,
                             int64_t rows, int32_t hidden, lsq_dtype dt, void* stream);

/* lsq_layernorm_bwd for callers that cannot allocate device memory or own no workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same operation, same
 * arguments (minus the workspace), same kernels and therefore the same bits as lsq_layernorm_bwd.
 * The partial rows of the dgamma / dbeta column sums go to an 8 MiB device array that the library
 * itself holds (one copy per GPU the library runs on, until the process ends); the call allocates
 * and frees nothing.  Limit: lsq_workspace_bytes(LSQ_OP_LAYERNORM_BWD, rows, hidden) <= 8 MiB
 * (hidden <= 4096 for any number of rows); beyond it the call returns LSQ_WORKSPACE_TOO_SMALL and
 * launches nothing.  Every call on a GPU uses that GPU's one array: calls that may overlap in time on
 * one GPU (different streams, concurrent graph launches) race and must be serialised by the caller.
 * Nothing in the array needs to start at zero (each launch overwrites what it later reads).
 * LSQ_LAUNCH_FAILED if the array's device address cannot be obtained. */
lsq_status lsq_layernorm_bwd_noalloc(void* dx, float* dgamma, float* dbeta,
                                     const void* dy, const void* x, const void* gamma,
                                     const float* mean, const float* rstd, const void* dres_in,
                                     int64_t rows, int32_t hidden, lsq_dtype dt, void* stream);

/* Fused bias + dropout + residual, forward (Sec. IV-A, Transformer layers: the
 * last kernel of the self-attention block):
 *   out[r,i] = residual[r,i] + keep[r,i] * (x[r,i] + bias[i]) / (1 - p)
 * x, residual, out: [rows, hidden] dt;  bias: nullable [hidden] dt.
 * out may alias x or residual.  p in [0,1).  Dropout contract above, flat index
 * e = r*hidden + i.
 * Speed: hidden a multiple of 8 takes the column-block kernels; any other hidden is walked as one
 * flat array in aligned 128-bit packs (a pack may straddle two rows; the bias is gathered per
 * element), forward and backward, about 1.5 x the time; the same holds for
 * lsq_bias_act_dropout_fwd/bwd (about 2 x). */
lsq_status lsq_bias_dropout_residual_fwd(void* out, const void* x, const void* bias,
                                         const void* residual, int64_t rows, int32_t hidden,
                                         float p, uint64_t seed, uint64_t offset,
                                         lsq_dtype dt, void* stream);

/* Backward of the above: dx = keep * dy / (1-p) with the mask regenerated from
 * (seed, offset);  dbias[i] = sum_rows dx[r,i] (nullable; fp32 [hidden],
 * overwritten).  The gradient of `residual` is dy itself: the caller aliases it.
 * dx may alias dy.  workspace: >= lsq_workspace_bytes(LSQ_OP_BIAS_DROPOUT_RESIDUAL_BWD,
 * rows, hidden) bytes, only read when dbias != NULL. */
lsq_status lsq_bias_dropout_residual_bwd(void* dx, float* dbias, const void* dy,
                                         int64_t rows, int32_t hidden,
                                         float p, uint64_t seed, uint64_t offset,
                                         void* workspace, size_t workspace_bytes,
                                         lsq_dtype dt, void* stream);

/* Attention softmax forward (Sec. IV-B, Softmax: the three-step stable form) over
 * the last axis of x[batch, heads, q_len, k_len], restricted to the allowed set
 *   A(b,i) = { j : j < key_len[b] }  intersected, if causal != 0, with
 *            { j : j <= i + (k_len - q_len) }:
 *   m = max_{j in A} scale*x_j;  Z = sum_{j in A} exp(scale*x_j - m);
 *   y_j = exp(scale*x_j - m) / Z for j in A, and exactly +0 for j not in A
 * (an empty A gives an all-zero row).  If p_attn > 0, y_drop = keep * y / (1-p_attn)
 * is written as well (dropout contract above, flat index over the whole tensor).
 * key_len: nullable int32[batch] (NULL = every key allowed), values clamped to
 * [0, k_len].  y_drop must be non-NULL iff p_attn > 0.  y may alias x.
 * Speed: key axes that are a multiple of 8 (any length up to 16384) take the 128-bit
 * register paths; other lengths up to 2048 go through LDS staging, 10-30 % slower.
 * scale: any finite value; a scale that is not positive (never an attention scale) takes
 * the LDS-staging kernels as well.  batch*heads*q_len must be below 2^31. */
lsq_status lsq_softmax_fwd(void* y, void* y_drop, const void* x, const int32_t* key_len,
                           int32_t batch, int32_t heads, int32_t q_len, int32_t k_len,
                           int32_t causal, float scale,
                           float p_attn, uint64_t seed, uint64_t offset,
                           lsq_dtype dt, void* stream);

/* Attention softmax backward (the softmax Jacobian of Sec. IV-A, criterion layer,
 * contracted with the upstream gradient):
 *   dx_j = scale * y_j * (dyy_j - sum_{k in A} dyy_k y_k),  0 outside A,
 * where dyy = dy if p_attn == 0, else keep * dy / (1-p_attn) with dy the
 * gradient of y_drop.  y is the tensor the forward stored.  dx may alias dy. */
lsq_status lsq_softmax_bwd(void* dx, const void* dy, const void* y, const int32_t* key_len,
                           int32_t batch, int32_t heads, int32_t q_len, int32_t k_len,
                           int32_t causal, float scale,
                           float p_attn, uint64_t seed, uint64_t offset,
                           lsq_dtype dt, void* stream);

/* Run-time choice of the softmax launch shape (Sec. IV-B, Softmax, last paragraph: several
 * templates, the best parameters searched before training starts).  For rows of up to 2048 keys
 * (k_len a multiple of 8) the library holds up to 4 launch shapes (lanes per row, packs per lane,
 * rows per lane group) per row length; lsq_softmax_candidates returns how many (1 where there is no
 * choice).  lsq_softmax_tune with force == -1 runs every candidate of the given problem on the
 * caller's buffers (arguments as lsq_softmax_varlen_fwd / _bwd; y, y_drop and dx are overwritten
 * with valid results), `reps` launches each between two events on `stream`, and records the fastest
 * per direction for (row-length bucket, mask kind, dropout on/off, storage width); later calls of
 * lsq_softmax_fwd/bwd and the varlen forms with such a problem use it.  force >= 0 records that
 * candidate without launching anything (all candidates give the same results up to summation order
 * inside a row; the tests run every one against the oracle); force == -2 forgets the record (the
 * built-in default, candidate 0, is used again).  best_fwd / best_bwd (nullable) receive the choice,
 * us (nullable, float[8]) the measured microseconds per launch, [direction][candidate], -1 where
 * there is none.  The search synchronises with `stream` (it waits for its events) and must not be
 * called under stream capture; it allocates no device memory.  The record is process-wide host
 * state, safe against concurrent host threads. */
int32_t lsq_softmax_candidates(int32_t k_len);
lsq_status lsq_softmax_tune(int32_t* best_fwd, int32_t* best_bwd, float* us,
                            void* y, void* y_drop, void* dx, const void* x, const void* dy,
                            const int32_t* key_len, const int32_t* query_len,
                            int32_t batch, int32_t heads, int32_t q_len, int32_t k_len,
                            int32_t causal, float scale, float p_attn, uint64_t seed, uint64_t offset,
                            lsq_dtype dt, int32_t force, int32_t reps, void* stream);

/* Label-smoothed cross-entropy forward (Sec. IV-A, criterion layer): per token,
 * with q = softmax(h) over the whole vocabulary and p = (1-alpha)*onehot(k) + alpha/V,
 *   loss = -sum_i p_i log q_i = lse - (1-alpha)*h_k - (alpha/V) * sum_i h_i,
 *   nll  = -log q_k = lse - h_k,        lse = log sum_i exp(h_i).
 * logits: [tokens, vocab] dt;  target: int32[tokens];  loss, lse: fp32[tokens];
 * nll: nullable fp32[tokens].  A token whose target equals ignore_index or lies
 * outside [0, vocab) is ignored (padding): its row is not read, loss = nll = lse = 0.
 * sums: nullable fp32[3] = { sum loss, sum nll, number of non-ignored tokens },
 * reduced in a fixed order (bit-reproducible); it is cheapest when nll is given
 * (without it the target logits are gathered a second time). */
lsq_status lsq_ls_xent_fwd(float* loss, float* nll, float* lse, float* sums,
                           const void* logits, const int32_t* target,
                           int64_t tokens, int32_t vocab, float alpha, int32_t ignore_index,
                           lsq_dtype dt, void* stream);

/* Backward of the criterion (Sec. IV-A, the final gradient to the decoder output):
 *   dlogits_i = grad_scale * (exp(h_i - lse) - alpha/V - (1-alpha)*[i == k]),
 * all zero for ignored tokens.  lse: as written by the forward.  dlogits may
 * alias logits (in-place). */
lsq_status lsq_ls_xent_bwd(void* dlogits, const void* logits, const float* lse,
                           const int32_t* target, int64_t tokens, int32_t vocab,
                           float alpha, int32_t ignore_index, float grad_scale,
                           lsq_dtype dt, void* stream);

/* Criterion forward and backward in ONE pass (Sec. IV-A, criterion layer: both formulas
 * above).  The scale of the loss gradient is known before the criterion runs, so the
 * gradient can be written while a token's row is still on chip: the logits are read
 * once and dlogits written once, two passes over [tokens, vocab] instead of the three
 * of the two calls (about a quarter less time when most tokens count; no gain on
 * masked-LM batches where most rows are ignored and only zeros are written).
 * Outputs as lsq_ls_xent_fwd (loss, nll nullable, lse, sums nullable) plus dlogits as
 * lsq_ls_xent_bwd.  dlogits is evaluated as e_i * (grad_scale / S) - grad_scale*alpha/V
 * with e_i = exp(h_i - max) rounded once to dt and S = sum_i e_i: it agrees with
 * lsq_ls_xent_bwd to two roundings of dt.  dlogits may alias logits (in place); in place,
 * `sums` needs `nll` (LSQ_INVALID_ARG if sums != NULL, nll == NULL and dlogits == logits:
 * the logits the sum of nll would be gathered from are overwritten by then).  Rows
 * of up to 65528 elements are held in registers; longer rows run the two operators
 * back to back. */
lsq_status lsq_ls_xent_fwd_bwd(float* loss, float* nll, float* lse, float* sums, void* dlogits,
                               const void* logits, const int32_t* target,
                               int64_t tokens, int32_t vocab, float alpha, int32_t ignore_index,
                               float grad_scale, lsq_dtype dt, void* stream);

/* Mixed-precision Adam over one flat workspace, one launch (Sec. IV-C): the
 * low-precision gradient is converted on the fly, the update runs in fp32
 * registers, and each element is read and written once.
 *   ghat = g * inv_grad_scale (+ weight_decay * p if adamw == 0)
 *   m = beta1*m + (1-beta1)*ghat;  v = beta2*v + (1-beta2)*ghat^2
 *   c1 = 1 - beta1^step, c2 = 1 - beta2^step (both 1 if bias_correction == 0)
 *   p = p - lr * ( (m/c1) / (sqrt(v/c2) + eps) + (adamw ? weight_decay*p : 0) )
 *   p_lp = round-to-nearest-even(p) in p_lp_dt   (nullable: the copy the next
 *   forward pass reads)
 * p, m, v: fp32[n], updated in place;  g: [n] g_dt (LSQ_F32 allowed);
 * p_lp: nullable [n] p_lp_dt.  Errors: step < 1, n < 0, beta outside [0,1). */
lsq_status lsq_adam_step(float* p, float* m, float* v, const void* g, void* p_lp,
                         int64_t n, float lr, float beta1, float beta2, float eps,
                         float weight_decay, int32_t step, int32_t adamw,
                         int32_t bias_correction, float inv_grad_scale,
                         lsq_dtype g_dt, lsq_dtype p_lp_dt, void* stream);

/* Fused bias + activation + dropout of the feed-forward block, forward (Sec. IV-A:
 * adjacent element-wise kernels fused; the paper names ReLU, the BERT / GPT-2
 * models of Sec. VI use GELU):
 *   out[r,i] = keep[r,i] * act(x[r,i] + bias[i]) / (1 - p)
 * x, out: [rows, hidden] dt;  bias: nullable [hidden] dt;  act: an lsq_act.
 * out may alias x (but backward needs x: keep it if you train). */
lsq_status lsq_bias_act_dropout_fwd(void* out, const void* x, const void* bias,
                                    int64_t rows, int32_t hidden, int32_t act,
                                    float p, uint64_t seed, uint64_t offset,
                                    lsq_dtype dt, void* stream);

/* Backward of the above: dx = act'(x + bias) * keep * dy / (1-p), mask regenerated,
 * slope recomputed from the saved pre-activation x (ReLU slope at 0 is 0);
 * dbias[i] = sum_rows dx[r,i] (nullable; fp32 [hidden], overwritten).  dx may
 * alias dy.  workspace: >= lsq_workspace_bytes(LSQ_OP_BIAS_ACT_DROPOUT_BWD, rows,
 * hidden) bytes, only used when dbias != NULL. */
lsq_status lsq_bias_act_dropout_bwd(void* dx, float* dbias, const void* dy, const void* x,
                                    const void* bias, int64_t rows, int32_t hidden, int32_t act,
                                    float p, uint64_t seed, uint64_t offset,
                                    void* workspace, size_t workspace_bytes,
                                    lsq_dtype dt, void* stream);

/* The paper's own trainer layout (Sec. IV-C): the workspace holds the parameter in
 * LOW precision; it is widened in registers, updated with the rule of
 * lsq_adam_step, narrowed (round to nearest even) and stored in place.
 * p_lp, g: [n] dt (LSQ_F16 or LSQ_BF16);  m, v: fp32[n] in place.  22 bytes/param. */
lsq_status lsq_adam_step_lp(void* p_lp, float* m, float* v, const void* g, int64_t n,
                            float lr, float beta1, float beta2, float eps, float weight_decay,
                            int32_t step, int32_t adamw, int32_t bias_correction,
                            float inv_grad_scale, lsq_dtype dt, void* stream);

/* The boundary between two sub-layers of a pre-LN Transformer in ONE pass: the paper
 * fuses "bias adding, dropout, and residual" (Sec. IV-A) and rewrites LayerNorm
 * (Sec. IV-B) as two kernels; the output of the first is the input of the second, so
 * here the row never leaves the registers in between.
 *   h = residual + Dropout_p(x + bias)          (stored: the next residual)
 *   y, mean, rstd = LayerNorm(h; gamma, beta)   (from the STORED, rounded h)
 * Bit for bit the result of lsq_bias_dropout_residual_fwd followed by
 * lsq_layernorm_fwd on its output; 8 instead of 10 bytes per element, one launch.
 * Arguments as in those two calls (h: [rows, hidden] dt, written), except that h and y must
 * not alias x or residual (the next rows of x and residual are being read while h is
 * written). */
lsq_status lsq_bdr_layernorm_fwd(void* h, void* y, float* mean, float* rstd, const void* x,
                                 const void* bias, const void* residual, const void* gamma,
                                 const void* beta, int64_t rows, int32_t hidden, float p,
                                 uint64_t seed, uint64_t offset, float eps, lsq_dtype dt, void* stream);

/* Its backward, also one pass:
 *   dh = LayerNorm_bwd(dy; h, gamma, mean, rstd) + dres_in   (stored: the gradient of the
 *                                                             residual branch; dres_in nullable)
 *   dx = keep * dh / (1-p)  from the STORED dh                (gradient of the projection)
 *   dgamma, dbeta (LayerNorm), dbias = column sums of dx      (fp32, overwritten)
 * dh and dx equal lsq_layernorm_bwd followed by lsq_bias_dropout_residual_bwd bit for
 * bit (the three column sums differ from theirs only in summation order); 10 instead
 * of 12 bytes per element, one second-stage launch instead of two.
 * workspace: >= lsq_workspace_bytes(LSQ_OP_BDR_LAYERNORM_BWD, rows, hidden) bytes. */
lsq_status lsq_bdr_layernorm_bwd(void* dh, void* dx, float* dgamma, float* dbeta, float* dbias,
                                 const void* dy, const void* h, const void* gamma, const float* mean,
                                 const float* rstd, const void* dres_in, void* workspace,
                                 size_t workspace_bytes, int64_t rows, int32_t hidden, float p,
                                 uint64_t seed, uint64_t offset, lsq_dtype dt, void* stream);

/* Adam with the trainer's private state in a blocked layout (Sec. IV-C builds one
 * workspace so that the update is one launch over contiguous memory; this goes one step
 * further for the three fp32 arrays that only the trainer reads).  `state` holds
 * ceil(n / LSQ_ADAM_BLOCK) blocks of 3 * LSQ_ADAM_BLOCK floats: the block's slice of
 * p, then of m, then of v.  Same arithmetic, same bytes as lsq_adam_step, one address
 * stream instead of three (measured 8 % faster at 774 M parameters).
 *
 * lsq_adam_state_bytes(n): size of `state` in bytes (0 for n <= 0).
 * lsq_adam_state_pack:     state <- (p, m, v); m and/or v NULL mean zeros (a fresh
 *                          optimizer); the padding of the last block is zero-filled.
 * lsq_adam_state_unpack:   (p, m, v) <- state; NULL outputs are skipped (checkpoints,
 *                          tests).  Both are bit-exact moves of fp32 values.
 * lsq_adam_step_blocked:   lsq_adam_step on that state; g, p_lp, the hyperparameters,
 *                          the dtypes and the errors are those of lsq_adam_step. */
#define LSQ_ADAM_BLOCK 8192
size_t lsq_adam_state_bytes(int64_t n);
lsq_status lsq_adam_state_pack(float* state, const float* p, const float* m, const float* v, int64_t n,
                               void* stream);
lsq_status lsq_adam_state_unpack(float* p, float* m, float* v, const float* state, int64_t n, void* stream);
lsq_status lsq_adam_step_blocked(float* state, const void* g, void* p_lp, int64_t n,
                                 float lr, float beta1, float beta2, float eps, float weight_decay,
                                 int32_t step, int32_t adamw, int32_t bias_correction,
                                 float inv_grad_scale, lsq_dtype g_dt, lsq_dtype p_lp_dt, void* stream);

/* The blocked layout for any trainer: `arrays` (1..3) fp32 arrays of n elements that only
 * the trainer reads, interleaved in blocks of LSQ_ADAM_BLOCK elements ([a0 | a1 | a2] per
 * block).  lsq_adam_state_bytes/pack/unpack are the arrays = 3 case (p, m, v).
 * pack: a0 required, a1 / a2 NULL mean zeros; unpack: NULL outputs are skipped. */
size_t lsq_trainer_state_bytes(int64_t n, int32_t arrays);
lsq_status lsq_trainer_state_pack(float* state, const float* a0, const float* a1, const float* a2,
                                  int64_t n, int32_t arrays, void* stream);
lsq_status lsq_trainer_state_unpack(float* a0, float* a1, float* a2, const float* state, int64_t n,
                                    int32_t arrays, void* stream);

/* lsq_sgd_step with the master parameters and the momentum buffer blocked as [p | buf]
 * (arrays = 2; the buffer's blocks are present but untouched when momentum == 0), and
 * lsq_adam_step_lp with both moments blocked as [m | v] (arrays = 2) next to the
 * low-precision parameters that stay flat.  Arithmetic, bytes and errors as in the
 * entry points they mirror; results are bit-identical. */
lsq_status lsq_sgd_step_blocked(float* state, const void* g, void* p_lp, int64_t n,
                                float lr, float momentum, float weight_decay, int32_t nesterov,
                                float inv_grad_scale, lsq_dtype g_dt, lsq_dtype p_lp_dt, void* stream);
lsq_status lsq_adam_step_lp_blocked(void* p_lp, float* state, const void* g, int64_t n,
                                    float lr, float beta1, float beta2, float eps, float weight_decay,
                                    int32_t step, int32_t adamw, int32_t bias_correction,
                                    float inv_grad_scale, lsq_dtype dt, void* stream);

/* SGD over the flat workspace, one launch (the paper's second trainer, Sec. VI-C):
 *   ghat = g * inv_grad_scale + weight_decay * p
 *   buf  = momentum * buf + ghat                    (momentum > 0; buf starts at 0)
 *   d    = nesterov ? ghat + momentum * buf : (momentum > 0 ? buf : ghat)
 *   p    = p - lr * d;   p_lp = round-to-nearest-even(p)  (nullable)
 * p: fp32[n] in place;  momentum_buf: fp32[n] in place, may be NULL iff momentum == 0;
 * g: [n] g_dt.  Errors: momentum < 0, nesterov without momentum. */
lsq_status lsq_sgd_step(float* p, float* momentum_buf, const void* g, void* p_lp, int64_t n,
                        float lr, float momentum, float weight_decay, int32_t nesterov,
                        float inv_grad_scale, lsq_dtype g_dt, lsq_dtype p_lp_dt, void* stream);

/* Head split (the "Reshape" of Sec. IV-A's element-wise operations): the projection
 * output `in` [batch*len, parts*hidden], columns ordered (part, head, head_dim), plus
 * an optional bias [parts*hidden], is written as `parts` tensors
 * out_k[batch, heads, len, head_dim] (k < parts; parts in 1..3: 3 for a fused QKV
 * projection).  hidden = heads*head_dim.  Unused out pointers may be NULL.
 * Without a bias the move is bit-exact.  batch*len must be below 2^31 (LSQ_INVALID_ARG beyond;
 * the same holds for the three calls that follow). */
lsq_status lsq_split_heads_fwd(void* out0, void* out1, void* out2, const void* in, const void* bias,
                               int32_t batch, int32_t len, int32_t heads, int32_t head_dim,
                               int32_t parts, lsq_dtype dt, void* stream);

/* Backward of the split: din[batch*len, parts*hidden] gathers d_k[batch, heads, len,
 * head_dim] (bit-exact), and dbias[parts*hidden] (nullable, fp32, overwritten) is
 * the column sum of din.  workspace: >= lsq_workspace_bytes(LSQ_OP_SPLIT_HEADS_BWD,
 * batch*len, parts*hidden) bytes, only used when dbias != NULL. */
lsq_status lsq_split_heads_bwd(void* din, float* dbias, const void* d0, const void* d1, const void* d2,
                               int32_t batch, int32_t len, int32_t heads, int32_t head_dim,
                               int32_t parts, void* workspace, size_t workspace_bytes,
                               lsq_dtype dt, void* stream);

/* Head merge of the attention output: x[batch, heads, len, head_dim] ->
 * out[batch*len, hidden]; and its backward, dy[batch*len, hidden] ->
 * dx[batch, heads, len, head_dim].  Both are bit-exact moves. */
lsq_status lsq_merge_heads_fwd(void* out, const void* x, int32_t batch, int32_t len, int32_t heads,
                               int32_t head_dim, lsq_dtype dt, void* stream);
lsq_status lsq_merge_heads_bwd(void* dx, const void* dy, int32_t batch, int32_t len, int32_t heads,
                               int32_t head_dim, lsq_dtype dt, void* stream);

/* Embedding forward (Sec. IV-A, embedding layer):
 *   out[t,:] = keep[t,:] * (scale * emb[tokens[t],:] + pos[t mod len,:]) / (1 - p)
 * tokens: int32[batch*len];  emb: [vocab, hidden] dt;  pos: [>= len, hidden] dt;
 * out: [batch*len, hidden] dt.  A token equal to pad_idx or outside [0, vocab)
 * gives a zero row.  Dropout contract as everywhere, flat index over out. */
lsq_status lsq_embedding_fwd(void* out, const int32_t* tokens, const void* emb, const void* pos,
                             int32_t batch, int32_t len, int32_t hidden, int32_t vocab, int32_t pad_idx,
                             float scale, float p, uint64_t seed, uint64_t offset,
                             lsq_dtype dt, void* stream);

/* Embedding backward (Sec. IV-A): the gradient rows of a repeated token are summed
 * (the paper uses atomicAdd; here the order is fixed, ascending position, so the
 * result is bit-reproducible):
 *   demb[w,:] += scale * sum_{t: tokens[t] == w} keep[t,:] * dy[t,:] / (1-p)
 *   dpos[l,:] += sum_b keep * dy[b*len + l,:] / (1-p)            (dpos nullable)
 * demb [vocab, hidden] and dpos [len, hidden] are dt and are ACCUMULATED INTO (one
 * rounding per row and call; rows of tokens that do not occur are not touched).
 * Padding tokens receive nothing.  workspace: >= lsq_workspace_bytes(
 * LSQ_OP_EMBEDDING_BWD, batch*len, hidden) bytes.  Errors: batch*len beyond 2^30. */
lsq_status lsq_embedding_bwd(void* demb, void* dpos, const void* dy, const int32_t* tokens,
                             int32_t batch, int32_t len, int32_t hidden, int32_t vocab, int32_t pad_idx,
                             float scale, float p, uint64_t seed, uint64_t offset,
                             void* workspace, size_t workspace_bytes, lsq_dtype dt, void* stream);

/* Padding removal (named in the paper's conclusion as the optimisation to do next):
 * the real rows of a padded [batch, max_len, hidden] tensor are stored back to back
 * as [sum(len), hidden], so the row-wise operators above run on sum(len) rows.
 *
 * lsq_pad_offsets writes offsets[b] = sum_{b' < b} len_b', offsets[batch] = sum(len),
 * with len_b = clamp(key_len[b], 0, max_len) (key_len NULL: every sentence is full).
 * offsets: int32[batch + 1], device.  batch * max_len must fit in int32. */
lsq_status lsq_pad_offsets(int32_t* offsets, const int32_t* key_len, int32_t batch, int32_t max_len,
                           void* stream);

/* packed[offsets[b] + i, :] = padded[b, i, :] for i < len_b (len_b = offsets[b+1] -
 * offsets[b]); a bit-exact move.  packed_rows is the capacity of `packed` in rows
 * (>= sum(len), which the caller's batching knows; the padded row count is always
 * enough): rows that would fall outside it are skipped, nothing is written beyond.
 * Rows of `packed` from sum(len) on are not touched.  Its backward is
 * lsq_pad_restore (the gradient of a dropped row is 0). */
lsq_status lsq_pad_remove(void* packed, const void* padded, const int32_t* offsets, int32_t batch,
                          int32_t max_len, int32_t hidden, int64_t packed_rows, lsq_dtype dt, void* stream);

/* padded[b, i, :] = packed[offsets[b] + i, :] for i < len_b, and +0 on the padding;
 * every element of `padded` is written.  Its backward is lsq_pad_remove. */
lsq_status lsq_pad_restore(void* padded, const void* packed, const int32_t* offsets, int32_t batch,
                           int32_t max_len, int32_t hidden, int64_t packed_rows, lsq_dtype dt, void* stream);

/* lsq_softmax_fwd / lsq_softmax_bwd with query lengths as well: query rows
 * i >= query_len[b] are padding, their allowed set is empty, so they are not read and
 * their outputs are exact zeros (finite, so that the batched products around the
 * softmax stay finite).  query_len: int32[batch], device, nullable (NULL gives
 * lsq_softmax_fwd / lsq_softmax_bwd exactly).  Everything else as documented there. */
lsq_status lsq_softmax_varlen_fwd(void* y, void* y_drop, const void* x, const int32_t* key_len,
                                  const int32_t* query_len, int32_t batch, int32_t heads, int32_t q_len,
                                  int32_t k_len, int32_t causal, float scale, float p_attn,
                                  uint64_t seed, uint64_t offset, lsq_dtype dt, void* stream);
lsq_status lsq_softmax_varlen_bwd(void* dx, const void* dy, const void* y, const int32_t* key_len,
                                  const int32_t* query_len, int32_t batch, int32_t heads, int32_t q_len,
                                  int32_t k_len, int32_t causal, float scale, float p_attn,
                                  uint64_t seed, uint64_t offset, lsq_dtype dt, void* stream);

/* Measurement aid, not an operator: a plain memory stream in the operators' launch style (128-bit
 * nontemporal accesses, one pack per thread), which the benchmark times beside the operators at the
 * operators' tensor sizes (the calibration ceiling).  kind 0: copy `bytes` from src to dst;
 * kind 1: read `bytes` of src (dst: 4 bytes that are written only if a pack of src equals an
 * unlikely constant); kind 2: write `bytes` of a constant to dst; kind 3: an empty kernel (launch
 * cost).  bytes: a multiple of 16. */
lsq_status lsq_calib_stream(int32_t kind, void* dst, const void* src, int64_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* LSQ_H_ */
