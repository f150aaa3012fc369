/*
 * lsq_oracle.c — TEST INFRASTRUCTURE, not the product.
 *
 * A plain, slow, double-precision CPU statement of what each operator on the hot
 * path computes, written from the paper's formulas (LightSeq2, arXiv 2110.05722,
 * Sec. IV-A criterion layer, Sec. IV-B LayerNorm / Softmax, Sec. IV-C trainer).
 * Only the tests, the smoke check and the benchmark's CPU-baseline leg may call
 * it.  It shares no code with the HIP library: its own storage decoders, its
 * own Philox, its own loops.
 *
 * Conventions
 *   - Inputs arrive in their STORAGE representation (dt: 0 = IEEE fp16 bits,
 *     1 = bfloat16 bits, 2 = float32) and are widened to double exactly.
 *   - All arithmetic is double; reductions are plain left-to-right sums, two
 *     passes where the definition is two passes.
 *   - Outputs are double and UNROUNDED: the caller compares the device result
 *     against them with the tolerance of the device's storage type.
 *   - Rows are independent; `#pragma omp parallel for` over rows is the only
 *     concession to run time (no blocking, fusion or reordering inside a row).
 *
 * Pins (tests/test_oracle_*.py): every function below is pinned by closed
 * forms, invariants, finite differences or brute force that do not call it to
 * produce their expected values.  No function is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

static const double PI = 3.14159265358979323846;

/* ------------------------------------------------------------------ storage */
static double half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int exp = (h >> 10) & 0x1F;
    int man = h & 0x3FF;
    double v;
    if (exp == 0)
        v = ldexp((double)man, -24);               /* subnormal or zero */
    else if (exp == 31)
        v = man ? NAN : INFINITY;
    else
        v = ldexp((double)(man | 0x400), exp - 25);
    return sign ? -v : v;
}

static double bf16_to_double(uint16_t b)
{
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static inline double load(const void* base, int64_t i, int dt)
{
    if (dt == 0) return half_to_double(((const uint16_t*)base)[i]);
    if (dt == 1) return bf16_to_double(((const uint16_t*)base)[i]);
    return (double)((const float*)base)[i];
}

/* ------------------------------------------------------------------- Philox */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy
 * as 1, 2, 3", SC'11): a 4-word counter, a 2-word key, ten rounds of two
 * 32x32->64 multiplies and a word permutation; the key is bumped by the Weyl
 * constants between rounds. */
void lsqo_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = M0 * c0;
        uint64_t p1 = M1 * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += W0; k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Dropout threshold: keep iff r16 >= T16, T16 = round(p * 2^16) clamped. */
static uint32_t threshold16(double p)
{
    double t = floor(p * 65536.0 + 0.5);
    if (t < 0.0) t = 0.0;
    if (t > 65535.0) t = 65535.0;
    return (uint32_t)t;
}

/* The 16 random bits that belong to flat element e. */
static uint32_t dropout_bits(uint64_t e, uint64_t seed, uint64_t offset)
{
    uint64_t g = e >> 3;
    uint32_t ctr[4] = { (uint32_t)g, (uint32_t)(g >> 32), (uint32_t)offset, (uint32_t)(offset >> 32) };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t w[4];
    lsqo_philox4x32_10(ctr, key, w);
    unsigned lane = (unsigned)(e & 7);
    return (w[lane >> 1] >> (16 * (lane & 1))) & 0xFFFFu;
}

static int keep_element(uint64_t e, double p, uint32_t t16, uint64_t seed, uint64_t offset)
{
    if (p == 0.0) return 1;
    return dropout_bits(e, seed, offset) >= t16;
}

/* keep[i] = 1 iff flat element e0+i survives dropout. */
void lsqo_dropout_mask(uint8_t* keep, uint64_t e0, int64_t n, double p, uint64_t seed, uint64_t offset)
{
    uint32_t t16 = threshold16(p);
    for (int64_t i = 0; i < n; ++i)
        keep[i] = (uint8_t)keep_element(e0 + (uint64_t)i, p, t16, seed, offset);
}

/* ---------------------------------------------------------------- LayerNorm */
/* Forward, Sec. IV-B LayerNorm equation, textbook two-pass statistics:
 * biased variance, eps inside the root. */
void lsqo_layernorm_fwd(double* y, double* mean, double* rstd, const void* x, const void* gamma,
                        const void* beta, int64_t rows, int32_t hidden, double eps, int dt)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const int64_t o = r * hidden;
        double s = 0.0;
        for (int i = 0; i < hidden; ++i) s += load(x, o + i, dt);
        double mu = s / hidden;
        double q = 0.0;
        for (int i = 0; i < hidden; ++i) {
            double d = load(x, o + i, dt) - mu;
            q += d * d;
        }
        double rs = 1.0 / sqrt(q / hidden + eps);
        mean[r] = mu;
        rstd[r] = rs;
        for (int i = 0; i < hidden; ++i)
            y[o + i] = load(gamma, i, dt) * ((load(x, o + i, dt) - mu) * rs) + load(beta, i, dt);
    }
}

/* Backward, Sec. IV-B: the "final gradient" equation written with xhat, with
 * sigma = sqrt(var + eps); statistics recomputed here from x in double.
 * dgamma / dbeta are the standard column sums (the paper prints only dx). */
void lsqo_layernorm_bwd(double* dx, double* dgamma, double* dbeta, const void* dy, const void* x,
                        const void* gamma, const void* dres_in, int64_t rows, int32_t hidden,
                        double eps, int dt)
{
    for (int i = 0; i < hidden; ++i) { dgamma[i] = 0.0; dbeta[i] = 0.0; }
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const int64_t o = r * hidden;
        double s = 0.0;
        for (int i = 0; i < hidden; ++i) s += load(x, o + i, dt);
        double mu = s / hidden;
        double q = 0.0;
        for (int i = 0; i < hidden; ++i) { double d = load(x, o + i, dt) - mu; q += d * d; }
        double sigma = sqrt(q / hidden + eps);
        double s1 = 0.0, s2 = 0.0;
        for (int j = 0; j < hidden; ++j) {
            double g = load(dy, o + j, dt) * load(gamma, j, dt);
            double xh = (load(x, o + j, dt) - mu) / sigma;
            s1 += g;
            s2 += g * xh;
        }
        for (int i = 0; i < hidden; ++i) {
            double g = load(dy, o + i, dt) * load(gamma, i, dt);
            double xh = (load(x, o + i, dt) - mu) / sigma;
            double v = g / sigma - (s1 + xh * s2) / (hidden * sigma);
            if (dres_in) v += load(dres_in, o + i, dt);
            dx[o + i] = v;
        }
    }
    /* column sums, rows in order (serial: a fixed summation order) */
    for (int64_t r = 0; r < rows; ++r) {
        const int64_t o = r * hidden;
        double s = 0.0;
        for (int i = 0; i < hidden; ++i) s += load(x, o + i, dt);
        double mu = s / hidden;
        double q = 0.0;
        for (int i = 0; i < hidden; ++i) { double d = load(x, o + i, dt) - mu; q += d * d; }
        double sigma = sqrt(q / hidden + eps);
        for (int i = 0; i < hidden; ++i) {
            double g = load(dy, o + i, dt);
            dgamma[i] += g * ((load(x, o + i, dt) - mu) / sigma);
            dbeta[i] += g;
        }
    }
}

/* The paper's rearranged gradient (Sec. IV-B, the equation with coefficients
 * alpha and beta): the two sums run over raw x, so neither waits for the mean.
 * Kept as a second, separately coded statement of dx; the tests require it to
 * agree with lsqo_layernorm_bwd.  (The text after the equation misprints the
 * second sum; the equation itself, sum_j w_j dy_j x_j, is what is coded.) */
void lsqo_layernorm_bwd_rearranged(double* dx, const void* dy, const void* x, const void* gamma,
                                   int64_t rows, int32_t hidden, double eps, int dt)
{
    for (int64_t r = 0; r < rows; ++r) {
        const int64_t o = r * hidden;
        const double m = hidden;
        double sx = 0.0, sxx = 0.0, a = 0.0, b = 0.0;
        for (int j = 0; j < hidden; ++j) {
            double xj = load(x, o + j, dt);
            double wg = load(gamma, j, dt) * load(dy, o + j, dt);
            sx += xj;
            sxx += xj * xj;
            a += wg;            /* sum_j w_j dy_j      */
            b += wg * xj;       /* sum_j w_j dy_j x_j  */
        }
        double mu = sx / m;
        double sigma = sqrt(sxx / m - mu * mu + eps);
        double s3 = sigma * sigma * sigma;
        for (int i = 0; i < hidden; ++i) {
            double xi = load(x, o + i, dt);
            double ca = ((xi - mu) * mu - sigma * sigma) / (m * s3);
            double cb = (mu - xi) / (m * s3);
            dx[o + i] = load(gamma, i, dt) * load(dy, o + i, dt) / sigma + ca * a + cb * b;
        }
    }
}

/* ------------------------------------------------- bias + dropout + residual */
/* Sec. IV-A: bias adding, dropout, residual, in that order.  e0 = flat index
 * of element [0,0] in the full tensor (non-zero when the caller passes a slice
 * of rows of a larger tensor). */
void lsqo_bias_dropout_residual_fwd(double* out, const void* x, const void* bias, const void* residual,
                                    int64_t rows, int32_t hidden, double p, uint64_t seed,
                                    uint64_t offset, uint64_t e0, int dt)
{
    const uint32_t t16 = threshold16(p);
    const double scale = 1.0 / (1.0 - p);
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int i = 0; i < hidden; ++i) {
            int64_t e = r * hidden + i;
            double z = load(x, e, dt) + (bias ? load(bias, i, dt) : 0.0);
            double d = keep_element(e0 + (uint64_t)e, p, t16, seed, offset) ? z * scale : 0.0;
            out[e] = load(residual, e, dt) + d;
        }
}

void lsqo_bias_dropout_residual_bwd(double* dx, double* dbias, const void* dy, int64_t rows,
                                    int32_t hidden, double p, uint64_t seed, uint64_t offset,
                                    uint64_t e0, int dt)
{
    const uint32_t t16 = threshold16(p);
    const double scale = 1.0 / (1.0 - p);
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int i = 0; i < hidden; ++i) {
            int64_t e = r * hidden + i;
            dx[e] = keep_element(e0 + (uint64_t)e, p, t16, seed, offset) ? load(dy, e, dt) * scale : 0.0;
        }
    if (dbias) {
        for (int i = 0; i < hidden; ++i) dbias[i] = 0.0;
        for (int64_t r = 0; r < rows; ++r)
            for (int i = 0; i < hidden; ++i) dbias[i] += dx[r * hidden + i];
    }
}

/* ------------------------------------------------- bias + activation + dropout */
/* The feed-forward half of Sec. IV-A's fused element-wise kernels: bias adding,
 * activation, dropout.  The paper names ReLU; BERT and GPT-2 (Sec. VI) use GELU,
 * in its erf form and its tanh approximation respectively.
 * act: 0 = ReLU, 1 = GELU (erf), 2 = GELU (tanh approximation). */
static double act_value(double z, int act)
{
    if (act == 0) return z > 0.0 ? z : 0.0;
    if (act == 1) return 0.5 * z * erfc(-z / sqrt(2.0));   /* = z*Phi(z); erfc keeps the negative tail exact */
    double u = sqrt(2.0 / PI) * (z + 0.044715 * z * z * z);
    return 0.5 * z * (1.0 + tanh(u));
}

static double act_slope(double z, int act)
{
    if (act == 0) return z > 0.0 ? 1.0 : 0.0;
    if (act == 1) return 0.5 * erfc(-z / sqrt(2.0)) + z * exp(-0.5 * z * z) / sqrt(2.0 * PI);
    double c = sqrt(2.0 / PI);
    double u = c * (z + 0.044715 * z * z * z);
    double t = tanh(u);
    return 0.5 * (1.0 + t) + 0.5 * z * (1.0 - t * t) * c * (1.0 + 3.0 * 0.044715 * z * z);
}

void lsqo_bias_act_dropout_fwd(double* out, const void* x, const void* bias, int64_t rows, int32_t hidden,
                               int32_t act, double p, uint64_t seed, uint64_t offset, uint64_t e0, int dt)
{
    const uint32_t t16 = threshold16(p);
    const double scale = 1.0 / (1.0 - p);
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int i = 0; i < hidden; ++i) {
            int64_t e = r * hidden + i;
            double z = load(x, e, dt) + (bias ? load(bias, i, dt) : 0.0);
            double a = act_value(z, act);
            out[e] = keep_element(e0 + (uint64_t)e, p, t16, seed, offset) ? a * scale : 0.0;
        }
}

/* dx = act'(x + bias) * keep * dy / (1-p);  dbias = column sums of dx. */
void lsqo_bias_act_dropout_bwd(double* dx, double* dbias, const void* dy, const void* x, const void* bias,
                               int64_t rows, int32_t hidden, int32_t act, double p, uint64_t seed,
                               uint64_t offset, uint64_t e0, int dt)
{
    const uint32_t t16 = threshold16(p);
    const double scale = 1.0 / (1.0 - p);
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int i = 0; i < hidden; ++i) {
            int64_t e = r * hidden + i;
            double z = load(x, e, dt) + (bias ? load(bias, i, dt) : 0.0);
            double g = keep_element(e0 + (uint64_t)e, p, t16, seed, offset) ? load(dy, e, dt) * scale : 0.0;
            dx[e] = g * act_slope(z, act);
        }
    if (dbias) {
        for (int i = 0; i < hidden; ++i) dbias[i] = 0.0;
        for (int64_t r = 0; r < rows; ++r)
            for (int i = 0; i < hidden; ++i) dbias[i] += dx[r * hidden + i];
    }
}

/* ------------------------------------------------------------------ softmax */
static int allowed(int j, int i, int klen_b, int causal, int q_len, int k_len)
{
    if (j >= klen_b) return 0;
    if (causal && j > i + (k_len - q_len)) return 0;
    return 1;
}

static int clamp_len(const int32_t* key_len, int b, int k_len)
{
    if (!key_len) return k_len;
    int v = key_len[b];
    if (v < 0) v = 0;
    if (v > k_len) v = k_len;
    return v;
}

/* Sec. IV-B Softmax, the three steps in order, over the allowed set only;
 * positions outside it are exactly 0.  y_drop may be NULL.  query_len (nullable):
 * query rows at or beyond query_len[b] are padding, their allowed set is empty. */
void lsqo_softmax_varlen_fwd(double* y, double* y_drop, const void* x, const int32_t* key_len,
                             const int32_t* query_len, int32_t batch, int32_t heads, int32_t q_len,
                             int32_t k_len, int32_t causal, double scale, double p, uint64_t seed,
                             uint64_t offset, uint64_t e0, int dt)
{
    const uint32_t t16 = threshold16(p);
    const double dscale = 1.0 / (1.0 - p);
    const int64_t nrows = (int64_t)batch * heads * q_len;
#pragma omp parallel for schedule(static)
    for (int64_t row = 0; row < nrows; ++row) {
        int b = (int)(row / ((int64_t)heads * q_len));
        int i = (int)(row % q_len);
        int kl = clamp_len(key_len, b, k_len);
        if (query_len && i >= query_len[b]) kl = 0;
        const int64_t o = row * k_len;
        /* step 1: the maximum */
        int any = 0;
        double mx = 0.0;
        for (int j = 0; j < k_len; ++j)
            if (allowed(j, i, kl, causal, q_len, k_len)) {
                double v = scale * load(x, o + j, dt);
                if (!any || v > mx) mx = v;
                any = 1;
            }
        /* step 2: the partition function */
        double Z = 0.0;
        for (int j = 0; j < k_len; ++j)
            if (allowed(j, i, kl, causal, q_len, k_len)) Z += exp(scale * load(x, o + j, dt) - mx);
        /* step 3: normalise */
        for (int j = 0; j < k_len; ++j) {
            double v = 0.0;
            if (allowed(j, i, kl, causal, q_len, k_len)) v = exp(scale * load(x, o + j, dt) - mx) / Z;
            y[o + j] = v;
            if (y_drop)
                y_drop[o + j] = keep_element(e0 + (uint64_t)(o + j), p, t16, seed, offset) ? v * dscale : 0.0;
        }
    }
}

void lsqo_softmax_fwd(double* y, double* y_drop, const void* x, const int32_t* key_len,
                      int32_t batch, int32_t heads, int32_t q_len, int32_t k_len, int32_t causal,
                      double scale, double p, uint64_t seed, uint64_t offset, uint64_t e0, int dt)
{
    lsqo_softmax_varlen_fwd(y, y_drop, x, key_len, NULL, batch, heads, q_len, k_len, causal, scale, p, seed,
                            offset, e0, dt);
}

/* Contraction of the softmax Jacobian (Sec. IV-A, criterion layer: dq_i/dh_j)
 * with the upstream gradient; y is the STORED forward output. */
void lsqo_softmax_varlen_bwd(double* dx, const void* dy, const void* y, const int32_t* key_len,
                             const int32_t* query_len, int32_t batch, int32_t heads, int32_t q_len,
                             int32_t k_len, int32_t causal, double scale, double p, uint64_t seed,
                             uint64_t offset, uint64_t e0, int dt)
{
    const uint32_t t16 = threshold16(p);
    const double dscale = 1.0 / (1.0 - p);
    const int64_t nrows = (int64_t)batch * heads * q_len;
#pragma omp parallel for schedule(static)
    for (int64_t row = 0; row < nrows; ++row) {
        int b = (int)(row / ((int64_t)heads * q_len));
        int i = (int)(row % q_len);
        int kl = clamp_len(key_len, b, k_len);
        if (query_len && i >= query_len[b]) kl = 0;
        const int64_t o = row * k_len;
        double dot = 0.0;
        for (int j = 0; j < k_len; ++j)
            if (allowed(j, i, kl, causal, q_len, k_len)) {
                double g = load(dy, o + j, dt);
                if (p != 0.0) g = keep_element(e0 + (uint64_t)(o + j), p, t16, seed, offset) ? g * dscale : 0.0;
                dot += g * load(y, o + j, dt);
            }
        for (int j = 0; j < k_len; ++j) {
            double v = 0.0;
            if (allowed(j, i, kl, causal, q_len, k_len)) {
                double g = load(dy, o + j, dt);
                if (p != 0.0) g = keep_element(e0 + (uint64_t)(o + j), p, t16, seed, offset) ? g * dscale : 0.0;
                v = scale * load(y, o + j, dt) * (g - dot);
            }
            dx[o + j] = v;
        }
    }
}

void lsqo_softmax_bwd(double* dx, const void* dy, const void* y, const int32_t* key_len,
                      int32_t batch, int32_t heads, int32_t q_len, int32_t k_len, int32_t causal,
                      double scale, double p, uint64_t seed, uint64_t offset, uint64_t e0, int dt)
{
    lsqo_softmax_varlen_bwd(dx, dy, y, key_len, NULL, batch, heads, q_len, k_len, causal, scale, p, seed,
                            offset, e0, dt);
}

/* ---------------------------------------------------------------- criterion */
static int ignored(int32_t k, int32_t vocab, int32_t ignore_index)
{
    return k == ignore_index || k < 0 || k >= vocab;
}

/* Sec. IV-A criterion layer, literally: q = softmax(h), p = (1-alpha) onehot + alpha/V,
 * loss = -sum_i p_i log q_i with log q_i = h_i - lse.  sums (nullable) =
 * { sum loss, sum nll, count of non-ignored tokens }. */
void lsqo_ls_xent_fwd(double* loss, double* nll, double* lse, double* sums, const void* logits,
                      const int32_t* target, int64_t tokens, int32_t vocab, double alpha,
                      int32_t ignore_index, int dt)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < tokens; ++t) {
        const int64_t o = t * vocab;
        int32_t k = target[t];
        /* a padded token contributes nothing and nothing of it is needed later: all three outputs are 0 */
        if (ignored(k, vocab, ignore_index)) { loss[t] = 0.0; nll[t] = 0.0; lse[t] = 0.0; continue; }
        double mx = load(logits, o, dt);
        for (int i = 1; i < vocab; ++i) { double h = load(logits, o + i, dt); if (h > mx) mx = h; }
        double z = 0.0;
        for (int i = 0; i < vocab; ++i) z += exp(load(logits, o + i, dt) - mx);
        double l = mx + log(z);
        lse[t] = l;
        double acc = 0.0;
        for (int i = 0; i < vocab; ++i) {
            double pi = alpha / vocab + (i == k ? 1.0 - alpha : 0.0);
            double logq = load(logits, o + i, dt) - l;
            acc -= pi * logq;
        }
        loss[t] = acc;
        nll[t] = -(load(logits, o + k, dt) - l);
    }
    if (sums) {
        double a = 0.0, b = 0.0, c = 0.0;
        for (int64_t t = 0; t < tokens; ++t)
            if (!ignored(target[t], vocab, ignore_index)) { a += loss[t]; b += nll[t]; c += 1.0; }
        sums[0] = a; sums[1] = b; sums[2] = c;
    }
}

/* Sec. IV-A, the final gradient to the decoder output, times the upstream
 * scalar grad_scale; lse recomputed here in double. */
void lsqo_ls_xent_bwd(double* dlogits, const void* logits, const int32_t* target, int64_t tokens,
                      int32_t vocab, double alpha, int32_t ignore_index, double grad_scale, int dt)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < tokens; ++t) {
        const int64_t o = t * vocab;
        int32_t k = target[t];
        if (ignored(k, vocab, ignore_index)) {
            for (int i = 0; i < vocab; ++i) dlogits[o + i] = 0.0;
            continue;
        }
        double mx = load(logits, o, dt);
        for (int i = 1; i < vocab; ++i) { double h = load(logits, o + i, dt); if (h > mx) mx = h; }
        double z = 0.0;
        for (int i = 0; i < vocab; ++i) z += exp(load(logits, o + i, dt) - mx);
        double l = mx + log(z);
        for (int i = 0; i < vocab; ++i) {
            double q = exp(load(logits, o + i, dt) - l);
            double gr = q - alpha / vocab;
            if (i == k) gr -= 1.0 - alpha;
            dlogits[o + i] = grad_scale * gr;
        }
    }
}

/* --------------------------------------------------------------------- Adam */
/* Sec. IV-C describes the data movement (one flat workspace, on-the-fly
 * conversion, one pass); the update itself is textbook Adam (Kingma & Ba),
 * eps outside the root after bias correction, optional L2 / decoupled decay. */
void lsqo_adam_step(double* p_out, double* m_out, double* v_out, const float* p, const float* m,
                    const float* v, const void* g, int64_t n, double lr, double beta1, double beta2,
                    double eps, double weight_decay, int32_t step, int32_t adamw,
                    int32_t bias_correction, double inv_grad_scale, int g_dt)
{
    double c1 = 1.0, c2 = 1.0;
    if (bias_correction) {
        c1 = 1.0 - pow(beta1, (double)step);
        c2 = 1.0 - pow(beta2, (double)step);
    }
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double pi = (double)p[i];
        double gh = load(g, i, g_dt) * inv_grad_scale;
        if (!adamw) gh += weight_decay * pi;
        double mi = beta1 * (double)m[i] + (1.0 - beta1) * gh;
        double vi = beta2 * (double)v[i] + (1.0 - beta2) * gh * gh;
        double upd = (mi / c1) / (sqrt(vi / c2) + eps);
        if (adamw) upd += weight_decay * pi;
        p_out[i] = pi - lr * upd;
        m_out[i] = mi;
        v_out[i] = vi;
    }
}

/* The paper's own trainer layout (Sec. IV-C, Fig. "Mixed-precision trainer"): the
 * workspace holds the parameter in LOW precision; it is widened, updated in
 * higher precision and narrowed again in place.  Same update rule as above; p
 * arrives in storage type `dt` (as does g). */
void lsqo_adam_step_lp(double* p_out, double* m_out, double* v_out, const void* p_lp, const float* m,
                       const float* v, const void* g, int64_t n, double lr, double beta1, double beta2,
                       double eps, double weight_decay, int32_t step, int32_t adamw, int32_t bias_correction,
                       double inv_grad_scale, int dt)
{
    double c1 = 1.0, c2 = 1.0;
    if (bias_correction) {
        c1 = 1.0 - pow(beta1, (double)step);
        c2 = 1.0 - pow(beta2, (double)step);
    }
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double pi = load(p_lp, i, dt);
        double gh = load(g, i, dt) * inv_grad_scale;
        if (!adamw) gh += weight_decay * pi;
        double mi = beta1 * (double)m[i] + (1.0 - beta1) * gh;
        double vi = beta2 * (double)v[i] + (1.0 - beta2) * gh * gh;
        double upd = (mi / c1) / (sqrt(vi / c2) + eps);
        if (adamw) upd += weight_decay * pi;
        p_out[i] = pi - lr * upd;
        m_out[i] = mi;
        v_out[i] = vi;
    }
}

/* SGD trainer over the same flat workspace (Sec. VI-C names an SGD trainer next to
 * Adam; the rule is the textbook one): g' = g*inv_grad_scale + wd*p;
 * buf = momentum*buf + g' (momentum > 0; buf starts at 0); step direction
 * d = g' + momentum*buf if nesterov, buf if momentum > 0, else g';  p -= lr*d. */
void lsqo_sgd_step(double* p_out, double* buf_out, const float* p, const float* buf, const void* g,
                   int64_t n, double lr, double momentum, double weight_decay, int32_t nesterov,
                   double inv_grad_scale, int g_dt)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double pi = (double)p[i];
        double gh = load(g, i, g_dt) * inv_grad_scale + weight_decay * pi;
        double d = gh;
        if (momentum != 0.0) {
            double b = momentum * (double)buf[i] + gh;
            buf_out[i] = b;
            d = nesterov ? gh + momentum * b : b;
        }
        p_out[i] = pi - lr * d;
    }
}

/* --------------------------------------------------------- head split / merge */
/* The "Reshape" of Sec. IV-A's element-wise list: the projection output [batch*len,
 * parts*hidden] (columns ordered part, head, head_dim) plus its bias is laid out as
 * `parts` tensors [batch, heads, len, head_dim] for the batched attention GEMMs, and
 * the attention output is laid back.  Pure index permutations (+ the bias). */
void lsqo_split_heads_fwd(double* out0, double* out1, double* out2, const void* in, const void* bias,
                          int32_t batch, int32_t len, int32_t heads, int32_t head_dim, int32_t parts, int dt)
{
    double* outs[3] = { out0, out1, out2 };
    const int64_t hidden = (int64_t)heads * head_dim;
    for (int b = 0; b < batch; ++b)
        for (int l = 0; l < len; ++l)
            for (int part = 0; part < parts; ++part)
                for (int n = 0; n < heads; ++n)
                    for (int d = 0; d < head_dim; ++d) {
                        int64_t col = part * hidden + (int64_t)n * head_dim + d;
                        int64_t src = ((int64_t)b * len + l) * parts * hidden + col;
                        int64_t dst = (((int64_t)b * heads + n) * len + l) * head_dim + d;
                        outs[part][dst] = load(in, src, dt) + (bias ? load(bias, col, dt) : 0.0);
                    }
}

/* The inverse layout change, with the bias gradient (column sums) as a by-product. */
void lsqo_split_heads_bwd(double* din, double* dbias, const void* d0, const void* d1, const void* d2,
                          int32_t batch, int32_t len, int32_t heads, int32_t head_dim, int32_t parts, int dt)
{
    const void* ds[3] = { d0, d1, d2 };
    const int64_t hidden = (int64_t)heads * head_dim;
    if (dbias) for (int64_t c = 0; c < parts * hidden; ++c) dbias[c] = 0.0;
    for (int b = 0; b < batch; ++b)
        for (int l = 0; l < len; ++l)
            for (int part = 0; part < parts; ++part)
                for (int n = 0; n < heads; ++n)
                    for (int d = 0; d < head_dim; ++d) {
                        int64_t col = part * hidden + (int64_t)n * head_dim + d;
                        int64_t dst = ((int64_t)b * len + l) * parts * hidden + col;
                        int64_t src = (((int64_t)b * heads + n) * len + l) * head_dim + d;
                        double g = load(ds[part], src, dt);
                        din[dst] = g;
                        if (dbias) dbias[col] += g;
                    }
}

/* ------------------------------------------------------------------ embedding */
/* Sec. IV-A, embedding layer: y^(w,p) = Dropout(s * E_w + P_p) for the token w at
 * position p of its sentence.  tokens: [batch, len]; a token equal to pad_idx or
 * outside [0, vocab) produces a zero row (and receives no gradient). */
static int is_pad(int32_t w, int32_t vocab, int32_t pad_idx) { return w == pad_idx || w < 0 || w >= vocab; }

void lsqo_embedding_fwd(double* out, const int32_t* tokens, const void* emb, const void* pos, int32_t batch,
                        int32_t len, int32_t hidden, int32_t vocab, int32_t pad_idx, double scale, double p,
                        uint64_t seed, uint64_t offset, uint64_t e0, int dt)
{
    const uint32_t t16 = threshold16(p);
    const double dscale = 1.0 / (1.0 - p);
    const int64_t T = (int64_t)batch * len;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        const int32_t w = tokens[t];
        const int l = (int)(t % len);
        for (int i = 0; i < hidden; ++i) {
            const int64_t e = t * hidden + i;
            double v = 0.0;
            if (!is_pad(w, vocab, pad_idx)) {
                v = scale * load(emb, (int64_t)w * hidden + i, dt) + load(pos, (int64_t)l * hidden + i, dt);
                v = keep_element(e0 + (uint64_t)e, p, t16, seed, offset) ? v * dscale : 0.0;
            }
            out[e] = v;
        }
    }
}

/* Sec. IV-A: grad E_w = s * sum over the positions that hold token w of m (.) grad y, summed here in
 * ascending position order; grad P_l = the same sum over the batch for position l.  demb [vocab, hidden]
 * and dpos [len, hidden] receive the INCREMENTS (they are zeroed first); dpos may be NULL. */
void lsqo_embedding_bwd(double* demb, double* dpos, const void* dy, const int32_t* tokens, int32_t batch,
                        int32_t len, int32_t hidden, int32_t vocab, int32_t pad_idx, double scale, double p,
                        uint64_t seed, uint64_t offset, uint64_t e0, int dt)
{
    const uint32_t t16 = threshold16(p);
    const double dscale = 1.0 / (1.0 - p);
    const int64_t T = (int64_t)batch * len;
    for (int64_t i = 0; i < (int64_t)vocab * hidden; ++i) demb[i] = 0.0;
    if (dpos) for (int64_t i = 0; i < (int64_t)len * hidden; ++i) dpos[i] = 0.0;
    for (int64_t t = 0; t < T; ++t) {
        const int32_t w = tokens[t];
        if (is_pad(w, vocab, pad_idx)) continue;
        const int l = (int)(t % len);
        for (int i = 0; i < hidden; ++i) {
            const int64_t e = t * hidden + i;
            double g = keep_element(e0 + (uint64_t)e, p, t16, seed, offset) ? load(dy, e, dt) * dscale : 0.0;
            demb[(int64_t)w * hidden + i] += scale * g;
            if (dpos) dpos[(int64_t)l * hidden + i] += g;
        }
    }
}

/* ---------------------------------------------------------- padding removal */
/* Padding removal (the paper's conclusion names it as the next optimisation): the
 * len_b = clamp(key_len[b], 0, max_len) real rows of every sentence are stored
 * back to back.  offsets[b] = first packed row of sentence b, offsets[batch] = total. */
void lsqo_pad_offsets(int32_t* offsets, const int32_t* key_len, int32_t batch, int32_t max_len)
{
    int32_t run = 0;
    for (int b = 0; b < batch; ++b) {
        offsets[b] = run;
        run += clamp_len(key_len, b, max_len);
    }
    offsets[batch] = run;
}

/* packed[offsets[b] + i, :] = padded[b, i, :] for i < len_b */
void lsqo_pad_remove(double* packed, const void* padded, const int32_t* key_len, int32_t batch,
                     int32_t max_len, int32_t hidden, int dt)
{
    int64_t r = 0;
    for (int b = 0; b < batch; ++b)
        for (int i = 0; i < clamp_len(key_len, b, max_len); ++i, ++r)
            for (int c = 0; c < hidden; ++c)
                packed[r * hidden + c] = load(padded, ((int64_t)b * max_len + i) * hidden + c, dt);
}

/* padded[b, i, :] = packed[offsets[b] + i, :] for i < len_b, 0 on the padding */
void lsqo_pad_restore(double* padded, const void* packed, const int32_t* key_len, int32_t batch,
                      int32_t max_len, int32_t hidden, int dt)
{
    int64_t r = 0;
    for (int b = 0; b < batch; ++b) {
        const int lb = clamp_len(key_len, b, max_len);
        for (int i = 0; i < max_len; ++i) {
            for (int c = 0; c < hidden; ++c)
                padded[((int64_t)b * max_len + i) * hidden + c] = i < lb ? load(packed, r * hidden + c, dt) : 0.0;
            if (i < lb) ++r;
        }
    }
}
