// Fused bias + activation + dropout of the feed-forward block, forward and backward
// (Sec. IV-A of the paper: adjacent element-wise kernels — bias adding, activation,
// dropout — fused into one launch).  The paper names ReLU; the BERT and GPT-2
// models of its Sec. VI use GELU (erf form and tanh approximation).
//
// A wave owns 64 consecutive packs of one row and walks down the rows with the bias
// pack in registers, the next row's packs loaded before this row's are used; the
// dropout mask is rebuilt from the Philox counter of the pack in both directions;
// backward recomputes the activation slope from the saved pre-activation input
// and accumulates dbias per lane (no atomics; partial rows + ordered second stage).
// HBM traffic: forward 2 tensors, backward 3.  Rows of up to 32 packs, and rows that are not whole
// packs, take the flat walk of host.hpp instead.
#include "host.hpp"

namespace lsq {

constexpr bool kNT = true;

constexpr int kBadWaves = 4;
enum { ACT_RELU = 0, ACT_GELU = 1, ACT_GELU_TANH = 2 };

// sigmoid(2u) for the tanh form of GELU, 2u = 2 sqrt(2/pi) (z + 0.044715 z^3), with the constants of the
// argument and of the base-2 exponential folded into one cubic: z * (c1 + c3 z^2) = -2u log2(e)
// (the kernels that call this are bound by vector-ALU issue slots: every instruction counts).  One v_exp_f32 and
// one v_rcp_f32 (1 ulp; an IEEE division costs ten instructions).
__device__ __forceinline__ float sigmoid_2u(float z, float z2)
{
    constexpr float c1 = -1.5957691216057308f * 1.4426950408889634f;
    constexpr float c3 = c1 * 0.044715f;
    return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(z * fmaf(c3, z2, c1)));
}

// Standard normal CDF Phi(z).  erfc(u / sqrt 2) = 2 Phi(-u), u >= 0, is evaluated as
// 2^q(u) with q a degree-10 least-squares fit of log2 erfc(u / sqrt 2) on Chebyshev nodes
// of [0, 6.5] (relative error 5e-7 in exact arithmetic, 5e-6 in fp32 Horner form; beyond
// 6.5 the tail is held at 8e-11).  The lower tail comes out with that RELATIVE accuracy
// (no 1 + erf cancellation), the upper one as 1 - tail.  Branch-free, one v_exp_f32:
// about half the instructions of a library erff, which made the GELU kernels ALU-bound.
__device__ __forceinline__ float normal_cdf(float z)
{
    const float u = fminf(fabsf(z), 6.5f);
    float q = -7.934565005e-09f;
    q = fmaf(q, u, 2.847633596e-07f);
    q = fmaf(q, u, -4.305318271e-06f);
    q = fmaf(q, u, 3.393354200e-05f);
    q = fmaf(q, u, -1.167951486e-04f);
    q = fmaf(q, u, -3.832164512e-04f);
    q = fmaf(q, u, 7.491793949e-03f);
    q = fmaf(q, u, -5.288341269e-02f);
    q = fmaf(q, u, -4.590395689e-01f);
    q = fmaf(q, u, -1.151132941e+00f);
    q = fmaf(q, u, 7.463755196e-07f - 1.0f);                    // the factor 1/2 of Phi(-u) = erfc(u / sqrt 2) / 2
    const float tail = __builtin_amdgcn_exp2f(q);               // Phi(-|z|)
    return z < 0.0f ? tail : 1.0f - tail;
}

template <int ACT> __device__ __forceinline__ float act_value(float z)
{
    if constexpr (ACT == ACT_RELU) return fmaxf(z, 0.0f);
    else if constexpr (ACT == ACT_GELU) return z * normal_cdf(z);
    else {
        // 0.5*(1 + tanh(u)) == sigmoid(2u): no cancellation in the negative tail, no tanh call
        return z * sigmoid_2u(z, z * z);
    }
}

template <int ACT> __device__ __forceinline__ float act_slope(float z)
{
    if constexpr (ACT == ACT_RELU) return z > 0.0f ? 1.0f : 0.0f;
    else if constexpr (ACT == ACT_GELU)
        // Phi(z) + z * phi(z), phi = exp(-z^2/2) / sqrt(2 pi) through one v_exp_f32
        return fmaf(z * 0.3989422804014327f, __builtin_amdgcn_exp2f(-0.72134752044448170f * z * z), normal_cdf(z));
    else {
        // d/dz [z*sigmoid(2u)] = s + z*s*(1-s)*d(2u)/dz
        const float z2 = z * z;
        const float s = sigmoid_2u(z, z2);
        const float du2 = fmaf(3.0f * 0.044715f * 1.5957691216057308f, z2, 1.5957691216057308f);
        return fmaf(z * du2, fmaf(-s, s, s), s);
    }
}

template <typename T, int ACT, bool HAS_BIAS, bool DROP>
__global__ __launch_bounds__(256) void bad_fwd_cols(T* out, const T* x, const T* __restrict__ bias, int64_t rows,
                                                    int ppr, DropoutParams d)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int cp = blockIdx.x * 64 + lane;
    if (cp >= ppr) return;
    float b[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if constexpr (HAS_BIAS) load8<T>(bias + static_cast<int64_t>(cp) * kPack, b);
    const int64_t stride = static_cast<int64_t>(gridDim.y) * kBadWaves;
    // the pack of the next row is loaded before this row's is used
    int64_t r = static_cast<int64_t>(blockIdx.y) * kBadWaves + wave;
    RawPack<T> nx = r < rows ? load_raw<T, kNT>(x + (r * ppr + cp) * kPack) : zero_raw<T>();
    for (; r < rows; r += stride) {
        const RawPack<T> cx = nx;
        if (r + stride < rows) nx = load_raw<T, kNT>(x + ((r + stride) * ppr + cp) * kPack);
        const int64_t pack = r * ppr + cp;
        float xf[8], k[8];
        if constexpr (DROP) dropout_factors8(d, static_cast<uint64_t>(pack), k);
        unpack<T>(cx, xf);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float a = act_value<ACT>(xf[j] + b[j]);
            xf[j] = DROP ? a * k[j] : a;
        }
        store8<T, kNT>(out + pack * kPack, xf);
    }
}

template <typename T, int ACT, bool HAS_BIAS, bool DROP>
__global__ __launch_bounds__(256) void bad_bwd_cols(T* dx, float* __restrict__ partial, const T* dy, const T* x,
                                                    const T* __restrict__ bias, int64_t rows, int ppr, DropoutParams d)
{
    __shared__ float sm[kBadWaves][8][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int cp = blockIdx.x * 64 + lane;
    const bool active = cp < ppr;
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    const int64_t stride = static_cast<int64_t>(gridDim.y) * kBadWaves;
    if (active) {
        float b[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        if constexpr (HAS_BIAS) load8<T>(bias + static_cast<int64_t>(cp) * kPack, b);
        // the packs of the next row are loaded before this row's are used, and the dropout factors, which need
        // no data, are drawn while the loads are in flight
        int64_t r = static_cast<int64_t>(blockIdx.y) * kBadWaves + wave;
        RawPack<T> ng = zero_raw<T>(), nx = zero_raw<T>();
        if (r < rows) {
            ng = load_raw<T, kNT>(dy + (r * ppr + cp) * kPack);
            nx = load_raw<T, kNT>(x + (r * ppr + cp) * kPack);
        }
        for (; r < rows; r += stride) {
            const RawPack<T> cg = ng, cx = nx;
            const int64_t rn = r + stride;
            if (rn < rows) {
                ng = load_raw<T, kNT>(dy + (rn * ppr + cp) * kPack);
                nx = load_raw<T, kNT>(x + (rn * ppr + cp) * kPack);
            }
            const int64_t pack = r * ppr + cp;
            float g[8], xf[8], k[8];
            if constexpr (DROP) dropout_factors8(d, static_cast<uint64_t>(pack), k);
            unpack<T>(cg, g);
            unpack<T>(cx, xf);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float s = act_slope<ACT>(xf[j] + b[j]);
                g[j] = DROP ? g[j] * k[j] * s : g[j] * s;
                acc[j] += g[j];
            }
            store8<T, kNT>(dx + pack * kPack, g);
        }
    }
    if (partial == nullptr) return;        // uniform over the grid
#pragma unroll
    for (int j = 0; j < 8; ++j) sm[wave][j][lane] = acc[j];
    __syncthreads();
    if (wave == 0 && active) {
        float* dst = partial + static_cast<int64_t>(blockIdx.y) * ppr * kPack + static_cast<int64_t>(cp) * kPack;
        float s[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            float t = sm[0][j][lane];
#pragma unroll
            for (int w = 1; w < kBadWaves; ++w) t += sm[w][j][lane];
            s[j] = t;
        }
        store8<float>(dst, s);
    }
}

// ---- any hidden (rows are not a whole number of packs): the operators for flat_packs_kernel
template <typename T, int ACT>
struct BadFwdFlat {
    T* out;
    const T* x;
    const T* bias;
    int hidden;
    DropoutParams d;
    __device__ __forceinline__ void pack(int64_t e0, int c0, float (&g)[8]) const
    {
        const RawPack<T> xr = load_raw<T, kNT>(x + e0);
        float k[8];
        if (d.on) dropout_factors8(d, static_cast<uint64_t>(e0 >> 3), k);
        unpack<T>(xr, g);
        int c = c0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float z = bias ? g[j] + to_f32<T>(bias[c]) : g[j];
            const float a = act_value<ACT>(z);
            g[j] = d.on ? a * k[j] : a;
            c = c + 1 == hidden ? 0 : c + 1;
        }
        store8<T, kNT>(out + e0, g);
    }
    __device__ __forceinline__ float one(int64_t e, int c) const
    {
        float z = to_f32<T>(x[e]);
        if (bias) z += to_f32<T>(bias[c]);
        float a = act_value<ACT>(z);
        if (d.on) a *= dropout_factor1(d, static_cast<uint64_t>(e));
        out[e] = from_f32<T>(a);
        return a;
    }
};

template <typename T, int ACT>
struct BadBwdFlat {
    T* dx;
    const T* dy;
    const T* x;
    const T* bias;
    int hidden;
    DropoutParams d;
    __device__ __forceinline__ void pack(int64_t e0, int c0, float (&g)[8]) const
    {
        const RawPack<T> gr = load_raw<T, kNT>(dy + e0), xr = load_raw<T, kNT>(x + e0);
        float k[8];
        if (d.on) dropout_factors8(d, static_cast<uint64_t>(e0 >> 3), k);
        float xf[8];
        unpack<T>(gr, g);
        unpack<T>(xr, xf);
        int c = c0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float z = bias ? xf[j] + to_f32<T>(bias[c]) : xf[j];
            const float v = g[j] * act_slope<ACT>(z);
            g[j] = d.on ? v * k[j] : v;
            c = c + 1 == hidden ? 0 : c + 1;
        }
        store8<T, kNT>(dx + e0, g);
    }
    __device__ __forceinline__ float one(int64_t e, int c) const
    {
        float z = to_f32<T>(x[e]);
        if (bias) z += to_f32<T>(bias[c]);
        float v = to_f32<T>(dy[e]) * act_slope<ACT>(z);
        if (d.on) v *= dropout_factor1(d, static_cast<uint64_t>(e));
        dx[e] = from_f32<T>(v);
        return v;
    }
};

template <typename T, int ACT>
static lsq_status bad_fwd_dispatch(void* out, const void* x, const void* bias, int64_t rows, int32_t hidden,
                                   const DropoutParams& d, hipStream_t s)
{
    T* o = static_cast<T*>(out);
    const T* xp = static_cast<const T*>(x);
    const T* bp = static_cast<const T*>(bias);
    if (!bad_is_flat(hidden)) {
        const int ppr = hidden / kPack;
        // two rows per wave: 28.1 / 23.1 us at 8192 x 5120 / 4096 x 4096 against 29.0 / 23.8 with four and 28.1 / 24.3 with one
        int64_t rb = ceil_div(rows, 2 * kBadWaves);
        if (rb > 8192) rb = 8192;
        const dim3 grid(static_cast<unsigned>(ceil_div(ppr, 64)), static_cast<unsigned>(rb)), block(256);
        const bool drop = d.on != 0;
        if (bp && drop) hipLaunchKernelGGL((bad_fwd_cols<T, ACT, true, true>), grid, block, 0, s, o, xp, bp, rows, ppr, d);
        else if (bp) hipLaunchKernelGGL((bad_fwd_cols<T, ACT, true, false>), grid, block, 0, s, o, xp, bp, rows, ppr, d);
        else if (drop) hipLaunchKernelGGL((bad_fwd_cols<T, ACT, false, true>), grid, block, 0, s, o, xp, bp, rows, ppr, d);
        else hipLaunchKernelGGL((bad_fwd_cols<T, ACT, false, false>), grid, block, 0, s, o, xp, bp, rows, ppr, d);
    } else {
        launch_flat_packs(BadFwdFlat<T, ACT>{o, xp, bp, hidden, d}, nullptr, nullptr, rows, hidden, s);
    }
    return launch_status();
}

template <typename T, int ACT>
static lsq_status bad_bwd_dispatch(void* dx, float* dbias, const void* dy, const void* x, const void* bias, int64_t rows,
                                   int32_t hidden, const DropoutParams& d, void* workspace, hipStream_t s)
{
    T* o = static_cast<T*>(dx);
    const T* g = static_cast<const T*>(dy);
    const T* xp = static_cast<const T*>(x);
    const T* bp = static_cast<const T*>(bias);
    if (!bad_is_flat(hidden)) {
        const int ppr = hidden / kPack;
        const int rb = bad_bwd_row_blocks(rows, hidden);
        const dim3 grid(static_cast<unsigned>(ceil_div(ppr, 64)), static_cast<unsigned>(rb)), block(256);
        float* partial = dbias ? static_cast<float*>(workspace) : nullptr;
        const bool drop = d.on != 0;
        if (bp && drop) hipLaunchKernelGGL((bad_bwd_cols<T, ACT, true, true>), grid, block, 0, s, o, partial, g, xp, bp, rows, ppr, d);
        else if (bp) hipLaunchKernelGGL((bad_bwd_cols<T, ACT, true, false>), grid, block, 0, s, o, partial, g, xp, bp, rows, ppr, d);
        else if (drop) hipLaunchKernelGGL((bad_bwd_cols<T, ACT, false, true>), grid, block, 0, s, o, partial, g, xp, bp, rows, ppr, d);
        else hipLaunchKernelGGL((bad_bwd_cols<T, ACT, false, false>), grid, block, 0, s, o, partial, g, xp, bp, rows, ppr, d);
        if (dbias) launch_colsum_finalize(dbias, dbias, hidden, partial, rb, hidden, s);
    } else {
        launch_flat_packs(BadBwdFlat<T, ACT>{o, g, xp, bp, hidden, d}, dbias, workspace, rows, hidden, s);
    }
    return launch_status();
}

template <typename T>
static lsq_status bad_fwd_act(int act, void* out, const void* x, const void* bias, int64_t rows, int32_t hidden,
                              const DropoutParams& d, hipStream_t s)
{
    switch (act) {
        case ACT_RELU: return bad_fwd_dispatch<T, ACT_RELU>(out, x, bias, rows, hidden, d, s);
        case ACT_GELU: return bad_fwd_dispatch<T, ACT_GELU>(out, x, bias, rows, hidden, d, s);
        default: return bad_fwd_dispatch<T, ACT_GELU_TANH>(out, x, bias, rows, hidden, d, s);
    }
}

template <typename T>
static lsq_status bad_bwd_act(int act, void* dx, float* dbias, const void* dy, const void* x, const void* bias,
                              int64_t rows, int32_t hidden, const DropoutParams& d, void* ws, hipStream_t s)
{
    switch (act) {
        case ACT_RELU: return bad_bwd_dispatch<T, ACT_RELU>(dx, dbias, dy, x, bias, rows, hidden, d, ws, s);
        case ACT_GELU: return bad_bwd_dispatch<T, ACT_GELU>(dx, dbias, dy, x, bias, rows, hidden, d, ws, s);
        default: return bad_bwd_dispatch<T, ACT_GELU_TANH>(dx, dbias, dy, x, bias, rows, hidden, d, ws, s);
    }
}

}  // namespace lsq

extern "C" lsq_status lsq_bias_act_dropout_fwd(void* out, const void* x, const void* bias, int64_t rows, int32_t hidden,
                                               int32_t act, float p, uint64_t seed, uint64_t offset, lsq_dtype dt,
                                               void* stream)
{
    using namespace lsq;
    LSQ_REQUIRE(rows >= 0 && hidden > 0);
    LSQ_REQUIRE(act == LSQ_ACT_RELU || act == LSQ_ACT_GELU || act == LSQ_ACT_GELU_TANH);
    if (!valid_dtype(dt)) return LSQ_UNSUPPORTED_DTYPE;
    DropoutParams d;
    LSQ_REQUIRE(make_dropout(p, seed, offset, &d));
    if (rows == 0) return LSQ_OK;
    LSQ_REQUIRE(out && x);
    LSQ_ALIGNED(out); LSQ_ALIGNED(x); LSQ_ALIGNED(bias);
    LSQ_REQUIRE(ceil_div(rows * hidden, 256) <= 0x7FFFFFFF);
    hipStream_t s = static_cast<hipStream_t>(stream);
    switch (dt) {
        case LSQ_F16: return bad_fwd_act<f16>(act, out, x, bias, rows, hidden, d, s);
        case LSQ_BF16: return bad_fwd_act<bf16>(act, out, x, bias, rows, hidden, d, s);
        default: return bad_fwd_act<float>(act, out, x, bias, rows, hidden, d, s);
    }
}

extern "C" lsq_status lsq_bias_act_dropout_bwd(void* dx, float* dbias, const void* dy, const void* x, const void* bias,
                                               int64_t rows, int32_t hidden, int32_t act, float p, uint64_t seed,
                                               uint64_t offset, void* workspace, size_t workspace_bytes, lsq_dtype dt,
                                               void* stream)
{
    using namespace lsq;
    LSQ_REQUIRE(rows >= 0 && hidden > 0);
    LSQ_REQUIRE(act == LSQ_ACT_RELU || act == LSQ_ACT_GELU || act == LSQ_ACT_GELU_TANH);
    if (!valid_dtype(dt)) return LSQ_UNSUPPORTED_DTYPE;
    DropoutParams d;
    LSQ_REQUIRE(make_dropout(p, seed, offset, &d));
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (rows == 0) return dbias ? zero_fill(dbias, hidden, s) : LSQ_OK;
    LSQ_REQUIRE(dx && dy && x);
    LSQ_ALIGNED(dx); LSQ_ALIGNED(dy); LSQ_ALIGNED(x); LSQ_ALIGNED(bias); LSQ_ALIGNED(dbias); LSQ_ALIGNED(workspace);
    LSQ_REQUIRE(ceil_div(rows * hidden, 256) <= 0x7FFFFFFF);
    if (dbias) {
        const size_t need = lsq_workspace_bytes(LSQ_OP_BIAS_ACT_DROPOUT_BWD, rows, hidden);
        if (need && (!workspace || workspace_bytes < need)) return LSQ_WORKSPACE_TOO_SMALL;
    }
    switch (dt) {
        case LSQ_F16: return bad_bwd_act<f16>(act, dx, dbias, dy, x, bias, rows, hidden, d, workspace, s);
        case LSQ_BF16: return bad_bwd_act<bf16>(act, dx, dbias, dy, x, bias, rows, hidden, d, workspace, s);
        default: return bad_bwd_act<float>(act, dx, dbias, dy, x, bias, rows, hidden, d, workspace, s);
    }
}
