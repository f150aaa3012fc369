// Fused bias + dropout + residual, forward and backward (Sec. IV-A of the paper,
// Transformer layers: "bias adding, dropout, and residual" in one launch).
//
// Layout of the fast path (hidden % 8 == 0): a wave owns 64 consecutive packs of
// one row (512 columns, 1 KiB of fp16) and walks down the rows, so the bias pack
// is loaded once into registers, every access is a 128-bit one, and in backward
// each lane accumulates the column sums of its own 8 columns with no atomics.
// The dropout mask is never stored: both directions rebuild it from the Philox
// counter of the pack.  HBM traffic: forward 3 tensors, backward 2.
#include "host.hpp"

namespace lsq {

#ifndef LSQ_NT
#define LSQ_NT 1
#endif
constexpr bool kNT = LSQ_NT != 0;   // nontemporal hint on the streamed tensors (not on gamma/beta/bias)

constexpr int kBdrWaves = 4;   // waves per workgroup; each takes its own rows
#ifndef LSQ_BDR_UNROLL
#define LSQ_BDR_UNROLL 4
#endif
constexpr int kBdrUnroll = LSQ_BDR_UNROLL;   // rows a wave has in flight in backward

template <typename T, bool HAS_BIAS, bool DROP>
__global__ __launch_bounds__(256) void bdr_fwd_cols(T* out, const T* x,
                                                    const T* __restrict__ bias, const T* res,
                                                    int64_t rows, int ppr, DropoutParams d)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int cp = blockIdx.x * 64 + lane;
    if (cp >= ppr) return;
    float b[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if constexpr (HAS_BIAS) load8<T>(bias + static_cast<int64_t>(cp) * kPack, b);
    const int64_t stride = static_cast<int64_t>(gridDim.y) * kBdrWaves;
    for (int64_t r = static_cast<int64_t>(blockIdx.y) * kBdrWaves + wave; r < rows; r += stride) {
        const int64_t pack = r * ppr + cp;
        float xf[8], rf[8], k[8];
        load8<T, kNT>(x + pack * kPack, xf);
        load8<T, kNT>(res + pack * kPack, rf);
        if constexpr (DROP) dropout_factors8(d, static_cast<uint64_t>(pack), k);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float z = xf[j] + b[j];
            rf[j] = DROP ? fmaf(z, k[j], rf[j]) : rf[j] + z;
        }
        store8<T, kNT>(out + pack * kPack, rf);
    }
}

// Backward.  partial: [gridDim.y][hidden] fp32 column sums of this workgroup's rows
// (nullptr: dbias not wanted).
template <typename T, bool DROP>
__global__ __launch_bounds__(256) void bdr_bwd_cols(T* dx, float* __restrict__ partial,
                                                    const T* dy, int64_t rows, int ppr,
                                                    DropoutParams d)
{
    __shared__ float sm[kBdrWaves][8][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int cp = blockIdx.x * 64 + lane;
    const bool active = cp < ppr;
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    const int64_t stride = static_cast<int64_t>(gridDim.y) * kBdrWaves;
    if (active) {
        // kBdrUnroll rows per trip: their loads are issued before the first Philox call
        for (int64_t r0 = static_cast<int64_t>(blockIdx.y) * kBdrWaves + wave; r0 < rows; r0 += stride * kBdrUnroll) {
            RawPack<T> raw[kBdrUnroll];
#pragma unroll
            for (int u = 0; u < kBdrUnroll; ++u) {
                const int64_t r = r0 + u * stride;
                if (r < rows) raw[u] = load_raw<T, kNT>(dy + (r * ppr + cp) * kPack);
                else raw[u] = zero_raw<T>();
            }
#pragma unroll
            for (int u = 0; u < kBdrUnroll; ++u) {
                const int64_t r = r0 + u * stride;
                if (r < rows) {
                    const int64_t pack = r * ppr + cp;
                    float g[8], k[8];
                    unpack<T>(raw[u], g);
                    if constexpr (DROP) {
                        dropout_factors8(d, static_cast<uint64_t>(pack), k);
#pragma unroll
                        for (int j = 0; j < 8; ++j) g[j] *= k[j];
                    }
                    store8<T, kNT>(dx + pack * kPack, g);
#pragma unroll
                    for (int j = 0; j < 8; ++j) acc[j] += g[j];
                }
            }
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
            for (int w = 1; w < kBdrWaves; ++w) t += sm[w][j][lane];
            s[j] = t;
        }
        store8<float>(dst, s);
    }
}

// ---- generic paths: any hidden (rows are not 16-byte aligned), one element per thread
template <typename T>
__global__ __launch_bounds__(256) void bdr_fwd_flat(T* out, const T* x,
                                                    const T* __restrict__ bias, const T* res,
                                                    int64_t total, int hidden, DropoutParams d)
{
    const int64_t e = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (e >= total) return;
    float z = to_f32<T>(x[e]);
    if (bias) z += to_f32<T>(bias[e % hidden]);
    const float k = d.t16 ? dropout_factor1(d, static_cast<uint64_t>(e)) : 1.0f;
    out[e] = from_f32<T>(d.t16 ? fmaf(z, k, to_f32<T>(res[e])) : to_f32<T>(res[e]) + z);
}

template <typename T>
__global__ __launch_bounds__(256) void bdr_bwd_flat(T* dx, const T* dy,
                                                    int64_t total, DropoutParams d)
{
    const int64_t e = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (e >= total) return;
    float g = to_f32<T>(dy[e]);
    if (d.t16) g *= dropout_factor1(d, static_cast<uint64_t>(e));
    dx[e] = from_f32<T>(g);
}

// one thread per column walks down the rows (coalesced across the wave)
template <typename T>
__global__ __launch_bounds__(256) void bdr_dbias_flat(float* __restrict__ dbias, const T* __restrict__ dy,
                                                      int64_t rows, int hidden, DropoutParams d)
{
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= hidden) return;
    float s = 0.0f;
    for (int64_t r = 0; r < rows; ++r) {
        const int64_t e = r * hidden + c;
        float g = to_f32<T>(dy[e]);
        if (d.t16) g *= dropout_factor1(d, static_cast<uint64_t>(e));
        s += g;
    }
    dbias[c] = s;
}

inline dim3 bdr_grid(int64_t rows, int ppr, int row_blocks)
{
    return dim3(static_cast<unsigned>(ceil_div(ppr, 64)), static_cast<unsigned>(row_blocks));
}

template <typename T>
static lsq_status bdr_fwd_dispatch(void* out, const void* x, const void* bias, const void* res, int64_t rows,
                                   int32_t hidden, const DropoutParams& d, hipStream_t s)
{
    T* o = static_cast<T*>(out);
    const T* xp = static_cast<const T*>(x);
    const T* bp = static_cast<const T*>(bias);
    const T* rp = static_cast<const T*>(res);
    if (hidden % kPack == 0) {
        const int ppr = hidden / kPack;
        int64_t rb = ceil_div(rows, 4 * kBdrWaves);
        if (rb > 4096) rb = 4096;
        const dim3 grid = bdr_grid(rows, ppr, static_cast<int>(rb)), block(256);
        const bool drop = d.t16 != 0;
        if (bp && drop) hipLaunchKernelGGL((bdr_fwd_cols<T, true, true>), grid, block, 0, s, o, xp, bp, rp, rows, ppr, d);
        else if (bp) hipLaunchKernelGGL((bdr_fwd_cols<T, true, false>), grid, block, 0, s, o, xp, bp, rp, rows, ppr, d);
        else if (drop) hipLaunchKernelGGL((bdr_fwd_cols<T, false, true>), grid, block, 0, s, o, xp, bp, rp, rows, ppr, d);
        else hipLaunchKernelGGL((bdr_fwd_cols<T, false, false>), grid, block, 0, s, o, xp, bp, rp, rows, ppr, d);
    } else {
        const int64_t total = rows * hidden;
        hipLaunchKernelGGL((bdr_fwd_flat<T>), dim3(static_cast<unsigned>(ceil_div(total, 256))), dim3(256), 0, s,
                           o, xp, bp, rp, total, hidden, d);
    }
    return launch_status();
}

template <typename T>
static lsq_status bdr_bwd_dispatch(void* dx, float* dbias, const void* dy, int64_t rows, int32_t hidden,
                                   const DropoutParams& d, void* workspace, hipStream_t s)
{
    T* o = static_cast<T*>(dx);
    const T* g = static_cast<const T*>(dy);
    if (hidden % kPack == 0) {
        const int ppr = hidden / kPack;
        const int rb = bdr_bwd_row_blocks(rows, hidden);
        const dim3 grid = bdr_grid(rows, ppr, rb), block(256);
        float* partial = dbias ? static_cast<float*>(workspace) : nullptr;
        if (d.t16) hipLaunchKernelGGL((bdr_bwd_cols<T, true>), grid, block, 0, s, o, partial, g, rows, ppr, d);
        else hipLaunchKernelGGL((bdr_bwd_cols<T, false>), grid, block, 0, s, o, partial, g, rows, ppr, d);
        if (dbias)
            launch_colsum_finalize(dbias, dbias, hidden, partial, rb, hidden, s);
    } else {
        const int64_t total = rows * hidden;
        hipLaunchKernelGGL((bdr_bwd_flat<T>), dim3(static_cast<unsigned>(ceil_div(total, 256))), dim3(256), 0, s,
                           o, g, total, d);
        if (dbias)
            hipLaunchKernelGGL((bdr_dbias_flat<T>), dim3(static_cast<unsigned>(ceil_div(hidden, 256))), dim3(256), 0, s,
                               dbias, g, rows, hidden, d);
    }
    return launch_status();
}

}  // namespace lsq

extern "C" lsq_status lsq_bias_dropout_residual_fwd(void* out, const void* x, const void* bias, const void* residual,
                                                    int64_t rows, int32_t hidden, float p, uint64_t seed,
                                                    uint64_t offset, lsq_dtype dt, void* stream)
{
    using namespace lsq;
    LSQ_REQUIRE(rows >= 0 && hidden > 0);
    if (!valid_dtype(dt)) return LSQ_UNSUPPORTED_DTYPE;
    DropoutParams d;
    LSQ_REQUIRE(make_dropout(p, seed, offset, &d));
    if (rows == 0) return LSQ_OK;
    LSQ_REQUIRE(out && x && residual);
    LSQ_ALIGNED(out); LSQ_ALIGNED(x); LSQ_ALIGNED(bias); LSQ_ALIGNED(residual);
    LSQ_REQUIRE(ceil_div(rows * hidden, 256) <= 0x7FFFFFFF);
    hipStream_t s = static_cast<hipStream_t>(stream);
    switch (dt) {
        case LSQ_F16: return bdr_fwd_dispatch<f16>(out, x, bias, residual, rows, hidden, d, s);
        case LSQ_BF16: return bdr_fwd_dispatch<bf16>(out, x, bias, residual, rows, hidden, d, s);
        default: return bdr_fwd_dispatch<float>(out, x, bias, residual, rows, hidden, d, s);
    }
}

extern "C" lsq_status lsq_bias_dropout_residual_bwd(void* dx, float* dbias, const void* dy, int64_t rows,
                                                    int32_t hidden, float p, uint64_t seed, uint64_t offset,
                                                    void* workspace, size_t workspace_bytes, lsq_dtype dt,
                                                    void* stream)
{
    using namespace lsq;
    LSQ_REQUIRE(rows >= 0 && hidden > 0);
    if (!valid_dtype(dt)) return LSQ_UNSUPPORTED_DTYPE;
    DropoutParams d;
    LSQ_REQUIRE(make_dropout(p, seed, offset, &d));
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (rows == 0) {
        if (dbias) return zero_fill(dbias, hidden, s);
        return LSQ_OK;
    }
    LSQ_REQUIRE(dx && dy);
    LSQ_ALIGNED(dx); LSQ_ALIGNED(dy); LSQ_ALIGNED(dbias); LSQ_ALIGNED(workspace);
    LSQ_REQUIRE(ceil_div(rows * hidden, 256) <= 0x7FFFFFFF);
    if (dbias) {
        const size_t need = lsq_workspace_bytes(LSQ_OP_BIAS_DROPOUT_RESIDUAL_BWD, rows, hidden);
        if (need && (!workspace || workspace_bytes < need)) return LSQ_WORKSPACE_TOO_SMALL;
    }
    switch (dt) {
        case LSQ_F16: return bdr_bwd_dispatch<f16>(dx, dbias, dy, rows, hidden, d, workspace, s);
        case LSQ_BF16: return bdr_bwd_dispatch<bf16>(dx, dbias, dy, rows, hidden, d, workspace, s);
        default: return bdr_bwd_dispatch<float>(dx, dbias, dy, rows, hidden, d, workspace, s);
    }
}
