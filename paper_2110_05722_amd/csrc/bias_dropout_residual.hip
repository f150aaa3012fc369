// Fused bias + dropout + residual, forward and backward (Sec. IV-A of the paper,
// Transformer layers: "bias adding, dropout, and residual" in one launch).
//
// Layout of the fast path (hidden % 8 == 0): W lanes of a wave (W = 32 or 16, the wider
// that divides the packs of a row, so no lane idles on a ragged last column block) own W
// consecutive packs of one row and the wave covers 64 / W rows at a time; a workgroup's column
// block is fixed, so the bias pack is loaded once into registers, every access is a 128-bit one,
// and in backward each lane accumulates the column sums of its own 8 columns with no atomics.
// The dropout mask is never stored: both directions rebuild it from the Philox
// counter of the pack.  HBM traffic: forward 3 tensors, backward 2.
//
// Backward column sums (dbias): a workgroup adds up its lanes' sums through LDS in a fixed order and
// writes one partial row of its column block to the workspace; a second small kernel sums the
// partial rows in a fixed order (bit-reproducible; no atomics).
#include "host.hpp"

namespace lsq {

constexpr bool kNT = true;    // nontemporal hint on the streamed tensors (not on gamma/beta/bias)

// A wave as 64 / W row segments of W packs: lane -> (row of the group, pack of the column block).
template <int W> struct BdrLane {
    static constexpr int SUB = 64 / W;
    int col, sub;
    __device__ __forceinline__ BdrLane() : col((threadIdx.x & 63) % W), sub((threadIdx.x & 63) / W) {}
};

template <typename T, bool HAS_BIAS, bool DROP, int W>
__global__ __launch_bounds__(64 * kBdrFwdWaves) void bdr_fwd_cols(T* out, const T* x, const T* __restrict__ bias,
                                                                  const T* res, int64_t rows, int ppr, DropoutParams d)
{
    constexpr int SUB = 64 / W, U = kBdrFwdUnroll, RPI = kBdrFwdWaves * SUB * U;
    const BdrLane<W> ln;
    const int wave = threadIdx.x >> 6;
    const int cp = blockIdx.x * W + ln.col;
    if (cp >= ppr) return;
    // the bias stays packed and is widened where it is used: widening it here would make the
    // row loads below wait for its arrival
    RawPack<T> braw = zero_raw<T>();
    if constexpr (HAS_BIAS) braw = load_raw<T>(bias + static_cast<int64_t>(cp) * kPack);
    for (int64_t base = static_cast<int64_t>(blockIdx.y) * RPI; base < rows; base += static_cast<int64_t>(gridDim.y) * RPI) {
        RawPack<T> xr[U], rr[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t r = base + (u * kBdrFwdWaves + wave) * SUB + ln.sub;
            if (r < rows) {
                xr[u] = load_raw<T, kNT>(x + (r * ppr + cp) * kPack);
                rr[u] = load_raw<T, kNT>(res + (r * ppr + cp) * kPack);
            } else {
                xr[u] = zero_raw<T>();
                rr[u] = zero_raw<T>();
            }
        }
        // the dropout factors need no data: they are drawn while the loads are in flight
        float k[DROP ? U : 1][8];
        if constexpr (DROP) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t r = base + (u * kBdrFwdWaves + wave) * SUB + ln.sub;
                dropout_factors8(d, static_cast<uint64_t>(r * ppr + cp), k[u]);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t r = base + (u * kBdrFwdWaves + wave) * SUB + ln.sub;
            if (r < rows) {
                const int64_t pack = r * ppr + cp;
                float xf[8], rf[8], b[8];
                unpack<T>(xr[u], xf);
                unpack<T>(rr[u], rf);
                if constexpr (HAS_BIAS) opaque<T>(braw);
                unpack<T>(braw, b);
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const float z = xf[j] + b[j];
                    rf[j] = DROP ? fmaf(z, k[DROP ? u : 0][j], rf[j]) : rf[j] + z;
                }
                pin_f32(rf);                  // rounds like the kernel that fuses the LayerNorm behind it
                store8<T, kNT>(out + pack * kPack, rf);
            }
        }
    }
}

// Backward.  partial: [gridDim.y][hidden] fp32 column sums of the workgroups' rows (nullptr:
// dbias not wanted), summed over the row blocks by colsum_finalize_kernel.
template <typename T, bool DROP, int W>
__global__ __launch_bounds__(64 * kBdrBwdWaves) void bdr_bwd_cols(T* dx, float* __restrict__ partial, const T* dy,
                                                                  int64_t rows, int ppr, int trips, DropoutParams d)
{
    constexpr int SUB = 64 / W, NW = kBdrBwdWaves, THREADS = 64 * NW;
    __shared__ float sm[NW * 8 * 64];      // the lanes' sums
    const BdrLane<W> ln;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int cp = blockIdx.x * W + ln.col;
    const bool active = cp < ppr;
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (active) {
        // A workgroup walks `trips` consecutive groups of NW * SUB rows; the pack of the next trip is
        // loaded before this trip's is used, and the dropout factors, which need no data, are
        // drawn while the loads are in flight.
        const int64_t first = static_cast<int64_t>(blockIdx.y) * trips * (NW * SUB) + wave * SUB + ln.sub;
        RawPack<T> nxt = first < rows ? load_raw<T, kNT>(dy + (first * ppr + cp) * kPack) : zero_raw<T>();
        for (int t = 0; t < trips; ++t) {
            const int64_t r = first + static_cast<int64_t>(t) * (NW * SUB);
            const RawPack<T> cur = nxt;
            const int64_t rn = r + NW * SUB;
            if (t + 1 < trips && rn < rows) nxt = load_raw<T, kNT>(dy + (rn * ppr + cp) * kPack);
            if (r < rows) {
                const int64_t pack = r * ppr + cp;
                float g[8], k[8];
                if constexpr (DROP) dropout_factors8(d, static_cast<uint64_t>(pack), k);
                unpack<T>(cur, g);
                if constexpr (DROP) {
#pragma unroll
                    for (int j = 0; j < 8; ++j) g[j] *= k[j];
                }
                pin_f32(g);
                store8<T, kNT>(dx + pack * kPack, g);
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[j] += g[j];
            }
        }
    }
    if (partial == nullptr) return;        // uniform over the grid
    // the workgroup's sums: wave by wave, row of the group by row of the group, in that order
#pragma unroll
    for (int j = 0; j < 8; ++j) sm[(wave * 8 + j) * 64 + lane] = acc[j];
    __syncthreads();
    const int hidden = ppr * kPack;
    const int c0 = blockIdx.x * W * kPack;                       // first column of the block
    const int ncols = min(W * kPack, hidden - c0);
    float* prow = partial + static_cast<int64_t>(blockIdx.y) * hidden + c0;
    for (int c = threadIdx.x; c < W * kPack; c += THREADS) {
        const int j = c / W, col = c % W;                        // consecutive threads read consecutive LDS words
        float t = 0.0f;
#pragma unroll
        for (int w = 0; w < NW; ++w)
#pragma unroll
            for (int sb = 0; sb < SUB; ++sb) t += sm[(w * 8 + j) * 64 + sb * W + col];
        if (col * kPack + j < ncols) prow[col * kPack + j] = t;
    }
}

// ---- any hidden (rows are not a whole number of packs): the operators for flat_packs_kernel
template <typename T>
struct BdrFwdFlat {
    T* out;
    const T* x;
    const T* bias;
    const T* res;
    int hidden;
    DropoutParams d;
    __device__ __forceinline__ void pack(int64_t e0, int c0, float (&g)[8]) const
    {
        const RawPack<T> xr = load_raw<T, kNT>(x + e0), rr = load_raw<T, kNT>(res + e0);
        float k[8];
        if (d.on) dropout_factors8(d, static_cast<uint64_t>(e0 >> 3), k);
        float xf[8];
        unpack<T>(xr, xf);
        unpack<T>(rr, g);
        int c = c0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float z = bias ? xf[j] + to_f32<T>(bias[c]) : xf[j];
            g[j] = d.on ? fmaf(z, k[j], g[j]) : g[j] + z;
            c = c + 1 == hidden ? 0 : c + 1;
        }
        pin_f32(g);
        store8<T, kNT>(out + e0, g);
    }
    __device__ __forceinline__ float one(int64_t e, int c) const
    {
        float z = to_f32<T>(x[e]);
        if (bias) z += to_f32<T>(bias[c]);
        const float r = to_f32<T>(res[e]);
        const float v = d.on ? fmaf(z, dropout_factor1(d, static_cast<uint64_t>(e)), r) : r + z;
        out[e] = from_f32<T>(v);
        return v;
    }
};

template <typename T>
struct BdrBwdFlat {
    T* dx;
    const T* dy;
    DropoutParams d;
    __device__ __forceinline__ void pack(int64_t e0, int, float (&g)[8]) const
    {
        const RawPack<T> cur = load_raw<T, kNT>(dy + e0);
        float k[8];
        if (d.on) dropout_factors8(d, static_cast<uint64_t>(e0 >> 3), k);
        unpack<T>(cur, g);
        if (d.on) {
#pragma unroll
            for (int j = 0; j < 8; ++j) g[j] *= k[j];
        }
        pin_f32(g);
        store8<T, kNT>(dx + e0, g);
    }
    __device__ __forceinline__ float one(int64_t e, int) const
    {
        float g = to_f32<T>(dy[e]);
        if (d.on) g *= dropout_factor1(d, static_cast<uint64_t>(e));
        dx[e] = from_f32<T>(g);
        return g;
    }
};

template <typename T>
static lsq_status bdr_fwd_dispatch(void* out, const void* x, const void* bias, const void* res, int64_t rows,
                                   int32_t hidden, const DropoutParams& d, hipStream_t s)
{
    T* o = static_cast<T*>(out);
    const T* xp = static_cast<const T*>(x);
    const T* bp = static_cast<const T*>(bias);
    const T* rp = static_cast<const T*>(res);
    if (!bdr_fwd_is_flat(hidden)) {
        const int ppr = hidden / kPack;
        const int w = bdr_lanes_per_row(ppr);
        const int64_t rpi = static_cast<int64_t>(kBdrFwdWaves) * (64 / w) * kBdrFwdUnroll;     // rows of a workgroup's trip
        int64_t rb = ceil_div(rows, rpi);
        if (rb > 8192) rb = 8192;
        const dim3 grid(static_cast<unsigned>(ceil_div(ppr, w)), static_cast<unsigned>(rb)), block(64 * kBdrFwdWaves);
        const bool drop = d.on != 0;
#define LSQ_BDR_FWD(W)                                                                                                  \
        if (w == W) {                                                                                                   \
            if (bp && drop) hipLaunchKernelGGL((bdr_fwd_cols<T, true, true, W>), grid, block, 0, s, o, xp, bp, rp, rows, ppr, d);    \
            else if (bp) hipLaunchKernelGGL((bdr_fwd_cols<T, true, false, W>), grid, block, 0, s, o, xp, bp, rp, rows, ppr, d);     \
            else if (drop) hipLaunchKernelGGL((bdr_fwd_cols<T, false, true, W>), grid, block, 0, s, o, xp, bp, rp, rows, ppr, d);   \
            else hipLaunchKernelGGL((bdr_fwd_cols<T, false, false, W>), grid, block, 0, s, o, xp, bp, rp, rows, ppr, d);            \
        }
        LSQ_BDR_FWD(32) LSQ_BDR_FWD(16)
#undef LSQ_BDR_FWD
    } else {
        launch_flat_packs(BdrFwdFlat<T>{o, xp, bp, rp, hidden, d}, nullptr, nullptr, rows, hidden, s);
    }
    return launch_status();
}

template <typename T>
static lsq_status bdr_bwd_dispatch(void* dx, float* dbias, const void* dy, int64_t rows, int32_t hidden,
                                   const DropoutParams& d, void* workspace, hipStream_t s)
{
    T* o = static_cast<T*>(dx);
    const T* g = static_cast<const T*>(dy);
    if (!bdr_bwd_is_flat(hidden)) {
        const int ppr = hidden / kPack;
        const BdrBwdPlan pl = bdr_bwd_plan(rows, hidden);
        const dim3 grid(static_cast<unsigned>(pl.col_blocks), static_cast<unsigned>(pl.row_blocks)), block(64 * kBdrBwdWaves);
        float* partial = dbias ? static_cast<float*>(workspace) : nullptr;
#define LSQ_BDR_BWD(W)                                                                                                  \
        if (pl.w == W) {                                                                                                \
            if (d.on) hipLaunchKernelGGL((bdr_bwd_cols<T, true, W>), grid, block, 0, s, o, partial, g, rows, ppr, pl.trips, d);    \
            else hipLaunchKernelGGL((bdr_bwd_cols<T, false, W>), grid, block, 0, s, o, partial, g, rows, ppr, pl.trips, d);         \
        }
        LSQ_BDR_BWD(32) LSQ_BDR_BWD(16)
        if (dbias) launch_colsum_finalize(dbias, dbias, hidden, partial, pl.row_blocks, hidden, s);
#undef LSQ_BDR_BWD
    } else {
        // every pack is read and written by one thread, which also hands its fp32 results to the column sums: in place is fine
        launch_flat_packs(BdrBwdFlat<T>{o, g, d}, dbias, workspace, rows, hidden, s);
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
