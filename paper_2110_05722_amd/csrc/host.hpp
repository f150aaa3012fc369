// Host-side helpers shared by the entry points: argument checks, dropout
// parameter packing, launch bookkeeping.  Nothing here touches device memory.
#pragma once
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "../../include/lsq.h"
#include "device.hpp"

namespace lsq {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

#define LSQ_REQUIRE(cond) do { if (!(cond)) return LSQ_INVALID_ARG; } while (0)
#define LSQ_ALIGNED(ptr) do { if ((ptr) && !::lsq::aligned16(ptr)) return LSQ_MISALIGNED; } while (0)

inline bool valid_dtype(int dt) { return dt == LSQ_F16 || dt == LSQ_BF16 || dt == LSQ_F32; }

// p must lie in [0, 1).  T16 = round(p * 65536) in double, clamped to [0, 65535].
inline bool make_dropout(float p, uint64_t seed, uint64_t offset, DropoutParams* d)
{
    if (!(p >= 0.0f) || !(p < 1.0f)) return false;
    double t = floor(static_cast<double>(p) * 65536.0 + 0.5);
    if (t < 0.0) t = 0.0;
    if (t > 65535.0) t = 65535.0;
    d->key0 = static_cast<uint32_t>(seed);
    d->key1 = static_cast<uint32_t>(seed >> 32);
    d->ctr2 = static_cast<uint32_t>(offset);
    d->ctr3 = static_cast<uint32_t>(offset >> 32);
    d->t16 = p == 0.0f ? 0u : static_cast<uint32_t>(t);
    d->on = p > 0.0f ? 1u : 0u;
    d->scale = static_cast<float>(1.0 / (1.0 - static_cast<double>(p)));
    return true;
}

inline lsq_status launch_status()
{
    return hipGetLastError() == hipSuccess ? LSQ_OK : LSQ_LAUNCH_FAILED;
}

// Zero fill by a kernel (a memset node inside a captured graph is avoided on purpose).
template <int = 0>
__global__ __launch_bounds__(256) void zero_f32_kernel(float* p, int64_t n)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i < n) p[i] = 0.0f;
}

inline lsq_status zero_fill(float* p, int64_t n, hipStream_t s)
{
    if (n <= 0) return LSQ_OK;
    hipLaunchKernelGGL((zero_f32_kernel<0>), dim3(static_cast<unsigned>((n + 255) / 256)), dim3(256), 0, s, p, n);
    return launch_status();
}

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Division of a row index (below 2^32) by a launch constant: multiply-high by a host-made reciprocal, two shifts
// (Granlund and Montgomery's round-up form) -- 5 integer instructions where the 64-bit division the compiler emits
// for an int64 row index takes about 40 per row (a tenth of a short softmax row's vector-ALU work).
struct FastDiv {
    uint32_t m;
    int sh1, sh2;
};
inline FastDiv make_fastdiv(uint32_t d)
{
    if (d == 0) d = 1;
    int l = 0;
    while ((1ull << l) < d) ++l;                                   // ceil(log2 d)
    FastDiv f;
    f.m = static_cast<uint32_t>(((1ull << 32) * ((1ull << l) - d)) / d + 1);
    f.sh1 = l < 1 ? l : 1;
    f.sh2 = l - f.sh1;
    return f;
}
__device__ __forceinline__ uint32_t fastdiv(uint32_t n, const FastDiv& f)
{
    const uint32_t t = __umulhi(f.m, n);
    return (t + ((n - t) >> f.sh1)) >> f.sh2;
}

// Second stage of the column reductions: out[c] = sum over the P partial rows of
// partial[y][c], C columns, in a fixed order (reproducible).  Columns below `split`
// go to out0, those below `split2` to out1, the rest to out2.  A workgroup owns 32 columns; its 8 row slices each
// sum a contiguous chunk of rows with the loads of 32 rows in flight at a time (a
// plain loop would pay one memory latency per row; 256 partial rows are one batch per thread), then the
// slices are combined in slice order through LDS.  Measured behind a 21 MB producer kernel, 256 x 2560
// partials: 2.5 us against 2.7 us as 32 slices x 8 loads in a 1024-thread workgroup (an empty dependent
// kernel: 1.4 us).
constexpr int kFinalizeSlices = 8, kFinalizeLoads = 32;

template <int = 0>
__global__ __launch_bounds__(32 * kFinalizeSlices) void colsum_finalize_kernel(float* __restrict__ out0,
                                                                               float* __restrict__ out1,
                                                                               float* __restrict__ out2, int split,
                                                                               int split2,
                                                                               const float* __restrict__ partial,
                                                                               int P, int C)
{
    __shared__ float sm[kFinalizeSlices][33];
    const int lane = threadIdx.x & 31, slice = threadIdx.x >> 5;
    const int c = blockIdx.x * 32 + lane;
    const int chunk = (P + kFinalizeSlices - 1) / kFinalizeSlices;
    const int y0 = slice * chunk, y1 = min(P, y0 + chunk);
    float s = 0.0f;
    if (c < C) {
        int y = y0;
        for (; y + kFinalizeLoads <= y1; y += kFinalizeLoads) {
            float t[kFinalizeLoads];
#pragma unroll
            for (int k = 0; k < kFinalizeLoads; ++k) t[k] = partial[static_cast<int64_t>(y + k) * C + c];
#pragma unroll
            for (int k = 0; k < kFinalizeLoads; ++k) s += t[k];
        }
        for (; y + 8 <= y1; y += 8) {
            float t[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) t[k] = partial[static_cast<int64_t>(y + k) * C + c];
#pragma unroll
            for (int k = 0; k < 8; ++k) s += t[k];
        }
        for (; y < y1; ++y) s += partial[static_cast<int64_t>(y) * C + c];
    }
    sm[slice][lane] = s;
    __syncthreads();
    if (slice == 0 && c < C) {
        float t = sm[0][lane];
#pragma unroll
        for (int w = 1; w < kFinalizeSlices; ++w) t += sm[w][lane];
        if (c < split) out0[c] = t;
        else if (c < split2) out1[c - split] = t;
        else out2[c - split2] = t;
    }
}

inline void launch_colsum_finalize(float* out0, float* out1, int split, const float* partial, int P, int C, hipStream_t s,
                                   float* out2 = nullptr, int split2 = 0x7FFFFFFF)
{
    hipLaunchKernelGGL((colsum_finalize_kernel<0>), dim3(static_cast<unsigned>((C + 31) / 32)), dim3(32 * kFinalizeSlices), 0, s,
                       out0, out1, out2, split, split2, partial, P, C);
}

// ---- rows that are not a whole number of packs (hidden % 8 != 0): element-wise operators
// The tensor is walked as ONE flat array in aligned packs (a pack may straddle two rows), so every
// access stays a 128-bit one and a pack still costs one Philox call (the dropout contract counts
// packs over the flat tensor).  F supplies the operator:
//   void  pack(int64_t e0, int c0, float (&g)[8])   loads, computes and stores the pack at element e0,
//                                                   whose first column is c0; g = the fp32 results
//   float one(int64_t e, int c)                      the same for one element of the ragged last pack
// With COLS the fp32 results also feed column sums (a bias gradient): a workgroup parks the
// results of a trip (256 threads x 4 packs, consecutive) in LDS, then every thread adds up, in
// ascending element order, the entries of the columns it owns (c = thread, thread + 256, ...); the
// owner alone touches a column's accumulator (in LDS up to 8192 columns, else straight in the
// workgroup's partial row), so no atomics and a fixed order.  One partial row per workgroup, summed
// by colsum_finalize_kernel.
constexpr int kFlatPacks = 4;                                    // packs per thread and trip
constexpr int kFlatChunk = 256 * kFlatPacks * kPack;             // elements per trip
constexpr int kFlatMaxBlocks = 512;                              // partial rows at most
constexpr int kFlatLdsColumns = 8192;                            // accumulators in LDS up to this row length

struct FlatPlan { int blocks, trips; };
inline FlatPlan flat_plan(int64_t total, bool cols)
{
    const int64_t chunks = ceil_div(total, kFlatChunk);
    FlatPlan p;
    if (!cols) { p.blocks = static_cast<int>(chunks); p.trips = 1; return p; }
    p.trips = static_cast<int>(ceil_div(chunks, kFlatMaxBlocks));
    if (p.trips < 1) p.trips = 1;
    p.blocks = static_cast<int>(ceil_div(chunks, p.trips));
    if (p.blocks < 1) p.blocks = 1;
    return p;
}

template <typename F, bool COLS, bool ACC_LDS>
__global__ __launch_bounds__(256) void flat_packs_kernel(F f, float* __restrict__ partial, int64_t total, int hidden, int trips)
{
    extern __shared__ float flat_lds[];        // COLS: [kFlatChunk] results of the trip (, [hidden] accumulators)
    const int tid = threadIdx.x;
    float* acc = nullptr;
    if constexpr (COLS) {
        acc = ACC_LDS ? flat_lds + kFlatChunk : partial + static_cast<int64_t>(blockIdx.x) * hidden;
        for (int c = tid; c < hidden; c += 256) acc[c] = 0.0f;     // read again by this thread only
    }
    for (int t = 0; t < trips; ++t) {
        const int64_t base = (static_cast<int64_t>(blockIdx.x) * trips + t) * kFlatChunk;
        if (base >= total) break;                                  // uniform over the workgroup
        const int cb = static_cast<int>(base % hidden);            // column of the trip's first element
#pragma unroll
        for (int u = 0; u < kFlatPacks; ++u) {
            const int off = (u * 256 + tid) * kPack;
            const int64_t e0 = base + off;
            float g[8] = {0, 0, 0, 0, 0, 0, 0, 0};
            if (e0 + kPack <= total) {
                f.pack(e0, static_cast<int>(static_cast<uint32_t>(cb + off) % static_cast<uint32_t>(hidden)), g);
            } else if (e0 < total) {
                int c = static_cast<int>(static_cast<uint32_t>(cb + off) % static_cast<uint32_t>(hidden));
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    if (e0 + j < total) g[j] = f.one(e0 + j, c);
                    c = c + 1 == hidden ? 0 : c + 1;
                }
            }
            if constexpr (COLS) store8<float>(flat_lds + off, g);
        }
        if constexpr (COLS) {
            __syncthreads();
            const int64_t left = total - base;
            const int n = left < kFlatChunk ? static_cast<int>(left) : kFlatChunk;
            if (hidden >= 256) {
                for (int c = tid; c < hidden; c += 256) {
                    int i = c - cb;
                    if (i < 0) i += hidden;
                    float a = acc[c];
                    for (; i < n; i += hidden) a += flat_lds[i];
                    acc[c] = a;
                }
                __syncthreads();                                   // the next trip overwrites the results
            } else {
                // short rows: 256 / hidden threads share a column (every slices-th entry each, ascending), their
                // sums are added in slice order by the column's owner
                const int slices = 256 / hidden, c = tid % hidden, sl = tid / hidden;
                float a = 0.0f;
                if (sl < slices) {
                    int i = c - cb;
                    if (i < 0) i += hidden;
                    for (i += sl * hidden; i < n; i += slices * hidden) a += flat_lds[i];
                }
                __syncthreads();                                   // all entries read: the results' place is reused
                if (sl < slices) flat_lds[sl * hidden + c] = a;
                __syncthreads();
                if (tid < hidden) {
                    float tsum = acc[tid];
                    for (int k = 0; k < slices; ++k) tsum += flat_lds[k * hidden + tid];
                    acc[tid] = tsum;
                }
                __syncthreads();
            }
        }
    }
    if constexpr (COLS && ACC_LDS) {
        float* prow = partial + static_cast<int64_t>(blockIdx.x) * hidden;
        for (int c = tid; c < hidden; c += 256) prow[c] = acc[c];
    }
}

// dbias == nullptr: the element-wise part only.  workspace: flat_plan(total, true).blocks rows of hidden floats.
template <typename F>
inline void launch_flat_packs(const F& f, float* dbias, void* workspace, int64_t rows, int hidden, hipStream_t s)
{
    const int64_t total = rows * hidden;
    const FlatPlan pl = flat_plan(total, dbias != nullptr);
    const dim3 grid(static_cast<unsigned>(pl.blocks)), block(256);
    if (!dbias) {
        hipLaunchKernelGGL((flat_packs_kernel<F, false, false>), grid, block, 0, s, f, nullptr, total, hidden, 1);
        return;
    }
    float* partial = static_cast<float*>(workspace);
    if (hidden <= kFlatLdsColumns)
        hipLaunchKernelGGL((flat_packs_kernel<F, true, true>), grid, block, (kFlatChunk + hidden) * sizeof(float), s, f, partial,
                           total, hidden, pl.trips);
    else
        hipLaunchKernelGGL((flat_packs_kernel<F, true, false>), grid, block, kFlatChunk * sizeof(float), s, f, partial, total,
                           hidden, pl.trips);
    launch_colsum_finalize(dbias, dbias, hidden, partial, pl.blocks, hidden, s);
}

inline size_t flat_workspace_bytes(int64_t rows, int32_t hidden)
{
    return static_cast<size_t>(flat_plan(rows * hidden, true).blocks) * static_cast<size_t>(hidden) * sizeof(float);
}

// Number of partial-sum rows the column reductions write to the workspace.
// One per workgroup; sized so the grid fills 256 compute units a few times over
// while the partials stay a small fraction of the tensor traffic.
inline int ln_bwd_blocks(int64_t rows, int32_t /*hidden*/)
{
    int64_t b = ceil_div(rows, 8);       // at least 8 rows per workgroup
    if (b > 256) b = 256;   // one workgroup per compute unit: measured best at 8192 rows
    if (b < 1) b = 1;
    return static_cast<int>(b);
}

// ---- bias + dropout + residual: launch shapes (shared with the workspace sizing)
// Measured at 8192 x 1280 / 8192 x 1024 (fp16, p = 0.1): forward one row per lane 11.4 / 9.9 us, two 11.5 / 10.8, four
// 13.4 / 10.6; backward (without the column sums) 4 waves per workgroup 8.9 / 7.6 us, 8 waves 9.2 / 7.3, 16 waves 9.5 / 8.0;
// column blocks of 32 packs against 16: forward 11.4 / 9.7 against 11.5 / 10.2.
constexpr int kBdrFwdWaves = 4;                   // waves per forward workgroup; each takes its own rows
constexpr int kBdrFwdUnroll = 1;                  // rows a lane has in flight in forward
constexpr int kBdrBwdWaves = 4;                   // waves per backward workgroup
constexpr int kBdrMaxLanes = 32;                  // widest column block (packs) the kernels are built for

// Lanes of a wave that share a row: 32 or 16, the wider that divides the packs of a row; 16 with a
// ragged last column block if none does.
inline int bdr_lanes_per_row(int ppr)
{
    for (int w = kBdrMaxLanes; w >= 16; w >>= 1)
        if (ppr % w == 0) return w;
    return 16;
}

// Rows of very few packs leave most lanes of a 16-lane row segment idle; they take the flat walk like the
// rows that are not whole packs (measured at 32 Mi elements: forward 187 / 94 / 63 us at 8 / 16 / 24 columns
// against 47 us flat; backward 860 / 439 / 175 / 83 / 80 us at 8 / 16 / 24 / 64 / 72 columns against 48 us flat).
inline bool bdr_fwd_is_flat(int hidden) { return hidden % kPack != 0 || hidden <= 32; }
inline bool bdr_bwd_is_flat(int hidden) { return hidden % kPack != 0 || hidden < 128; }
// bias + activation + dropout works in column blocks of 64 packs: rows of up to 32 packs take the flat walk
// (8 columns: 1629 / 10103 us in column blocks at 32 Mi elements, 51 / 95 us flat; 256 columns: 56 / 138 us).
inline bool bad_is_flat(int hidden) { return hidden % kPack != 0 || hidden <= 256; }

// Backward launch shape: column blocks of w packs; row blocks (= partial rows of the column sums) of
// `trips` consecutive groups of waves * 64 / w rows.
constexpr int kBdrBwdWorkgroups = 1280;           // about five per compute unit: fewer (640, 768) cost 0.5-1.5 us at 8192 rows
constexpr int kBdrBwdMaxPartials = 256;           // partial rows the second stage sums
struct BdrBwdPlan { int w, col_blocks, row_blocks, trips; };
inline BdrBwdPlan bdr_bwd_plan(int64_t rows, int32_t hidden)
{
    BdrBwdPlan p;
    const int ppr = hidden / kPack;
    p.w = bdr_lanes_per_row(ppr);
    p.col_blocks = static_cast<int>(ceil_div(ppr, p.w));
    const int64_t units = ceil_div(rows, static_cast<int64_t>(kBdrBwdWaves) * (64 / p.w));     // row groups of one trip
    int64_t rb_max = kBdrBwdWorkgroups / p.col_blocks;
    if (rb_max > kBdrBwdMaxPartials) rb_max = kBdrBwdMaxPartials;
    if (rb_max < 1) rb_max = 1;
    const int64_t trips = ceil_div(units, rb_max);
    p.trips = static_cast<int>(trips < 1 ? 1 : trips);
    const int64_t rb = ceil_div(units, p.trips);
    p.row_blocks = static_cast<int>(rb < 1 ? 1 : rb);
    return p;
}

// Row blocks of the column-blocked backward kernels that leave one partial row of column sums per row block
// (feed-forward bias+activation+dropout, head merge): as many as give about `target` workgroups over the
// hidden / 512 column blocks.  Measured at 8192 x 5120 (GELU, dropout) and 4096 x 4096 (ReLU): 512 workgroups, two per
// compute unit, 45.2 / 35.2 us; 384: 49.8 / 40.7; 640: 47.5 / 37.9; 1024: 46.9 / 36.8; 2560 (one row block per
// 32 rows, the earlier choice): 49.8 / 38.4 -- totals that are not a multiple of the 256 compute units leave some
// of them with one workgroup more, and fewer, longer workgroups pay prologue, LDS epilogue and partial row less often.
// The head merge (no arithmetic, 128-byte pieces) wants more loads in flight: 1024 workgroups 26.5 us at
// 8192 x 3840, 768: 28.4, 1536: 27.6, 2048: 29.2, 512: 34.
constexpr int kBadBwdWorkgroups = 512, kHeadsBwdWorkgroups = 1024;
inline int colsum_row_blocks(int64_t rows, int32_t hidden, int target)
{
    const int64_t col_blocks = ceil_div(hidden, 64 * kPack);
    int64_t b = target / col_blocks;
    const int64_t most = ceil_div(rows, 16);
    if (b > most) b = most;
    return static_cast<int>(b < 1 ? 1 : b);
}
inline int bad_bwd_row_blocks(int64_t rows, int32_t hidden) { return colsum_row_blocks(rows, hidden, kBadBwdWorkgroups); }
inline int heads_bwd_row_blocks(int64_t rows, int32_t hidden) { return colsum_row_blocks(rows, hidden, kHeadsBwdWorkgroups); }

// Workspace of the embedding backward:
//   order  [rows] (token position, sort key), 8 bytes each
//   window rows [2 * windows][hidden rounded up to 8] fp32: the partial sums of id segments
//          that cross a window of kEmbWin sorted entries (at most two per window)
//   rank counts [spans][rows] int32: token i against the tokens of span js (a span is a run
//          of 256-token tiles, at most 64 spans); beyond kEmbCountMax tokens the same region holds
//          the radix sort's [256][workgroups] digit counts and its second (token, key) buffer
constexpr int kEmbTile = 256;
constexpr int64_t kEmbCountMax = 16384;
constexpr int kEmbWin = 8;
struct EmbBwdPlan {
    int ntiles, span_tiles, nspans, radix_blocks;
    size_t radix_hist_bytes;
    int64_t nwin;
    size_t order_bytes, win_bytes, rank_bytes;
    size_t total() const { return order_bytes + win_bytes + rank_bytes; }
};
inline EmbBwdPlan emb_bwd_plan(int64_t rows, int32_t hidden)
{
    EmbBwdPlan p;
    p.ntiles = static_cast<int>(ceil_div(rows, kEmbTile));
    p.span_tiles = static_cast<int>(ceil_div(p.ntiles, 64));
    p.nspans = static_cast<int>(ceil_div(p.ntiles, p.span_tiles));
    p.nwin = ceil_div(rows, kEmbWin);
    const size_t colsp = (static_cast<size_t>(hidden) + 7u) / 8u * 8u;
    p.order_bytes = (static_cast<size_t>(rows) * 8u + 15u) / 16u * 16u;
    p.win_bytes = 2u * static_cast<size_t>(p.nwin) * colsp * sizeof(float);
    p.rank_bytes = static_cast<size_t>(p.nspans) * static_cast<size_t>(rows) * sizeof(int32_t);
    p.radix_blocks = static_cast<int>(ceil_div(rows, 2048));
    p.radix_hist_bytes = (static_cast<size_t>(256) * static_cast<size_t>(p.radix_blocks) * sizeof(int32_t) + 15u) / 16u * 16u;
    if (rows > kEmbCountMax) p.rank_bytes = p.radix_hist_bytes + static_cast<size_t>(rows) * 8u;
    return p;
}

}  // namespace lsq
