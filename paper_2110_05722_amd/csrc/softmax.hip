// Masked, variable-length attention softmax, forward and backward (Sec. IV-B of
// the paper, Softmax: maximum, partition function, normalisation; backward is
// the softmax Jacobian of Sec. IV-A contracted with the upstream gradient).
//
// The paper copes with the spread of shapes ("a few to thousands" of columns,
// "thousands to millions" of rows) by tuning templates at run time.  Here the
// shape picks a compile-time bucket instead: LPR lanes share a row (1..64 lanes
// of a wave64), each lane keeps VPL packs of 8 scores in registers, so a row is
// read from HBM once, both reductions run on DPP inside the wave, and nothing
// goes through LDS.  Short rows put many rows in one wave (k_len 32 -> 16 rows per
// wave) so lanes are never idle.  Rows of 2049..16384 keys take one workgroup
// each (the reductions cross its four waves through LDS).  Rows whose length is
// not a multiple of 8 (up to 2048) use the same scheme with element-granular lanes
// working on LDS, which is filled and drained in aligned 128-bit packs (10-30 %
// slower than a length that is a multiple of 8);
// anything else falls to a three-pass kernel that re-reads the row from cache.
//
// Masks restrict the SET the softmax runs over: packs that lie wholly beyond the
// row's limit (key padding, or the causal diagonal) are not even loaded, and
// their outputs are written as exact zeros.  Attention-probability dropout is
// fused (Philox per pack, mask regenerated in backward).
#include <atomic>
#include <mutex>

#include "host.hpp"

namespace lsq {
// Threads per workgroup of the packed kernels (lanes per row <= 64: the waves of a workgroup share nothing).  The
// backward is 2-3 % faster as one-wave workgroups (106 against 109 us at 8 x 20 x 1024 x 1024 causal, 62.6 against 64 us
// with key padding at 512 keys, 16.8 against 17.1 us at 256 keys), the forward 3-4 % slower at 256 keys and equal elsewhere.
constexpr int kSmWgFwd = 256, kSmWgBwd = 64;

constexpr bool kNT = true;    // nontemporal hint on the streamed tensors

constexpr float kLog2e = 1.4426950408889634f;

struct SoftmaxGeom {
    int64_t nrows;        // batch * heads * q_len (below 2^31)
    int rows_per_batch;   // heads * q_len
    FastDiv by_rows_per_batch, by_q_len;
    int q_len, k_len;
    int causal;           // 0 / 1
    int shift;            // k_len - q_len (end-aligned causal mask)
    float scale;
};

// key and query lengths of the batch (either may be absent)
struct SoftmaxLens {
    const int32_t* __restrict__ key;
    const int32_t* __restrict__ query;
};

// number of allowed keys (a prefix of the row) for query row `row`; 0 for a padded query
__device__ __forceinline__ int row_limit(const SoftmaxGeom& g, const SoftmaxLens& len, int64_t row)
{
    int limit = g.k_len;
    const uint32_t r32 = static_cast<uint32_t>(row);
    const int i = static_cast<int>(r32 - fastdiv(r32, g.by_q_len) * static_cast<uint32_t>(g.q_len));
    if (len.key || len.query) {
        // the rows of a wave almost always belong to one sentence: its lengths come through
        // the scalar path (one cached load per wave), the vector path serves a straddling wave
        const int b = static_cast<int>(fastdiv(r32, g.by_rows_per_batch));
        const int b0 = __builtin_amdgcn_readfirstlane(b);
        if (len.key) {
            int kl = len.key[b0];
            if (b != b0) kl = len.key[b];
            limit = min(max(kl, 0), g.k_len);
        }
        if (len.query) {
            int ql = len.query[b0];
            if (b != b0) ql = len.query[b];
            if (i >= ql) limit = 0;
        }
    }
    if (g.causal) limit = min(limit, max(i + 1 + g.shift, 0));
    return limit;
}

// RPT rows per lane group: the loads of all RPT rows are issued before the first
// reduction, so a wave has RPT*VPL packs per lane in flight and the two dependent
// round trips (lengths, then scores) are paid once per RPT rows.
template <typename T, int LPR, int VPL, int RPT, bool DROP>
__global__ __launch_bounds__(kSmWgFwd) void softmax_fwd_kernel(T* y, T* __restrict__ yd, const T* x,
                                                          SoftmaxLens len, SoftmaxGeom g, DropoutParams d)
{
    constexpr int RPB = kSmWgFwd / LPR;
    const int sub = threadIdx.x % LPR;
    const int nv = g.k_len / kPack;
    int64_t row[RPT];
    int limit[RPT];
    // Loads first, arithmetic after.  The packs of a row's first 128 bytes are loaded before the
    // row's limit is known (unless the row is empty that line is needed whatever the limit, and
    // what lies beyond the limit is masked in registers): with a key-padding mask the limit comes
    // from memory, and waiting for it first would put two dependent round trips in front of
    // every row.  The other packs are loaded only if they reach into the allowed prefix.
    // (a limit that is computed from the row index alone, causal or none, waits for nothing)
    const int kEarly = (len.key || len.query) ? 128 / static_cast<int>(sizeof(T)) : 0;
    RawPack<T> raw[RPT][VPL];
#pragma unroll
    for (int r = 0; r < RPT; ++r) {
        row[r] = (static_cast<int64_t>(blockIdx.x) * RPT + r) * RPB + threadIdx.x / LPR;
#pragma unroll
        for (int k = 0; k < VPL; ++k) {
            const int j0 = (sub + k * LPR) * kPack;
            if (j0 < kEarly) {
                if (row[r] < g.nrows && j0 < g.k_len) raw[r][k] = load_raw<T, kNT>(x + row[r] * g.k_len + j0);
                else raw[r][k] = zero_raw<T>();
            }
        }
    }
#pragma unroll
    for (int r = 0; r < RPT; ++r) limit[r] = row[r] < g.nrows ? row_limit(g, len, row[r]) : 0;
#pragma unroll
    for (int r = 0; r < RPT; ++r)
#pragma unroll
        for (int k = 0; k < VPL; ++k) {
            const int j0 = (sub + k * LPR) * kPack;
            if (j0 >= kEarly) {
                if (j0 < limit[r]) raw[r][k] = load_raw<T, kNT>(x + row[r] * g.k_len + j0);   // implies a valid row and pack
                else raw[r][k] = zero_raw<T>();
            }
        }
#pragma unroll
    for (int r = 0; r < RPT; ++r) {
        const int64_t ro = row[r] * g.k_len;
        const int lim = limit[r];
        float v[VPL][8];
        bool live[VPL];       // wave-uniform: does any lane of the wave hold an allowed element of pack k?
        float mx = -INFINITY;
#pragma unroll
        for (int k = 0; k < VPL; ++k) {
            const int j0 = (sub + k * LPR) * kPack;
            live[k] = __ballot(j0 < lim) != 0;
            if (live[k]) {    // a pack that is masked for the whole wave costs no arithmetic
                unpack<T>(raw[r][k], v[k]);
                const int allowed = lim - j0;             // of this pack's 8 elements (<= 0: none, >= 8: all)
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    v[k][j] = (j < allowed) ? v[k][j] : -INFINITY;
                    mx = fmaxf(mx, v[k][j]);
                }
            }
        }
        // The scale is positive here (the dispatch sends other scales to the element kernels), so the maximum of the
        // scaled scores is the scaled maximum and the scale folds into the exponent's fma: one multiplication per
        // element less in a kernel that is bound by vector-ALU issue slots.
        mx = group_max<LPR>(mx);
        const float c = g.scale * kLog2e;
        const float mxs = (lim > 0 ? mx : 0.0f) * c;
        float z = 0.0f;
#pragma unroll
        for (int k = 0; k < VPL; ++k) {
            if (live[k]) {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const float e = __builtin_amdgcn_exp2f(fmaf(v[k][j], c, -mxs));   // exp2(-inf) = 0 on masked lanes
                    v[k][j] = e;
                    z += e;
                }
            }
        }
        z = group_sum<LPR>(z);
        const float inv = lim > 0 ? 1.0f / z : 0.0f;
#pragma unroll
        for (int k = 0; k < VPL; ++k) {
            const int idx = sub + k * LPR;
            if (row[r] < g.nrows && idx < nv) {
                float o[8] = {0, 0, 0, 0, 0, 0, 0, 0};
                if (live[k]) {
#pragma unroll
                    for (int j = 0; j < 8; ++j) o[j] = v[k][j] * inv;
                }
                store8<T, kNT>(y + ro + idx * kPack, o);
                if constexpr (DROP) {
                    if (idx * kPack < lim) {    // packs beyond the mask are zeros whatever the draw
                        float kf[8];
                        dropout_factors8(d, static_cast<uint64_t>(row[r]) * nv + idx, kf);
#pragma unroll
                        for (int j = 0; j < 8; ++j) o[j] *= kf[j];
                    }
                    store8<T, kNT>(yd + ro + idx * kPack, o);
                }
            }
        }
    }
}

template <typename T, int LPR, int VPL, int RPT, bool DROP>
__global__ __launch_bounds__(kSmWgBwd) void softmax_bwd_kernel(T* dx, const T* dy, const T* __restrict__ y,
                                                          SoftmaxLens len, SoftmaxGeom g, DropoutParams d)
{
    constexpr int RPB = kSmWgBwd / LPR;
    const int sub = threadIdx.x % LPR;
    const int nv = g.k_len / kPack;
    int64_t row[RPT];
    int limit[RPT];
    // as in forward: the first 128 bytes of a row are loaded before its limit is known
    const int kEarly = (len.key || len.query) ? 128 / static_cast<int>(sizeof(T)) : 0;
    RawPack<T> ry[RPT][VPL], rg[RPT][VPL];
#pragma unroll
    for (int r = 0; r < RPT; ++r) {
        row[r] = (static_cast<int64_t>(blockIdx.x) * RPT + r) * RPB + threadIdx.x / LPR;
#pragma unroll
        for (int k = 0; k < VPL; ++k) {
            const int j0 = (sub + k * LPR) * kPack;
            if (j0 < kEarly) {
                if (row[r] < g.nrows && j0 < g.k_len) {
                    ry[r][k] = load_raw<T, kNT>(y + row[r] * g.k_len + j0);
                    rg[r][k] = load_raw<T, kNT>(dy + row[r] * g.k_len + j0);
                } else {
                    ry[r][k] = zero_raw<T>();
                    rg[r][k] = zero_raw<T>();
                }
            }
        }
    }
#pragma unroll
    for (int r = 0; r < RPT; ++r) limit[r] = row[r] < g.nrows ? row_limit(g, len, row[r]) : 0;
#pragma unroll
    for (int r = 0; r < RPT; ++r)
#pragma unroll
        for (int k = 0; k < VPL; ++k) {
            const int j0 = (sub + k * LPR) * kPack;
            if (j0 >= kEarly) {
                if (j0 < limit[r]) {
                    ry[r][k] = load_raw<T, kNT>(y + row[r] * g.k_len + j0);
                    rg[r][k] = load_raw<T, kNT>(dy + row[r] * g.k_len + j0);
                } else {
                    ry[r][k] = zero_raw<T>();
                    rg[r][k] = zero_raw<T>();
                }
            }
        }
#pragma unroll
    for (int r = 0; r < RPT; ++r) {
        const int64_t ro = row[r] * g.k_len;
        const int lim = limit[r];
        float yv[VPL][8], gv[VPL][8];
        float dot = 0.0f;
#pragma unroll
        for (int k = 0; k < VPL; ++k) {
            const int idx = sub + k * LPR;
            const int j0 = idx * kPack;
            unpack<T>(ry[r][k], yv[k]);
            unpack<T>(rg[r][k], gv[k]);
            if constexpr (DROP) {
                if (j0 < lim) {
                    float kf[8];
                    dropout_factors8(d, static_cast<uint64_t>(row[r]) * nv + idx, kf);
#pragma unroll
                    for (int j = 0; j < 8; ++j) gv[k][j] *= kf[j];
                }
            }
            const int allowed = lim - j0;                 // of this pack's 8 elements (<= 0: none, >= 8: all)
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if (j >= allowed) { yv[k][j] = 0.0f; gv[k][j] = 0.0f; }       // whatever sits beyond the mask never counts
                dot = fmaf(gv[k][j], yv[k][j], dot);
            }
        }
        dot = group_sum<LPR>(dot);
#pragma unroll
        for (int k = 0; k < VPL; ++k) {
            const int idx = sub + k * LPR;
            if (row[r] < g.nrows && idx < nv) {
                float o[8];
#pragma unroll
                for (int j = 0; j < 8; ++j)      // outside the allowed set y and dy are zero here: the sum with +0 turns the product's -0 into +0
                    o[j] = g.scale * yv[k][j] * (gv[k][j] - dot) + 0.0f;
                store8<T, kNT>(dx + ro + idx * kPack, o);
            }
        }
    }
}

// ---- long rows (2048 < k_len <= 16384): one workgroup per row, VPL packs per thread in
// registers, the two reductions cross the four waves through LDS.  Still one read of the row.
template <typename T, int VPL, bool DROP>
__global__ __launch_bounds__(256) void softmax_fwd_wide(T* y, T* __restrict__ yd, const T* x,
                                                        SoftmaxLens len, SoftmaxGeom g, DropoutParams d)
{
    __shared__ float red[4];
    const int64_t row = blockIdx.x;
    const int nv = g.k_len / kPack;
    const int limit = row_limit(g, len, row);
    const int64_t ro = row * g.k_len;
    RawPack<T> raw[VPL];
#pragma unroll
    for (int k = 0; k < VPL; ++k) {
        const int j0 = (threadIdx.x + k * 256) * kPack;
        if (j0 < limit) raw[k] = load_raw<T, kNT>(x + ro + j0);
        else raw[k] = zero_raw<T>();
    }
    float v[VPL][8];
    float mx = -INFINITY;
#pragma unroll
    for (int k = 0; k < VPL; ++k) {
        const int j0 = (threadIdx.x + k * 256) * kPack;
        unpack<T>(raw[k], v[k]);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            v[k][j] = (j0 + j < limit) ? v[k][j] * g.scale : -INFINITY;
            mx = fmaxf(mx, v[k][j]);
        }
    }
    mx = block_allreduce<4, OpMax>(mx, red);
    const float mxs = (limit > 0 ? mx : 0.0f) * kLog2e;
    float z = 0.0f;
#pragma unroll
    for (int k = 0; k < VPL; ++k)
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float e = __builtin_amdgcn_exp2f(fmaf(v[k][j], kLog2e, -mxs));
            v[k][j] = e;
            z += e;
        }
    z = block_allreduce<4, OpSum>(z, red);
    const float inv = limit > 0 ? 1.0f / z : 0.0f;
#pragma unroll
    for (int k = 0; k < VPL; ++k) {
        const int idx = threadIdx.x + k * 256;
        if (idx < nv) {
            float o[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) o[j] = v[k][j] * inv;
            store8<T, kNT>(y + ro + idx * kPack, o);
            if constexpr (DROP) {
                if (idx * kPack < limit) {
                    float kf[8];
                    dropout_factors8(d, static_cast<uint64_t>(row) * nv + idx, kf);
#pragma unroll
                    for (int j = 0; j < 8; ++j) o[j] *= kf[j];
                }
                store8<T, kNT>(yd + ro + idx * kPack, o);
            }
        }
    }
}

template <typename T, int VPL, bool DROP>
__global__ __launch_bounds__(256) void softmax_bwd_wide(T* dx, const T* dy, const T* __restrict__ y,
                                                        SoftmaxLens len, SoftmaxGeom g, DropoutParams d)
{
    __shared__ float red[4];
    const int64_t row = blockIdx.x;
    const int nv = g.k_len / kPack;
    const int limit = row_limit(g, len, row);
    const int64_t ro = row * g.k_len;
    RawPack<T> ry[VPL], rg[VPL];
#pragma unroll
    for (int k = 0; k < VPL; ++k) {
        const int j0 = (threadIdx.x + k * 256) * kPack;
        if (j0 < limit) {
            ry[k] = load_raw<T, kNT>(y + ro + j0);
            rg[k] = load_raw<T, kNT>(dy + ro + j0);
        } else {
            ry[k] = zero_raw<T>();
            rg[k] = zero_raw<T>();
        }
    }
    float yv[VPL][8], gv[VPL][8];
    float dot = 0.0f;
#pragma unroll
    for (int k = 0; k < VPL; ++k) {
        const int idx = threadIdx.x + k * 256;
        const int j0 = idx * kPack;
        unpack<T>(ry[k], yv[k]);
        unpack<T>(rg[k], gv[k]);
        if constexpr (DROP) {
            if (j0 < limit) {
                float kf[8];
                dropout_factors8(d, static_cast<uint64_t>(row) * nv + idx, kf);
#pragma unroll
                for (int j = 0; j < 8; ++j) gv[k][j] *= kf[j];
            }
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (j0 + j >= limit) yv[k][j] = 0.0f;
            dot = fmaf(gv[k][j], yv[k][j], dot);
        }
    }
    dot = block_allreduce<4, OpSum>(dot, red);
#pragma unroll
    for (int k = 0; k < VPL; ++k) {
        const int idx = threadIdx.x + k * 256;
        if (idx < nv) {
            float o[8];
#pragma unroll
            for (int j = 0; j < 8; ++j)
                o[j] = (idx * kPack + j < limit) ? g.scale * yv[k][j] * (gv[k][j] - dot) : 0.0f;
            store8<T, kNT>(dx + ro + idx * kPack, o);
        }
    }
}

// ---- rows whose length is not a multiple of 8 (or whose tensors are not 16-byte aligned), up
// to 2048 keys: the common case of a sequence-to-sequence batch.  Same register-resident,
// read-once scheme with ELEMENT-granular lanes: lane `sub` of a row's group holds elements
// sub, sub + LPR, ... (2-byte accesses, contiguous across the wave).  Dropout decisions are
// still one Philox call per aligned pack of the flat tensor: the workgroup's rows cover one
// contiguous element range, its threads compute the keep bits of the packs of that range
// into LDS, and every element then picks its bit.
template <int LPR>
__device__ __forceinline__ float elem_max(float v, float* lds)
{
    if constexpr (LPR == 256) return block_allreduce<4, OpMax>(v, lds);
    else return group_max<LPR>(v);
}
template <int LPR>
__device__ __forceinline__ float elem_sum(float v, float* lds)
{
    if constexpr (LPR == 256) return block_allreduce<4, OpSum>(v, lds);
    else return group_sum<LPR>(v);
}

// keep bits of the packs that the rows [row0, row0 + rpb) touch; returns the first pack's index
template <int NBYTES>
__device__ __forceinline__ int64_t elem_keep_mask(uint8_t (&keep)[NBYTES], const SoftmaxGeom& g, const DropoutParams& d,
                                                  int64_t row0, int rpb)
{
    const int64_t e_begin = row0 * g.k_len;
    const int64_t r_end = row0 + rpb < g.nrows ? row0 + rpb : g.nrows;
    const int64_t p_begin = e_begin >> 3, p_end = (r_end * g.k_len + 7) >> 3;
    for (int64_t pk = p_begin + threadIdx.x; pk < p_end; pk += 256)
        keep[pk - p_begin] = static_cast<uint8_t>(dropout_keep_bits8(d, static_cast<uint64_t>(pk)));
    __syncthreads();
    return p_begin;
}

// The rows of a workgroup are one contiguous element range [e0, e1) of the tensor.  Global memory
// is touched in aligned 128-bit packs only: the packs that cover the range are copied to LDS (and
// results back from LDS), the lanes work on LDS with 2-byte accesses.  The first and the last pack
// may be shared with the neighbouring workgroups: reading them is harmless, writing is done element
// by element for the part that belongs here.  Element i of LDS = element (e0 & ~7) + i of the tensor.
constexpr bool kSmStage = true;

template <typename T>
__device__ __forceinline__ void stage_in(T* buf, const T* src, int64_t e0, int64_t e1, int64_t total)
{
    const int64_t p0 = e0 >> 3, p1 = (e1 + 7) >> 3;
    for (int64_t pk = p0 + threadIdx.x; pk < p1; pk += 256) {
        T* dst = buf + (pk - p0) * kPack;
        const int64_t base = pk * kPack;
        if (base + kPack <= total) {
            *reinterpret_cast<RawPack<T>*>(dst) = load_raw<T, kNT>(src + base);
        } else {
            for (int j = 0; j < kPack; ++j)
                if (base + j < total) dst[j] = src[base + j];
        }
    }
}

template <typename T>
__device__ __forceinline__ void stage_out(T* dstg, const T* buf, int64_t e0, int64_t e1)
{
    const int64_t p0 = e0 >> 3, p1 = (e1 + 7) >> 3;
    for (int64_t pk = p0 + threadIdx.x; pk < p1; pk += 256) {
        const T* from = buf + (pk - p0) * kPack;
        const int64_t base = pk * kPack;
        if (base >= e0 && base + kPack <= e1) {
            store_raw<T, kNT>(dstg + base, *reinterpret_cast<const RawPack<T>*>(from));
        } else {
            for (int j = 0; j < kPack; ++j)
                if (base + j >= e0 && base + j < e1) dstg[base + j] = from[j];
        }
    }
}

template <typename T, int LPR, int EPL, bool DROP>
__global__ __launch_bounds__(256) void softmax_fwd_elem(T* y, T* __restrict__ yd, const T* x,
                                                        SoftmaxLens len, SoftmaxGeom g, DropoutParams d)
{
    constexpr int RPB = 256 / LPR;
    constexpr int NBUF = kSmStage ? 256 * EPL + 16 : 8;      // elements per staged tensor
    __shared__ float red[4];
    __shared__ uint8_t keep[DROP ? 256 * EPL / 8 + 8 : 1];
    __shared__ __align__(16) T xs[NBUF];
    __shared__ __align__(16) T ys[NBUF];
    __shared__ __align__(16) T yds[DROP ? NBUF : 8];
    const int sub = threadIdx.x % LPR;
    const int64_t row0 = static_cast<int64_t>(blockIdx.x) * RPB;
    const int64_t row = row0 + threadIdx.x / LPR;
    const bool rv = row < g.nrows;
    const int limit = rv ? row_limit(g, len, row) : 0;
    const int64_t ro = row * g.k_len;
    const int64_t e0 = row0 * g.k_len;
    const int64_t e1 = (row0 + RPB < g.nrows ? row0 + RPB : g.nrows) * g.k_len;
    const int lo = static_cast<int>(ro - (e0 & ~static_cast<int64_t>(7)));     // this row's first element in LDS
    if constexpr (kSmStage) {
        stage_in<T>(xs, x, e0, e1, g.nrows * g.k_len);
        __syncthreads();
    }
    float v[EPL];
#pragma unroll
    for (int m = 0; m < EPL; ++m) {
        const int j = sub + m * LPR;
        if constexpr (kSmStage) v[m] = j < limit ? to_f32<T>(xs[lo + j]) * g.scale : -INFINITY;
        else v[m] = j < limit ? to_f32<T>(x[ro + j]) * g.scale : -INFINITY;
    }
    int64_t p_begin = 0;
    if constexpr (DROP) p_begin = elem_keep_mask(keep, g, d, row0, RPB);
    float mx = v[0];
#pragma unroll
    for (int m = 1; m < EPL; ++m) mx = fmaxf(mx, v[m]);
    mx = elem_max<LPR>(mx, red);
    const float mxs = (limit > 0 ? mx : 0.0f) * kLog2e;
    float z = 0.0f;
#pragma unroll
    for (int m = 0; m < EPL; ++m) {
        v[m] = __builtin_amdgcn_exp2f(fmaf(v[m], kLog2e, -mxs));
        z += v[m];
    }
    z = elem_sum<LPR>(z, red);
    const float inv = limit > 0 ? 1.0f / z : 0.0f;
#pragma unroll
    for (int m = 0; m < EPL; ++m) {
        const int j = sub + m * LPR;
        if (rv && j < g.k_len) {
            const float o = v[m] * inv;           // 0 beyond the limit (exp2(-inf)), and on empty rows
            if constexpr (kSmStage) ys[lo + j] = from_f32<T>(o);
            else y[ro + j] = from_f32<T>(o);
            if constexpr (DROP) {
                const int64_t e = ro + j;
                const bool kept = (keep[(e >> 3) - p_begin] >> (e & 7)) & 1;
                if constexpr (kSmStage) yds[lo + j] = from_f32<T>(kept ? o * d.scale : 0.0f);
                else yd[e] = from_f32<T>(kept ? o * d.scale : 0.0f);
            }
        }
    }
    if constexpr (kSmStage) {
        __syncthreads();
        stage_out<T>(y, ys, e0, e1);
        if constexpr (DROP) stage_out<T>(yd, yds, e0, e1);
    }
}

template <typename T, int LPR, int EPL, bool DROP>
__global__ __launch_bounds__(256) void softmax_bwd_elem(T* dx, const T* dy, const T* __restrict__ y,
                                                        SoftmaxLens len, SoftmaxGeom g, DropoutParams d)
{
    constexpr int RPB = 256 / LPR;
    constexpr int NBUF = kSmStage ? 256 * EPL + 16 : 8;
    __shared__ float red[4];
    __shared__ uint8_t keep[DROP ? 256 * EPL / 8 + 8 : 1];
    __shared__ __align__(16) T ysh[NBUF];
    __shared__ __align__(16) T gsh[NBUF];        // dy in, dx out
    const int sub = threadIdx.x % LPR;
    const int64_t row0 = static_cast<int64_t>(blockIdx.x) * RPB;
    const int64_t row = row0 + threadIdx.x / LPR;
    const bool rv = row < g.nrows;
    const int limit = rv ? row_limit(g, len, row) : 0;
    const int64_t ro = row * g.k_len;
    const int64_t e0 = row0 * g.k_len;
    const int64_t e1 = (row0 + RPB < g.nrows ? row0 + RPB : g.nrows) * g.k_len;
    const int lo = static_cast<int>(ro - (e0 & ~static_cast<int64_t>(7)));
    if constexpr (kSmStage) {
        stage_in<T>(ysh, y, e0, e1, g.nrows * g.k_len);
        stage_in<T>(gsh, dy, e0, e1, g.nrows * g.k_len);
        __syncthreads();
    }
    float yv[EPL], gv[EPL];
#pragma unroll
    for (int m = 0; m < EPL; ++m) {
        const int j = sub + m * LPR;
        if constexpr (kSmStage) {
            yv[m] = j < limit ? to_f32<T>(ysh[lo + j]) : 0.0f;
            gv[m] = j < limit ? to_f32<T>(gsh[lo + j]) : 0.0f;
        } else {
            yv[m] = j < limit ? to_f32<T>(y[ro + j]) : 0.0f;
            gv[m] = j < limit ? to_f32<T>(dy[ro + j]) : 0.0f;
        }
    }
    if constexpr (DROP) {
        const int64_t p_begin = elem_keep_mask(keep, g, d, row0, RPB);
#pragma unroll
        for (int m = 0; m < EPL; ++m) {
            const int j = sub + m * LPR;
            if (j < limit) {
                const int64_t e = ro + j;
                const bool kept = (keep[(e >> 3) - p_begin] >> (e & 7)) & 1;
                gv[m] = kept ? gv[m] * d.scale : 0.0f;
            }
        }
    }
    float dot = 0.0f;
#pragma unroll
    for (int m = 0; m < EPL; ++m) dot = fmaf(gv[m], yv[m], dot);
    dot = elem_sum<LPR>(dot, red);
#pragma unroll
    for (int m = 0; m < EPL; ++m) {
        const int j = sub + m * LPR;
        if (rv && j < g.k_len) {
            const T o = from_f32<T>(j < limit ? g.scale * yv[m] * (gv[m] - dot) : 0.0f);
            if constexpr (kSmStage) gsh[lo + j] = o;      // every element is read and written by one lane only
            else dx[ro + j] = o;
        }
    }
    if constexpr (kSmStage) {
        __syncthreads();
        stage_out<T>(dx, gsh, e0, e1);
    }
}

// ---- generic path: any k_len; TH = 64 (one wave per row) or 256 lanes (one workgroup per row), element-strided,
// row re-read from cache
template <typename T, int TH>
__global__ __launch_bounds__(256) void softmax_fwd_generic(T* y, T* __restrict__ yd, const T* x,
                                                           SoftmaxLens key_len, SoftmaxGeom g,
                                                           DropoutParams d)
{
    __shared__ float lds[4];
    constexpr int R = 256 / TH;
    const int lane = threadIdx.x % TH;
    const int64_t row = static_cast<int64_t>(blockIdx.x) * R + threadIdx.x / TH;
    if (row >= g.nrows) return;               // whole waves (TH = 64) or the whole workgroup (TH = 256) leave together
    const int limit = row_limit(g, key_len, row);
    const int64_t ro = row * g.k_len;
    float mx = -INFINITY;
    for (int j = lane; j < limit; j += TH) mx = fmaxf(mx, to_f32<T>(x[ro + j]) * g.scale);
    if constexpr (TH == 64) mx = group_max<64>(mx);
    else mx = block_allreduce<4, OpMax>(mx, lds);
    const float mxs = (limit > 0 ? mx : 0.0f) * kLog2e;
    float z = 0.0f;
    for (int j = lane; j < limit; j += TH) z += __builtin_amdgcn_exp2f(fmaf(to_f32<T>(x[ro + j]) * g.scale, kLog2e, -mxs));
    if constexpr (TH == 64) z = group_sum<64>(z);
    else z = block_allreduce<4, OpSum>(z, lds);
    const float inv = limit > 0 ? 1.0f / z : 0.0f;
    for (int j = lane; j < g.k_len; j += TH) {
        float o = 0.0f;
        if (j < limit) o = __builtin_amdgcn_exp2f(fmaf(to_f32<T>(x[ro + j]) * g.scale, kLog2e, -mxs)) * inv;
        y[ro + j] = from_f32<T>(o);
        if (yd) yd[ro + j] = from_f32<T>(o * dropout_factor1(d, static_cast<uint64_t>(ro + j)));
    }
}

template <typename T, int TH>
__global__ __launch_bounds__(256) void softmax_bwd_generic(T* dx, const T* dy, const T* __restrict__ y,
                                                           SoftmaxLens key_len, SoftmaxGeom g,
                                                           DropoutParams d)
{
    __shared__ float lds[4];
    constexpr int R = 256 / TH;
    const int lane = threadIdx.x % TH;
    const int64_t row = static_cast<int64_t>(blockIdx.x) * R + threadIdx.x / TH;
    if (row >= g.nrows) return;
    const int limit = row_limit(g, key_len, row);
    const int64_t ro = row * g.k_len;
    float dot = 0.0f;
    for (int j = lane; j < limit; j += TH) {
        float gg = to_f32<T>(dy[ro + j]);
        if (d.on) gg *= dropout_factor1(d, static_cast<uint64_t>(ro + j));
        dot = fmaf(gg, to_f32<T>(y[ro + j]), dot);
    }
    if constexpr (TH == 64) dot = group_sum<64>(dot);
    else dot = block_allreduce<4, OpSum>(dot, lds);
    for (int j = lane; j < g.k_len; j += TH) {
        float o = 0.0f;
        if (j < limit) {
            float gg = to_f32<T>(dy[ro + j]);
            if (d.on) gg *= dropout_factor1(d, static_cast<uint64_t>(ro + j));
            o = g.scale * to_f32<T>(y[ro + j]) * (gg - dot);
        }
        dx[ro + j] = from_f32<T>(o);
    }
}

// ------------------------------------------------------------------ dispatch
struct SmShape { int lpr, vpl; };

inline SmShape softmax_shape(int k_len)
{
    if (k_len % kPack != 0) return {0, 0};
    const int nv = k_len / kPack;
    if (nv <= 1) return {1, 1};
    if (nv <= 2) return {2, 1};
    if (nv <= 4) return {4, 1};
    if (nv <= 8) return {8, 1};
    if (nv <= 16) return {16, 1};
    if (nv <= 32) return {32, 1};
    if (nv <= 64) return {64, 1};
    if (nv <= 128) return {64, 2};
    if (nv <= 192) return {64, 3};
    if (nv <= 256) return {64, 4};
    if (nv <= 512) return {256, 2};      // one workgroup per row from here on
    if (nv <= 1024) return {256, 4};
    if (nv <= 2048) return {256, 8};
    return {0, 0};
}

// element-granular buckets: lanes per row, elements per lane.  Few lanes per row with up to 8
// elements each (more rows per workgroup, more loads in flight per lane) measured 2x faster
// than one element per lane on 64 lanes.
inline SmShape softmax_elem_shape(int k_len)
{
    if (k_len <= 8) return {8, 1};
    if (k_len <= 16) return {8, 2};
    if (k_len <= 32) return {8, 4};
    if (k_len <= 64) return {8, 8};
    if (k_len <= 128) return {16, 8};
    if (k_len <= 256) return {32, 8};
    if (k_len <= 512) return {64, 8};
    if (k_len <= 1024) return {256, 4};
    if (k_len <= 2048) return {256, 8};
    return {0, 0};
}
#define LSQ_SM_ELEM_CASES(X) X(8, 1) X(8, 2) X(8, 4) X(8, 8) X(16, 8) X(32, 8) X(64, 8) X(256, 4) X(256, 8)

// ---- launch shapes of the register path for rows of up to 2048 keys, and their choice at run time.
// The paper copes with the spread of softmax shapes by keeping several templates and searching for
// the best parameters before training starts (Sec. IV-B, Softmax, last paragraph).  Here a template
// is (lanes per row, packs per lane, rows per lane group); every row length has a short list of
// candidates, the first of which is the default, and lsq_softmax_tune times them on the caller's
// own buffers and records the winner per (row-length bucket, mask kind, dropout, storage width,
// direction), which the dispatch then uses.
struct SmCand { int lpr, vpl, rpt; };
constexpr int kSmBuckets = 10, kSmMaxCand = 4;
struct SmBucket { int max_packs, n; SmCand c[kSmMaxCand]; };
// Defaults measured on MI355X at the shapes of the five configurations (fp16): rows of 128 keys under a
// key-padding mask take 18.3 / 16.3 us (forward with attention dropout / backward) as 8 lanes x 2 packs
// against 20.6 / 18.2 us as 16 lanes x 1 pack, two rows per group: each of a lane's two loads then covers
// whole 128-byte lines of 8 rows, the first of which is issued before the sentence length has arrived.
static const SmBucket kSmTable[kSmBuckets] = {
    {1, 2, {{1, 1, 2}, {1, 1, 1}}},
    {2, 2, {{2, 1, 2}, {2, 1, 1}}},
    {4, 2, {{4, 1, 2}, {4, 1, 1}}},
    {8, 3, {{8, 1, 2}, {8, 1, 1}, {4, 2, 1}}},
    {16, 4, {{8, 2, 1}, {16, 1, 2}, {16, 1, 1}, {8, 2, 2}}},
    {32, 4, {{16, 2, 1}, {32, 1, 2}, {32, 1, 1}, {8, 4, 1}}},      // 256 keys, key padding: 32.0 / 26.7 us against 38.5 / 34.6 us as 32 x 1, two rows
    {64, 3, {{32, 2, 1}, {64, 1, 2}, {64, 1, 1}}},      // 512 keys, no mask: 44.5 / 63.9 us against 45.5 / 66.6 us as 64 x 1, two rows
    {128, 2, {{64, 2, 1}, {32, 4, 1}}},
    {192, 1, {{64, 3, 1}}},
    {256, 1, {{64, 4, 1}}},
};
#define LSQ_SM_CASES(X)                                                                                      \
    X(1, 1, 1) X(1, 1, 2) X(2, 1, 1) X(2, 1, 2) X(4, 1, 1) X(4, 1, 2) X(8, 1, 1) X(8, 1, 2) X(4, 2, 1)       \
    X(8, 2, 1) X(8, 2, 2) X(16, 1, 1) X(16, 1, 2) X(32, 1, 1) X(32, 1, 2) X(16, 2, 1) X(8, 4, 1)             \
    X(64, 1, 1) X(64, 1, 2) X(32, 2, 1) X(64, 2, 1) X(32, 4, 1) X(64, 3, 1) X(64, 4, 1)

inline int sm_bucket(int k_len)
{
    const int nv = k_len / kPack;
    for (int b = 0; b < kSmBuckets; ++b)
        if (nv <= kSmTable[b].max_packs) return b;
    return -1;
}

// what lsq_softmax_tune has recorded: [bucket][mask kind][dropout][storage width][direction], -1 = default
static std::atomic<signed char> sm_tuned[kSmBuckets][4][2][2][2];
static std::atomic<bool> sm_tuned_init{false};
static std::mutex sm_tuned_mutex;

inline void sm_tuned_prepare()
{
    if (sm_tuned_init.load(std::memory_order_acquire)) return;
    std::lock_guard<std::mutex> lock(sm_tuned_mutex);
    if (sm_tuned_init.load(std::memory_order_relaxed)) return;
    for (auto& a : sm_tuned) for (auto& b : a) for (auto& c : b) for (auto& e : c) for (auto& f : e) f.store(-1, std::memory_order_relaxed);
    sm_tuned_init.store(true, std::memory_order_release);
}

inline std::atomic<signed char>& sm_slot(int bucket, const SoftmaxLens& len, const SoftmaxGeom& g, bool drop, size_t elem, int dir)
{
    sm_tuned_prepare();
    const int mask = ((len.key || len.query) ? 1 : 0) + (g.causal ? 2 : 0);
    return sm_tuned[bucket][mask][drop ? 1 : 0][elem == 2 ? 0 : 1][dir];
}

// `forced` >= 0 picks that candidate of the row length's list; -1 the recorded one, else the default.
// A candidate with several rows per lane group falls back to one row when the grid would
// otherwise drop under kSmMinBlocks workgroups.
constexpr int64_t kSmMinBlocks = 1024;
inline SmCand sm_choose(const SoftmaxLens& len, const SoftmaxGeom& g, bool drop, size_t elem, int dir, int forced)
{
    const int b = sm_bucket(g.k_len);
    int pick = forced;
    if (pick < 0) pick = sm_slot(b, len, g, drop, elem, dir).load(std::memory_order_relaxed);
    if (pick < 0 || pick >= kSmTable[b].n) pick = 0;
    SmCand c = kSmTable[b].c[pick];
    if (c.rpt > 1 && ceil_div(g.nrows, 256 / c.lpr) < kSmMinBlocks * c.rpt) c.rpt = 1;
    return c;
}

template <typename T>
static lsq_status softmax_fwd_dispatch(void* y, void* yd, const void* x, SoftmaxLens key_len, const SoftmaxGeom& g,
                                       const DropoutParams& d, hipStream_t s, int forced = -1)
{
    T* yp = static_cast<T*>(y);
    T* ydp = static_cast<T*>(yd);
    const T* xp = static_cast<const T*>(x);
    const bool packs_ok = g.k_len % kPack == 0 && aligned16(y) && aligned16(yd) && aligned16(x);
    SmShape sh = packs_ok ? softmax_shape(g.k_len) : SmShape{0, 0};
    // the packed kernel of rows up to 2048 keys folds the scale into its exponent and needs it positive;
    // other scales (never an attention scale) take the element kernels, which multiply first
    if (sh.lpr != 0 && sh.lpr <= 64 && !(g.scale > 0.0f)) sh = SmShape{0, 0};
    const bool drop = d.on != 0;
    const SmShape es = softmax_elem_shape(g.k_len);
    if (sh.lpr == 0 && es.lpr != 0) {
        const dim3 egrid(static_cast<unsigned>(ceil_div(g.nrows, 256 / es.lpr)));
#define X(L, E)                                                                                              \
        if (es.lpr == L && es.vpl == E) {                                                                    \
            if (drop) hipLaunchKernelGGL((softmax_fwd_elem<T, L, E, true>), egrid, dim3(256), 0, s, yp, ydp, xp, key_len, g, d); \
            else hipLaunchKernelGGL((softmax_fwd_elem<T, L, E, false>), egrid, dim3(256), 0, s, yp, ydp, xp, key_len, g, d);    \
        }
        LSQ_SM_ELEM_CASES(X)
#undef X
        return launch_status();
    }
    if (sh.lpr == 0) {
        // long rows: a whole workgroup per row (four times the lanes, and rows of this length come in small numbers)
        if (g.k_len > 2048)
            hipLaunchKernelGGL((softmax_fwd_generic<T, 256>), dim3(static_cast<unsigned>(g.nrows)), dim3(256), 0, s,
                               yp, ydp, xp, key_len, g, d);
        else
            hipLaunchKernelGGL((softmax_fwd_generic<T, 64>), dim3(static_cast<unsigned>(ceil_div(g.nrows, 4))), dim3(256), 0, s,
                               yp, ydp, xp, key_len, g, d);
        return launch_status();
    }
    const dim3 block(256);
#define W(V)                                                                                                 \
    if (sh.lpr == 256 && sh.vpl == V) {                                                                      \
        const dim3 grid(static_cast<unsigned>(g.nrows));                                                     \
        if (drop) hipLaunchKernelGGL((softmax_fwd_wide<T, V, true>), grid, block, 0, s, yp, ydp, xp, key_len, g, d); \
        else hipLaunchKernelGGL((softmax_fwd_wide<T, V, false>), grid, block, 0, s, yp, ydp, xp, key_len, g, d);    \
    }
    W(2) W(4) W(8)
#undef W
    if (sh.lpr == 256) return launch_status();
    const SmCand c = sm_choose(key_len, g, drop, sizeof(T), 0, forced);
    const dim3 grid(static_cast<unsigned>(ceil_div(ceil_div(g.nrows, kSmWgFwd / c.lpr), c.rpt)));
#define X(L, V, R)                                                                                           \
    if (c.lpr == L && c.vpl == V && c.rpt == R) {                                                            \
        if (drop) hipLaunchKernelGGL((softmax_fwd_kernel<T, L, V, R, true>), grid, dim3(kSmWgFwd), 0, s, yp, ydp, xp, key_len, g, d); \
        else hipLaunchKernelGGL((softmax_fwd_kernel<T, L, V, R, false>), grid, dim3(kSmWgFwd), 0, s, yp, ydp, xp, key_len, g, d);    \
    }
    LSQ_SM_CASES(X)
#undef X
    return launch_status();
}

template <typename T>
static lsq_status softmax_bwd_dispatch(void* dx, const void* dy, const void* y, SoftmaxLens key_len,
                                       const SoftmaxGeom& g, const DropoutParams& d, hipStream_t s, int forced = -1)
{
    T* dxp = static_cast<T*>(dx);
    const T* dyp = static_cast<const T*>(dy);
    const T* yp = static_cast<const T*>(y);
    const bool packs_ok = g.k_len % kPack == 0 && aligned16(dx) && aligned16(dy) && aligned16(y);
    const SmShape sh = packs_ok ? softmax_shape(g.k_len) : SmShape{0, 0};
    const bool drop = d.on != 0;
    const SmShape es = softmax_elem_shape(g.k_len);
    if (sh.lpr == 0 && es.lpr != 0) {
        const dim3 egrid(static_cast<unsigned>(ceil_div(g.nrows, 256 / es.lpr)));
#define X(L, E)                                                                                              \
        if (es.lpr == L && es.vpl == E) {                                                                    \
            if (drop) hipLaunchKernelGGL((softmax_bwd_elem<T, L, E, true>), egrid, dim3(256), 0, s, dxp, dyp, yp, key_len, g, d); \
            else hipLaunchKernelGGL((softmax_bwd_elem<T, L, E, false>), egrid, dim3(256), 0, s, dxp, dyp, yp, key_len, g, d);    \
        }
        LSQ_SM_ELEM_CASES(X)
#undef X
        return launch_status();
    }
    if (sh.lpr == 0) {
        if (g.k_len > 2048)
            hipLaunchKernelGGL((softmax_bwd_generic<T, 256>), dim3(static_cast<unsigned>(g.nrows)), dim3(256), 0, s,
                               dxp, dyp, yp, key_len, g, d);
        else
            hipLaunchKernelGGL((softmax_bwd_generic<T, 64>), dim3(static_cast<unsigned>(ceil_div(g.nrows, 4))), dim3(256), 0, s,
                               dxp, dyp, yp, key_len, g, d);
        return launch_status();
    }
    const dim3 block(256);
#define W(V)                                                                                                 \
    if (sh.lpr == 256 && sh.vpl == V) {                                                                      \
        const dim3 grid(static_cast<unsigned>(g.nrows));                                                     \
        if (drop) hipLaunchKernelGGL((softmax_bwd_wide<T, V, true>), grid, block, 0, s, dxp, dyp, yp, key_len, g, d); \
        else hipLaunchKernelGGL((softmax_bwd_wide<T, V, false>), grid, block, 0, s, dxp, dyp, yp, key_len, g, d);    \
    }
    W(2) W(4) W(8)
#undef W
    if (sh.lpr == 256) return launch_status();
    const SmCand c = sm_choose(key_len, g, drop, sizeof(T), 1, forced);
    const dim3 grid(static_cast<unsigned>(ceil_div(ceil_div(g.nrows, kSmWgBwd / c.lpr), c.rpt)));
#define X(L, V, R)                                                                                           \
    if (c.lpr == L && c.vpl == V && c.rpt == R) {                                                            \
        if (drop) hipLaunchKernelGGL((softmax_bwd_kernel<T, L, V, R, true>), grid, dim3(kSmWgBwd), 0, s, dxp, dyp, yp, key_len, g, d); \
        else hipLaunchKernelGGL((softmax_bwd_kernel<T, L, V, R, false>), grid, dim3(kSmWgBwd), 0, s, dxp, dyp, yp, key_len, g, d);    \
    }
    LSQ_SM_CASES(X)
#undef X
    return launch_status();
}

static lsq_status softmax_check(const void* a, const void* b, int32_t batch, int32_t heads, int32_t q_len,
                                int32_t k_len, float scale, int dt, SoftmaxGeom* g)
{
    (void)a; (void)b;
    if (batch < 0 || heads < 0 || q_len < 0 || k_len < 0) return LSQ_INVALID_ARG;
    if (!(scale == scale) || isinf(scale)) return LSQ_INVALID_ARG;
    if (!valid_dtype(dt)) return LSQ_UNSUPPORTED_DTYPE;
    const int64_t rpb = static_cast<int64_t>(heads) * q_len;
    if (rpb > 0x7FFFFFFF) return LSQ_INVALID_ARG;
    g->nrows = static_cast<int64_t>(batch) * rpb;
    g->rows_per_batch = static_cast<int>(rpb);
    g->by_rows_per_batch = make_fastdiv(static_cast<uint32_t>(rpb));
    g->by_q_len = make_fastdiv(static_cast<uint32_t>(q_len));
    g->q_len = q_len;
    g->k_len = k_len;
    g->shift = k_len - q_len;
    g->scale = scale;
    if (g->nrows > 0x7FFFFFFF) return LSQ_INVALID_ARG;
    return LSQ_OK;
}

}  // namespace lsq

extern "C" lsq_status lsq_softmax_varlen_fwd(void* y, void* y_drop, const void* x, const int32_t* key_len,
                                             const int32_t* query_len, int32_t batch, int32_t heads, int32_t q_len,
                                             int32_t k_len, int32_t causal, float scale, float p_attn, uint64_t seed,
                                             uint64_t offset, lsq_dtype dt, void* stream)
{
    using namespace lsq;
    const SoftmaxLens len{key_len, query_len};
    SoftmaxGeom g;
    lsq_status st = softmax_check(y, x, batch, heads, q_len, k_len, scale, dt, &g);
    if (st != LSQ_OK) return st;
    g.causal = causal != 0;
    DropoutParams d;
    LSQ_REQUIRE(make_dropout(p_attn, seed, offset, &d));
    LSQ_REQUIRE((d.on != 0) == (y_drop != nullptr));
    if (g.nrows == 0 || k_len == 0) return LSQ_OK;
    LSQ_REQUIRE(y && x);
    LSQ_ALIGNED(y); LSQ_ALIGNED(y_drop); LSQ_ALIGNED(x);
    hipStream_t s = static_cast<hipStream_t>(stream);
    switch (dt) {
        case LSQ_F16: return softmax_fwd_dispatch<f16>(y, y_drop, x, len, g, d, s);
        case LSQ_BF16: return softmax_fwd_dispatch<bf16>(y, y_drop, x, len, g, d, s);
        default: return softmax_fwd_dispatch<float>(y, y_drop, x, len, g, d, s);
    }
}

extern "C" lsq_status lsq_softmax_fwd(void* y, void* y_drop, const void* x, const int32_t* key_len, int32_t batch,
                                      int32_t heads, int32_t q_len, int32_t k_len, int32_t causal, float scale,
                                      float p_attn, uint64_t seed, uint64_t offset, lsq_dtype dt, void* stream)
{
    return lsq_softmax_varlen_fwd(y, y_drop, x, key_len, nullptr, batch, heads, q_len, k_len, causal, scale, p_attn,
                                  seed, offset, dt, stream);
}

extern "C" lsq_status lsq_softmax_varlen_bwd(void* dx, const void* dy, const void* y, const int32_t* key_len,
                                             const int32_t* query_len, int32_t batch, int32_t heads, int32_t q_len,
                                             int32_t k_len, int32_t causal, float scale, float p_attn, uint64_t seed,
                                             uint64_t offset, lsq_dtype dt, void* stream)
{
    using namespace lsq;
    const SoftmaxLens len{key_len, query_len};
    SoftmaxGeom g;
    lsq_status st = softmax_check(dx, dy, batch, heads, q_len, k_len, scale, dt, &g);
    if (st != LSQ_OK) return st;
    g.causal = causal != 0;
    DropoutParams d;
    LSQ_REQUIRE(make_dropout(p_attn, seed, offset, &d));
    if (g.nrows == 0 || k_len == 0) return LSQ_OK;
    LSQ_REQUIRE(dx && dy && y);
    LSQ_ALIGNED(dx); LSQ_ALIGNED(dy); LSQ_ALIGNED(y);
    hipStream_t s = static_cast<hipStream_t>(stream);
    switch (dt) {
        case LSQ_F16: return softmax_bwd_dispatch<f16>(dx, dy, y, len, g, d, s);
        case LSQ_BF16: return softmax_bwd_dispatch<bf16>(dx, dy, y, len, g, d, s);
        default: return softmax_bwd_dispatch<float>(dx, dy, y, len, g, d, s);
    }
}

extern "C" lsq_status lsq_softmax_bwd(void* dx, const void* dy, const void* y, const int32_t* key_len, int32_t batch,
                                      int32_t heads, int32_t q_len, int32_t k_len, int32_t causal, float scale,
                                      float p_attn, uint64_t seed, uint64_t offset, lsq_dtype dt, void* stream)
{
    return lsq_softmax_varlen_bwd(dx, dy, y, key_len, nullptr, batch, heads, q_len, k_len, causal, scale, p_attn, seed,
                                  offset, dt, stream);
}

// ---- run-time choice of the launch shape (Sec. IV-B, Softmax: templates + parameter search before training)
extern "C" int32_t lsq_softmax_candidates(int32_t k_len)
{
    using namespace lsq;
    if (k_len <= 0 || k_len % kPack != 0) return 1;
    const int b = sm_bucket(k_len);
    return b < 0 ? 1 : kSmTable[b].n;
}

extern "C" lsq_status lsq_softmax_tune(int32_t* best_fwd, int32_t* best_bwd, float* us, void* y, void* y_drop, void* dx,
                                       const void* x, const void* dy, const int32_t* key_len, const int32_t* query_len,
                                       int32_t batch, int32_t heads, int32_t q_len, int32_t k_len, int32_t causal,
                                       float scale, float p_attn, uint64_t seed, uint64_t offset, lsq_dtype dt,
                                       int32_t force, int32_t reps, void* stream)
{
    using namespace lsq;
    const SoftmaxLens len{key_len, query_len};
    SoftmaxGeom g;
    lsq_status st = softmax_check(y, x, batch, heads, q_len, k_len, scale, dt, &g);
    if (st != LSQ_OK) return st;
    g.causal = causal != 0;
    DropoutParams d;
    LSQ_REQUIRE(make_dropout(p_attn, seed, offset, &d));
    LSQ_REQUIRE(force >= -2 && reps >= 1 && reps <= 10000);
    if (best_fwd) *best_fwd = 0;
    if (best_bwd) *best_bwd = 0;
    if (us)
        for (int i = 0; i < 2 * kSmMaxCand; ++i) us[i] = -1.0f;
    const int ncand = lsq_softmax_candidates(k_len);
    const size_t elem = dt == LSQ_F32 ? 4 : 2;
    const bool drop = d.on != 0;
    const int b = sm_bucket(k_len);
    if (force != -1) {                       // set (>= 0) or forget (-2): nothing is launched
        LSQ_REQUIRE(force < ncand);
        if (ncand > 1) {
            sm_slot(b, len, g, drop, elem, 0).store(static_cast<signed char>(force < 0 ? -1 : force));
            sm_slot(b, len, g, drop, elem, 1).store(static_cast<signed char>(force < 0 ? -1 : force));
        }
        if (best_fwd) *best_fwd = force < 0 ? 0 : force;
        if (best_bwd) *best_bwd = force < 0 ? 0 : force;
        return LSQ_OK;
    }
    if (g.nrows == 0 || k_len == 0 || ncand <= 1) return LSQ_OK;
    LSQ_REQUIRE(y && x && dx && dy);
    LSQ_REQUIRE(drop == (y_drop != nullptr));
    LSQ_ALIGNED(y); LSQ_ALIGNED(y_drop); LSQ_ALIGNED(x); LSQ_ALIGNED(dx); LSQ_ALIGNED(dy);
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return LSQ_LAUNCH_FAILED;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return LSQ_LAUNCH_FAILED; }
    auto launch = [&](int dir, int cand) -> lsq_status {
        if (dir == 0) {
            switch (dt) {
                case LSQ_F16: return softmax_fwd_dispatch<f16>(y, y_drop, x, len, g, d, s, cand);
                case LSQ_BF16: return softmax_fwd_dispatch<bf16>(y, y_drop, x, len, g, d, s, cand);
                default: return softmax_fwd_dispatch<float>(y, y_drop, x, len, g, d, s, cand);
            }
        }
        switch (dt) {
            case LSQ_F16: return softmax_bwd_dispatch<f16>(dx, dy, y, len, g, d, s, cand);
            case LSQ_BF16: return softmax_bwd_dispatch<bf16>(dx, dy, y, len, g, d, s, cand);
            default: return softmax_bwd_dispatch<float>(dx, dy, y, len, g, d, s, cand);
        }
    };
    st = LSQ_OK;
    for (int dir = 0; dir < 2 && st == LSQ_OK; ++dir) {
        int best = 0;
        float best_ms = 0.0f;
        for (int c = 0; c < ncand && st == LSQ_OK; ++c) {
            for (int i = 0; i < 2 && st == LSQ_OK; ++i) st = launch(dir, c);          // warm-up
            if (st != LSQ_OK) break;
            float ms = 0.0f;
            bool ok = hipEventRecord(e0, s) == hipSuccess;
            for (int i = 0; i < reps && st == LSQ_OK; ++i) st = launch(dir, c);
            ok = ok && hipEventRecord(e1, s) == hipSuccess && hipEventSynchronize(e1) == hipSuccess &&
                 hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
            if (!ok) st = LSQ_LAUNCH_FAILED;
            if (st != LSQ_OK) break;
            if (us) us[dir * kSmMaxCand + c] = ms * 1000.0f / static_cast<float>(reps);
            if (c == 0 || ms < best_ms) { best = c; best_ms = ms; }
        }
        if (st == LSQ_OK) {
            sm_slot(b, len, g, drop, elem, dir).store(static_cast<signed char>(best));
            if (dir == 0 && best_fwd) *best_fwd = best;
            if (dir == 1 && best_bwd) *best_bwd = best;
        }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return st;
}
