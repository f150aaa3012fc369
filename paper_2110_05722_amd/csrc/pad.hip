// Padding removal: the real rows of every sentence of a padded [batch, max_len, hidden]
// tensor are stored back to back in a packed [sum(len), hidden] tensor, so that the
// row-wise operators (LayerNorm, bias+dropout+residual, bias+activation+dropout and
// the projections around them) run on sum(len) rows instead of batch*max_len.  The
// paper's conclusion names this as the optimisation to do next; its kernels as
// published always work on the padded batch.
//
// Pure data movement, bit-exact.  A wave owns 64 consecutive packs of a row (1 KiB)
// and walks down the padded rows four at a time (four loads in flight before the
// first store); rows of padding cost one scalar compare.  The packed position of a
// row comes from the prefix sums written by pad_offsets_kernel, so nothing is
// copied to the host and the sequence can be captured in a graph.
#include "host.hpp"

namespace lsq {

constexpr bool kNT = true;
constexpr int kPadWaves = 4;    // waves per workgroup
constexpr int kPadRows = 1;     // rows a wave has in flight: 6.1 / 6.9 us (remove / restore) at 4096 x 1024 and 9.6 / 9.7 at 8192 x 1280 against 7.5 / 8.3 and 10.1 / 10.1 with four

struct PadGeom {
    int64_t rows;           // batch * max_len
    int64_t packed_rows;    // capacity of the packed tensor, rows
    int batch, max_len, hidden;
    int ppr;                // packs per row (hidden / 8), pack path only
    FastDiv by_max_len;     // padded row -> sentence (rows are below 2^31)
};

// offsets[b] = number of real rows before sentence b; offsets[batch] = total.  One
// workgroup; chunks of 256 sentences are scanned with wave shifts and a running carry.
__global__ __launch_bounds__(256) void pad_offsets_kernel(int32_t* __restrict__ offsets,
                                                          const int32_t* __restrict__ key_len, int batch, int max_len)
{
    __shared__ int wave_total[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int carry = 0;
    for (int base = 0; base < batch; base += 256) {
        const int b = base + threadIdx.x;
        int v = 0;
        if (b < batch) v = key_len ? min(max(key_len[b], 0), max_len) : max_len;
        int incl = v;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int up = __shfl_up(incl, d, 64);
            if (lane >= d) incl += up;
        }
        if (lane == 63) wave_total[wave] = incl;
        __syncthreads();
        int before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const int t = wave_total[w];
            if (w < wave) before += t;
            total += t;
        }
        if (b < batch) offsets[b] = carry + before + incl - v;
        carry += total;
        __syncthreads();
    }
    if (threadIdx.x == 0) offsets[batch] = carry;
}

// packed row of padded row t, or -1 when t is padding (or would fall outside the packed tensor)
__device__ __forceinline__ int64_t packed_row(const PadGeom& g, const int32_t* __restrict__ offsets, int64_t t)
{
    if (t >= g.rows) return -1;
    const int b = static_cast<int>(fastdiv(static_cast<uint32_t>(t), g.by_max_len));
    const int i = static_cast<int>(t - static_cast<int64_t>(b) * g.max_len);
    const int first = offsets[b];
    const int lb = min(offsets[b + 1] - first, g.max_len);
    const int64_t r = static_cast<int64_t>(first) + i;
    return (i < lb && first >= 0 && r < g.packed_rows) ? r : -1;
}

// RESTORE = false: packed <- padded (rows of padding skipped);
// RESTORE = true:  padded <- packed, zeros on the padding.
template <typename T, bool RESTORE>
__global__ __launch_bounds__(256) void pad_move_kernel(T* __restrict__ dst, const T* __restrict__ src,
                                                       const int32_t* __restrict__ offsets, PadGeom g)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int cp = blockIdx.x * 64 + lane;
    if (cp >= g.ppr) return;
    const int64_t stride = static_cast<int64_t>(gridDim.y) * (kPadWaves * kPadRows);
    for (int64_t t0 = (static_cast<int64_t>(blockIdx.y) * kPadWaves + wave) * kPadRows; t0 < g.rows; t0 += stride) {
        int64_t pr[kPadRows];
        RawPack<T> raw[kPadRows];
#pragma unroll
        for (int k = 0; k < kPadRows; ++k) {
            pr[k] = packed_row(g, offsets, t0 + k);      // wave-uniform
            const int64_t from = RESTORE ? pr[k] : t0 + k;
            if (pr[k] >= 0) raw[k] = load_raw<T, kNT>(src + (from * g.ppr + cp) * kPack);
            else raw[k] = zero_raw<T>();
        }
#pragma unroll
        for (int k = 0; k < kPadRows; ++k) {
            if (RESTORE) {
                if (t0 + k < g.rows) store_raw<T, kNT>(dst + ((t0 + k) * g.ppr + cp) * kPack, raw[k]);
            } else {
                if (pr[k] >= 0) store_raw<T, kNT>(dst + (pr[k] * g.ppr + cp) * kPack, raw[k]);
            }
        }
    }
}

// any hidden size / alignment: one element per thread over the padded tensor
template <typename T, bool RESTORE>
__global__ __launch_bounds__(256) void pad_move_flat(T* __restrict__ dst, const T* __restrict__ src,
                                                     const int32_t* __restrict__ offsets, PadGeom g)
{
    const int64_t e = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (e >= g.rows * g.hidden) return;
    const int64_t t = e / g.hidden;
    const int c = static_cast<int>(e - t * g.hidden);
    const int64_t r = packed_row(g, offsets, t);
    if (RESTORE) {
        T zero;
        __builtin_memset(&zero, 0, sizeof(T));
        dst[e] = r >= 0 ? src[r * g.hidden + c] : zero;
    } else if (r >= 0) {
        dst[r * g.hidden + c] = src[e];
    }
}

template <typename T, bool RESTORE>
static lsq_status pad_dispatch(void* dst, const void* src, const int32_t* offsets, const PadGeom& g, hipStream_t s)
{
    T* d = static_cast<T*>(dst);
    const T* a = static_cast<const T*>(src);
    if (g.hidden % kPack == 0 && aligned16(dst) && aligned16(src)) {
        const int gx = static_cast<int>(ceil_div(g.ppr, 64));
        int64_t gy = ceil_div(g.rows, kPadWaves * kPadRows);
        const int64_t cap = 16384 / gx > 1 ? 16384 / gx : 1;      // about 64 workgroups per compute unit
        if (gy > cap) gy = cap;
        hipLaunchKernelGGL((pad_move_kernel<T, RESTORE>), dim3(static_cast<unsigned>(gx), static_cast<unsigned>(gy)),
                           dim3(256), 0, s, d, a, offsets, g);
    } else {
        hipLaunchKernelGGL((pad_move_flat<T, RESTORE>), dim3(static_cast<unsigned>(ceil_div(g.rows * g.hidden, 256))),
                           dim3(256), 0, s, d, a, offsets, g);
    }
    return launch_status();
}

static lsq_status pad_geom(PadGeom* g, int32_t batch, int32_t max_len, int32_t hidden, int64_t packed_rows, int dt)
{
    if (batch < 0 || max_len < 0 || hidden < 0 || packed_rows < 0) return LSQ_INVALID_ARG;
    if (!valid_dtype(dt)) return LSQ_UNSUPPORTED_DTYPE;
    g->rows = static_cast<int64_t>(batch) * max_len;
    if (g->rows > 0x7FFFFFFF) return LSQ_INVALID_ARG;          // offsets are int32
    g->packed_rows = packed_rows;
    g->batch = batch; g->max_len = max_len; g->hidden = hidden;
    g->by_max_len = make_fastdiv(static_cast<uint32_t>(max_len));
    g->ppr = hidden / kPack;
    if (ceil_div(g->rows * hidden, 256) > 0x7FFFFFFF) return LSQ_INVALID_ARG;
    return LSQ_OK;
}

template <bool RESTORE>
static lsq_status pad_move(void* dst, const void* src, const int32_t* offsets, int32_t batch, int32_t max_len,
                           int32_t hidden, int64_t packed_rows, int dt, void* stream)
{
    PadGeom g;
    lsq_status st = pad_geom(&g, batch, max_len, hidden, packed_rows, dt);
    if (st != LSQ_OK) return st;
    if (g.rows == 0 || hidden == 0) return LSQ_OK;
    const void* packed = RESTORE ? src : dst;
    const void* padded = RESTORE ? static_cast<const void*>(dst) : src;
    LSQ_REQUIRE(padded && offsets && (packed || packed_rows == 0));
    if (!RESTORE && packed_rows == 0) return LSQ_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    switch (dt) {
        case LSQ_F16: return pad_dispatch<f16, RESTORE>(dst, src, offsets, g, s);
        case LSQ_BF16: return pad_dispatch<bf16, RESTORE>(dst, src, offsets, g, s);
        default: return pad_dispatch<float, RESTORE>(dst, src, offsets, g, s);
    }
}

}  // namespace lsq

extern "C" lsq_status lsq_pad_offsets(int32_t* offsets, const int32_t* key_len, int32_t batch, int32_t max_len,
                                      void* stream)
{
    using namespace lsq;
    if (batch < 0 || max_len < 0) return LSQ_INVALID_ARG;
    if (static_cast<int64_t>(batch) * max_len > 0x7FFFFFFF) return LSQ_INVALID_ARG;
    LSQ_REQUIRE(offsets);
    hipLaunchKernelGGL(pad_offsets_kernel, dim3(1), dim3(256), 0, static_cast<hipStream_t>(stream), offsets, key_len,
                       batch, max_len);
    return launch_status();
}

extern "C" lsq_status lsq_pad_remove(void* packed, const void* padded, const int32_t* offsets, int32_t batch,
                                     int32_t max_len, int32_t hidden, int64_t packed_rows, lsq_dtype dt, void* stream)
{
    return lsq::pad_move<false>(packed, padded, offsets, batch, max_len, hidden, packed_rows, dt, stream);
}

extern "C" lsq_status lsq_pad_restore(void* padded, const void* packed, const int32_t* offsets, int32_t batch,
                                      int32_t max_len, int32_t hidden, int64_t packed_rows, lsq_dtype dt, void* stream)
{
    return lsq::pad_move<true>(padded, packed, offsets, batch, max_len, hidden, packed_rows, dt, stream);
}
