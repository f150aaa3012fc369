// Embedding layer, forward and backward (Sec. IV-A of the paper, embedding layer):
//   forward   y[t,:] = Dropout_p(scale * E[w_t,:] + P[l_t,:])
//   backward  dE[w,:] += scale * sum_{t: w_t = w} m_t (.) dy[t,:]      dP[l,:] += sum_b m (.) dy[b,l,:]
//
// The paper sums the gradient rows of a repeated token with atomicAdd.  Floating-point
// atomics make the result depend on the arrival order; here the sum has a fixed order
// instead, with no atomics at all:
//   1. rank: every token's position in the order sorted by (token id, position) is
//      COUNTED — tile against tile, 256 x 256 comparisons per workgroup out of LDS —
//      rather than sorted: counting is order-free, so the result is deterministic; the
//      same counts give the start and the length of each id segment;
//   2. scatter: order[rank[t]] = (t, id, segment start, segment length);
//   3. accumulate: a segment is cut into chunks of 32 rows; one workgroup per chunk sums
//      m (.) dy rows in ascending position in fp32 (eight rows in flight).  A segment of one
//      chunk is added to dE[w,:] at once; a longer one (a frequent token) leaves fp32 chunk
//      rows that a last kernel adds in chunk order: one rounding of dE per call either way.
// Tokens equal to pad_idx (or outside the vocabulary) produce zero rows and no gradient.
#include <limits.h>

#include "host.hpp"

namespace lsq {

#ifndef LSQ_NT
#define LSQ_NT 1
#endif
constexpr bool kNT = LSQ_NT != 0;
constexpr int kEmbWaves = 4;
constexpr int kTile = 256;

__device__ __forceinline__ bool emb_is_pad(int w, int vocab, int pad_idx) { return w == pad_idx || w < 0 || w >= vocab; }

template <typename T, bool DROP>
__global__ __launch_bounds__(256) void emb_fwd_cols(T* __restrict__ out, const int32_t* __restrict__ tokens,
                                                    const T* __restrict__ emb, const T* __restrict__ pos, int64_t rows,
                                                    int len, int ppr, int vocab, int pad_idx, float scale,
                                                    DropoutParams d)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int cp = blockIdx.x * 64 + lane;
    if (cp >= ppr) return;
    const int64_t stride = static_cast<int64_t>(gridDim.y) * kEmbWaves;
    for (int64_t t = static_cast<int64_t>(blockIdx.y) * kEmbWaves + wave; t < rows; t += stride) {
        const int w = tokens[t];
        const int64_t pack = t * ppr + cp;
        float o[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        if (!emb_is_pad(w, vocab, pad_idx)) {
            const int l = static_cast<int>(t % len);
            float e[8], pp[8];
            load8<T>(emb + (static_cast<int64_t>(w) * ppr + cp) * kPack, e);
            load8<T>(pos + (static_cast<int64_t>(l) * ppr + cp) * kPack, pp);
#pragma unroll
            for (int j = 0; j < 8; ++j) o[j] = fmaf(scale, e[j], pp[j]);
            if constexpr (DROP) {
                float k[8];
                dropout_factors8(d, static_cast<uint64_t>(pack), k);
#pragma unroll
                for (int j = 0; j < 8; ++j) o[j] *= k[j];
            }
        }
        store8<T, kNT>(out + pack * kPack, o);
    }
}

// sort key of a token: its id, with padding last
__device__ __forceinline__ int emb_key(int w, int vocab, int pad_idx) { return emb_is_pad(w, vocab, pad_idx) ? INT_MAX : w; }

// Three counts per (token i, tile jt), tile against tile out of LDS:
//   less[jt][i]   tokens j of the tile with key_j <  key_i          -> start of i's id segment
//   before[jt][i] tokens j of the tile with key_j == key_i, j < i   -> i's place inside the segment
//   equal[jt][i]  tokens j of the tile with key_j == key_i          -> length of the segment
__global__ __launch_bounds__(kTile) void emb_rank_partial(int32_t* __restrict__ partial, const int32_t* __restrict__ tokens,
                                                          int64_t rows, int ntiles, int vocab, int pad_idx)
{
    __shared__ int keys[kTile];
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kTile + threadIdx.x;
    const int64_t j0 = static_cast<int64_t>(blockIdx.y) * kTile;
    const int64_t jl = j0 + threadIdx.x;
    keys[threadIdx.x] = jl < rows ? emb_key(tokens[jl], vocab, pad_idx) : INT_MAX;
    __syncthreads();
    if (i >= rows) return;
    const int ki = emb_key(tokens[i], vocab, pad_idx);
    const int nj = static_cast<int>(min(static_cast<int64_t>(kTile), rows - j0));
    int less = 0, before = 0, equal = 0;
    for (int jj = 0; jj < nj; ++jj) {
        const int kj = keys[jj];                       // LDS broadcast
        less += kj < ki ? 1 : 0;
        equal += kj == ki ? 1 : 0;
        before += (kj == ki && j0 + jj < i) ? 1 : 0;
    }
    const int64_t plane = static_cast<int64_t>(ntiles) * rows;
    const int64_t o = static_cast<int64_t>(blockIdx.y) * rows + i;
    partial[o] = less;
    partial[plane + o] = before;
    partial[2 * plane + o] = equal;
}

// order[q] = { token position, key, segment start, segment length } for sorted position q
__global__ __launch_bounds__(256) void emb_scatter(int4* __restrict__ order, const int32_t* __restrict__ partial,
                                                   const int32_t* __restrict__ tokens, int64_t rows, int ntiles,
                                                   int vocab, int pad_idx)
{
    const int64_t t = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (t >= rows) return;
    const int64_t plane = static_cast<int64_t>(ntiles) * rows;
    int less = 0, before = 0, equal = 0;
    int jt = 0;
    for (; jt + 4 <= ntiles; jt += 4) {               // twelve loads in flight per trip (integer sums: any order)
        int a[4], b[4], c[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int64_t o = static_cast<int64_t>(jt + k) * rows + t;
            a[k] = partial[o]; b[k] = partial[plane + o]; c[k] = partial[2 * plane + o];
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) { less += a[k]; before += b[k]; equal += c[k]; }
    }
    for (; jt < ntiles; ++jt) {
        const int64_t o = static_cast<int64_t>(jt) * rows + t;
        less += partial[o];
        before += partial[plane + o];
        equal += partial[2 * plane + o];
    }
    order[less + before] = make_int4(static_cast<int>(t), emb_key(tokens[t], vocab, pad_idx), less, equal);
}

constexpr int kEmbChunk = 32;    // rows of one id summed by one workgroup

// slot of the partial row written by the chunk that starts at sorted position q (segment start s):
// a window of kEmbChunk sorted positions holds at most one chunk head that is not a segment start
// and at most one start of a segment longer than a chunk
__device__ __forceinline__ int64_t emb_slot(int64_t q, int64_t s) { return 2 * (q / kEmbChunk) + (q == s ? 1 : 0); }

// One workgroup per sorted entry; only chunk heads work.  A chunk sums up to kEmbChunk rows of one id
// in ascending position.  Segments of one chunk are added to dE at once; longer ones leave fp32
// partial rows that emb_combine sums in chunk order.
template <typename T, bool DROP>
__global__ __launch_bounds__(256) void emb_accumulate(T* __restrict__ demb, float* __restrict__ chunk_rows,
                                                      const T* __restrict__ dy, const int4* __restrict__ order,
                                                      int ppr, float scale, DropoutParams d)
{
    const int64_t q = blockIdx.x;
    const int4 me = order[q];                                    // uniform
    const int key = me.y;
    const int64_t s = me.z;
    const int len = me.w;
    if (key == INT_MAX) return;                                  // padding
    if ((q - s) % kEmbChunk != 0) return;                        // not a chunk head
    const int cnt = static_cast<int>(min(static_cast<int64_t>(kEmbChunk), s + len - q));
    const int lane = threadIdx.x & 63;
    const int tt = lane < cnt ? order[q + lane].x : 0;           // the chunk's token positions, one per lane
    for (int cp = threadIdx.x; cp < ppr; cp += 256) {
        float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        for (int u0 = 0; u0 < cnt; u0 += 8) {
            // eight rows in flight, then added in order
            RawPack<T> raw[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                if (u0 + k < cnt) {
                    const int64_t t = __builtin_amdgcn_readlane(tt, u0 + k);
                    raw[k] = load_raw<T, kNT>(dy + (t * ppr + cp) * kPack);
                } else {
                    raw[k] = zero_raw<T>();
                }
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                if (u0 + k < cnt) {
                    float g[8];
                    unpack<T>(raw[k], g);
                    if constexpr (DROP) {
                        const int64_t t = __builtin_amdgcn_readlane(tt, u0 + k);
                        float kf[8];
                        dropout_factors8(d, static_cast<uint64_t>(t * ppr + cp), kf);
#pragma unroll
                        for (int j = 0; j < 8; ++j) acc[j] = fmaf(g[j], kf[j], acc[j]);
                    } else {
#pragma unroll
                        for (int j = 0; j < 8; ++j) acc[j] += g[j];
                    }
                }
            }
        }
        if (len <= kEmbChunk) {
            T* dst = demb + (static_cast<int64_t>(key) * ppr + cp) * kPack;
            float o[8];
            load8<T>(dst, o);
#pragma unroll
            for (int j = 0; j < 8; ++j) o[j] = fmaf(scale, acc[j], o[j]);
            store8<T>(dst, o);
        } else {
            store8<float>(chunk_rows + (emb_slot(q, s) * ppr + cp) * kPack, acc);
        }
    }
}

// segments longer than a chunk: the workgroup of the segment start adds the chunk rows in chunk order
template <typename T>
__global__ __launch_bounds__(256) void emb_combine(T* __restrict__ demb, const float* __restrict__ chunk_rows,
                                                   const int4* __restrict__ order, int ppr, float scale)
{
    const int64_t q = blockIdx.x;
    const int4 me = order[q];
    if (me.y == INT_MAX || me.z != q || me.w <= kEmbChunk) return;
    const int nchunks = (me.w + kEmbChunk - 1) / kEmbChunk;
    for (int cp = threadIdx.x; cp < ppr; cp += 256) {
        float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        for (int c = 0; c < nchunks; ++c) {
            float r[8];
            load8<float>(chunk_rows + (emb_slot(q + static_cast<int64_t>(c) * kEmbChunk, q) * ppr + cp) * kPack, r);
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] += r[j];
        }
        T* dst = demb + (static_cast<int64_t>(me.y) * ppr + cp) * kPack;
        float o[8];
        load8<T>(dst, o);
#pragma unroll
        for (int j = 0; j < 8; ++j) o[j] = fmaf(scale, acc[j], o[j]);
        store8<T>(dst, o);
    }
}

// dP[l,:] += sum over the batch.  A workgroup owns 64 packs of one position; its four
// waves take every fourth sentence each (four loads in flight per wave) and their
// partial sums are added in wave order, so the result does not depend on timing.
template <typename T, bool DROP>
__global__ __launch_bounds__(256) void emb_dpos(T* __restrict__ dpos, const T* __restrict__ dy,
                                                const int32_t* __restrict__ tokens, int batch, int len, int ppr,
                                                int vocab, int pad_idx, DropoutParams d)
{
    constexpr int U = 4;
    __shared__ float sm[kEmbWaves - 1][8][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l = blockIdx.y;
    const int cp = blockIdx.x * 64 + lane;
    const bool active = cp < ppr;
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (active) {
        for (int b0 = wave; b0 < batch; b0 += kEmbWaves * U) {
            RawPack<T> raw[U];
            bool ok[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int b = b0 + u * kEmbWaves;
                ok[u] = false;
                if (b < batch) {
                    const int64_t t = static_cast<int64_t>(b) * len + l;
                    ok[u] = !emb_is_pad(tokens[t], vocab, pad_idx);
                    if (ok[u]) raw[u] = load_raw<T, true>(dy + (t * ppr + cp) * kPack);
                }
                if (!ok[u]) raw[u] = zero_raw<T>();
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (!ok[u]) continue;
                const int64_t pack = (static_cast<int64_t>(b0 + u * kEmbWaves) * len + l) * ppr + cp;
                float g[8];
                unpack<T>(raw[u], g);
                if constexpr (DROP) {
                    float kf[8];
                    dropout_factors8(d, static_cast<uint64_t>(pack), kf);
#pragma unroll
                    for (int j = 0; j < 8; ++j) acc[j] = fmaf(g[j], kf[j], acc[j]);
                } else {
#pragma unroll
                    for (int j = 0; j < 8; ++j) acc[j] += g[j];
                }
            }
        }
    }
    if (wave > 0) {
#pragma unroll
        for (int j = 0; j < 8; ++j) sm[wave - 1][j][lane] = acc[j];
    }
    __syncthreads();
    if (wave == 0 && active) {
#pragma unroll
        for (int w = 0; w < kEmbWaves - 1; ++w)
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] += sm[w][j][lane];
        T* dst = dpos + (static_cast<int64_t>(l) * ppr + cp) * kPack;
        float o[8];
        load8<T>(dst, o);
#pragma unroll
        for (int j = 0; j < 8; ++j) o[j] += acc[j];
        store8<T>(dst, o);
    }
}

// ---- generic paths (hidden not a multiple of 8): one element per thread
template <typename T>
__global__ __launch_bounds__(256) void emb_fwd_flat(T* __restrict__ out, const int32_t* __restrict__ tokens,
                                                    const T* __restrict__ emb, const T* __restrict__ pos, int64_t rows,
                                                    int len, int hidden, int vocab, int pad_idx, float scale,
                                                    DropoutParams d)
{
    const int64_t e = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (e >= rows * hidden) return;
    const int64_t t = e / hidden;
    const int i = static_cast<int>(e - t * hidden);
    const int w = tokens[t];
    float v = 0.0f;
    if (!emb_is_pad(w, vocab, pad_idx)) {
        v = fmaf(scale, to_f32<T>(emb[static_cast<int64_t>(w) * hidden + i]), to_f32<T>(pos[(t % len) * hidden + i]));
        if (d.t16) v *= dropout_factor1(d, static_cast<uint64_t>(e));
    }
    out[e] = from_f32<T>(v);
}

// one thread per (id segment head, column): walks the segment sequentially
template <typename T>
__global__ __launch_bounds__(256) void emb_accumulate_flat(T* __restrict__ demb, const T* __restrict__ dy,
                                                           const int4* __restrict__ order, int hidden, float scale,
                                                           DropoutParams d)
{
    const int64_t q = blockIdx.x;
    const int4 me = order[q];
    if (me.y == INT_MAX || me.z != q) return;
    for (int i = threadIdx.x; i < hidden; i += 256) {
        float acc = 0.0f;
        for (int c = 0; c < me.w; ++c) {
            const int64_t e = static_cast<int64_t>(order[q + c].x) * hidden + i;
            float g = to_f32<T>(dy[e]);
            if (d.t16) g *= dropout_factor1(d, static_cast<uint64_t>(e));
            acc += g;
        }
        T* dst = demb + static_cast<int64_t>(me.y) * hidden + i;
        *dst = from_f32<T>(fmaf(scale, acc, to_f32<T>(*dst)));
    }
}

template <typename T>
__global__ __launch_bounds__(256) void emb_dpos_flat(T* __restrict__ dpos, const T* __restrict__ dy,
                                                     const int32_t* __restrict__ tokens, int batch, int len, int hidden,
                                                     int vocab, int pad_idx, DropoutParams d)
{
    const int l = blockIdx.x;
    for (int i = threadIdx.x; i < hidden; i += 256) {
        float acc = 0.0f;
        for (int b = 0; b < batch; ++b) {
            const int64_t t = static_cast<int64_t>(b) * len + l;
            if (emb_is_pad(tokens[t], vocab, pad_idx)) continue;
            const int64_t e = t * hidden + i;
            float g = to_f32<T>(dy[e]);
            if (d.t16) g *= dropout_factor1(d, static_cast<uint64_t>(e));
            acc += g;
        }
        T* dst = dpos + static_cast<int64_t>(l) * hidden + i;
        *dst = from_f32<T>(to_f32<T>(*dst) + acc);
    }
}

template <typename T>
static lsq_status emb_fwd_dispatch(void* out, const int32_t* tokens, const void* emb, const void* pos, int64_t rows,
                                   int len, int hidden, int vocab, int pad_idx, float scale, const DropoutParams& d,
                                   hipStream_t s)
{
    T* o = static_cast<T*>(out);
    const T* e = static_cast<const T*>(emb);
    const T* p = static_cast<const T*>(pos);
    if (hidden % kPack == 0) {
        const int ppr = hidden / kPack;
        int64_t rb = ceil_div(rows, 4 * kEmbWaves);
        if (rb > 4096) rb = 4096;
        const dim3 grid(static_cast<unsigned>(ceil_div(ppr, 64)), static_cast<unsigned>(rb)), block(256);
        if (d.t16) hipLaunchKernelGGL((emb_fwd_cols<T, true>), grid, block, 0, s, o, tokens, e, p, rows, len, ppr, vocab, pad_idx, scale, d);
        else hipLaunchKernelGGL((emb_fwd_cols<T, false>), grid, block, 0, s, o, tokens, e, p, rows, len, ppr, vocab, pad_idx, scale, d);
    } else {
        hipLaunchKernelGGL((emb_fwd_flat<T>), dim3(static_cast<unsigned>(ceil_div(rows * hidden, 256))), dim3(256), 0, s,
                           o, tokens, e, p, rows, len, hidden, vocab, pad_idx, scale, d);
    }
    return launch_status();
}

template <typename T>
static lsq_status emb_bwd_dispatch(void* demb, void* dpos, const void* dy, const int32_t* tokens, void* ws,
                                   int batch, int len, int hidden, int vocab, int pad_idx, float scale,
                                   const DropoutParams& d, hipStream_t s)
{
    const int64_t rows = static_cast<int64_t>(batch) * len;
    const int ntiles = static_cast<int>(ceil_div(rows, kTile));
    // workspace: order[rows] (int4) | chunk rows [2*ceil(rows/chunk)][hidden] fp32 | rank counts [3][ntiles][rows] int32
    int4* order = reinterpret_cast<int4*>(ws);
    float* chunk_rows = reinterpret_cast<float*>(order + rows);
    int32_t* partial = reinterpret_cast<int32_t*>(chunk_rows + 2 * ceil_div(rows, kEmbChunk) * ((hidden + 7) / 8 * 8));
    T* de = static_cast<T*>(demb);
    T* dp = static_cast<T*>(dpos);
    const T* g = static_cast<const T*>(dy);
    // the dropout scale 1/(1-p) is carried by the per-element factors; `scale` is the embedding scale
    hipLaunchKernelGGL(emb_rank_partial, dim3(ntiles, ntiles), dim3(kTile), 0, s, partial, tokens, rows, ntiles, vocab, pad_idx);
    hipLaunchKernelGGL(emb_scatter, dim3(static_cast<unsigned>(ceil_div(rows, 256))), dim3(256), 0, s, order, partial,
                       tokens, rows, ntiles, vocab, pad_idx);
    const dim3 grid(static_cast<unsigned>(rows)), block(256);
    if (hidden % kPack == 0) {
        const int ppr = hidden / kPack;
        if (d.t16) hipLaunchKernelGGL((emb_accumulate<T, true>), grid, block, 0, s, de, chunk_rows, g, order, ppr, scale, d);
        else hipLaunchKernelGGL((emb_accumulate<T, false>), grid, block, 0, s, de, chunk_rows, g, order, ppr, scale, d);
        hipLaunchKernelGGL((emb_combine<T>), grid, block, 0, s, de, chunk_rows, order, ppr, scale);
        if (dp) {
            const dim3 pgrid(static_cast<unsigned>(ceil_div(ppr, 64)), static_cast<unsigned>(len));
            if (d.t16) hipLaunchKernelGGL((emb_dpos<T, true>), pgrid, dim3(256), 0, s, dp, g, tokens, batch, len, ppr, vocab, pad_idx, d);
            else hipLaunchKernelGGL((emb_dpos<T, false>), pgrid, dim3(256), 0, s, dp, g, tokens, batch, len, ppr, vocab, pad_idx, d);
        }
    } else {
        hipLaunchKernelGGL((emb_accumulate_flat<T>), grid, block, 0, s, de, g, order, hidden, scale, d);
        if (dp)
            hipLaunchKernelGGL((emb_dpos_flat<T>), dim3(len), dim3(256), 0, s, dp, g, tokens, batch, len, hidden, vocab,
                               pad_idx, d);
    }
    return launch_status();
}

}  // namespace lsq

extern "C" lsq_status lsq_embedding_fwd(void* out, const int32_t* tokens, const void* emb, const void* pos,
                                        int32_t batch, int32_t len, int32_t hidden, int32_t vocab, int32_t pad_idx,
                                        float scale, float p, uint64_t seed, uint64_t offset, lsq_dtype dt, void* stream)
{
    using namespace lsq;
    LSQ_REQUIRE(batch >= 0 && len >= 0 && hidden > 0 && vocab > 0);
    if (!valid_dtype(dt)) return LSQ_UNSUPPORTED_DTYPE;
    DropoutParams d;
    LSQ_REQUIRE(make_dropout(p, seed, offset, &d));
    const int64_t rows = static_cast<int64_t>(batch) * len;
    if (rows == 0) return LSQ_OK;
    LSQ_REQUIRE(out && tokens && emb && pos);
    LSQ_ALIGNED(out); LSQ_ALIGNED(emb); LSQ_ALIGNED(pos);
    LSQ_REQUIRE(ceil_div(rows * hidden, 256) <= 0x7FFFFFFF);
    hipStream_t s = static_cast<hipStream_t>(stream);
    switch (dt) {
        case LSQ_F16: return emb_fwd_dispatch<f16>(out, tokens, emb, pos, rows, len, hidden, vocab, pad_idx, scale, d, s);
        case LSQ_BF16: return emb_fwd_dispatch<bf16>(out, tokens, emb, pos, rows, len, hidden, vocab, pad_idx, scale, d, s);
        default: return emb_fwd_dispatch<float>(out, tokens, emb, pos, rows, len, hidden, vocab, pad_idx, scale, d, s);
    }
}

extern "C" lsq_status lsq_embedding_bwd(void* demb, void* dpos, const void* dy, const int32_t* tokens, int32_t batch,
                                        int32_t len, int32_t hidden, int32_t vocab, int32_t pad_idx, float scale,
                                        float p, uint64_t seed, uint64_t offset, void* workspace, size_t workspace_bytes,
                                        lsq_dtype dt, void* stream)
{
    using namespace lsq;
    LSQ_REQUIRE(batch >= 0 && len >= 0 && hidden > 0 && vocab > 0);
    if (!valid_dtype(dt)) return LSQ_UNSUPPORTED_DTYPE;
    DropoutParams d;
    LSQ_REQUIRE(make_dropout(p, seed, offset, &d));
    const int64_t rows = static_cast<int64_t>(batch) * len;
    if (rows == 0) return LSQ_OK;
    LSQ_REQUIRE(rows <= 0x7FFFFFFF / 2 && ceil_div(rows, kTile) <= 65535);
    LSQ_REQUIRE(!dpos || len <= 65535);       // one grid row per position
    LSQ_REQUIRE(demb && dy && tokens);
    LSQ_ALIGNED(demb); LSQ_ALIGNED(dpos); LSQ_ALIGNED(dy); LSQ_ALIGNED(workspace);
    const size_t need = lsq_workspace_bytes(LSQ_OP_EMBEDDING_BWD, rows, hidden);
    if (!workspace || workspace_bytes < need) return LSQ_WORKSPACE_TOO_SMALL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    void* ws = workspace;
    switch (dt) {
        case LSQ_F16: return emb_bwd_dispatch<f16>(demb, dpos, dy, tokens, ws, batch, len, hidden, vocab, pad_idx, scale, d, s);
        case LSQ_BF16: return emb_bwd_dispatch<bf16>(demb, dpos, dy, tokens, ws, batch, len, hidden, vocab, pad_idx, scale, d, s);
        default: return emb_bwd_dispatch<float>(demb, dpos, dy, tokens, ws, batch, len, hidden, vocab, pad_idx, scale, d, s);
    }
}
