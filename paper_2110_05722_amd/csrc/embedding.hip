// Embedding layer, forward and backward (Sec. IV-A of the paper, embedding layer):
//   forward   y[t,:] = Dropout_p(scale * E[w_t,:] + P[l_t,:])
//   backward  dE[w,:] += scale * sum_{t: w_t = w} m_t (.) dy[t,:]      dP[l,:] += sum_b m (.) dy[b,l,:]
//
// The paper sums the gradient rows of a repeated token with atomicAdd.  Floating-point
// atomics make the result depend on the arrival order; here the sum has a fixed order
// instead, with no atomics at all:
//   1. rank: every token's position in the order sorted by (token id, position) is
//      COUNTED — tile against tile, 256 x 256 comparisons per workgroup out of LDS —
//      rather than sorted: counting is order-free, so the result is deterministic;
//   2. scatter: sorted[rank[t]] = t, sorted_id[rank[t]] = w_t;
//   3. accumulate: the workgroup of the first entry of each id segment walks the segment
//      (64 entries per read, in ascending position), sums m (.) dy rows in fp32 and adds
//      the total to dE[w,:] once (one rounding per call).
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

// partial[jt][i] = number of tokens j in tile jt with (key_j, j) < (key_i, i)
__global__ __launch_bounds__(kTile) void emb_rank_partial(int32_t* __restrict__ partial, const int32_t* __restrict__ tokens,
                                                          int64_t rows, int vocab, int pad_idx)
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
    int count = 0;
    for (int jj = 0; jj < nj; ++jj) {
        const int kj = keys[jj];                       // LDS broadcast
        count += (kj < ki || (kj == ki && j0 + jj < i)) ? 1 : 0;
    }
    partial[static_cast<int64_t>(blockIdx.y) * rows + i] = count;
}

__global__ __launch_bounds__(256) void emb_scatter(int32_t* __restrict__ sorted, int32_t* __restrict__ sorted_key,
                                                   const int32_t* __restrict__ partial, const int32_t* __restrict__ tokens,
                                                   int64_t rows, int ntiles, int vocab, int pad_idx)
{
    const int64_t t = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (t >= rows) return;
    int rank = 0;
    for (int jt = 0; jt < ntiles; ++jt) rank += partial[static_cast<int64_t>(jt) * rows + t];
    sorted[rank] = static_cast<int32_t>(t);
    sorted_key[rank] = emb_key(tokens[t], vocab, pad_idx);
}

// one workgroup per sorted entry; only the first entry of an id segment works
template <typename T, bool DROP>
__global__ __launch_bounds__(256) void emb_accumulate(T* __restrict__ demb, const T* __restrict__ dy,
                                                      const int32_t* __restrict__ sorted,
                                                      const int32_t* __restrict__ sorted_key, int64_t rows, int ppr,
                                                      float scale, DropoutParams d)
{
    const int64_t q = blockIdx.x;
    const int key = sorted_key[q];
    if (key == INT_MAX) return;                                  // padding
    if (q > 0 && sorted_key[q - 1] == key) return;               // not the head of its segment
    const int lane = threadIdx.x & 63;
    // the trip count is uniform over the wave: the ballot below needs all 64 lanes
    for (int cp0 = (threadIdx.x & ~63); cp0 < ppr; cp0 += 256) {
        const int cp = cp0 + lane;
        const bool active = cp < ppr;
        float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        for (int64_t c = q; c < rows; c += 64) {
            // 64 entries of the sorted order per read; the segment ends at the first other key
            const int64_t qq = c + lane;
            const int k = qq < rows ? sorted_key[qq] : INT_MAX;
            const int tt = qq < rows ? sorted[qq] : 0;
            const unsigned long long same = __ballot(k == key);
            const int run = same == ~0ull ? 64 : __builtin_ctzll(~same);   // leading entries of this id
            if (active) {
                for (int u = 0; u < run; ++u) {
                    const int64_t t = __builtin_amdgcn_readlane(tt, u);
                    const int64_t pack = t * ppr + cp;
                    float g[8];
                    load8<T, kNT>(dy + pack * kPack, g);
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
            if (run < 64) break;
        }
        if (active) {
            T* dst = demb + (static_cast<int64_t>(key) * ppr + cp) * kPack;
            float o[8];
            load8<T>(dst, o);
#pragma unroll
            for (int j = 0; j < 8; ++j) o[j] = fmaf(scale, acc[j], o[j]);
            store8<T>(dst, o);
        }
    }
}

// dP[l,:] += sum over the batch, in batch order; one workgroup per position
template <typename T, bool DROP>
__global__ __launch_bounds__(256) void emb_dpos(T* __restrict__ dpos, const T* __restrict__ dy,
                                                const int32_t* __restrict__ tokens, int batch, int len, int ppr,
                                                int vocab, int pad_idx, DropoutParams d)
{
    const int l = blockIdx.x;
    for (int cp = threadIdx.x; cp < ppr; cp += 256) {
        float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        for (int b = 0; b < batch; ++b) {
            const int64_t t = static_cast<int64_t>(b) * len + l;
            if (emb_is_pad(tokens[t], vocab, pad_idx)) continue;
            const int64_t pack = t * ppr + cp;
            float g[8];
            load8<T>(dy + pack * kPack, g);
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
                                                           const int32_t* __restrict__ sorted,
                                                           const int32_t* __restrict__ sorted_key, int64_t rows,
                                                           int hidden, float scale, DropoutParams d)
{
    const int64_t q = blockIdx.x;
    const int key = sorted_key[q];
    if (key == INT_MAX) return;
    if (q > 0 && sorted_key[q - 1] == key) return;
    for (int i = threadIdx.x; i < hidden; i += 256) {
        float acc = 0.0f;
        for (int64_t c = q; c < rows && sorted_key[c] == key; ++c) {
            const int64_t e = static_cast<int64_t>(sorted[c]) * hidden + i;
            float g = to_f32<T>(dy[e]);
            if (d.t16) g *= dropout_factor1(d, static_cast<uint64_t>(e));
            acc += g;
        }
        T* dst = demb + static_cast<int64_t>(key) * hidden + i;
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
static lsq_status emb_bwd_dispatch(void* demb, void* dpos, const void* dy, const int32_t* tokens, int32_t* ws,
                                   int batch, int len, int hidden, int vocab, int pad_idx, float scale,
                                   const DropoutParams& d, hipStream_t s)
{
    const int64_t rows = static_cast<int64_t>(batch) * len;
    const int ntiles = static_cast<int>(ceil_div(rows, kTile));
    int32_t* partial = ws;
    int32_t* sorted = ws + static_cast<int64_t>(ntiles) * rows;
    int32_t* sorted_key = sorted + rows;
    T* de = static_cast<T*>(demb);
    T* dp = static_cast<T*>(dpos);
    const T* g = static_cast<const T*>(dy);
    // the dropout scale 1/(1-p) is carried by the per-element factors; `scale` is the embedding scale
    hipLaunchKernelGGL(emb_rank_partial, dim3(ntiles, ntiles), dim3(kTile), 0, s, partial, tokens, rows, vocab, pad_idx);
    hipLaunchKernelGGL(emb_scatter, dim3(static_cast<unsigned>(ceil_div(rows, 256))), dim3(256), 0, s, sorted, sorted_key,
                       partial, tokens, rows, ntiles, vocab, pad_idx);
    if (hidden % kPack == 0) {
        const int ppr = hidden / kPack;
        if (d.t16) hipLaunchKernelGGL((emb_accumulate<T, true>), dim3(static_cast<unsigned>(rows)), dim3(256), 0, s, de, g, sorted, sorted_key, rows, ppr, scale, d);
        else hipLaunchKernelGGL((emb_accumulate<T, false>), dim3(static_cast<unsigned>(rows)), dim3(256), 0, s, de, g, sorted, sorted_key, rows, ppr, scale, d);
        if (dp) {
            if (d.t16) hipLaunchKernelGGL((emb_dpos<T, true>), dim3(len), dim3(256), 0, s, dp, g, tokens, batch, len, ppr, vocab, pad_idx, d);
            else hipLaunchKernelGGL((emb_dpos<T, false>), dim3(len), dim3(256), 0, s, dp, g, tokens, batch, len, ppr, vocab, pad_idx, d);
        }
    } else {
        hipLaunchKernelGGL((emb_accumulate_flat<T>), dim3(static_cast<unsigned>(rows)), dim3(256), 0, s, de, g, sorted,
                           sorted_key, rows, hidden, scale, d);
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
    LSQ_REQUIRE(demb && dy && tokens);
    LSQ_ALIGNED(demb); LSQ_ALIGNED(dpos); LSQ_ALIGNED(dy); LSQ_ALIGNED(workspace);
    const size_t need = lsq_workspace_bytes(LSQ_OP_EMBEDDING_BWD, rows, hidden);
    if (!workspace || workspace_bytes < need) return LSQ_WORKSPACE_TOO_SMALL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int32_t* ws = static_cast<int32_t*>(workspace);
    switch (dt) {
        case LSQ_F16: return emb_bwd_dispatch<f16>(demb, dpos, dy, tokens, ws, batch, len, hidden, vocab, pad_idx, scale, d, s);
        case LSQ_BF16: return emb_bwd_dispatch<bf16>(demb, dpos, dy, tokens, ws, batch, len, hidden, vocab, pad_idx, scale, d, s);
        default: return emb_bwd_dispatch<float>(demb, dpos, dy, tokens, ws, batch, len, hidden, vocab, pad_idx, scale, d, s);
    }
}
