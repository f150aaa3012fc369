// Embedding layer, forward and backward (Sec. IV-A of the paper, embedding layer):
//   forward   y[t,:] = Dropout_p(scale * E[w_t,:] + P[l_t,:])
//   backward  dE[w,:] += scale * sum_{t: w_t = w} m_t (.) dy[t,:]      dP[l,:] += sum_b m (.) dy[b,l,:]
//
// The paper sums the gradient rows of a repeated token with atomicAdd.  Floating-point
// atomics make the result depend on the arrival order; here the sum has a fixed order
// instead, with no atomics at all:
//   1. rank: every token's position in the order sorted by (token id, position) is
//      COUNTED — tile against tile, 256 x 256 comparisons per workgroup out of LDS, one
//      compare per pair — rather than sorted: counting is order-free, so the result is
//      deterministic; beyond 16384 tokens (counting is quadratic) a stable radix sort of
//      (position, id) by id produces the same order;
//   2. scatter: order[rank[t]] = (t, id);
//   3. accumulate: the sorted order is cut into windows of 8 entries; one wave per (window,
//      64-pack column block) sums m (.) dy in ascending position in fp32, the eight rows and
//      the destination rows in flight together.  An id whose rows lie inside one window is
//      added to dE[w,:] at once; a more frequent one leaves one fp32 row per window that a
//      last kernel adds in window order: one rounding of dE per call either way.
// Tokens equal to pad_idx (or outside the vocabulary) produce zero rows and no gradient.
#include <limits.h>

#include "host.hpp"

namespace lsq {

constexpr bool kNT = true;
constexpr int kEmbWaves = 4;
constexpr int kTile = kEmbTile;

__device__ __forceinline__ bool emb_is_pad(int w, int vocab, int pad_idx) { return w == pad_idx || w < 0 || w >= vocab; }

template <typename T, bool DROP>
__global__ __launch_bounds__(256) void emb_fwd_cols(T* __restrict__ out, const int32_t* __restrict__ tokens,
                                                    const T* __restrict__ emb, const T* __restrict__ pos, int64_t rows,
                                                    int len, int ppr, int vocab, int pad_idx, float scale,
                                                    DropoutParams d, FastDiv by_len)
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
            const uint32_t t32 = static_cast<uint32_t>(t);           // tokens of a call are below 2^31 (checked at the entry)
            const int l = static_cast<int>(t32 - fastdiv(t32, by_len) * static_cast<uint32_t>(len));
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

// sort key of a token: its id, with padding last; kNoKey stands for "beyond the data"
constexpr unsigned kPadKey = 0x7FFFFFFFu;
constexpr unsigned kNoKey = 0xFFFFFFFFu;
__device__ __forceinline__ unsigned emb_key(int w, int vocab, int pad_idx)
{
    return emb_is_pad(w, vocab, pad_idx) ? kPadKey : static_cast<unsigned>(w);
}

// Workgroup (it, js): for the 256 tokens i of tile `it`, how many tokens j of span `js` sort
// before i by (key, position).  Every j of an earlier tile has j < i, so key_j <= key_i decides;
// in a later tile key_j < key_i does; both are one unsigned compare against key_i + 1 or key_i.
// Only the tile's own diagonal looks at the position.  Keys come out of LDS four at a time.
__device__ __forceinline__ void emb_rank_body(int it, int js, int32_t* __restrict__ partial, const int32_t* __restrict__ tokens,
                                              int64_t rows, int ntiles, int span_tiles, int vocab, int pad_idx)
{
    __shared__ __align__(16) unsigned keys[kTile];
    const int me = threadIdx.x;
    const int64_t i = static_cast<int64_t>(it) * kTile + me;
    const unsigned ki = i < rows ? emb_key(tokens[i], vocab, pad_idx) : 0u;
    const int jt0 = js * span_tiles;
    const int jt1 = min(ntiles, jt0 + span_tiles);
    const uint4* k4 = reinterpret_cast<const uint4*>(keys);
    int count = 0;
    for (int jt = jt0; jt < jt1; ++jt) {                   // uniform: every thread reaches both barriers
        const int64_t j = static_cast<int64_t>(jt) * kTile + me;
        __syncthreads();
        keys[me] = j < rows ? emb_key(tokens[j], vocab, pad_idx) : kNoKey;   // kNoKey is below no bound
        __syncthreads();
        if (jt != it) {
            const unsigned bound = ki + (jt < it ? 1u : 0u);
#pragma unroll 8
            for (int q = 0; q < kTile / 4; ++q) {
                const uint4 k = k4[q];                     // LDS broadcast
                count += (k.x < bound ? 1 : 0) + (k.y < bound ? 1 : 0) + (k.z < bound ? 1 : 0) + (k.w < bound ? 1 : 0);
            }
        } else {
#pragma unroll 4
            for (int q = 0; q < kTile / 4; ++q) {
                const uint4 k = k4[q];
                const int j4 = 4 * q;
                count += (k.x < ki || (k.x == ki && j4 + 0 < me) ? 1 : 0) + (k.y < ki || (k.y == ki && j4 + 1 < me) ? 1 : 0)
                       + (k.z < ki || (k.z == ki && j4 + 2 < me) ? 1 : 0) + (k.w < ki || (k.w == ki && j4 + 3 < me) ? 1 : 0);
            }
        }
    }
    if (i < rows) partial[static_cast<int64_t>(js) * rows + i] = count;
}

__global__ __launch_bounds__(kTile) void emb_rank_partial(int32_t* __restrict__ partial, const int32_t* __restrict__ tokens,
                                                          int64_t rows, int ntiles, int span_tiles, int vocab, int pad_idx)
{
    emb_rank_body(blockIdx.x % ntiles, blockIdx.x / ntiles, partial, tokens, rows, ntiles, span_tiles, vocab, pad_idx);
}

// order[rank of t] = (t, key of t): the counts are a permutation of 0..rows-1.  Four lanes per
// token add every fourth span each (integer sums: any order).
__global__ __launch_bounds__(256) void emb_scatter(int2* __restrict__ order, const int32_t* __restrict__ partial,
                                                   const int32_t* __restrict__ tokens, int64_t rows, int nspans,
                                                   int vocab, int pad_idx)
{
    const int part = threadIdx.x >> 6;                                       // the wave: tokens stay coalesced
    const int64_t t = static_cast<int64_t>(blockIdx.x) * 64 + (threadIdx.x & 63);
    __shared__ int sm[3][64];
    int rank = 0;
    if (t < rows) {
        int js = part;
        for (; js + 12 < nspans; js += 16) {            // four loads in flight per trip
            int a[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) a[k] = partial[static_cast<int64_t>(js + 4 * k) * rows + t];
            rank += a[0] + a[1] + a[2] + a[3];
        }
        for (; js < nspans; js += 4) rank += partial[static_cast<int64_t>(js) * rows + t];
    }
    if (part > 0) sm[part - 1][threadIdx.x & 63] = rank;
    __syncthreads();
    if (part == 0 && t < rows) {
        rank += sm[0][threadIdx.x] + sm[1][threadIdx.x] + sm[2][threadIdx.x];
        order[rank] = make_int2(static_cast<int>(t), static_cast<int>(emb_key(tokens[t], vocab, pad_idx)));
    }
}

// ---- the same order for MANY tokens.  Counting pairs is quadratic in the tokens of a call (10 us at
// 8192, 270 us at 65536); beyond 16384 tokens the (token, key) pairs go through a stable
// least-significant-digit radix sort instead, 8 bits per pass over the bits an id can have (two
// passes up to 65535 ids): a stable sort by key leaves equal ids in ascending position, which is the
// order the accumulation wants.  A workgroup owns 2048 consecutive entries, striped over its 256
// threads (entry j*256 + i is item j of thread i), so that "round j, wave w, lane l" is ascending
// position.  Per pass: digit histogram per workgroup (integer LDS atomics: the counts do not depend
// on arrival order), exclusive scan of the [digit][workgroup] table (its own kernel only for very
// many workgroups), and the scatter, which hands out slots in position order: the lanes of a wave that hold the same digit find
// each other with 8 ballots, and the four waves take their turns on the running LDS counters.
constexpr int kRadixItems = 8;
constexpr int kRadixBlock = 256 * kRadixItems;
constexpr int kRadixFuseScan = 512;       // up to this many workgroups (2^20 tokens) the scatter scans its own offsets

__device__ __forceinline__ int2 radix_item(const int2* __restrict__ src, const int32_t* __restrict__ tokens, int64_t i,
                                           int vocab, int pad_idx)
{
    if (src) return src[i];
    return make_int2(static_cast<int>(i), static_cast<int>(emb_key(tokens[i], vocab, pad_idx)));   // first pass: the ids themselves
}

__global__ __launch_bounds__(256) void emb_radix_hist(int32_t* __restrict__ hist, const int2* __restrict__ src,
                                                      const int32_t* __restrict__ tokens, int64_t rows, int nblocks,
                                                      int shift, int vocab, int pad_idx)
{
    __shared__ int cnt[256];
    cnt[threadIdx.x] = 0;
    __syncthreads();
    const int64_t base = static_cast<int64_t>(blockIdx.x) * kRadixBlock;
#pragma unroll
    for (int j = 0; j < kRadixItems; ++j) {
        const int64_t i = base + j * 256 + threadIdx.x;
        if (i < rows) atomicAdd(&cnt[(radix_item(src, tokens, i, vocab, pad_idx).y >> shift) & 255], 1);
    }
    __syncthreads();
    hist[static_cast<int64_t>(threadIdx.x) * nblocks + blockIdx.x] = cnt[threadIdx.x];      // digit-major
}

// exclusive scan of n counts in place, one workgroup: every thread owns a contiguous piece
__global__ __launch_bounds__(1024) void emb_radix_scan(int32_t* __restrict__ hist, int64_t n)
{
    __shared__ int wave_sum[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t per = (n + 1023) / 1024;
    const int64_t lo = min(n, tid * per), hi = min(n, lo + per);
    int sum = 0;
    for (int64_t i = lo; i < hi; ++i) sum += hist[i];
    int incl = sum;                                              // inclusive scan over the wave
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int v = __shfl_up(incl, o);
        if (lane >= o) incl += v;
    }
    if (lane == 63) wave_sum[wave] = incl;
    __syncthreads();
    int before = incl - sum;
    for (int w = 0; w < wave; ++w) before += wave_sum[w];
    for (int64_t i = lo; i < hi; ++i) {
        const int c = hist[i];
        hist[i] = before;
        before += c;
    }
}

// SCANNED: `offs` went through emb_radix_scan.  Otherwise it holds the raw counts and the workgroup
// derives its own 256 offsets: thread = digit adds up its row of the table (all of it, and the part
// before this workgroup), and an exclusive scan over the 256 row sums finishes it; one launch less per
// pass, worth it while a row of the table is short.
template <bool SCANNED>
__global__ __launch_bounds__(256) void emb_radix_scatter(int2* __restrict__ dst, const int32_t* __restrict__ offs,
                                                         const int2* __restrict__ src, const int32_t* __restrict__ tokens,
                                                         int64_t rows, int nblocks, int shift, int vocab, int pad_idx)
{
    __shared__ int next[256];                  // next slot of each digit, for this workgroup's entries
    __shared__ int wave_sum[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if constexpr (SCANNED) {
        next[tid] = offs[static_cast<int64_t>(tid) * nblocks + blockIdx.x];
    } else {
        const int32_t* row = offs + static_cast<int64_t>(tid) * nblocks;
        int total = 0, mine = 0;
        const int me = blockIdx.x;
#pragma unroll 8
        for (int b = 0; b < nblocks; ++b) {
            const int c = row[b];
            total += c;
            mine += b < me ? c : 0;
        }
        int incl = total;                                        // inclusive scan of the row sums over the wave
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int v = __shfl_up(incl, o);
            if (lane >= o) incl += v;
        }
        if (lane == 63) wave_sum[wave] = incl;
        __syncthreads();
        int before = incl - total;
        for (int w = 0; w < wave; ++w) before += wave_sum[w];
        next[tid] = before + mine;
    }
    __syncthreads();
    const int64_t base = static_cast<int64_t>(blockIdx.x) * kRadixBlock;
    for (int j = 0; j < kRadixItems; ++j) {                      // uniform trip count: every thread reaches every barrier
        const int64_t i = base + j * 256 + tid;
        const bool valid = i < rows;
        const int2 item = valid ? radix_item(src, tokens, i, vocab, pad_idx) : make_int2(0, 0);
        const int digit = (item.y >> shift) & 255;
        uint64_t same = __ballot(valid);                         // lanes of this wave with my digit
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const uint64_t has = __ballot((digit >> b) & 1);
            same &= ((digit >> b) & 1) ? has : ~has;
        }
        if (!valid) same = 0;
        const int below = __popcll(same & ((1ull << lane) - 1ull));
        const int leader = same ? __builtin_ctzll(same) : lane;
        int slot = 0;
        for (int w = 0; w < 4; ++w) {                            // waves in order: ascending position
            if (wave == w && valid && lane == leader) {          // one lane per digit present in the wave
                slot = next[digit];
                next[digit] = slot + __popcll(same);
            }
            __syncthreads();
        }
        slot = __shfl(slot, leader);
        if (valid) dst[slot + below] = item;
    }
}

// The sorted order is cut into windows of kEmbWin entries and 64-pack column blocks; one wave
// takes one (window, column block).  Lane 0 gets the entry before the window, lanes
// 1..kEmbWin the window, lane kEmbWin+1 the entry after it; beyond the data the key is kNoKey
// (-1 as int), which equals no token's key.
__device__ __forceinline__ int2 emb_window(const int2* __restrict__ order, int64_t win, int64_t rows, int lane)
{
    const int64_t idx = win * kEmbWin - 1 + lane;
    int2 e = make_int2(0, static_cast<int>(kNoKey));
    if (lane <= kEmbWin + 1 && idx >= 0 && idx < rows) e = order[idx];
    return e;
}

__device__ __forceinline__ bool emb_live_key(int key) { return key >= 0 && key != static_cast<int>(kPadKey); }

// Sums m (.) dy over each run of equal ids inside the window, in ascending position.  A run
// that starts and ends inside the window is added to dE[w,:] at once (the destination row is
// fetched together with the dy rows).  A run that comes from the previous window or goes on
// into the next leaves an fp32 row for emb_combine: slot 0 of the window if it is the window's
// first run, slot 1 otherwise (only the last run can be the other one).
template <typename T, bool DROP>
__global__ __launch_bounds__(256) void emb_accumulate(T* __restrict__ demb, float* __restrict__ win_rows,
                                                      const T* __restrict__ dy, const int2* __restrict__ order,
                                                      int64_t rows, int64_t nwin, int ncb, int ppr, float scale,
                                                      DropoutParams d)
{
    const int lane = threadIdx.x & 63;
    const int64_t gw = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
    if (gw >= nwin * ncb) return;                                   // wave-uniform
    const int64_t win = gw / ncb;
    const int cp = static_cast<int>(gw % ncb) * 64 + lane;
    const int2 e = emb_window(order, win, rows, lane);
    int key[kEmbWin + 2], tok[kEmbWin];
#pragma unroll
    for (int k = 0; k < kEmbWin + 2; ++k) key[k] = __builtin_amdgcn_readlane(e.y, k);
#pragma unroll
    for (int k = 0; k < kEmbWin; ++k) tok[k] = __builtin_amdgcn_readlane(e.x, k + 1);
    if (cp >= ppr) return;

    // what happens after entry k (all wave-uniform): 0 nothing, 1 add to dE, 2 / 3 leave slot 0 / 1
    int action[kEmbWin];
    {
        bool open_partial = key[1] == key[0], first_run = true;
#pragma unroll
        for (int k = 0; k < kEmbWin; ++k) {
            const bool live = emb_live_key(key[k + 1]);
            const bool tail = key[k + 1] != key[k + 2];
            action[k] = 0;
            if (live && tail) action[k] = open_partial ? 2 : 1;            // a run from the previous window is the first run
            else if (live && k == kEmbWin - 1) action[k] = first_run ? 2 : 3;
            if (tail) { open_partial = false; first_run = false; }
        }
    }
    RawPack<T> raw[kEmbWin], dst_raw[kEmbWin];
#pragma unroll
    for (int k = 0; k < kEmbWin; ++k) {
        if (emb_live_key(key[k + 1])) raw[k] = load_raw<T, kNT>(dy + (static_cast<int64_t>(tok[k]) * ppr + cp) * kPack);
        else raw[k] = zero_raw<T>();
    }
#pragma unroll
    for (int k = 0; k < kEmbWin; ++k) {
        if (action[k] == 1) dst_raw[k] = load_raw<T, false>(demb + (static_cast<int64_t>(key[k + 1]) * ppr + cp) * kPack);
        else dst_raw[k] = zero_raw<T>();
    }
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int k = 0; k < kEmbWin; ++k) {
        if (emb_live_key(key[k + 1])) {
            float g[8];
            unpack<T>(raw[k], g);
            if constexpr (DROP) {
                float kf[8];
                dropout_factors8(d, static_cast<uint64_t>(static_cast<int64_t>(tok[k]) * ppr + cp), kf);
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[j] = fmaf(g[j], kf[j], acc[j]);
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[j] += g[j];
            }
        }
        if (action[k] == 1) {
            float o[8];
            unpack<T>(dst_raw[k], o);
#pragma unroll
            for (int j = 0; j < 8; ++j) o[j] = fmaf(scale, acc[j], o[j]);
            store8<T>(demb + (static_cast<int64_t>(key[k + 1]) * ppr + cp) * kPack, o);
        } else if (action[k] >= 2) {
            store8<float>(win_rows + ((2 * win + (action[k] - 2)) * ppr + cp) * kPack, acc);
        }
        if (action[k] != 0) {
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] = 0.0f;
        }
    }
}

// The workgroup of the (window, column block) in which a window-crossing id segment ENDS adds
// the segment's fp32 rows and rounds dE[w,:] once.  The segment's first window is found by looking
// back, 64 windows per trip: window v is the first one if the entry before it has another key
// (or v = 0).  The four waves take every fourth row each, eight in flight, and their sums are
// added in wave order: a fixed association, so the result does not depend on timing.
template <typename T>
__global__ __launch_bounds__(256) void emb_combine(T* __restrict__ demb, const float* __restrict__ win_rows,
                                                   const int2* __restrict__ order, int64_t rows, int ncb, int ppr,
                                                   float scale)
{
    __shared__ float sm[kEmbWaves - 1][8][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t win = blockIdx.x / ncb;
    const int cp = static_cast<int>(blockIdx.x % ncb) * 64 + lane;
    // every wave reads the same entries and takes the same decisions: the exits are workgroup-uniform
    const int2 e = emb_window(order, win, rows, lane);
    const int key = __builtin_amdgcn_readlane(e.y, 1);
    if (!emb_live_key(key) || __builtin_amdgcn_readlane(e.y, 0) != key) return;   // first run starts here: nothing to combine
    constexpr uint64_t kAll = ((1ull << (kEmbWin + 1)) - 1) << 1;  // lanes 1..kEmbWin+1
    if ((__ballot(e.y == key) & kAll) == kAll) return;              // the run goes on into the next window
    // here win >= 1 (the entry before the window exists), so the search starts at a valid window
    int64_t head = 0;
    int head_first_key = 0;
    for (int64_t base = win - 1;; base -= 64) {
        const int64_t v = base - lane;
        bool stop = false;
        int first_key = 0;
        if (v >= 0) {
            first_key = order[v * kEmbWin].y;
            stop = v == 0 || order[v * kEmbWin - 1].y != key;
        }
        const uint64_t m = __ballot(stop);
        if (m != 0) {                                               // v = 0 stops: every wave leaves the loop
            const int l = __builtin_ctzll(m);
            head = base - l;
            head_first_key = __builtin_amdgcn_readlane(first_key, l);
            break;
        }
    }
    const bool active = cp < ppr;
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (active) {
        // the segment is the first run of its first window exactly if it starts at that window's first entry
        if (wave == 0) load8<float>(win_rows + ((2 * head + (head_first_key == key ? 0 : 1)) * ppr + cp) * kPack, acc);
        constexpr int U = 8;
        for (int64_t v0 = head + 1 + wave; v0 <= win; v0 += U * kEmbWaves) {
            float r[U][8];
#pragma unroll
            for (int k = 0; k < U; ++k) {
                const int64_t v = v0 + k * kEmbWaves;
                if (v <= win) {
                    load8<float>(win_rows + (2 * v * ppr + cp) * kPack, r[k]);
                } else {
#pragma unroll
                    for (int j = 0; j < 8; ++j) r[k][j] = 0.0f;
                }
            }
#pragma unroll
            for (int k = 0; k < U; ++k)
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[j] += r[k][j];
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
        T* dst = demb + (static_cast<int64_t>(key) * ppr + cp) * kPack;
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
__device__ __forceinline__ void emb_dpos_body(int cb, int l, T* __restrict__ dpos, const T* __restrict__ dy,
                                              const int32_t* __restrict__ tokens, int batch, int len, int ppr,
                                              int vocab, int pad_idx, const DropoutParams& d)
{
    constexpr int U = 4;
    __shared__ float sm[kEmbWaves - 1][8][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int cp = cb * 64 + lane;
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

// The rank count is arithmetic out of LDS, the position gradient a stream over dy; neither
// needs the other.  One launch holds the workgroups of both (the rank ones first, so that they
// all start at once and the streaming ones fill the remaining wave slots): the two overlap
// instead of running back to back.
template <typename T, bool DROP>
__global__ __launch_bounds__(256) void emb_rank_dpos(int32_t* __restrict__ partial, const int32_t* __restrict__ tokens,
                                                     int64_t rows, int ntiles, int span_tiles, int rank_blocks,
                                                     T* __restrict__ dpos, const T* __restrict__ dy, int batch, int len,
                                                     int ppr, int ncb, int vocab, int pad_idx, DropoutParams d)
{
    static_assert(kTile == 256, "one block size for both bodies");
    if (static_cast<int>(blockIdx.x) < rank_blocks) {            // workgroup-uniform
        emb_rank_body(blockIdx.x % ntiles, blockIdx.x / ntiles, partial, tokens, rows, ntiles, span_tiles, vocab, pad_idx);
    } else {
        const int b = static_cast<int>(blockIdx.x) - rank_blocks;
        emb_dpos_body<T, DROP>(b % ncb, b / ncb, dpos, dy, tokens, batch, len, ppr, vocab, pad_idx, d);
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
        if (d.on) v *= dropout_factor1(d, static_cast<uint64_t>(e));
    }
    out[e] = from_f32<T>(v);
}

// one thread per (id segment head, column): walks the segment sequentially
template <typename T>
__global__ __launch_bounds__(256) void emb_accumulate_flat(T* __restrict__ demb, const T* __restrict__ dy,
                                                           const int2* __restrict__ order, int64_t rows, int hidden,
                                                           float scale, DropoutParams d)
{
    const int64_t q = blockIdx.x;
    const int key = order[q].y;
    if (!emb_live_key(key) || (q > 0 && order[q - 1].y == key)) return;    // padding, or not the head of its segment
    for (int i = threadIdx.x; i < hidden; i += 256) {
        float acc = 0.0f;
        for (int64_t c = q; c < rows; ++c) {
            const int2 o = order[c];
            if (o.y != key) break;
            const int64_t e = static_cast<int64_t>(o.x) * hidden + i;
            float g = to_f32<T>(dy[e]);
            if (d.on) g *= dropout_factor1(d, static_cast<uint64_t>(e));
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
            if (d.on) g *= dropout_factor1(d, static_cast<uint64_t>(e));
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
        // one row per wave up to 65536 rows: 5.9 / 8.0 us at 4096 x 1024 / 8192 x 1280 against 6.6 / 8.15 with four
        int64_t rb = ceil_div(rows, kEmbWaves);
        if (rb > 16384) rb = 16384;
        const dim3 grid(static_cast<unsigned>(ceil_div(ppr, 64)), static_cast<unsigned>(rb)), block(256);
        const FastDiv by_len = make_fastdiv(static_cast<uint32_t>(len));
        if (d.on) hipLaunchKernelGGL((emb_fwd_cols<T, true>), grid, block, 0, s, o, tokens, e, p, rows, len, ppr, vocab, pad_idx, scale, d, by_len);
        else hipLaunchKernelGGL((emb_fwd_cols<T, false>), grid, block, 0, s, o, tokens, e, p, rows, len, ppr, vocab, pad_idx, scale, d, by_len);
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
    const EmbBwdPlan plan = emb_bwd_plan(rows, hidden);
    int2* order = reinterpret_cast<int2*>(ws);
    float* win_rows = reinterpret_cast<float*>(static_cast<char*>(ws) + plan.order_bytes);
    int32_t* partial = reinterpret_cast<int32_t*>(static_cast<char*>(ws) + plan.order_bytes + plan.win_bytes);
    T* de = static_cast<T*>(demb);
    T* dp = static_cast<T*>(dpos);
    const T* g = static_cast<const T*>(dy);
    // the dropout scale 1/(1-p) is carried by the per-element factors; `scale` is the embedding scale
    const bool packed = hidden % kPack == 0;
    const int ppr = hidden / kPack;
    const int ncb = static_cast<int>(ceil_div(ppr, 64));
    if (rows <= kEmbCountMax) {
        // few tokens: order[rank of t] = (t, key), the rank counted pair by pair
        const unsigned rank_blocks = static_cast<unsigned>(plan.ntiles) * static_cast<unsigned>(plan.nspans);
        if (packed && dp) {
            // the position gradient rides along with the rank count
            const dim3 rgrid(rank_blocks + static_cast<unsigned>(ncb) * static_cast<unsigned>(len));
            if (d.on) hipLaunchKernelGGL((emb_rank_dpos<T, true>), rgrid, dim3(256), 0, s, partial, tokens, rows, plan.ntiles, plan.span_tiles,
                                          static_cast<int>(rank_blocks), dp, g, batch, len, ppr, ncb, vocab, pad_idx, d);
            else hipLaunchKernelGGL((emb_rank_dpos<T, false>), rgrid, dim3(256), 0, s, partial, tokens, rows, plan.ntiles, plan.span_tiles,
                                    static_cast<int>(rank_blocks), dp, g, batch, len, ppr, ncb, vocab, pad_idx, d);
        } else {
            hipLaunchKernelGGL(emb_rank_partial, dim3(rank_blocks), dim3(kTile), 0, s, partial, tokens, rows, plan.ntiles,
                               plan.span_tiles, vocab, pad_idx);
        }
        hipLaunchKernelGGL(emb_scatter, dim3(static_cast<unsigned>(ceil_div(rows, 64))), dim3(256), 0, s, order, partial,
                           tokens, rows, plan.nspans, vocab, pad_idx);
    } else {
        // many tokens: stable radix sort of (t, key) by the bits an id can have; padding (all ones) comes last
        int bits = 1;
        while ((static_cast<int64_t>(1) << bits) <= vocab) ++bits;                 // 2^bits > vocab
        const int passes = (bits + 7) / 8;
        const int nblocks = plan.radix_blocks;
        int32_t* hist = partial;                                                     // [256][nblocks]
        int2* tmp = reinterpret_cast<int2*>(reinterpret_cast<char*>(partial) + plan.radix_hist_bytes);
        const int2* src = nullptr;
        for (int pass = 0; pass < passes; ++pass) {
            int2* dst = (passes - pass) % 2 == 1 ? order : tmp;                      // the last pass lands in `order`
            hipLaunchKernelGGL(emb_radix_hist, dim3(nblocks), dim3(256), 0, s, hist, src, tokens, rows, nblocks, 8 * pass, vocab, pad_idx);
            if (nblocks <= kRadixFuseScan) {
                hipLaunchKernelGGL((emb_radix_scatter<false>), dim3(nblocks), dim3(256), 0, s, dst, hist, src, tokens, rows, nblocks, 8 * pass, vocab, pad_idx);
            } else {
                hipLaunchKernelGGL(emb_radix_scan, dim3(1), dim3(1024), 0, s, hist, static_cast<int64_t>(256) * nblocks);
                hipLaunchKernelGGL((emb_radix_scatter<true>), dim3(nblocks), dim3(256), 0, s, dst, hist, src, tokens, rows, nblocks, 8 * pass, vocab, pad_idx);
            }
            src = dst;
        }
        if (packed && dp) {            // the position gradient on its own (no rank workgroups in the launch)
            const dim3 rgrid(static_cast<unsigned>(ncb) * static_cast<unsigned>(len));
            if (d.on) hipLaunchKernelGGL((emb_rank_dpos<T, true>), rgrid, dim3(256), 0, s, partial, tokens, rows, 1, 1, 0, dp, g, batch, len, ppr, ncb, vocab, pad_idx, d);
            else hipLaunchKernelGGL((emb_rank_dpos<T, false>), rgrid, dim3(256), 0, s, partial, tokens, rows, 1, 1, 0, dp, g, batch, len, ppr, ncb, vocab, pad_idx, d);
        }
    }
    if (packed) {
        const unsigned pairs = static_cast<unsigned>(plan.nwin * ncb);      // (window, column block) pairs
        const dim3 grid(static_cast<unsigned>(ceil_div(pairs, 4))), block(256);   // one wave per pair
        if (d.on) hipLaunchKernelGGL((emb_accumulate<T, true>), grid, block, 0, s, de, win_rows, g, order, rows, plan.nwin, ncb, ppr, scale, d);
        else hipLaunchKernelGGL((emb_accumulate<T, false>), grid, block, 0, s, de, win_rows, g, order, rows, plan.nwin, ncb, ppr, scale, d);
        hipLaunchKernelGGL((emb_combine<T>), dim3(pairs), block, 0, s, de, win_rows, order, rows, ncb, ppr, scale);   // one workgroup per pair
    } else {
        hipLaunchKernelGGL((emb_accumulate_flat<T>), dim3(static_cast<unsigned>(rows)), dim3(256), 0, s, de, g, order, rows, hidden, scale, d);
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
    LSQ_REQUIRE(rows <= 0x7FFFFFFF);
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
    LSQ_REQUIRE(rows <= 0x7FFFFFFF / 2);
    LSQ_REQUIRE(ceil_div(rows, kEmbWin) * ceil_div(hidden, 8 * 64) < 0x7FFFFFFF);   // one workgroup per (window, column block)
    LSQ_REQUIRE(ceil_div(rows, kTile) * 64 + ceil_div(hidden, 8 * 64) * static_cast<int64_t>(len) < 0x7FFFFFFF);
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
