// Label-smoothed cross-entropy, forward and backward (Sec. IV-A of the paper,
// criterion layer).  The loss is evaluated through log-softmax, as the paper
// does: loss = lse - (1-alpha)*h_k - (alpha/V)*sum_i h_i, and the gradient is the
// element-wise expression q_i - alpha/V - (1-alpha)[i == k] with q_i rebuilt as
// exp(h_i - lse) from the saved lse, so neither direction ever materialises the
// softmax.
//
// One workgroup per token.  The vocabulary row is read ONCE in forward: every
// thread keeps a running (max, sum) pair in the base-2 domain and rescales its
// sum when the maximum moves (9 exponentials per 8 logits), and the pairs are
// merged across the workgroup at the end.  Rows of odd vocabularies (50257,
// 30522) do not start on 16-byte boundaries: a row is split into a scalar head up
// to the next pack boundary of the flat tensor, a body of aligned 128-bit packs,
// and a scalar tail, so the body keeps full-width accesses for any vocab.
#include "host.hpp"

namespace lsq {

constexpr bool kNT = true;   // nontemporal hint on the streamed tensors
constexpr bool kBwdNTL = true, kBwdNTS = true;

constexpr float kLog2eX = 1.4426950408889634f;
constexpr float kLn2X = 0.6931471805599453f;
// measured at 8192 x 30522 / 32768 / 50257 logits: 512 or 1024 threads per row and 8 packs in flight per thread are
// no faster (within 2 %) or slower (1024 threads: -10 %)
constexpr int kXentThreads = 256;
// the flat backward runs as one-wave workgroups: 259 against 263 us at 8192 x 50257, 134 against 137 us at the
// transformer-big shape, 103 against 109 us on a masked-LM batch (256 threads per workgroup; 128: 266 / 136 / 102)
constexpr int kXbThreads = 64;
constexpr int kXentUnroll = 4;

struct RowSplit {
    int64_t begin, head_end, pack_begin, pack_end, tail_begin, end;
};

// [begin, head_end) scalar, packs [pack_begin, pack_end) aligned, [tail_begin, end) scalar.
__device__ __forceinline__ RowSplit split_row(int64_t t, int vocab)
{
    RowSplit r;
    r.begin = t * vocab;
    r.end = r.begin + vocab;
    r.pack_begin = (r.begin + kPack - 1) / kPack;
    r.pack_end = r.end / kPack;
    if (r.pack_begin > r.pack_end) {          // the row lies inside one pack
        r.pack_end = r.pack_begin;
        r.head_end = r.end;
        r.tail_begin = r.end;
    } else {
        r.head_end = r.pack_begin * kPack;
        r.tail_begin = r.pack_end * kPack;
    }
    return r;
}

__device__ __forceinline__ bool is_ignored(int k, int vocab, int ignore_index)
{
    return k == ignore_index || k < 0 || k >= vocab;
}

typedef _Float16 half2v __attribute__((ext_vector_type(2)));
struct Half8 { half2v v[4]; };
template <typename T> constexpr bool kIsF16 = false;
template <> constexpr bool kIsF16<f16> = true;

struct OnlineLse {
    float m = -INFINITY;   // running maximum of h*log2(e)
    float s = 0.0f;        // sum of exp2(h*log2e - m)
    float sh = 0.0f;       // sum of h
    __device__ __forceinline__ void add1(float h)
    {
        const float hs = h * kLog2eX;
        const float mn = fmaxf(m, hs);
        s = fmaf(s, __builtin_amdgcn_exp2f(m - mn), __builtin_amdgcn_exp2f(hs - mn));
        m = mn;
        sh += h;
    }
    __device__ __forceinline__ void add8(const float (&h)[8])
    {
        float hs[8];
        float vm = h[0] * kLog2eX;
        hs[0] = vm;
#pragma unroll
        for (int j = 1; j < 8; ++j) { hs[j] = h[j] * kLog2eX; vm = fmaxf(vm, hs[j]); }
        const float mn = fmaxf(m, vm);
        float acc = s * __builtin_amdgcn_exp2f(m - mn);
        float hsum = 0.0f;
#pragma unroll
        for (int j = 0; j < 8; ++j) { acc += __builtin_amdgcn_exp2f(hs[j] - mn); hsum += h[j]; }
        s = acc;
        m = mn;
        sh += hsum;
    }
    // The same for a pack of fp16 logits, on the packed halves: the maximum two elements per instruction (exact,
    // and max(h) * log2e = max(h * log2e) because rounding is monotonic), the sum of the logits by dot products
    // with ones, the exponent by one fma that reads the half directly.  A quarter fewer vector instructions per
    // element than add8, on a kernel whose vector ALU is 85 % busy.
    __device__ __forceinline__ void add_pack_f16(const Half8& h)
    {
        const half2v m01 = __builtin_elementwise_max(h.v[0], h.v[1]), m23 = __builtin_elementwise_max(h.v[2], h.v[3]);
        const half2v mm = __builtin_elementwise_max(m01, m23);
        const float vm = fmaxf(static_cast<float>(mm.x), static_cast<float>(mm.y)) * kLog2eX;
        const float mn = fmaxf(m, vm);
        float acc = s * __builtin_amdgcn_exp2f(m - mn);
        const half2v ones = {static_cast<_Float16>(1.0f), static_cast<_Float16>(1.0f)};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            acc += __builtin_amdgcn_exp2f(fmaf(static_cast<float>(h.v[c].x), kLog2eX, -mn));
            acc += __builtin_amdgcn_exp2f(fmaf(static_cast<float>(h.v[c].y), kLog2eX, -mn));
            sh = __builtin_amdgcn_fdot2(h.v[c], ones, sh, false);
        }
        s = acc;
        m = mn;
    }
};

// TH threads share a row and a workgroup holds R rows.  Long rows: TH = 256, R = 1.  Short rows
// (up to 2048 logits): TH = 64, R = 4: every wave has its own token, its reductions stay inside the
// wave (no barrier anywhere, so waves may leave on their own), and no thread idles on a row that
// is shorter than the workgroup.
template <typename T, int TH = kXentThreads, int R = 1>
__global__ __launch_bounds__(TH * R) void xent_fwd_kernel(float* __restrict__ loss, float* __restrict__ nll,
                                                          float* __restrict__ lse,
                                                          const T* __restrict__ logits,
                                                          const int32_t* __restrict__ target, int64_t tokens, int vocab,
                                                          float alpha, int ignore_index)
{
    static_assert(R == 1 || TH == 64, "several rows per workgroup only with one wave per row");
    __shared__ float lds[TH / 64];
    const int64_t t = static_cast<int64_t>(blockIdx.x) * R + threadIdx.x / TH;
    const int tid = threadIdx.x % TH;
    if (t >= tokens) return;                      // whole waves (R > 1 only)
    const int k0 = target[t];
    if (is_ignored(k0, vocab, ignore_index)) {    // uniform over the row's threads: a padded token's row is not read
        if (tid == 0) {
            loss[t] = 0.0f;
            lse[t] = 0.0f;
            if (nll) nll[t] = 0.0f;
        }
        return;
    }
    // (Issuing the first loads before the target is known was measured too: no faster on rows
    // that count, 15-60 % slower on batches with padding.)
    const RowSplit r = split_row(t, vocab);
    OnlineLse st;
    if (r.begin + tid < r.head_end) st.add1(to_f32<T>(logits[r.begin + tid]));
    if (r.tail_begin + tid < r.end) st.add1(to_f32<T>(logits[r.tail_begin + tid]));
    // kXentUnroll packs in flight per thread.  The sweep starts at the 128-byte line that
    // holds the row's first pack, not at the pack itself: every wave request is then
    // line-aligned.  (Started at the pack, each 1 KiB request straddles nine lines and,
    // with nontemporal loads, the shared line is fetched from HBM twice: +6 % traffic.)
    const int64_t base = r.pack_begin & ~static_cast<int64_t>(7);
    for (int64_t p = base + tid; p < r.pack_end; p += kXentUnroll * TH) {
        RawPack<T> raw[kXentUnroll];
        bool ok[kXentUnroll];
#pragma unroll
        for (int u = 0; u < kXentUnroll; ++u) {
            const int64_t q = p + u * TH;
            ok[u] = q >= r.pack_begin && q < r.pack_end;
            if (ok[u]) raw[u] = load_raw<T, kNT>(logits + q * kPack);
            else raw[u] = zero_raw<T>();
        }
#pragma unroll
        for (int u = 0; u < kXentUnroll; ++u) {
            if (ok[u]) {
                if constexpr (kIsF16<T>) {
                    st.add_pack_f16(__builtin_bit_cast(Half8, raw[u].u));
                } else {
                    float h[8];
                    unpack<T>(raw[u], h);
                    st.add8(h);
                }
            }
        }
    }
    const float M = block_allreduce<TH / 64, OpMax>(st.m, lds);
    const float S = block_allreduce<TH / 64, OpSum>(st.s * __builtin_amdgcn_exp2f(st.m - M), lds);
    const float SH = block_allreduce<TH / 64, OpSum>(st.sh, lds);
    if (tid == 0) {
        const float l = (M + __builtin_amdgcn_logf(S)) * kLn2X;     // v_log_f32 is log2
        lse[t] = l;
        const float hk = to_f32<T>(logits[r.begin + k0]);
        loss[t] = l - (1.0f - alpha) * hk - (alpha / static_cast<float>(vocab)) * SH;
        if (nll) nll[t] = l - hk;
    }
}

template <typename T>
__global__ __launch_bounds__(kXentThreads) void xent_bwd_kernel(T* dlogits, const T* logits,
                                                               const float* __restrict__ lse,
                                                               const int32_t* __restrict__ target, int vocab,
                                                               float alpha, int ignore_index, float grad_scale)
{
    const int64_t t = blockIdx.x;
    const RowSplit r = split_row(t, vocab);
    const int tid = threadIdx.x;
    const int k = target[t];
    if (is_ignored(k, vocab, ignore_index)) {           // uniform over the workgroup
        if (r.begin + tid < r.head_end) dlogits[r.begin + tid] = from_f32<T>(0.0f);
        if (r.tail_begin + tid < r.end) dlogits[r.tail_begin + tid] = from_f32<T>(0.0f);
        const float z[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        for (int64_t p = r.pack_begin + tid; p < r.pack_end; p += kXentThreads) store8<T, kBwdNTS>(dlogits + p * kPack, z);
        return;
    }
    const float ls = lse[t] * kLog2eX;
    const float smooth = alpha / static_cast<float>(vocab);
    const float hit = grad_scale * (1.0f - alpha);
    const int64_t kpos = r.begin + k;
    auto one = [&](int64_t e) {
        float gq = grad_scale * (__builtin_amdgcn_exp2f(fmaf(to_f32<T>(logits[e]), kLog2eX, -ls)) - smooth);
        if (e == kpos) gq -= hit;
        dlogits[e] = from_f32<T>(gq);
    };
    if (r.begin + tid < r.head_end) one(r.begin + tid);
    if (r.tail_begin + tid < r.end) one(r.tail_begin + tid);
    const int64_t kpack = kpos >> 3;
    auto pack = [&](int64_t q, float (&h)[8]) {
#pragma unroll
        for (int j = 0; j < 8; ++j) h[j] = grad_scale * (__builtin_amdgcn_exp2f(fmaf(h[j], kLog2eX, -ls)) - smooth);
        if (q == kpack) {
            const int jj = static_cast<int>(kpos & 7);
#pragma unroll
            for (int j = 0; j < 8; ++j) h[j] -= (j == jj) ? hit : 0.0f;
        }
        store8<T, kBwdNTS>(dlogits + q * kPack, h);
    };
    int64_t p = r.pack_begin + tid;
    for (; p + (kXentUnroll - 1) * kXentThreads < r.pack_end; p += kXentUnroll * kXentThreads) {
        float h[kXentUnroll][8];
#pragma unroll
        for (int u = 0; u < kXentUnroll; ++u) load8<T, kBwdNTL>(logits + (p + u * kXentThreads) * kPack, h[u]);
#pragma unroll
        for (int u = 0; u < kXentUnroll; ++u) pack(p + u * kXentThreads, h[u]);
    }
    for (; p < r.pack_end; p += kXentThreads) {
        float h[8];
        load8<T, kBwdNTL>(logits + p * kPack, h);
        pack(p, h);
    }
}

// Backward over the FLAT [tokens*vocab] tensor: a workgroup owns a contiguous chunk
// of U*64 aligned packs whatever rows they fall in, so the access pattern is that
// of a plain copy (few DRAM pages open at a time, every access 128-bit and aligned,
// no scalar head/tail per row).  Measured on MI355X a copy laid out one row per
// workgroup reaches 4.8 TB/s at vocab 50257, the flat one 6.6 TB/s.  The chunk is
// never longer than a row, so it touches at most two rows, A and B: their lse and
// target are wave-uniform and sit in scalar registers.  Only the one pack that
// straddles the boundary (vocab % 8 != 0) selects per element.  Packs of ignored
// rows are not read at all.
template <typename T, int U>
__global__ __launch_bounds__(kXbThreads) void xent_bwd_flat_kernel(T* dlogits, const T* logits,
                                                            const float* __restrict__ lse,
                                                            const int32_t* __restrict__ target, int64_t tokens,
                                                            int vocab, float alpha, int ignore_index, float grad_scale)
{
    const int64_t total = tokens * vocab;
    const int64_t npacks = total / kPack;                     // full packs; the ragged end is handled below
    const int64_t pb = static_cast<int64_t>(blockIdx.x) * (U * kXbThreads);
    const int64_t tA = (pb * kPack) / vocab;                  // row of the chunk's first element (uniform)
    const int64_t baseA = tA * vocab;
    const int64_t bnd = baseA + vocab;                        // first element of row B
    const bool hasB = tA + 1 < tokens;
    const float smooth = alpha / static_cast<float>(vocab);
    const float hit = grad_scale * (1.0f - alpha);
    const int kA = target[tA];
    const int kB = hasB ? target[tA + 1] : ignore_index;
    const bool liveA = !is_ignored(kA, vocab, ignore_index);
    const bool liveB = hasB && !is_ignored(kB, vocab, ignore_index);
    const float lsA = lse[tA] * kLog2eX;
    const float lsB = hasB ? lse[tA + 1] * kLog2eX : 0.0f;
    const int64_t hitA = baseA + (liveA ? kA : -1);           // flat index of the target element, if live
    const int64_t hitB = bnd + (liveB ? kB : -1);

    if (!liveA && !liveB && blockIdx.x != gridDim.x - 1) {    // a chunk of ignored rows only (masked-LM: most): zeros, nothing else
        const float zero[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t q = pb + u * kXbThreads + threadIdx.x;
            if (q < npacks) store8<T, kBwdNTS>(dlogits + q * kPack, zero);
        }
        return;
    }

    float h[U][8];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t q = pb + u * kXbThreads + threadIdx.x;
        const int64_t e0 = q * kPack;
        const bool need = q < npacks && ((e0 < bnd && liveA) || (e0 + kPack > bnd && liveB));
        if (need) {
            load8<T, kBwdNTL>(logits + e0, h[u]);
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) h[u][j] = 0.0f;
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t q = pb + u * kXbThreads + threadIdx.x;
        if (q >= npacks) continue;
        const int64_t e0 = q * kPack;
        float o[8];
        if (e0 + kPack <= bnd || e0 >= bnd) {                 // the whole pack lies in one row
            const bool inB = e0 >= bnd;
            const bool live = inB ? liveB : liveA;
            const float ls = inB ? lsB : lsA;
            const int64_t hp = (inB ? hitB : hitA) - e0;      // 0..7 iff the target element is in this pack
#pragma unroll
            for (int j = 0; j < 8; ++j)
                o[j] = live ? grad_scale * (__builtin_amdgcn_exp2f(fmaf(h[u][j], kLog2eX, -ls)) - smooth) : 0.0f;
            if (live && hp >= 0 && hp < kPack) {
#pragma unroll
                for (int j = 0; j < 8; ++j) o[j] -= (j == static_cast<int>(hp)) ? hit : 0.0f;
            }
        } else {                                              // straddles the boundary: select per element
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const bool inB = e0 + j >= bnd;
                const bool live = inB ? liveB : liveA;
                const float ls = inB ? lsB : lsA;
                float gq = grad_scale * (__builtin_amdgcn_exp2f(fmaf(h[u][j], kLog2eX, -ls)) - smooth);
                if (e0 + j == (inB ? hitB : hitA)) gq -= hit;
                o[j] = live ? gq : 0.0f;
            }
        }
        store8<T, kBwdNTS>(dlogits + e0, o);
    }
    // ragged end of the whole tensor (total % 8 elements): last workgroup, scalar
    if (blockIdx.x == gridDim.x - 1) {
        const int64_t e = npacks * kPack + threadIdx.x;
        if (e < total) {
            const int64_t t = e / vocab;
            const int k = target[t];
            float gq = 0.0f;
            if (!is_ignored(k, vocab, ignore_index)) {
                gq = grad_scale * (__builtin_amdgcn_exp2f(fmaf(to_f32<T>(logits[e]), kLog2eX, -lse[t] * kLog2eX)) - smooth);
                if (e == t * vocab + k) gq -= hit;
            }
            dlogits[e] = from_f32<T>(gq);
        }
    }
}

// ---- forward and backward in one pass over the logits.
// The loss scale of a training step is known before the criterion runs, so the gradient can be
// written while the row is still in registers: the logits are read once and dlogits written once
// (two passes over [tokens, vocab] instead of the three of forward + backward).  One workgroup
// per token holds the whole row as NP packs per thread.  Two exponentials per element would make
// the pass ALU-bound (v_exp_f32 runs at a quarter of the vector rate), so there is one: pass 1
// takes the maximum, pass 2 replaces each logit IN the registers by e = exp2(h log2e - max),
// rounded to the storage type, while summing e and h, and pass 3 is one fma per element,
// dlogits = e * (grad_scale / S) - grad_scale * alpha / V (- grad_scale (1 - alpha) at the target).
// The extra rounding of e is of the size of the rounding of dlogits itself (fp32 storage: none).
// Rows of odd vocabularies share their first and last pack of the flat tensor with the
// neighbouring rows: those two packs are read and written element by element, everything else in
// aligned 128-bit packs.  Every load of the row (and of the target logit) precedes every store,
// and a workgroup writes only its own row's elements, so dlogits may be the logits buffer itself.

// which of the 8 elements of window pack i lie in [lo, hi) (element offsets from the window's first pack)
__device__ __forceinline__ unsigned row_mask(int i, int lo, int hi)
{
    unsigned m = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) m |= (i * kPack + j >= lo && i * kPack + j < hi) ? (1u << j) : 0u;
    return m;
}

template <typename T, int THREADS, int NP, int R = 1>
__global__ __launch_bounds__(THREADS * R) void xent_fused_kernel(
    float* __restrict__ loss, float* __restrict__ nll, float* __restrict__ lse, T* dlogits, const T* logits,
    const int32_t* __restrict__ target, int64_t tokens, int vocab, float alpha, int ignore_index, float grad_scale)
{
    static_assert(R == 1 || THREADS == 64, "several rows per workgroup only with one wave per row (no barriers then)");
    constexpr int NW = THREADS / 64;
    __shared__ float lds[2][NW];
    // each XCD takes runs of 12 consecutive workgroups (1.2 MB of logits at vocab 50257), the runs rotating from group to
    // group so that padded sentence tails spread over the XCDs: 289 against 301 us at 8192 x 50257, 148 against 154 us
    // at the transformer-big shape (padded), 133 against 138 us on a masked-LM batch.  The separate forward gains 1 %
    // from the same and the flat backward nothing, so they keep workgroup = row / tile.
    const int64_t t = xcd_chunked_rotating<12>(blockIdx.x, gridDim.x) * R + threadIdx.x / THREADS;
    const int tid = threadIdx.x % THREADS;
    if (t >= tokens) return;                                   // whole waves (R > 1 only)
    const int64_t begin = t * vocab, end = begin + vocab;
    const int64_t p0 = begin >> 3, p1 = (end - 1) >> 3;        // packs of the flat tensor that hold the row
    const int np = static_cast<int>(p1 - p0) + 1;
    const int lo = static_cast<int>(begin - p0 * kPack), hi = lo + vocab;   // the row inside its window of packs
    // only the row's first and last pack can be shared with a neighbouring row (or overhang the tensor)
    const int ragged_first = (begin & 7) != 0 || np == 1 ? 0 : -1;
    const int ragged_last = (end & 7) != 0 || np == 1 ? np - 1 : -1;
    const T* src = logits + p0 * kPack;
    T* dst = dlogits + p0 * kPack;
    const int k0 = target[t];
    if (is_ignored(k0, vocab, ignore_index)) {                 // uniform over the workgroup: zeros, nothing is read
        const float z[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int k = 0; k < NP; ++k) {
            const int i = tid + k * THREADS;
            if (i >= np) continue;
            if (i != ragged_first && i != ragged_last) {
                store8<T, kBwdNTS>(dst + i * kPack, z);
            } else {
                const unsigned mask = row_mask(i, lo, hi);
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (mask >> j & 1u) dst[i * kPack + j] = from_f32<T>(0.0f);
            }
        }
        if (tid == 0) {
            loss[t] = 0.0f;
            lse[t] = 0.0f;
            if (nll) nll[t] = 0.0f;
        }
        return;
    }
    const float hk = tid == 0 ? to_f32<T>(logits[begin + k0]) : 0.0f;
    // Elements of a ragged pack that belong to another row, and packs past the row, are held as
    // -inf: neutral for the maximum and for the sum of exponentials, so the wide passes carry no
    // per-element conditions; the sum of the logits skips them explicitly.
    // Iterations whose packs all lie past the row are skipped as a whole.  That uniform test also keeps
    // the compiler from interleaving the iterations: 16-bit rows of 8 packs per thread then fit 64
    // registers, so two 1024-thread workgroups share a compute unit and one streams while the other
    // computes (measured: 385 us with one workgroup per unit, 301 us with two, at 8192 x 50257).
    RawPack<T> raw[NP];
#pragma unroll
    for (int k = 0; k < NP; ++k) {
        const int i = tid + k * THREADS;
        if (k * THREADS >= np) {
            raw[k] = zero_raw<T>();
        } else if (i < np && i != ragged_first && i != ragged_last) {
            raw[k] = load_raw<T, kNT>(src + i * kPack);
        } else if (i < np) {
            const unsigned mask = row_mask(i, lo, hi);
            float h[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) h[j] = (mask >> j & 1u) ? to_f32<T>(src[i * kPack + j]) : -INFINITY;
            raw[k] = pack_raw<T>(h);                           // exact: the values come from T, and -inf exists in T
        } else {
            float h[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) h[j] = -INFINITY;
            raw[k] = pack_raw<T>(h);
        }
    }
    // pass 1: the maximum (fp16: two elements per instruction, no widening)
    float m = -INFINITY;
    if constexpr (kIsF16<T>) {
        half2v mm = {static_cast<_Float16>(-INFINITY), static_cast<_Float16>(-INFINITY)};
#pragma unroll
        for (int k = 0; k < NP; ++k) {
            if (k * THREADS >= np) continue;
            const Half8 h = __builtin_bit_cast(Half8, raw[k].u);
#pragma unroll
            for (int c = 0; c < 4; ++c) mm = __builtin_elementwise_max(mm, h.v[c]);
        }
        m = fmaxf(static_cast<float>(mm.x), static_cast<float>(mm.y));
    } else {
#pragma unroll
        for (int k = 0; k < NP; ++k) {
            if (k * THREADS >= np) continue;
            float h[8];
            unpack<T>(raw[k], h);
#pragma unroll
            for (int j = 0; j < 8; ++j) m = fmaxf(m, h[j]);
        }
    }
    // the maximum of h * log2(e) is the maximum of h times log2(e): rounding is monotonic.  The
    // exponentials are kept for pass 3 in the storage type, so fp16 shifts them up by 2^14: the
    // largest is 16384 and relative precision holds down to 2^-28 of it.
    constexpr float kShift = kIsF16<T> ? 14.0f : 0.0f;
    const float Ms = block_allreduce<NW, OpMax>(m, lds[0]) * kLog2eX - kShift;
    // pass 2: e = exp2(h log2e - Ms) replaces h in the registers; sums of e (before its rounding) and of h
    float sx = 0.0f, sh = 0.0f;
#pragma unroll
    for (int k = 0; k < NP; ++k) {
        const int i = tid + k * THREADS;
        if (k * THREADS >= np) continue;
        opaque<T>(raw[k]);                                     // widened again in each pass: the row stays packed in between
        const bool whole = i < np && i != ragged_first && i != ragged_last;
        if constexpr (kIsF16<T>) {
            if (whole) {                                       // sum of the logits: two per instruction, fp32 accumulator
                const Half8 h2 = __builtin_bit_cast(Half8, raw[k].u);
                const half2v ones = {static_cast<_Float16>(1.0f), static_cast<_Float16>(1.0f)};
#pragma unroll
                for (int c = 0; c < 4; ++c) sh = __builtin_amdgcn_fdot2(h2.v[c], ones, sh, false);
            }
        }
        float h[8];
        unpack<T>(raw[k], h);
        if (!kIsF16<T> && whole) {
#pragma unroll
            for (int j = 0; j < 8; ++j) sh += h[j];
        }
        if (!whole && i < np) {
#pragma unroll
            for (int j = 0; j < 8; ++j) sh += h[j] == -INFINITY ? 0.0f : h[j];
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            h[j] = __builtin_amdgcn_exp2f(fmaf(h[j], kLog2eX, -Ms));     // exp2(-inf) = 0
            sx += h[j];
        }
        raw[k] = pack_raw<T>(h);
    }
    sx = group_allreduce<64, OpSum>(sx);
    sh = group_allreduce<64, OpSum>(sh);
    float S = sx, SH = sh;
    if constexpr (NW > 1) {                                    // both sums through LDS in one exchange
        __syncthreads();                                       // lds[0] was read by the maximum
        if ((tid & 63) == 0) {
            lds[0][tid >> 6] = sx;
            lds[1][tid >> 6] = sh;
        }
        __syncthreads();
        S = lds[0][0];
        SH = lds[1][0];
#pragma unroll
        for (int w = 1; w < NW; ++w) { S += lds[0][w]; SH += lds[1][w]; }
    }
    const float l = (Ms + __builtin_amdgcn_logf(S)) * kLn2X;       // v_log_f32 is log2
    if (tid == 0) {
        lse[t] = l;
        loss[t] = l - (1.0f - alpha) * hk - (alpha / static_cast<float>(vocab)) * SH;
        if (nll) nll[t] = l - hk;
    }
    // pass 3: dlogits = grad_scale * (e / S - alpha/V) - grad_scale * (1 - alpha) [target], one fma per element
    const float c1 = grad_scale / S;
    const float c0 = -grad_scale * (alpha / static_cast<float>(vocab));
    const float hit = grad_scale * (1.0f - alpha);
    const int ki = static_cast<int>(((begin + k0) >> 3) - p0);  // the pack of the target logit, and its place there
    const int kj = static_cast<int>((begin + k0) & 7);
#pragma unroll
    for (int k = 0; k < NP; ++k) {
        const int i = tid + k * THREADS;
        if (i >= np) continue;
        float h[8];
        opaque<T>(raw[k]);
        unpack<T>(raw[k], h);
#pragma unroll
        for (int j = 0; j < 8; ++j) h[j] = fmaf(h[j], c1, c0);
        if (i == ki) {
#pragma unroll
            for (int j = 0; j < 8; ++j) h[j] -= (j == kj) ? hit : 0.0f;
        }
        if (i != ragged_first && i != ragged_last) {
            store8<T, kBwdNTS>(dst + i * kPack, h);
        } else {
            const unsigned mask = row_mask(i, lo, hi);
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (mask >> j & 1u) dst[i * kPack + j] = from_f32<T>(h[j]);
        }
    }
}

// sums = { sum loss, sum nll, count } over non-ignored tokens: one workgroup, double
// accumulators, fixed strided order and a fixed LDS tree.  With the per-token nll at
// hand every input is a contiguous array; without it the target logits are gathered
// (one DRAM page each), 8 per thread in flight.
template <typename T>
__global__ __launch_bounds__(1024) void xent_sums_kernel(float* __restrict__ sums, const float* __restrict__ loss,
                                                         const float* __restrict__ nll, const float* __restrict__ lse,
                                                         const T* __restrict__ logits,
                                                         const int32_t* __restrict__ target, int64_t tokens, int vocab,
                                                         int ignore_index)
{
    __shared__ double sm[3][16];
    const int tid = threadIdx.x;
    double a = 0.0, b = 0.0, c = 0.0;
    // One workgroup walks all tokens, 8 x 1024 per trip; the next trip's loads are issued before this
    // trip's values are used (one compute unit alone is bound by latency, not bandwidth: without the
    // prefetch a quarter of a million tokens took 120 us, four times the forward kernel's share).
    int k[8], nk[8];
    float ls[8], lo[8], nls[8], nlo[8];
    auto fetch = [&](int64_t t0, int (&kk)[8], float (&llo)[8], float (&lls)[8]) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int64_t t = t0 + u * 1024;
            kk[u] = t < tokens ? target[t] : ignore_index;
            llo[u] = t < tokens ? loss[t] : 0.0f;
            lls[u] = t < tokens ? (nll ? nll[t] : lse[t]) : 0.0f;
        }
    };
    fetch(tid, nk, nlo, nls);
    for (int64_t t0 = tid; t0 < tokens; t0 += 8 * 1024) {
#pragma unroll
        for (int u = 0; u < 8; ++u) { k[u] = nk[u]; lo[u] = nlo[u]; ls[u] = nls[u]; }
        if (t0 + 8 * 1024 < tokens) fetch(t0 + 8 * 1024, nk, nlo, nls);
        float hk[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) hk[u] = 0.0f;
        if (!nll) {
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int64_t t = t0 + u * 1024;
                const bool live = t < tokens && !is_ignored(k[u], vocab, ignore_index);
                hk[u] = live ? to_f32<T>(logits[t * vocab + k[u]]) : 0.0f;
            }
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int64_t t = t0 + u * 1024;
            if (t < tokens && !is_ignored(k[u], vocab, ignore_index)) {
                a += static_cast<double>(lo[u]);
                b += static_cast<double>(ls[u]) - static_cast<double>(hk[u]);
                c += 1.0;
            }
        }
    }
    // fixed butterfly inside each wave, then the 16 wave totals in wave order: one barrier
#pragma unroll
    for (int w = 32; w > 0; w >>= 1) {
        a += __shfl_xor(a, w, 64);
        b += __shfl_xor(b, w, 64);
        c += __shfl_xor(c, w, 64);
    }
    if ((tid & 63) == 0) { sm[0][tid >> 6] = a; sm[1][tid >> 6] = b; sm[2][tid >> 6] = c; }
    __syncthreads();
    if (tid < 3) {
        double t = 0.0;
#pragma unroll
        for (int w = 0; w < 16; ++w) t += sm[tid][w];
        sums[tid] = static_cast<float>(t);
    }
}

template <typename T>
static lsq_status xent_fwd_dispatch(float* loss, float* nll, float* lse, float* sums, const void* logits, const int32_t* target,
                                    int64_t tokens, int32_t vocab, float alpha, int32_t ignore_index, hipStream_t s)
{
    const T* lp = static_cast<const T*>(logits);
    if (vocab <= 2048)
        hipLaunchKernelGGL((xent_fwd_kernel<T, 64, 4>), dim3(static_cast<unsigned>(ceil_div(tokens, 4))), dim3(256), 0, s,
                           loss, nll, lse, lp, target, tokens, vocab, alpha, ignore_index);
    else
        hipLaunchKernelGGL((xent_fwd_kernel<T>), dim3(static_cast<unsigned>(tokens)), dim3(kXentThreads), 0, s,
                           loss, nll, lse, lp, target, tokens, vocab, alpha, ignore_index);
    if (sums)
        hipLaunchKernelGGL((xent_sums_kernel<T>), dim3(1), dim3(1024), 0, s, sums, loss, nll, lse, lp, target, tokens,
                           vocab, ignore_index);
    return launch_status();
}

template <typename T>
static lsq_status xent_bwd_dispatch(void* dlogits, const void* logits, const float* lse, const int32_t* target,
                                    int64_t tokens, int32_t vocab, float alpha, int32_t ignore_index, float grad_scale,
                                    hipStream_t s)
{
    // the flat kernel needs chunk <= vocab (a chunk touches at most two rows): pick the unroll by vocab
    const int64_t npacks = tokens * vocab / kPack;
    const int U = vocab >= 4 * kXbThreads * kPack ? 4 : vocab >= 2 * kXbThreads * kPack ? 2 : vocab >= kXbThreads * kPack ? 1 : 0;
    const int64_t blocks = U ? ceil_div(npacks, U * kXbThreads) : 0;
    T* dp = static_cast<T*>(dlogits);
    const T* lp = static_cast<const T*>(logits);
    if (U == 4 && blocks <= 0x7FFFFFFF)
        hipLaunchKernelGGL((xent_bwd_flat_kernel<T, 4>), dim3(static_cast<unsigned>(blocks)), dim3(kXbThreads), 0, s, dp, lp, lse,
                           target, tokens, vocab, alpha, ignore_index, grad_scale);
    else if (U == 2 && blocks <= 0x7FFFFFFF)
        hipLaunchKernelGGL((xent_bwd_flat_kernel<T, 2>), dim3(static_cast<unsigned>(blocks)), dim3(kXbThreads), 0, s, dp, lp, lse,
                           target, tokens, vocab, alpha, ignore_index, grad_scale);
    else if (U == 1 && blocks <= 0x7FFFFFFF)
        hipLaunchKernelGGL((xent_bwd_flat_kernel<T, 1>), dim3(static_cast<unsigned>(blocks)), dim3(kXbThreads), 0, s, dp, lp, lse,
                           target, tokens, vocab, alpha, ignore_index, grad_scale);
    else
        hipLaunchKernelGGL((xent_bwd_kernel<T>), dim3(static_cast<unsigned>(tokens)), dim3(kXentThreads), 0, s, dp, lp,
                           lse, target, vocab, alpha, ignore_index, grad_scale);
    return launch_status();
}

// Rows of up to 1024 x 8 packs stay in registers; longer ones take the two operators back to back.
template <typename T>
static lsq_status xent_fused_dispatch(float* loss, float* nll, float* lse, float* sums, void* dlogits, const void* logits,
                                      const int32_t* target, int64_t tokens, int32_t vocab, float alpha,
                                      int32_t ignore_index, float grad_scale, hipStream_t s)
{
    const int64_t rp = (static_cast<int64_t>(vocab) + 7) / 8 + 1;       // packs a row can touch
    T* dp = static_cast<T*>(dlogits);
    const T* lp = static_cast<const T*>(logits);
#define LSQ_XF(TH, NPK, ROWS)                                                                                        \
    hipLaunchKernelGGL((xent_fused_kernel<T, TH, NPK, ROWS>), dim3(static_cast<unsigned>(ceil_div(tokens, ROWS))), dim3(TH * ROWS), 0, s, \
                       loss, nll, lse, dp, lp, target, tokens, vocab, alpha, ignore_index, grad_scale)
    if (rp <= 64 * 2) LSQ_XF(64, 2, 4);         // short rows: one wave per token, four tokens per workgroup, no barriers
    else if (rp <= 64 * 4) LSQ_XF(64, 4, 4);
    else if (rp <= 256 * 2) LSQ_XF(256, 2, 1);
    else if (rp <= 256 * 4) LSQ_XF(256, 4, 1);
    else if (rp <= 256 * 8) LSQ_XF(256, 8, 1);
    else if (rp <= 1024 * 4) LSQ_XF(1024, 4, 1);
    else if (rp <= 1024 * 8) LSQ_XF(1024, 8, 1);
    else {
        const lsq_status st = xent_fwd_dispatch<T>(loss, nll, lse, nullptr, logits, target, tokens, vocab, alpha, ignore_index, s);
        if (st != LSQ_OK) return st;
        const lsq_status sb = xent_bwd_dispatch<T>(dlogits, logits, lse, target, tokens, vocab, alpha, ignore_index, grad_scale, s);
        if (sb != LSQ_OK) return sb;
    }
#undef LSQ_XF
    if (sums)
        hipLaunchKernelGGL((xent_sums_kernel<T>), dim3(1), dim3(1024), 0, s, sums, loss, nll, lse, lp, target, tokens,
                           vocab, ignore_index);
    return launch_status();
}

}  // namespace lsq

extern "C" lsq_status lsq_ls_xent_fwd(float* loss, float* nll, float* lse, float* sums, const void* logits, const int32_t* target,
                                      int64_t tokens, int32_t vocab, float alpha, int32_t ignore_index, lsq_dtype dt,
                                      void* stream)
{
    using namespace lsq;
    LSQ_REQUIRE(tokens >= 0 && tokens <= 0x7FFFFFFF && vocab > 0);
    LSQ_REQUIRE(alpha >= 0.0f && alpha <= 1.0f);
    if (!valid_dtype(dt)) return LSQ_UNSUPPORTED_DTYPE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (tokens == 0) return sums ? zero_fill(sums, 3, s) : LSQ_OK;
    LSQ_REQUIRE(loss && lse && logits && target);
    LSQ_ALIGNED(logits);
    switch (dt) {
        case LSQ_F16: return xent_fwd_dispatch<f16>(loss, nll, lse, sums, logits, target, tokens, vocab, alpha, ignore_index, s);
        case LSQ_BF16: return xent_fwd_dispatch<bf16>(loss, nll, lse, sums, logits, target, tokens, vocab, alpha, ignore_index, s);
        default: return xent_fwd_dispatch<float>(loss, nll, lse, sums, logits, target, tokens, vocab, alpha, ignore_index, s);
    }
}

extern "C" lsq_status lsq_ls_xent_bwd(void* dlogits, const void* logits, const float* lse, const int32_t* target,
                                      int64_t tokens, int32_t vocab, float alpha, int32_t ignore_index,
                                      float grad_scale, lsq_dtype dt, void* stream)
{
    using namespace lsq;
    LSQ_REQUIRE(tokens >= 0 && tokens <= 0x7FFFFFFF && vocab > 0);
    LSQ_REQUIRE(alpha >= 0.0f && alpha <= 1.0f);
    if (!valid_dtype(dt)) return LSQ_UNSUPPORTED_DTYPE;
    if (tokens == 0) return LSQ_OK;
    LSQ_REQUIRE(dlogits && logits && lse && target);
    LSQ_ALIGNED(dlogits); LSQ_ALIGNED(logits);
    hipStream_t s = static_cast<hipStream_t>(stream);
    switch (dt) {
        case LSQ_F16: return xent_bwd_dispatch<f16>(dlogits, logits, lse, target, tokens, vocab, alpha, ignore_index, grad_scale, s);
        case LSQ_BF16: return xent_bwd_dispatch<bf16>(dlogits, logits, lse, target, tokens, vocab, alpha, ignore_index, grad_scale, s);
        default: return xent_bwd_dispatch<float>(dlogits, logits, lse, target, tokens, vocab, alpha, ignore_index, grad_scale, s);
    }
}

extern "C" lsq_status lsq_ls_xent_fwd_bwd(float* loss, float* nll, float* lse, float* sums, void* dlogits, const void* logits,
                                          const int32_t* target, int64_t tokens, int32_t vocab, float alpha,
                                          int32_t ignore_index, float grad_scale, lsq_dtype dt, void* stream)
{
    using namespace lsq;
    LSQ_REQUIRE(tokens >= 0 && tokens <= 0x7FFFFFFF && vocab > 0);
    LSQ_REQUIRE(alpha >= 0.0f && alpha <= 1.0f);
    if (!valid_dtype(dt)) return LSQ_UNSUPPORTED_DTYPE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (tokens == 0) return sums ? zero_fill(sums, 3, s) : LSQ_OK;
    LSQ_REQUIRE(loss && lse && dlogits && logits && target);
    LSQ_ALIGNED(dlogits); LSQ_ALIGNED(logits);
    // in place, the logits are gone by the time the sums are taken: the sum of nll then has to come
    // from the per-token nll, which the caller must ask for
    LSQ_REQUIRE(!(sums && !nll && dlogits == logits));
    switch (dt) {
        case LSQ_F16: return xent_fused_dispatch<f16>(loss, nll, lse, sums, dlogits, logits, target, tokens, vocab, alpha, ignore_index, grad_scale, s);
        case LSQ_BF16: return xent_fused_dispatch<bf16>(loss, nll, lse, sums, dlogits, logits, target, tokens, vocab, alpha, ignore_index, grad_scale, s);
        default: return xent_fused_dispatch<float>(loss, nll, lse, sums, dlogits, logits, target, tokens, vocab, alpha, ignore_index, grad_scale, s);
    }
}
