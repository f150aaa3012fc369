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

#ifndef LSQ_NT
#define LSQ_NT 1
#endif
constexpr bool kNT = LSQ_NT != 0;   // nontemporal hint on the streamed tensors
#ifndef LSQ_XB_NTL
#define LSQ_XB_NTL 1
#endif
#ifndef LSQ_XB_NTS
#define LSQ_XB_NTS 1
#endif
constexpr bool kBwdNTL = LSQ_XB_NTL != 0, kBwdNTS = LSQ_XB_NTS != 0;

constexpr float kLog2eX = 1.4426950408889634f;
constexpr float kLn2X = 0.6931471805599453f;
#ifndef LSQ_XENT_THREADS
#define LSQ_XENT_THREADS 256
#endif
#ifndef LSQ_XENT_UNROLL
#define LSQ_XENT_UNROLL 4
#endif
constexpr int kXentThreads = LSQ_XENT_THREADS;
constexpr int kXentUnroll = LSQ_XENT_UNROLL;

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
};

template <typename T>
__global__ __launch_bounds__(kXentThreads) void xent_fwd_kernel(float* __restrict__ loss, float* __restrict__ nll,
                                                               float* __restrict__ lse,
                                                               const T* __restrict__ logits,
                                                               const int32_t* __restrict__ target, int vocab,
                                                               float alpha, int ignore_index)
{
    __shared__ float lds[kXentThreads / 64];
    const int64_t t = blockIdx.x;
    const int tid = threadIdx.x;
    const int k0 = target[t];
    if (is_ignored(k0, vocab, ignore_index)) {    // uniform over the workgroup: a padded token's row is not read
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
    for (int64_t p = base + tid; p < r.pack_end; p += kXentUnroll * kXentThreads) {
        RawPack<T> raw[kXentUnroll];
        bool ok[kXentUnroll];
#pragma unroll
        for (int u = 0; u < kXentUnroll; ++u) {
            const int64_t q = p + u * kXentThreads;
            ok[u] = q >= r.pack_begin && q < r.pack_end;
            if (ok[u]) raw[u] = load_raw<T, kNT>(logits + q * kPack);
            else raw[u] = zero_raw<T>();
        }
#pragma unroll
        for (int u = 0; u < kXentUnroll; ++u) {
            if (ok[u]) {
                float h[8];
                unpack<T>(raw[u], h);
                st.add8(h);
            }
        }
    }
    const float M = block_allreduce<kXentThreads / 64, OpMax>(st.m, lds);
    const float S = block_allreduce<kXentThreads / 64, OpSum>(st.s * __builtin_amdgcn_exp2f(st.m - M), lds);
    const float SH = block_allreduce<kXentThreads / 64, OpSum>(st.sh, lds);
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
// of U*256 aligned packs whatever rows they fall in, so the access pattern is that
// of a plain copy (few DRAM pages open at a time, every access 128-bit and aligned,
// no scalar head/tail per row).  Measured on MI355X a copy laid out one row per
// workgroup reaches 4.8 TB/s at vocab 50257, the flat one 6.6 TB/s.  The chunk is
// never longer than a row, so it touches at most two rows, A and B: their lse and
// target are wave-uniform and sit in scalar registers.  Only the one pack that
// straddles the boundary (vocab % 8 != 0) selects per element.  Packs of ignored
// rows are not read at all.
template <typename T, int U>
__global__ __launch_bounds__(256) void xent_bwd_flat_kernel(T* dlogits, const T* logits,
                                                            const float* __restrict__ lse,
                                                            const int32_t* __restrict__ target, int64_t tokens,
                                                            int vocab, float alpha, int ignore_index, float grad_scale)
{
    const int64_t total = tokens * vocab;
    const int64_t npacks = total / kPack;                     // full packs; the ragged end is handled below
    const int64_t pb = static_cast<int64_t>(blockIdx.x) * (U * 256);
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
            const int64_t q = pb + u * 256 + threadIdx.x;
            if (q < npacks) store8<T, kBwdNTS>(dlogits + q * kPack, zero);
        }
        return;
    }

    float h[U][8];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t q = pb + u * 256 + threadIdx.x;
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
        const int64_t q = pb + u * 256 + threadIdx.x;
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
    for (int64_t t0 = tid; t0 < tokens; t0 += 8 * 1024) {
        int k[8];
        float ls[8], lo[8], hk[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int64_t t = t0 + u * 1024;
            k[u] = t < tokens ? target[t] : ignore_index;
            lo[u] = t < tokens ? loss[t] : 0.0f;
            if (nll) { ls[u] = t < tokens ? nll[t] : 0.0f; hk[u] = 0.0f; }
            else ls[u] = t < tokens ? lse[t] : 0.0f;
        }
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
    hipLaunchKernelGGL((xent_fwd_kernel<T>), dim3(static_cast<unsigned>(tokens)), dim3(kXentThreads), 0, s,
                       loss, nll, lse, lp, target, vocab, alpha, ignore_index);
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
    const int U = vocab >= 4 * 256 * kPack ? 4 : vocab >= 2 * 256 * kPack ? 2 : vocab >= 256 * kPack ? 1 : 0;
    const int64_t blocks = U ? ceil_div(npacks, U * 256) : 0;
    T* dp = static_cast<T*>(dlogits);
    const T* lp = static_cast<const T*>(logits);
    if (U == 4 && blocks <= 0x7FFFFFFF)
        hipLaunchKernelGGL((xent_bwd_flat_kernel<T, 4>), dim3(static_cast<unsigned>(blocks)), dim3(256), 0, s, dp, lp, lse,
                           target, tokens, vocab, alpha, ignore_index, grad_scale);
    else if (U == 2 && blocks <= 0x7FFFFFFF)
        hipLaunchKernelGGL((xent_bwd_flat_kernel<T, 2>), dim3(static_cast<unsigned>(blocks)), dim3(256), 0, s, dp, lp, lse,
                           target, tokens, vocab, alpha, ignore_index, grad_scale);
    else if (U == 1 && blocks <= 0x7FFFFFFF)
        hipLaunchKernelGGL((xent_bwd_flat_kernel<T, 1>), dim3(static_cast<unsigned>(blocks)), dim3(256), 0, s, dp, lp, lse,
                           target, tokens, vocab, alpha, ignore_index, grad_scale);
    else
        hipLaunchKernelGGL((xent_bwd_kernel<T>), dim3(static_cast<unsigned>(tokens)), dim3(kXentThreads), 0, s, dp, lp,
                           lse, target, vocab, alpha, ignore_index, grad_scale);
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
