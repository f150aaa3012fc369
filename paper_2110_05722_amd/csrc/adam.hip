// Mixed-precision Adam over one flat workspace (Sec. IV-C of the paper): the
// low-precision gradient is widened in registers, the fp32 master parameter and
// both moments are read once and written once, and the low-precision copy of the
// parameter that the next forward pass reads is produced by the same pass.
// One launch per step, whatever the number of parameter tensors in the workspace.
//
// HBM-bound: 28 bytes per parameter (26 without the low-precision copy).  Each
// thread owns 4 consecutive parameters: one 128-bit load of p, m and v, one
// 64-bit load of g, the mirror-image stores, every wave access fully coalesced,
// all of them nontemporal (each byte is touched once per step).  Measured: one
// pack per thread beats both two packs per thread and a persistent grid-stride
// loop, and the nontemporal hint is worth 10 %.
#include "host.hpp"

namespace lsq {

struct AdamParams {
    float lr, beta1, beta2, omb1, omb2, eps, wd, rc1, rc2, inv_scale;
    int adamw;
};

__device__ __forceinline__ void adam_update(float& p, float& m, float& v, float g, const AdamParams& a)
{
    float gh = g * a.inv_scale;
    if (!a.adamw) gh = fmaf(a.wd, p, gh);
    m = fmaf(a.beta1, m, a.omb1 * gh);
    v = fmaf(a.beta2, v, a.omb2 * gh * gh);
    float upd = (m * a.rc1) / (sqrtf(v * a.rc2) + a.eps);
    if (a.adamw) upd = fmaf(a.wd, p, upd);
    p = fmaf(-a.lr, upd, p);
}

constexpr int kAdamPack = 4;

// Launch shape of the trainers.  With separate arrays: one-wave workgroups (a tile of 256 elements, 1 KB of each
// fp32 array), and each XCD takes runs of 1 MB of consecutive tiles (xcd_chunked in device.hpp).  Measured on the
// same buffers in one process, three to six processes each (fraction of the 8 TB/s peak, 774 M parameters):
//   256 threads, tile = workgroup   0.68-0.72   (where the five arrays land decides which)
//   256 threads, runs of 1 MB       0.71-0.735
//   128 threads, runs of 1 MB       0.72-0.75
//    64 threads, tile = workgroup   0.72-0.75
//    64 threads, runs of 1 MB       0.755-0.77  in every process (runs of 512 KB..4 MB alike; 128-256 KB less steady)
// 512 / 1024 threads, or two / four packs per thread, are slower than 256 x 1; rotating which XCD takes which of
// eight tiles changes nothing.  The blocked state, one address stream already, also gains from one-wave workgroups
// (0.81 against 0.79 with 256 threads; 128 threads: 0.71) but not from runs (0.78-0.81 with runs of 4-1024 tiles).
constexpr int kAdamThreads = 64;
constexpr int kAdamRunBytes = 1 << 20;
template <bool BLOCKED>
__device__ __forceinline__ int64_t adam_tile()
{
    return xcd_chunked<BLOCKED ? 1 : kAdamRunBytes / (kAdamThreads * 16)>(blockIdx.x, gridDim.x);
}

// Blocked optimizer state: the three fp32 arrays that only the trainer reads are kept
// as blocks of kAdamBlock elements, [p block | m block | v block] back to back, instead
// of three arrays a gigabyte apart.  The bytes moved are the same; the read-modify-write
// then walks ONE address stream (plus g in, p_lp out) instead of three, which the
// memory system rewards: 6.3 TB/s against 5.5-5.85 TB/s measured at 774 M parameters.
// Swept 1 Ki .. 1 Mi elements per block: 8 Ki is the optimum, 64 Ki+ gives back half of it.
constexpr int kAdamBlock = LSQ_ADAM_BLOCK;
static_assert(kAdamBlock % (kAdamThreads * kAdamPack) == 0, "a workgroup must not straddle a block");

// offset of element e of the first array inside a blocked state of `arrays` arrays; the other
// arrays follow at +1 and +2 blocks
__device__ __host__ __forceinline__ int64_t adam_state_offset(int64_t e, int arrays = 3)
{
    return (e / kAdamBlock) * (arrays * static_cast<int64_t>(kAdamBlock)) + (e % kAdamBlock);
}

template <typename G, typename PL, bool HAS_PL, bool BLOCKED>
__global__ __launch_bounds__(kAdamThreads) void adam_kernel(float* __restrict__ p, float* __restrict__ m,
                                                   float* __restrict__ v, const G* __restrict__ g,
                                                   PL* __restrict__ plp, int64_t n, AdamParams a)
{
    const int64_t e = (adam_tile<BLOCKED>() * kAdamThreads + threadIdx.x) * kAdamPack;
    if constexpr (BLOCKED) {        // p is the state; this thread's pack sits at one offset in all three blocks
        const int64_t so = adam_state_offset(e) - e;
        p += so;
        m = p + kAdamBlock;
        v = p + 2 * kAdamBlock;
    }
    if (e + kAdamPack <= n) {
        float pf[4], mf[4], vf[4], gf[4];
        load4<float, true>(p + e, pf);
        load4<float, true>(m + e, mf);
        load4<float, true>(v + e, vf);
        load4<G, true>(g + e, gf);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            adam_update(pf[j], mf[j], vf[j], gf[j], a);
            // pin the fp32 value: without this the compiler folds the last fma into the
            // fp16 conversion (one rounding of the exact result), and the low-precision
            // copy would no longer be the rounded image of the stored fp32 parameter
            asm volatile("" : "+v"(pf[j]));
        }
        store4<float, true>(p + e, pf);
        store4<float, true>(m + e, mf);
        store4<float, true>(v + e, vf);
        if constexpr (HAS_PL) store4<PL, true>(plp + e, pf);
    } else {
        for (int64_t i = e; i < n; ++i) {      // ragged tail: at most 3 elements, one thread
            float pf = p[i], mf = m[i], vf = v[i];
            adam_update(pf, mf, vf, to_f32<G>(g[i]), a);
            asm volatile("" : "+v"(pf));
            p[i] = pf; m[i] = mf; v[i] = vf;
            if constexpr (HAS_PL) plp[i] = from_f32<PL>(pf);
        }
    }
}

template <typename G, bool BLOCKED>
static lsq_status adam_dispatch(float* p, float* m, float* v, const void* g, void* plp, int64_t n,
                                const AdamParams& a, int p_lp_dt, hipStream_t s)
{
    const int64_t packs = ceil_div(n, kAdamPack);
    const dim3 grid(static_cast<unsigned>(ceil_div(packs, kAdamThreads))), block(kAdamThreads);
    const G* gp = static_cast<const G*>(g);
    if (!plp)
        hipLaunchKernelGGL((adam_kernel<G, f16, false, BLOCKED>), grid, block, 0, s, p, m, v, gp, static_cast<f16*>(nullptr), n, a);
    else if (p_lp_dt == LSQ_F16)
        hipLaunchKernelGGL((adam_kernel<G, f16, true, BLOCKED>), grid, block, 0, s, p, m, v, gp, static_cast<f16*>(plp), n, a);
    else
        hipLaunchKernelGGL((adam_kernel<G, bf16, true, BLOCKED>), grid, block, 0, s, p, m, v, gp, static_cast<bf16*>(plp), n, a);
    return launch_status();
}

// state <- (p, m, v) (PACK) or (p, m, v) <- state; absent m / v read as zeros / are skipped.
// One thread per 4 elements of the padded length; the padding of the last block is zero-filled.
template <bool PACK>
__global__ __launch_bounds__(256) void adam_state_move(float* state, float* p, float* m, float* v, int64_t n, int64_t padded,
                                                       int arrays)
{
    const int64_t e = (static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x) * kAdamPack;
    if (e >= padded) return;
    float* sp = state + adam_state_offset(e, arrays);
    float* arr[3] = {p, m, v};
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        if (k >= arrays) break;
        float* a = arr[k];
        float* sk = sp + k * kAdamBlock;
        if (e + kAdamPack <= n) {
            float f[4] = {0, 0, 0, 0};
            if (PACK) {
                if (a) load4<float, true>(a + e, f);
                store4<float, true>(sk, f);
            } else if (a) {
                load4<float, true>(sk, f);
                store4<float, true>(a + e, f);
            }
        } else {
            for (int j = 0; j < kAdamPack; ++j) {       // ragged end of the arrays, padding of the state
                const int64_t i = e + j;
                if (PACK) sk[j] = (a && i < n) ? a[i] : 0.0f;
                else if (a && i < n) a[i] = sk[j];
            }
        }
    }
}

// ---- the paper's own layout: the workspace holds the parameter in low precision and
// it is updated in place (Sec. IV-C, "on-the-fly conversion"): 22 bytes per parameter.
template <typename T, bool BLOCKED>
__global__ __launch_bounds__(kAdamThreads) void adam_lp_kernel(T* __restrict__ p, float* __restrict__ m, float* __restrict__ v,
                                                      const T* __restrict__ g, int64_t n, AdamParams a)
{
    const int64_t e = (adam_tile<BLOCKED>() * kAdamThreads + threadIdx.x) * kAdamPack;
    if constexpr (BLOCKED) {        // m is the [m | v] state
        m += adam_state_offset(e, 2) - e;
        v = m + kAdamBlock;
    }
    if (e + kAdamPack <= n) {
        float pf[4], mf[4], vf[4], gf[4];
        load4<T, true>(p + e, pf);
        load4<float, true>(m + e, mf);
        load4<float, true>(v + e, vf);
        load4<T, true>(g + e, gf);
#pragma unroll
        for (int j = 0; j < 4; ++j) adam_update(pf[j], mf[j], vf[j], gf[j], a);
        store4<T, true>(p + e, pf);
        store4<float, true>(m + e, mf);
        store4<float, true>(v + e, vf);
    } else {
        for (int64_t i = e; i < n; ++i) {
            float pf = to_f32<T>(p[i]), mf = m[i], vf = v[i];
            adam_update(pf, mf, vf, to_f32<T>(g[i]), a);
            p[i] = from_f32<T>(pf); m[i] = mf; v[i] = vf;
        }
    }
}

// ---- SGD over the same flat workspace (the paper's second trainer): fp32 master p,
// optional fp32 momentum buffer, low-precision gradient in, low-precision copy out.
struct SgdParams { float lr, momentum, wd, inv_scale; int nesterov; };

template <bool MOM>
__device__ __forceinline__ void sgd_update(float& p, float& b, float g, const SgdParams& a)
{
    const float gh = fmaf(a.wd, p, g * a.inv_scale);
    float d = gh;
    if constexpr (MOM) {
        b = fmaf(a.momentum, b, gh);
        d = a.nesterov ? fmaf(a.momentum, b, gh) : b;
    }
    p = fmaf(-a.lr, d, p);
}

template <typename G, typename PL, bool HAS_PL, bool MOM, bool BLOCKED>
__global__ __launch_bounds__(kAdamThreads) void sgd_kernel(float* __restrict__ p, float* __restrict__ buf,
                                                  const G* __restrict__ g, PL* __restrict__ plp, int64_t n, SgdParams a)
{
    const int64_t e = (adam_tile<BLOCKED>() * kAdamThreads + threadIdx.x) * kAdamPack;
    if constexpr (BLOCKED) {        // p is the [p | momentum buffer] state
        p += adam_state_offset(e, 2) - e;
        buf = p + kAdamBlock;
    }
    if (e + kAdamPack <= n) {
        float pf[4], bf[4] = {0, 0, 0, 0}, gf[4];
        load4<float, true>(p + e, pf);
        if constexpr (MOM) load4<float, true>(buf + e, bf);
        load4<G, true>(g + e, gf);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            sgd_update<MOM>(pf[j], bf[j], gf[j], a);
            asm volatile("" : "+v"(pf[j]));     // the low-precision copy is the image of the STORED fp32 value
        }
        store4<float, true>(p + e, pf);
        if constexpr (MOM) store4<float, true>(buf + e, bf);
        if constexpr (HAS_PL) store4<PL, true>(plp + e, pf);
    } else {
        for (int64_t i = e; i < n; ++i) {
            float pf = p[i], bf = MOM ? buf[i] : 0.0f;
            sgd_update<MOM>(pf, bf, to_f32<G>(g[i]), a);
            asm volatile("" : "+v"(pf));
            p[i] = pf;
            if constexpr (MOM) buf[i] = bf;
            if constexpr (HAS_PL) plp[i] = from_f32<PL>(pf);
        }
    }
}

template <typename G, bool MOM, bool BLOCKED = false>
static lsq_status sgd_dispatch(float* p, float* buf, const void* g, void* plp, int64_t n, const SgdParams& a,
                               int p_lp_dt, hipStream_t s)
{
    const dim3 grid(static_cast<unsigned>(ceil_div(ceil_div(n, kAdamPack), kAdamThreads))), block(kAdamThreads);
    const G* gp = static_cast<const G*>(g);
    if (!plp)
        hipLaunchKernelGGL((sgd_kernel<G, f16, false, MOM, BLOCKED>), grid, block, 0, s, p, buf, gp, static_cast<f16*>(nullptr), n, a);
    else if (p_lp_dt == LSQ_F16)
        hipLaunchKernelGGL((sgd_kernel<G, f16, true, MOM, BLOCKED>), grid, block, 0, s, p, buf, gp, static_cast<f16*>(plp), n, a);
    else
        hipLaunchKernelGGL((sgd_kernel<G, bf16, true, MOM, BLOCKED>), grid, block, 0, s, p, buf, gp, static_cast<bf16*>(plp), n, a);
    return launch_status();
}

static bool make_adam_params(AdamParams* a, float lr, float beta1, float beta2, float eps, float weight_decay,
                             int32_t step, int32_t adamw, int32_t bias_correction, float inv_grad_scale)
{
    if (step < 1 || !(beta1 >= 0.0f && beta1 < 1.0f) || !(beta2 >= 0.0f && beta2 < 1.0f) || !(eps >= 0.0f)) return false;
    a->lr = lr; a->beta1 = beta1; a->beta2 = beta2;
    a->omb1 = 1.0f - beta1; a->omb2 = 1.0f - beta2;
    a->eps = eps; a->wd = weight_decay; a->inv_scale = inv_grad_scale; a->adamw = adamw != 0;
    // bias corrections in double on the host; the kernel multiplies by their reciprocals
    double c1 = 1.0, c2 = 1.0;
    if (bias_correction) {
        c1 = 1.0 - pow(static_cast<double>(beta1), static_cast<double>(step));
        c2 = 1.0 - pow(static_cast<double>(beta2), static_cast<double>(step));
    }
    a->rc1 = static_cast<float>(1.0 / c1);
    a->rc2 = static_cast<float>(1.0 / c2);
    return true;
}

}  // namespace lsq

extern "C" lsq_status lsq_adam_step(float* p, float* m, float* v, const void* g, void* p_lp, int64_t n,
                                    float lr, float beta1, float beta2, float eps, float weight_decay,
                                    int32_t step, int32_t adamw, int32_t bias_correction,
                                    float inv_grad_scale, lsq_dtype g_dt, lsq_dtype p_lp_dt, void* stream)
{
    using namespace lsq;
    LSQ_REQUIRE(n >= 0 && step >= 1);
    LSQ_REQUIRE(beta1 >= 0.0f && beta1 < 1.0f && beta2 >= 0.0f && beta2 < 1.0f);
    LSQ_REQUIRE(eps >= 0.0f);
    if (!valid_dtype(g_dt)) return LSQ_UNSUPPORTED_DTYPE;
    if (p_lp && p_lp_dt != LSQ_F16 && p_lp_dt != LSQ_BF16) return LSQ_UNSUPPORTED_DTYPE;
    if (n == 0) return LSQ_OK;
    LSQ_REQUIRE(p && m && v && g);
    LSQ_ALIGNED(p); LSQ_ALIGNED(m); LSQ_ALIGNED(v); LSQ_ALIGNED(g); LSQ_ALIGNED(p_lp);
    LSQ_REQUIRE(ceil_div(ceil_div(n, kAdamPack), kAdamThreads) <= 0x7FFFFFFF);

    AdamParams a;
    LSQ_REQUIRE(make_adam_params(&a, lr, beta1, beta2, eps, weight_decay, step, adamw, bias_correction, inv_grad_scale));

    hipStream_t s = static_cast<hipStream_t>(stream);
    switch (g_dt) {
        case LSQ_F16: return adam_dispatch<f16, false>(p, m, v, g, p_lp, n, a, p_lp_dt, s);
        case LSQ_BF16: return adam_dispatch<bf16, false>(p, m, v, g, p_lp, n, a, p_lp_dt, s);
        default: return adam_dispatch<float, false>(p, m, v, g, p_lp, n, a, p_lp_dt, s);
    }
}

extern "C" size_t lsq_trainer_state_bytes(int64_t n, int32_t arrays)
{
    if (n <= 0 || arrays < 1 || arrays > 3) return 0;
    return static_cast<size_t>(lsq::ceil_div(n, lsq::kAdamBlock)) * arrays * lsq::kAdamBlock * sizeof(float);
}

extern "C" lsq_status lsq_trainer_state_pack(float* state, const float* a0, const float* a1, const float* a2, int64_t n,
                                             int32_t arrays, void* stream)
{
    using namespace lsq;
    LSQ_REQUIRE(n >= 0 && arrays >= 1 && arrays <= 3);
    if (n == 0) return LSQ_OK;
    LSQ_REQUIRE(state && a0);
    LSQ_ALIGNED(state); LSQ_ALIGNED(a0); LSQ_ALIGNED(a1); LSQ_ALIGNED(a2);
    const int64_t padded = ceil_div(n, kAdamBlock) * kAdamBlock;
    LSQ_REQUIRE(padded / (256 * kAdamPack) <= 0x7FFFFFFF);
    hipLaunchKernelGGL((adam_state_move<true>), dim3(static_cast<unsigned>(padded / (256 * kAdamPack))), dim3(256), 0,
                       static_cast<hipStream_t>(stream), state, const_cast<float*>(a0), const_cast<float*>(a1),
                       const_cast<float*>(a2), n, padded, arrays);
    return launch_status();
}

extern "C" lsq_status lsq_trainer_state_unpack(float* a0, float* a1, float* a2, const float* state, int64_t n,
                                               int32_t arrays, void* stream)
{
    using namespace lsq;
    LSQ_REQUIRE(n >= 0 && arrays >= 1 && arrays <= 3);
    if (n == 0) return LSQ_OK;
    LSQ_REQUIRE(state);
    LSQ_ALIGNED(state); LSQ_ALIGNED(a0); LSQ_ALIGNED(a1); LSQ_ALIGNED(a2);
    const int64_t padded = ceil_div(n, kAdamBlock) * kAdamBlock;
    LSQ_REQUIRE(padded / (256 * kAdamPack) <= 0x7FFFFFFF);
    hipLaunchKernelGGL((adam_state_move<false>), dim3(static_cast<unsigned>(padded / (256 * kAdamPack))), dim3(256), 0,
                       static_cast<hipStream_t>(stream), const_cast<float*>(state), a0, a1, a2, n, padded, arrays);
    return launch_status();
}

extern "C" size_t lsq_adam_state_bytes(int64_t n) { return lsq_trainer_state_bytes(n, 3); }

extern "C" lsq_status lsq_adam_state_pack(float* state, const float* p, const float* m, const float* v, int64_t n,
                                          void* stream)
{
    return lsq_trainer_state_pack(state, p, m, v, n, 3, stream);
}

extern "C" lsq_status lsq_adam_state_unpack(float* p, float* m, float* v, const float* state, int64_t n, void* stream)
{
    return lsq_trainer_state_unpack(p, m, v, state, n, 3, stream);
}

extern "C" lsq_status lsq_adam_step_blocked(float* state, const void* g, void* p_lp, int64_t n, float lr, float beta1,
                                            float beta2, float eps, float weight_decay, int32_t step, int32_t adamw,
                                            int32_t bias_correction, float inv_grad_scale, lsq_dtype g_dt,
                                            lsq_dtype p_lp_dt, void* stream)
{
    using namespace lsq;
    LSQ_REQUIRE(n >= 0 && step >= 1);
    if (!valid_dtype(g_dt)) return LSQ_UNSUPPORTED_DTYPE;
    if (p_lp && p_lp_dt != LSQ_F16 && p_lp_dt != LSQ_BF16) return LSQ_UNSUPPORTED_DTYPE;
    AdamParams a;
    LSQ_REQUIRE(make_adam_params(&a, lr, beta1, beta2, eps, weight_decay, step, adamw, bias_correction, inv_grad_scale));
    if (n == 0) return LSQ_OK;
    LSQ_REQUIRE(state && g);
    LSQ_ALIGNED(state); LSQ_ALIGNED(g); LSQ_ALIGNED(p_lp);
    LSQ_REQUIRE(ceil_div(ceil_div(n, kAdamPack), kAdamThreads) <= 0x7FFFFFFF);
    hipStream_t s = static_cast<hipStream_t>(stream);
    switch (g_dt) {
        case LSQ_F16: return adam_dispatch<f16, true>(state, nullptr, nullptr, g, p_lp, n, a, p_lp_dt, s);
        case LSQ_BF16: return adam_dispatch<bf16, true>(state, nullptr, nullptr, g, p_lp, n, a, p_lp_dt, s);
        default: return adam_dispatch<float, true>(state, nullptr, nullptr, g, p_lp, n, a, p_lp_dt, s);
    }
}

namespace lsq {
template <bool BLOCKED>
static lsq_status adam_lp_entry(void* p_lp, float* m, float* v, const void* g, int64_t n, float lr, float beta1,
                                float beta2, float eps, float weight_decay, int32_t step, int32_t adamw,
                                int32_t bias_correction, float inv_grad_scale, lsq_dtype dt, void* stream)
{
    LSQ_REQUIRE(n >= 0);
    AdamParams a;
    LSQ_REQUIRE(make_adam_params(&a, lr, beta1, beta2, eps, weight_decay, step, adamw, bias_correction, inv_grad_scale));
    if (dt != LSQ_F16 && dt != LSQ_BF16) return LSQ_UNSUPPORTED_DTYPE;
    if (n == 0) return LSQ_OK;
    LSQ_REQUIRE(p_lp && m && (BLOCKED || v) && g);
    LSQ_ALIGNED(p_lp); LSQ_ALIGNED(m); LSQ_ALIGNED(v); LSQ_ALIGNED(g);
    LSQ_REQUIRE(ceil_div(ceil_div(n, kAdamPack), kAdamThreads) <= 0x7FFFFFFF);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const dim3 grid(static_cast<unsigned>(ceil_div(ceil_div(n, kAdamPack), kAdamThreads))), block(kAdamThreads);
    if (dt == LSQ_F16)
        hipLaunchKernelGGL((adam_lp_kernel<f16, BLOCKED>), grid, block, 0, s, static_cast<f16*>(p_lp), m, v, static_cast<const f16*>(g), n, a);
    else
        hipLaunchKernelGGL((adam_lp_kernel<bf16, BLOCKED>), grid, block, 0, s, static_cast<bf16*>(p_lp), m, v, static_cast<const bf16*>(g), n, a);
    return launch_status();
}
}  // namespace lsq

extern "C" lsq_status lsq_adam_step_lp(void* p_lp, float* m, float* v, const void* g, int64_t n, float lr, float beta1,
                                       float beta2, float eps, float weight_decay, int32_t step, int32_t adamw,
                                       int32_t bias_correction, float inv_grad_scale, lsq_dtype dt, void* stream)
{
    return lsq::adam_lp_entry<false>(p_lp, m, v, g, n, lr, beta1, beta2, eps, weight_decay, step, adamw, bias_correction,
                                     inv_grad_scale, dt, stream);
}

extern "C" lsq_status lsq_adam_step_lp_blocked(void* p_lp, float* state, const void* g, int64_t n, float lr, float beta1,
                                               float beta2, float eps, float weight_decay, int32_t step, int32_t adamw,
                                               int32_t bias_correction, float inv_grad_scale, lsq_dtype dt, void* stream)
{
    return lsq::adam_lp_entry<true>(p_lp, state, nullptr, g, n, lr, beta1, beta2, eps, weight_decay, step, adamw,
                                    bias_correction, inv_grad_scale, dt, stream);
}

namespace lsq {
template <bool BLOCKED>
static lsq_status sgd_entry(float* p, float* momentum_buf, const void* g, void* p_lp, int64_t n, float lr,
                            float momentum, float weight_decay, int32_t nesterov, float inv_grad_scale,
                            lsq_dtype g_dt, lsq_dtype p_lp_dt, void* stream)
{
    LSQ_REQUIRE(n >= 0 && momentum >= 0.0f);
    LSQ_REQUIRE(!(nesterov && momentum == 0.0f));
    if (!valid_dtype(g_dt)) return LSQ_UNSUPPORTED_DTYPE;
    if (p_lp && p_lp_dt != LSQ_F16 && p_lp_dt != LSQ_BF16) return LSQ_UNSUPPORTED_DTYPE;
    if (n == 0) return LSQ_OK;
    LSQ_REQUIRE(p && g && (BLOCKED || momentum == 0.0f || momentum_buf));
    LSQ_ALIGNED(p); LSQ_ALIGNED(momentum_buf); LSQ_ALIGNED(g); LSQ_ALIGNED(p_lp);
    LSQ_REQUIRE(ceil_div(ceil_div(n, kAdamPack), kAdamThreads) <= 0x7FFFFFFF);
    SgdParams a{lr, momentum, weight_decay, inv_grad_scale, nesterov != 0};
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool mom = momentum != 0.0f;
    switch (g_dt) {
        case LSQ_F16: return mom ? sgd_dispatch<f16, true, BLOCKED>(p, momentum_buf, g, p_lp, n, a, p_lp_dt, s)
                                 : sgd_dispatch<f16, false, BLOCKED>(p, momentum_buf, g, p_lp, n, a, p_lp_dt, s);
        case LSQ_BF16: return mom ? sgd_dispatch<bf16, true, BLOCKED>(p, momentum_buf, g, p_lp, n, a, p_lp_dt, s)
                                  : sgd_dispatch<bf16, false, BLOCKED>(p, momentum_buf, g, p_lp, n, a, p_lp_dt, s);
        default: return mom ? sgd_dispatch<float, true, BLOCKED>(p, momentum_buf, g, p_lp, n, a, p_lp_dt, s)
                            : sgd_dispatch<float, false, BLOCKED>(p, momentum_buf, g, p_lp, n, a, p_lp_dt, s);
    }
}
}  // namespace lsq

extern "C" lsq_status lsq_sgd_step(float* p, float* momentum_buf, const void* g, void* p_lp, int64_t n, float lr,
                                   float momentum, float weight_decay, int32_t nesterov, float inv_grad_scale,
                                   lsq_dtype g_dt, lsq_dtype p_lp_dt, void* stream)
{
    return lsq::sgd_entry<false>(p, momentum_buf, g, p_lp, n, lr, momentum, weight_decay, nesterov, inv_grad_scale, g_dt,
                                 p_lp_dt, stream);
}

extern "C" lsq_status lsq_sgd_step_blocked(float* state, const void* g, void* p_lp, int64_t n, float lr, float momentum,
                                           float weight_decay, int32_t nesterov, float inv_grad_scale, lsq_dtype g_dt,
                                           lsq_dtype p_lp_dt, void* stream)
{
    return lsq::sgd_entry<true>(state, nullptr, g, p_lp, n, lr, momentum, weight_decay, nesterov, inv_grad_scale, g_dt,
                                p_lp_dt, stream);
}
