// Device-side building blocks for the gfx950 kernels: storage types, 8-element
// packs (one 128-bit access for fp16/bf16), wave64 reductions on DPP, and the
// Philox4x32-10 dropout stream.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lsq {

using f16 = _Float16;
using bf16 = __bf16;

constexpr int kWave = 64;
constexpr int kPack = 8;   // elements per pack == elements per Philox call

template <typename T> struct alignas(sizeof(T) * 8 > 16 ? 16 : sizeof(T) * 8) Raw8 { T v[8]; };

template <typename T> __device__ __forceinline__ float to_f32(T v) { return static_cast<float>(v); }
template <typename T> __device__ __forceinline__ T from_f32(float v) { return static_cast<T>(v); }

// 128-bit vector types the nontemporal builtins accept.
typedef float fvec4 __attribute__((ext_vector_type(4)));
typedef uint32_t uvec4 __attribute__((ext_vector_type(4)));
typedef uint32_t uvec2 __attribute__((ext_vector_type(2)));

// Streaming accesses carry the nontemporal hint: the tensors on this path are far
// larger than L2 and are touched once per kernel, so keeping their lines only
// evicts data someone else could reuse.  Measured on MI355X it is worth 7 % on a
// plain copy and 10 % on the Adam kernel.
template <bool NT> __device__ __forceinline__ fvec4 ld_f4(const float* p)
{
    if constexpr (NT) return __builtin_nontemporal_load(reinterpret_cast<const fvec4*>(p));
    else return *reinterpret_cast<const fvec4*>(p);
}
template <bool NT> __device__ __forceinline__ void st_f4(float* p, fvec4 v)
{
    if constexpr (NT) __builtin_nontemporal_store(v, reinterpret_cast<fvec4*>(p));
    else *reinterpret_cast<fvec4*>(p) = v;
}
template <bool NT> __device__ __forceinline__ uvec4 ld_u4(const void* p)
{
    if constexpr (NT) return __builtin_nontemporal_load(reinterpret_cast<const uvec4*>(p));
    else return *reinterpret_cast<const uvec4*>(p);
}
template <bool NT> __device__ __forceinline__ void st_u4(void* p, uvec4 v)
{
    if constexpr (NT) __builtin_nontemporal_store(v, reinterpret_cast<uvec4*>(p));
    else *reinterpret_cast<uvec4*>(p) = v;
}
template <bool NT> __device__ __forceinline__ uvec2 ld_u2(const void* p)
{
    if constexpr (NT) return __builtin_nontemporal_load(reinterpret_cast<const uvec2*>(p));
    else return *reinterpret_cast<const uvec2*>(p);
}
template <bool NT> __device__ __forceinline__ void st_u2(void* p, uvec2 v)
{
    if constexpr (NT) __builtin_nontemporal_store(v, reinterpret_cast<uvec2*>(p));
    else *reinterpret_cast<uvec2*>(p) = v;
}

// 8 consecutive elements starting at a pack-aligned address, widened to fp32.
// fp16/bf16: one global_load_dwordx4; fp32: two.
template <typename T, bool NT = false>
__device__ __forceinline__ void load8(const T* __restrict__ p, float (&f)[8])
{
    if constexpr (sizeof(T) == 2) {
        const uvec4 u = ld_u4<NT>(p);
        const Raw8<T> r = __builtin_bit_cast(Raw8<T>, u);
#pragma unroll
        for (int j = 0; j < 8; ++j) f[j] = to_f32<T>(r.v[j]);
    } else {
        const fvec4 a = ld_f4<NT>(reinterpret_cast<const float*>(p));
        const fvec4 b = ld_f4<NT>(reinterpret_cast<const float*>(p) + 4);
        f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w;
        f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
    }
}

template <typename T, bool NT = false>
__device__ __forceinline__ void store8(T* __restrict__ p, const float (&f)[8])
{
    if constexpr (sizeof(T) == 2) {
        Raw8<T> r;
#pragma unroll
        for (int j = 0; j < 8; ++j) r.v[j] = from_f32<T>(f[j]);
        st_u4<NT>(p, __builtin_bit_cast(uvec4, r));
    } else {
        st_f4<NT>(reinterpret_cast<float*>(p), fvec4{f[0], f[1], f[2], f[3]});
        st_f4<NT>(reinterpret_cast<float*>(p) + 4, fvec4{f[4], f[5], f[6], f[7]});
    }
}

// A pack in its storage form (4 registers for fp16/bf16, 8 for fp32).  Kernels load the
// raw packs of a whole row first and widen them afterwards: all loads of the row are then
// in flight together, and a prefetched row costs half the registers of its fp32 form.
template <typename T, int = sizeof(T)> struct RawPack;
template <typename T> struct RawPack<T, 2> { uvec4 u; };
template <typename T> struct RawPack<T, 4> { fvec4 a, b; };

template <typename T, bool NT = false>
__device__ __forceinline__ RawPack<T> load_raw(const T* __restrict__ p)
{
    RawPack<T> r;
    if constexpr (sizeof(T) == 2) {
        r.u = ld_u4<NT>(p);
    } else {
        r.a = ld_f4<NT>(reinterpret_cast<const float*>(p));
        r.b = ld_f4<NT>(reinterpret_cast<const float*>(p) + 4);
    }
    return r;
}

template <typename T, bool NT = false>
__device__ __forceinline__ void store_raw(T* __restrict__ p, const RawPack<T>& r)
{
    if constexpr (sizeof(T) == 2) {
        st_u4<NT>(p, r.u);
    } else {
        st_f4<NT>(reinterpret_cast<float*>(p), r.a);
        st_f4<NT>(reinterpret_cast<float*>(p) + 4, r.b);
    }
}

template <typename T>
__device__ __forceinline__ RawPack<T> zero_raw()
{
    RawPack<T> r;
    if constexpr (sizeof(T) == 2) r.u = uvec4{0u, 0u, 0u, 0u};
    else { r.a = fvec4{0.f, 0.f, 0.f, 0.f}; r.b = r.a; }
    return r;
}

// Hide a packed row from the optimiser: a kernel that walks the same packs in several passes
// re-widens them in each pass instead of keeping 8 fp32 registers per pack alive in between.
template <typename T>
__device__ __forceinline__ void opaque(RawPack<T>& r)
{
    if constexpr (sizeof(T) == 2) asm volatile("" : "+v"(r.u));
    else asm volatile("" : "+v"(r.a), "+v"(r.b));
}

template <typename T>
__device__ __forceinline__ void unpack(const RawPack<T>& r, float (&f)[8])
{
    if constexpr (sizeof(T) == 2) {
        const Raw8<T> h = __builtin_bit_cast(Raw8<T>, r.u);
#pragma unroll
        for (int j = 0; j < 8; ++j) f[j] = to_f32<T>(h.v[j]);
    } else {
        f[0] = r.a.x; f[1] = r.a.y; f[2] = r.a.z; f[3] = r.a.w;
        f[4] = r.b.x; f[5] = r.b.y; f[6] = r.b.z; f[7] = r.b.w;
    }
}

// fp32 -> storage form (one rounding per element), the inverse of unpack
template <typename T>
__device__ __forceinline__ RawPack<T> pack_raw(const float (&f)[8])
{
    RawPack<T> r;
    if constexpr (sizeof(T) == 2) {
        Raw8<T> h;
#pragma unroll
        for (int j = 0; j < 8; ++j) h.v[j] = from_f32<T>(f[j]);
        r.u = __builtin_bit_cast(uvec4, h);
    } else {
        r.a = fvec4{f[0], f[1], f[2], f[3]};
        r.b = fvec4{f[4], f[5], f[6], f[7]};
    }
    return r;
}

// Make eight fp32 values exist as fp32 before they are narrowed: without it the compiler may fold
// a final fma into the conversion (v_fma_mixlo_f16: one rounding instead of two), and it takes
// that decision instantiation by instantiation, so two kernels that must agree bit for bit would not.
__device__ __forceinline__ void pin_f32(float (&f)[8])
{
#pragma unroll
    for (int j = 0; j < 8; ++j) asm volatile("" : "+v"(f[j]));
}

// 4 consecutive elements (one 128-bit access of fp32, one 64-bit access of fp16/bf16).
template <typename T> struct alignas(sizeof(T) * 4 > 16 ? 16 : sizeof(T) * 4) Raw4 { T v[4]; };

template <typename T, bool NT = false>
__device__ __forceinline__ void load4(const T* __restrict__ p, float (&f)[4])
{
    if constexpr (sizeof(T) == 2) {
        const uvec2 u = ld_u2<NT>(p);
        const Raw4<T> r = __builtin_bit_cast(Raw4<T>, u);
#pragma unroll
        for (int j = 0; j < 4; ++j) f[j] = to_f32<T>(r.v[j]);
    } else {
        const fvec4 a = ld_f4<NT>(reinterpret_cast<const float*>(p));
        f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w;
    }
}

template <typename T, bool NT = false>
__device__ __forceinline__ void store4(T* __restrict__ p, const float (&f)[4])
{
    if constexpr (sizeof(T) == 2) {
        Raw4<T> r;
#pragma unroll
        for (int j = 0; j < 4; ++j) r.v[j] = from_f32<T>(f[j]);
        st_u2<NT>(p, __builtin_bit_cast(uvec2, r));
    } else {
        st_f4<NT>(reinterpret_cast<float*>(p), fvec4{f[0], f[1], f[2], f[3]});
    }
}

// ---------------------------------------------------------------- reductions
// All-reduce over aligned groups of WIDTH lanes (a power of two <= 64) inside one
// wave64.  Lanes 1..15 apart are reached with DPP (quad permutes and row mirrors,
// no LDS traffic); 16 apart with a 32-lane swizzle; the last step of a full-wave
// reduction reads the four row results through scalar registers.
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, false));
}

struct OpSum { static __device__ __forceinline__ float apply(float a, float b) { return a + b; } };
struct OpMax { static __device__ __forceinline__ float apply(float a, float b) { return fmaxf(a, b); } };

template <int WIDTH, typename Op>
__device__ __forceinline__ float group_allreduce(float v)
{
    static_assert(WIDTH == 1 || WIDTH == 2 || WIDTH == 4 || WIDTH == 8 || WIDTH == 16 || WIDTH == 32 || WIDTH == 64, "");
    if constexpr (WIDTH >= 2) v = Op::apply(v, dpp_mov<0xB1>(v));    // quad_perm [1,0,3,2]
    if constexpr (WIDTH >= 4) v = Op::apply(v, dpp_mov<0x4E>(v));    // quad_perm [2,3,0,1]
    if constexpr (WIDTH >= 8) v = Op::apply(v, dpp_mov<0x141>(v));   // row_half_mirror
    if constexpr (WIDTH >= 16) v = Op::apply(v, dpp_mov<0x140>(v));  // row_mirror
    if constexpr (WIDTH == 32) {
        // swap with the lane 16 away inside each half-wave (bit-mask mode: and 0x1F, xor 0x10)
        float o = __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, v), 0x401F));
        v = Op::apply(v, o);
    }
    if constexpr (WIDTH == 64) {
        const int iv = __builtin_bit_cast(int, v);
        float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 0));
        float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 16));
        float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 32));
        float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 48));
        v = Op::apply(Op::apply(r0, r1), Op::apply(r2, r3));
    }
    return v;
}

template <int WIDTH> __device__ __forceinline__ float group_sum(float v) { return group_allreduce<WIDTH, OpSum>(v); }
template <int WIDTH> __device__ __forceinline__ float group_max(float v) { return group_allreduce<WIDTH, OpMax>(v); }

// Block-wide all-reduce for NWAVES waves; `scratch` holds NWAVES floats of LDS.
// Every thread of the block must call it; it contains two barriers.
template <int NWAVES, typename Op>
__device__ __forceinline__ float block_allreduce(float v, float* scratch)
{
    v = group_allreduce<64, Op>(v);
    if constexpr (NWAVES == 1) return v;
    const int wave = threadIdx.x >> 6;
    __syncthreads();                    // scratch may still be read from a previous call
    if ((threadIdx.x & 63) == 0) scratch[wave] = v;
    __syncthreads();
    float r = scratch[0];
#pragma unroll
    for (int w = 1; w < NWAVES; ++w) r = Op::apply(r, scratch[w]);
    return r;
}

// -------------------------------------------------------------------- Philox
// Philox4x32-10 (Salmon et al., SC'11).  One call yields 128 bits = eight 16-bit
// dropout lanes, so a pack of 8 elements costs one call.
struct DropoutParams {
    uint32_t key0, key1;      // seed
    uint32_t ctr2, ctr3;      // offset
    uint32_t t16;             // keep iff r16 >= t16
    uint32_t on;              // p > 0: draw and scale (a p so small that t16 rounds to 0 keeps everything, still scaled)
    float scale;              // 1 / (1 - p)
};

__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t (&out)[4])
{
    constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    constexpr uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint64_t p0 = static_cast<uint64_t>(M0) * c0;
        const uint64_t p1 = static_cast<uint64_t>(M1) * c2;
        // three-input xor in one VALU operation (truth table 0x96); the round keys stay scalar
        const uint32_t n0 = __builtin_amdgcn_bitop3_b32(static_cast<uint32_t>(p1 >> 32), c1, k0, 0x96);
        const uint32_t n2 = __builtin_amdgcn_bitop3_b32(static_cast<uint32_t>(p0 >> 32), c3, k1, 0x96);
        c1 = static_cast<uint32_t>(p1);
        c3 = static_cast<uint32_t>(p0);
        c0 = n0;
        c2 = n2;
        k0 += W0;
        k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Workgroup -> tile for kernels that stream large tensors one tile per workgroup.  Consecutive workgroups of a
// launch go to the eight XCDs in turn, each with its own L2 and address-translation cache; with tile = workgroup
// every XCD walks every small piece of every tensor.  Here an XCD takes a run of CHUNK consecutive tiles out of
// every eight runs, so that it streams about a megabyte of each tensor at a stretch.  The last, partial group of
// eight runs keeps its order; the map is a permutation of 0..nb-1.
template <int CHUNK>
__device__ __forceinline__ int64_t xcd_chunked(int64_t b, int64_t nb)
{
    if constexpr (CHUNK <= 1) return b;
    constexpr int64_t kGroup = 8 * static_cast<int64_t>(CHUNK);
    const int64_t first = b / kGroup * kGroup;
    if (first + kGroup > nb) return b;
    const int64_t r = b - first;
    return first + (r % 8) * CHUNK + r / 8;
}

// The same with the runs of a group handed to the XCDs in an order that rotates from group to group: XCDs receive
// their workgroups in strict rotation whatever their load, so when the cost of a tile depends on its position
// in a period that the group length divides (padded sentence tails in a criterion batch), fixed runs would give
// one XCD all the cheap tiles.
template <int CHUNK>
__device__ __forceinline__ int64_t xcd_chunked_rotating(int64_t b, int64_t nb)
{
    if constexpr (CHUNK <= 1) return b;
    constexpr int64_t kGroup = 8 * static_cast<int64_t>(CHUNK);
    const int64_t grp = b / kGroup, first = grp * kGroup;
    if (first + kGroup > nb) return b;
    const int64_t r = b - first;
    return first + ((r + grp) % 8) * CHUNK + r / 8;
}

// (column block, row block) of a workgroup of a [column blocks, row blocks] grid.
// ORDER 0: as launched (column blocks fastest); 1: row blocks fastest.
struct GridBlock { int col; int row; };
template <int ORDER>
__device__ __forceinline__ GridBlock grid_block()
{
    if constexpr (ORDER == 1) {
        const unsigned lin = blockIdx.x + gridDim.x * blockIdx.y;
        return {static_cast<int>(lin / gridDim.y), static_cast<int>(lin % gridDim.y)};
    } else {
        return {static_cast<int>(blockIdx.x), static_cast<int>(blockIdx.y)};
    }
}

// keep[j] (as 0.0f / scale) for the 8 elements of pack `g` (flat element index / 8).
__device__ __forceinline__ void dropout_factors8(const DropoutParams& d, uint64_t g, float (&k)[8])
{
    uint32_t w[4];
    philox4x32_10(static_cast<uint32_t>(g), static_cast<uint32_t>(g >> 32), d.ctr2, d.ctr3, d.key0, d.key1, w);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        k[2 * j] = (w[j] & 0xFFFFu) >= d.t16 ? d.scale : 0.0f;
        k[2 * j + 1] = (w[j] >> 16) >= d.t16 ? d.scale : 0.0f;
    }
}

// The keep decisions of pack `g` as 8 bits (bit j = element 8g + j survives): what a kernel whose
// lanes are not aligned with packs stores in LDS, one Philox call per pack instead of per element.
__device__ __forceinline__ uint32_t dropout_keep_bits8(const DropoutParams& d, uint64_t g)
{
    uint32_t w[4];
    philox4x32_10(static_cast<uint32_t>(g), static_cast<uint32_t>(g >> 32), d.ctr2, d.ctr3, d.key0, d.key1, w);
    uint32_t bits = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        bits |= ((w[j] & 0xFFFFu) >= d.t16 ? 1u : 0u) << (2 * j);
        bits |= ((w[j] >> 16) >= d.t16 ? 1u : 0u) << (2 * j + 1);
    }
    return bits;
}

// The factor for one element (element-strided paths and the ragged last pack of a flat walk: one Philox call per element).
__device__ __forceinline__ float dropout_factor1(const DropoutParams& d, uint64_t e)
{
    uint32_t w[4];
    const uint64_t g = e >> 3;
    philox4x32_10(static_cast<uint32_t>(g), static_cast<uint32_t>(g >> 32), d.ctr2, d.ctr3, d.key0, d.key1, w);
    const uint32_t lane = static_cast<uint32_t>(e) & 7u;
    const uint32_t word = lane < 2 ? w[0] : lane < 4 ? w[1] : lane < 6 ? w[2] : w[3];
    const uint32_t r16 = (word >> (16u * (lane & 1u))) & 0xFFFFu;
    return r16 >= d.t16 ? d.scale : 0.0f;
}

}  // namespace lsq
