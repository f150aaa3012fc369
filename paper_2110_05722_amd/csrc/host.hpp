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

// Number of partial-sum rows the column reductions write to the workspace.
// One per workgroup; sized so the grid fills 256 compute units a few times over
// while the partials stay a small fraction of the tensor traffic.
inline int ln_bwd_blocks(int64_t rows, int32_t /*hidden*/)
{
    int64_t b = ceil_div(rows, 8);       // at least 8 rows per workgroup
    if (b > 512) b = 512;
    if (b < 1) b = 1;
    return static_cast<int>(b);
}

inline int bdr_bwd_row_blocks(int64_t rows, int32_t /*hidden*/)
{
    int64_t b = ceil_div(rows, 16);
    if (b > 256) b = 256;
    if (b < 1) b = 1;
    return static_cast<int>(b);
}

}  // namespace lsq
