// Head split / merge: the "Reshape" in the paper's list of element-wise operations
// (Sec. IV-A).  The projection output [batch*len, parts*hidden] (+ bias) is laid out
// as `parts` tensors [batch, heads, len, head_dim] for the batched attention GEMMs;
// the backward (and the merge of the attention output) is the inverse permutation,
// with the bias gradient as a by-product.
//
// Pure data movement: read every element once, write it once.  A wave owns 64
// consecutive packs of a [T, parts*hidden] row (1 KiB contiguous) and walks down
// the rows; on the [batch, heads, len, head_dim] side the same packs fall into
// whole head rows (head_dim*2 bytes, 128 B at head_dim 64), so both sides move
// full cache lines.  The bias pack (forward) or the dbias accumulators (backward)
// stay in registers of the lane that owns the columns.
#include "host.hpp"

namespace lsq {

constexpr bool kNT = true;
constexpr int kHeadWaves = 4;

struct HeadGeom {
    int64_t rows;          // batch * len
    int len, heads, head_dim, parts;
    int hidden;            // heads * head_dim
    int ppr;               // packs per [T, parts*hidden] row
    FastDiv by_len;        // token index -> sentence
};

template <typename T>
__device__ __forceinline__ T* pick(T* a, T* b, T* c, int part) { return part == 0 ? a : part == 1 ? b : c; }

// element offset inside a [batch, heads, len, head_dim] tensor of column `within` (< hidden) of row t
__device__ __forceinline__ int64_t head_offset(const HeadGeom& g, int64_t t, int within)
{
    // tokens of a call are below 2^31 (checked at the entry): the batch index comes from a reciprocal
    const int64_t b = fastdiv(static_cast<uint32_t>(t), g.by_len);
    const int l = static_cast<int>(t - b * g.len);
    const int n = within / g.head_dim;
    const int dd = within - n * g.head_dim;
    return ((b * g.heads + n) * g.len + l) * static_cast<int64_t>(g.head_dim) + dd;
}

template <typename T, bool HAS_BIAS>
__global__ __launch_bounds__(256) void split_heads_kernel(T* __restrict__ o0, T* __restrict__ o1, T* __restrict__ o2,
                                                          const T* __restrict__ in, const T* __restrict__ bias,
                                                          HeadGeom g)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // row blocks fastest: consecutive workgroups (consecutive XCDs) take consecutive row blocks of one column block;
    // 18.5 against 19.5 us at 4096 x 3072 and 23.7 against 24.4 us at 8192 x 3840 (the merge is 1-3 % slower that way)
    const GridBlock gb = grid_block<1>();
    const int cp = gb.col * 64 + lane;
    if (cp >= g.ppr) return;
    const int col = cp * kPack;
    const int part = col / g.hidden;
    const int within = col - part * g.hidden;
    T* out = pick(o0, o1, o2, part);
    float b[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if constexpr (HAS_BIAS) load8<T>(bias + col, b);
    const int64_t stride = static_cast<int64_t>(gridDim.y) * kHeadWaves;
    // the pack of the next token is loaded before this token's is stored
    int64_t t = static_cast<int64_t>(gb.row) * kHeadWaves + wave;
    RawPack<T> nxt = t < g.rows ? load_raw<T, kNT>(in + (t * g.ppr + cp) * kPack) : zero_raw<T>();
    for (; t < g.rows; t += stride) {
        const RawPack<T> r = nxt;
        if (t + stride < g.rows) nxt = load_raw<T, kNT>(in + ((t + stride) * g.ppr + cp) * kPack);
        T* dst = out + head_offset(g, t, within);
        if constexpr (HAS_BIAS) {
            float f[8];
            unpack<T>(r, f);
#pragma unroll
            for (int j = 0; j < 8; ++j) f[j] += b[j];
            store8<T, kNT>(dst, f);
        } else {                                                 // a pure move: bit-exact
            if constexpr (sizeof(T) == 2) st_u4<kNT>(dst, r.u);
            else { st_f4<kNT>(reinterpret_cast<float*>(dst), r.a); st_f4<kNT>(reinterpret_cast<float*>(dst) + 4, r.b); }
        }
    }
}

// inverse: `parts` tensors [batch, heads, len, head_dim] -> [T, parts*hidden]; partial: dbias partial rows or nullptr
template <typename T>
__global__ __launch_bounds__(256) void merge_heads_kernel(T* __restrict__ out, float* __restrict__ partial,
                                                          const T* __restrict__ i0, const T* __restrict__ i1,
                                                          const T* __restrict__ i2, HeadGeom g)
{
    __shared__ float sm[kHeadWaves][8][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const GridBlock gb = grid_block<0>();
    const int cp = gb.col * 64 + lane;
    const bool active = cp < g.ppr;
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (active) {
        const int col = cp * kPack;
        const int part = col / g.hidden;
        const int within = col - part * g.hidden;
        const T* in = pick(i0, i1, i2, part);
        const int64_t stride = static_cast<int64_t>(gridDim.y) * kHeadWaves;
        for (int64_t t = static_cast<int64_t>(gb.row) * kHeadWaves + wave; t < g.rows; t += stride) {
            const RawPack<T> r = load_raw<T, kNT>(in + head_offset(g, t, within));
            T* dst = out + (t * g.ppr + cp) * kPack;
            if constexpr (sizeof(T) == 2) st_u4<kNT>(dst, r.u);
            else { st_f4<kNT>(reinterpret_cast<float*>(dst), r.a); st_f4<kNT>(reinterpret_cast<float*>(dst) + 4, r.b); }
            if (partial) {
                float f[8];
                unpack<T>(r, f);
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[j] += f[j];
            }
        }
    }
    if (partial == nullptr) return;        // uniform over the grid
#pragma unroll
    for (int j = 0; j < 8; ++j) sm[wave][j][lane] = acc[j];
    __syncthreads();
    if (wave == 0 && active) {
        float s[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            float t = sm[0][j][lane];
#pragma unroll
            for (int w = 1; w < kHeadWaves; ++w) t += sm[w][j][lane];
            s[j] = t;
        }
        store8<float>(partial + (static_cast<int64_t>(gb.row) * g.ppr + cp) * kPack, s);
    }
}

// ---- generic paths (head_dim not a multiple of 8): one element per thread
template <typename T>
__global__ __launch_bounds__(256) void split_heads_flat(T* o0, T* o1, T* o2, const T* __restrict__ in,
                                                        const T* __restrict__ bias, HeadGeom g)
{
    const int64_t e = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    const int64_t width = static_cast<int64_t>(g.parts) * g.hidden;
    if (e >= g.rows * width) return;
    const int64_t t = e / width;
    const int col = static_cast<int>(e - t * width);
    const int part = col / g.hidden;
    float v = to_f32<T>(in[e]);
    if (bias) v += to_f32<T>(bias[col]);
    pick(o0, o1, o2, part)[head_offset(g, t, col - part * g.hidden)] = bias ? from_f32<T>(v) : in[e];
}

template <typename T>
__global__ __launch_bounds__(256) void merge_heads_flat(T* __restrict__ out, const T* i0, const T* i1, const T* i2,
                                                        HeadGeom g)
{
    const int64_t e = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    const int64_t width = static_cast<int64_t>(g.parts) * g.hidden;
    if (e >= g.rows * width) return;
    const int64_t t = e / width;
    const int col = static_cast<int>(e - t * width);
    const int part = col / g.hidden;
    out[e] = pick(i0, i1, i2, part)[head_offset(g, t, col - part * g.hidden)];
}

// Column sums when rows are not a whole number of packs: one thread per column and row block walks its
// rows (a wave reads 64 consecutive elements per row), the row blocks' partial rows are summed by
// colsum_finalize_kernel.
template <typename T>
__global__ __launch_bounds__(256) void colsum_rows_flat(float* __restrict__ partial, const T* __restrict__ x, int64_t rows,
                                                        int cols, int rows_per_block)
{
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= cols) return;
    const int64_t r0 = static_cast<int64_t>(blockIdx.y) * rows_per_block;
    const int64_t r1 = r0 + rows_per_block < rows ? r0 + rows_per_block : rows;
    float s = 0.0f;
#pragma unroll 4
    for (int64_t r = r0; r < r1; ++r) s += to_f32<T>(x[r * cols + c]);
    partial[static_cast<int64_t>(blockIdx.y) * cols + c] = s;
}

// one row per wave up to 16384 rows (the merge 7.35 / 9.07 us at 4096 x 1024 / 8192 x 1280 against 7.9 / 9.4 with four;
// the split 22.8 against 23.4 us at 8192 x 3840 and 18.5 against 18.3 at 4096 x 3072)
inline int head_row_blocks(int64_t rows)
{
    int64_t b = ceil_div(rows, kHeadWaves);
    if (b > 4096) b = 4096;
    return static_cast<int>(b < 1 ? 1 : b);
}

template <typename T>
static lsq_status split_dispatch(void* o0, void* o1, void* o2, const void* in, const void* bias, const HeadGeom& g,
                                 hipStream_t s)
{
    T* a = static_cast<T*>(o0); T* b = static_cast<T*>(o1); T* c = static_cast<T*>(o2);
    const T* ip = static_cast<const T*>(in);
    const T* bp = static_cast<const T*>(bias);
    if (g.head_dim % kPack == 0) {
        const dim3 grid(static_cast<unsigned>(ceil_div(g.ppr, 64)), static_cast<unsigned>(head_row_blocks(g.rows))), block(256);
        if (bp) hipLaunchKernelGGL((split_heads_kernel<T, true>), grid, block, 0, s, a, b, c, ip, bp, g);
        else hipLaunchKernelGGL((split_heads_kernel<T, false>), grid, block, 0, s, a, b, c, ip, bp, g);
    } else {
        const int64_t total = g.rows * g.parts * g.hidden;
        hipLaunchKernelGGL((split_heads_flat<T>), dim3(static_cast<unsigned>(ceil_div(total, 256))), dim3(256), 0, s,
                           a, b, c, ip, bp, g);
    }
    return launch_status();
}

template <typename T>
static lsq_status merge_dispatch(void* out, float* dbias, const void* i0, const void* i1, const void* i2,
                                 const HeadGeom& g, void* workspace, hipStream_t s)
{
    T* o = static_cast<T*>(out);
    const T* a = static_cast<const T*>(i0); const T* b = static_cast<const T*>(i1); const T* c = static_cast<const T*>(i2);
    const int cols = g.parts * g.hidden;
    if (g.head_dim % kPack == 0) {
        const int rb = heads_bwd_row_blocks(g.rows, cols);
        const dim3 grid(static_cast<unsigned>(ceil_div(g.ppr, 64)), static_cast<unsigned>(dbias ? rb : head_row_blocks(g.rows))), block(256);
        float* partial = dbias ? static_cast<float*>(workspace) : nullptr;
        hipLaunchKernelGGL((merge_heads_kernel<T>), grid, block, 0, s, o, partial, a, b, c, g);
        if (dbias) launch_colsum_finalize(dbias, dbias, cols, partial, rb, cols, s);
    } else {
        const int64_t total = g.rows * cols;
        hipLaunchKernelGGL((merge_heads_flat<T>), dim3(static_cast<unsigned>(ceil_div(total, 256))), dim3(256), 0, s,
                           o, a, b, c, g);
        if (dbias) {
            const int rb = heads_bwd_row_blocks(g.rows, cols);
            float* partial = static_cast<float*>(workspace);
            hipLaunchKernelGGL((colsum_rows_flat<T>), dim3(static_cast<unsigned>(ceil_div(cols, 256)), static_cast<unsigned>(rb)), dim3(256), 0, s,
                               partial, static_cast<const T*>(o), g.rows, cols, static_cast<int>(ceil_div(g.rows, rb)));
            launch_colsum_finalize(dbias, dbias, cols, partial, rb, cols, s);
        }
    }
    return launch_status();
}

static lsq_status head_geom(HeadGeom* g, int32_t batch, int32_t len, int32_t heads, int32_t head_dim, int32_t parts, int dt)
{
    if (batch < 0 || len < 0 || heads <= 0 || head_dim <= 0 || parts < 1 || parts > 3) return LSQ_INVALID_ARG;
    if (!valid_dtype(dt)) return LSQ_UNSUPPORTED_DTYPE;
    const int64_t hidden = static_cast<int64_t>(heads) * head_dim;
    if (hidden * parts > 0x3FFFFFFF) return LSQ_INVALID_ARG;
    g->rows = static_cast<int64_t>(batch) * len;
    if (g->rows > 0x7FFFFFFF) return LSQ_INVALID_ARG;
    g->by_len = make_fastdiv(static_cast<uint32_t>(len));
    g->len = len; g->heads = heads; g->head_dim = head_dim; g->parts = parts;
    g->hidden = static_cast<int>(hidden);
    g->ppr = static_cast<int>(hidden * parts / kPack);
    if (ceil_div(g->rows * hidden * parts, 256) > 0x7FFFFFFF) return LSQ_INVALID_ARG;
    return LSQ_OK;
}

}  // namespace lsq

extern "C" lsq_status lsq_split_heads_fwd(void* out0, void* out1, void* out2, const void* in, const void* bias,
                                          int32_t batch, int32_t len, int32_t heads, int32_t head_dim, int32_t parts,
                                          lsq_dtype dt, void* stream)
{
    using namespace lsq;
    HeadGeom g;
    lsq_status st = head_geom(&g, batch, len, heads, head_dim, parts, dt);
    if (st != LSQ_OK) return st;
    if (g.rows == 0) return LSQ_OK;
    LSQ_REQUIRE(in && out0 && (parts < 2 || out1) && (parts < 3 || out2));
    LSQ_ALIGNED(out0); LSQ_ALIGNED(out1); LSQ_ALIGNED(out2); LSQ_ALIGNED(in); LSQ_ALIGNED(bias);
    hipStream_t s = static_cast<hipStream_t>(stream);
    switch (dt) {
        case LSQ_F16: return split_dispatch<f16>(out0, out1, out2, in, bias, g, s);
        case LSQ_BF16: return split_dispatch<bf16>(out0, out1, out2, in, bias, g, s);
        default: return split_dispatch<float>(out0, out1, out2, in, bias, g, s);
    }
}

extern "C" lsq_status lsq_split_heads_bwd(void* din, float* dbias, const void* d0, const void* d1, const void* d2,
                                          int32_t batch, int32_t len, int32_t heads, int32_t head_dim, int32_t parts,
                                          void* workspace, size_t workspace_bytes, lsq_dtype dt, void* stream)
{
    using namespace lsq;
    HeadGeom g;
    lsq_status st = head_geom(&g, batch, len, heads, head_dim, parts, dt);
    if (st != LSQ_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (g.rows == 0) return dbias ? zero_fill(dbias, static_cast<int64_t>(parts) * g.hidden, s) : LSQ_OK;
    LSQ_REQUIRE(din && d0 && (parts < 2 || d1) && (parts < 3 || d2));
    LSQ_ALIGNED(din); LSQ_ALIGNED(d0); LSQ_ALIGNED(d1); LSQ_ALIGNED(d2); LSQ_ALIGNED(dbias); LSQ_ALIGNED(workspace);
    if (dbias) {
        const size_t need = lsq_workspace_bytes(LSQ_OP_SPLIT_HEADS_BWD, g.rows, parts * g.hidden);
        if (need && (!workspace || workspace_bytes < need)) return LSQ_WORKSPACE_TOO_SMALL;
    }
    switch (dt) {
        case LSQ_F16: return merge_dispatch<f16>(din, dbias, d0, d1, d2, g, workspace, s);
        case LSQ_BF16: return merge_dispatch<bf16>(din, dbias, d0, d1, d2, g, workspace, s);
        default: return merge_dispatch<float>(din, dbias, d0, d1, d2, g, workspace, s);
    }
}

extern "C" lsq_status lsq_merge_heads_fwd(void* out, const void* x, int32_t batch, int32_t len, int32_t heads,
                                          int32_t head_dim, lsq_dtype dt, void* stream)
{
    return lsq_split_heads_bwd(out, nullptr, x, nullptr, nullptr, batch, len, heads, head_dim, 1, nullptr, 0, dt, stream);
}

extern "C" lsq_status lsq_merge_heads_bwd(void* dx, const void* dy, int32_t batch, int32_t len, int32_t heads,
                                          int32_t head_dim, lsq_dtype dt, void* stream)
{
    return lsq_split_heads_fwd(dx, nullptr, nullptr, dy, nullptr, batch, len, heads, head_dim, 1, dt, stream);
}
