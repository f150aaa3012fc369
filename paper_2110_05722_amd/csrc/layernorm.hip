// LayerNorm forward and backward (Sec. IV-B of the paper, "dependent reduction
// rewriting").
//
// The paper merges the mean and variance reductions by computing E[x^2]-E[x]^2
// so that neither waits for the other.  Here a row lives in registers after one
// 128-bit load per lane and pack, so the second reduction costs no memory traffic
// at all; it is therefore taken about the mean (two passes over registers), which
// cannot cancel catastrophically.  Backward uses the xhat form of the gradient:
// its two row sums (sum g, sum g*xhat) are independent given the saved mean and
// rstd, and run side by side in the same DPP reduction steps.
//
// Layout: LPR lanes share a row (8..64 lanes of one wave, or a whole 256- or 1024-thread
// workgroup for rows of 2049..8192 and 8193..16384 columns); each lane holds VPL packs of 8 columns, strided
// by LPR packs so that a wave's loads are contiguous.  gamma/beta stay in
// registers while the workgroup walks down its rows.  dgamma/dbeta: every lane
// accumulates its own columns over its rows, the row slots of a workgroup are
// summed in a fixed order through LDS, one partial row per workgroup goes to the
// workspace and a second small kernel sums the partial rows in order.  No atomics.
#include <mutex>

#include "host.hpp"

namespace lsq {

constexpr bool kNT = true;    // nontemporal hint on the streamed tensors (not on gamma/beta/bias)

template <int LPR>
__device__ __forceinline__ float row_sum(float v, float* lds)
{
    if constexpr (LPR >= 256) return block_allreduce<LPR / 64, OpSum>(v, lds);      // the row spans the workgroup
    else return group_sum<LPR>(v);
}

// Raw packs of row r for this lane (zeros where the row or the pack does not exist).
// Loads only, no arithmetic: every load of the row is in flight before the first use.
template <typename T, int LPR, int VPL>
__device__ __forceinline__ void ln_load_row(RawPack<T> (&raw)[VPL], const T* __restrict__ base, int64_t r, bool rv,
                                            int hidden, int nv, int sub)
{
#pragma unroll
    for (int k = 0; k < VPL; ++k) {
        const int idx = sub + k * LPR;
        if (rv && idx < nv) raw[k] = load_raw<T, kNT>(base + r * hidden + idx * kPack);
        else raw[k] = zero_raw<T>();
    }
}

// What the fused variants add around the LayerNorm (all unused, and compiled out, otherwise).
template <typename T>
struct BdrFuse {
    T* out;               // forward: h = residual + Dropout(x + bias), stored;  backward: dx of the projection
    const T* residual;    // forward only
    const T* bias;        // forward only, nullable
    DropoutParams d;
};

// FUSE: the row that is normalised is h = residual + Dropout(x + bias), built in registers from
// two loads, stored once (the next residual) and normalised from its STORED (rounded) value, so the
// result equals bias+dropout+residual followed by LayerNorm bit for bit while h is never re-read.
template <typename T, int LPR, int VPL, bool FUSE = false, bool DROP = false>
__global__ __launch_bounds__(LPR > 256 ? LPR : 256) void ln_fwd_kernel(T* __restrict__ y, float* __restrict__ mean,
                                                     float* __restrict__ rstd, const T* __restrict__ x,
                                                     const T* __restrict__ gamma, const T* __restrict__ beta,
                                                     int64_t rows, int hidden, float eps, BdrFuse<T> fz)
{
    __shared__ float lds[16];
    constexpr int RPB = LPR > 256 ? 1 : 256 / LPR;     // rows a workgroup handles at a time
    const int sub = threadIdx.x % LPR;
    const int slot = threadIdx.x / LPR;
    const int nv = hidden / kPack;
    const float inv_h = 1.0f / static_cast<float>(hidden);
    const int64_t gstride = static_cast<int64_t>(gridDim.x) * RPB;

    RawPack<T> gm[VPL], bt[VPL];              // gamma/beta stay packed; widened where used
    ln_load_row<T, LPR, VPL>(gm, gamma, 0, true, hidden, nv, sub);
    ln_load_row<T, LPR, VPL>(bt, beta, 0, true, hidden, nv, sub);

    RawPack<T> bs[FUSE ? VPL : 1];
    if constexpr (FUSE) {
        if (fz.bias) ln_load_row<T, LPR, VPL>(bs, fz.bias, 0, true, hidden, nv, sub);
        else {
#pragma unroll
            for (int k = 0; k < VPL; ++k) bs[k] = zero_raw<T>();
        }
    }

    int64_t base = static_cast<int64_t>(blockIdx.x) * RPB;
    RawPack<T> nxt[VPL], nres[FUSE ? VPL : 1];
    ln_load_row<T, LPR, VPL>(nxt, x, base + slot, base + slot < rows, hidden, nv, sub);
    if constexpr (FUSE) ln_load_row<T, LPR, VPL>(nres, fz.residual, base + slot, base + slot < rows, hidden, nv, sub);
    for (; base < rows; base += gstride) {
        const int64_t r = base + slot;
        const bool rv = r < rows;
        RawPack<T> cur[VPL], cres[FUSE ? VPL : 1];
#pragma unroll
        for (int k = 0; k < VPL; ++k) cur[k] = nxt[k];
        if constexpr (FUSE) {
#pragma unroll
            for (int k = 0; k < VPL; ++k) cres[k] = nres[k];
        }
        if (base + gstride < rows) {          // prefetch the next row group while this one is reduced
            ln_load_row<T, LPR, VPL>(nxt, x, r + gstride, r + gstride < rows, hidden, nv, sub);
            if constexpr (FUSE)
                ln_load_row<T, LPR, VPL>(nres, fz.residual, r + gstride, r + gstride < rows, hidden, nv, sub);
        }
        if constexpr (FUSE) {
            // same expressions as the stand-alone bias+dropout+residual kernel; the pack index of
            // the dropout stream is the flat one (row * packs per row + pack)
#pragma unroll
            for (int k = 0; k < VPL; ++k) {
                const int idx = sub + k * LPR;
                if (rv && idx < nv) {
                    float xf[8], rf[8], b8[8], kf[8];
                    unpack<T>(cur[k], xf);
                    unpack<T>(cres[k], rf);
                    unpack<T>(bs[k], b8);
                    if constexpr (DROP) dropout_factors8(fz.d, static_cast<uint64_t>(r) * nv + idx, kf);
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const float z = xf[j] + b8[j];
                        rf[j] = DROP ? fmaf(z, kf[j], rf[j]) : rf[j] + z;
                    }
                    pin_f32(rf);              // rounds like the stand-alone bias+dropout+residual kernel
                    cur[k] = pack_raw<T>(rf);
                    store_raw<T, kNT>(fz.out + r * hidden + idx * kPack, cur[k]);
                }
            }
        }

        float xv[VPL][8];
        float s = 0.0f;
#pragma unroll
        for (int k = 0; k < VPL; ++k) {
            unpack<T>(cur[k], xv[k]);         // absent packs are zeros: they add nothing
#pragma unroll
            for (int j = 0; j < 8; ++j) s += xv[k][j];
        }
        s = row_sum<LPR>(s, lds);
        const float mu = s * inv_h;
        float q = 0.0f;
#pragma unroll
        for (int k = 0; k < VPL; ++k) {
            const bool ok = sub + k * LPR < nv;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float dlt = xv[k][j] - mu;
                xv[k][j] = dlt;
                q = ok ? fmaf(dlt, dlt, q) : q;
            }
        }
        q = row_sum<LPR>(q, lds);
        const float rs = 1.0f / sqrtf(fmaf(q, inv_h, eps));
        if (rv && sub == 0) {
            mean[r] = mu;
            rstd[r] = rs;
        }
        T* yr = y + r * hidden;
#pragma unroll
        for (int k = 0; k < VPL; ++k) {
            const int idx = sub + k * LPR;
            if (rv && idx < nv) {
                float o[8], g8[8], b8[8];
                unpack<T>(gm[k], g8);
                unpack<T>(bt[k], b8);
#pragma unroll
                for (int j = 0; j < 8; ++j) o[j] = fmaf(xv[k][j] * rs, g8[j], b8[j]);
                pin_f32(o);                   // the fused and the plain kernel round alike
                store8<T, kNT>(yr + idx * kPack, o);
            }
        }
    }
}

constexpr int kLnBwdThreads = 256;

// Whether every row slot of a workgroup gets its own LDS copy of the column accumulators
// (one barrier in the epilogue) or the slots take turns on one copy: decided by the LDS
// it takes for the widest row of the bucket, kept under 64 KiB.
template <int LPR, int VPL, int THREADS, int NACC>
constexpr bool ln_bwd_slots_parallel()
{
    return LPR < 256 && static_cast<long>(THREADS / LPR) * NACC * 8 * ((LPR * VPL) | 1) * 4 <= 63 * 1024;
}

// partial: [gridDim.x][2][hidden] fp32 (dgamma row, then dbeta row).
// THREADS lanes per workgroup: THREADS/LPR rows in flight per workgroup (plus their
// prefetched successors).  With one wave per SIMD the kernel is bound by memory latency,
// not bandwidth: the bytes in flight per compute unit are what THREADS buys.
// FUSE: the LayerNorm gradient (plus dres) is the gradient of h = residual + Dropout(x + bias): it is
// stored (the residual branch's gradient), then masked and scaled from its STORED value into
// fz.out (the projection's gradient), whose column sums (dbias) join dgamma/dbeta as a third
// partial row.  Equal to LayerNorm backward followed by bias+dropout+residual backward, one pass.
// Rows wider than 8192 columns take one 1024-thread workgroup per row, which leaves a thread 128
// registers: too few for the row, its prefetched successor and the column accumulators.  There the
// accumulators live in LDS instead, each thread reading and writing only its own columns' entries
// (131 KB for 16384 columns: no barrier, no conflict, and the LDS traffic hides behind the row
// stream).  COLS = false computes dx only.
template <typename T, int LPR, int VPL, bool HAS_RES, int THREADS, bool FUSE = false, bool DROP = false, bool COLS = true>
__global__ __launch_bounds__(THREADS) void ln_bwd_kernel(T* dx, float* __restrict__ partial, const T* dy,
                                                         const T* __restrict__ x, const T* __restrict__ gamma,
                                                         const float* __restrict__ mean, const float* __restrict__ rstd,
                                                         const T* dres, int64_t rows, int hidden, BdrFuse<T> fz)
{
    constexpr int NACC = FUSE ? 3 : 2;        // column accumulators: dgamma, dbeta (, dbias)
    constexpr bool kColsInRegs = COLS && LPR <= 256, kColsInLds = COLS && LPR > 256;
    extern __shared__ float colbuf[];         // [NACC][8][packs | 1]: the slots' exchange when LPR < 256, the accumulators themselves when LPR > 256
    __shared__ float lds[16];
    static_assert(LPR < 256 || THREADS == LPR, "a whole-workgroup row takes the whole workgroup");
    static_assert(COLS || !FUSE, "the fused boundary needs the column sums");
    constexpr int RPB = THREADS / LPR;
    const int sub = threadIdx.x % LPR;
    const int slot = threadIdx.x / LPR;
    const int nv = hidden / kPack;
    const float inv_h = 1.0f / static_cast<float>(hidden);
    const int64_t gstride = static_cast<int64_t>(gridDim.x) * RPB;

    RawPack<T> gm[VPL];
    ln_load_row<T, LPR, VPL>(gm, gamma, 0, true, hidden, nv, sub);
    float dg[VPL][8], db[VPL][8], dbi[FUSE ? VPL : 1][8];
#pragma unroll
    for (int k = 0; k < VPL; ++k)
#pragma unroll
        for (int j = 0; j < 8; ++j) { dg[k][j] = 0.0f; db[k][j] = 0.0f; }
    if constexpr (FUSE) {
#pragma unroll
        for (int k = 0; k < VPL; ++k)
#pragma unroll
            for (int j = 0; j < 8; ++j) dbi[k][j] = 0.0f;
    }

    const int cstride = nv | 1;               // odd: consecutive lanes fall in consecutive banks
    if constexpr (kColsInLds) {
#pragma unroll
        for (int k = 0; k < VPL; ++k) {
            const int idx = sub + k * LPR;
            if (idx < nv) {
#pragma unroll
                for (int j = 0; j < 16; ++j) colbuf[j * cstride + idx] = 0.0f;
            }
        }
    }

    int64_t base = static_cast<int64_t>(blockIdx.x) * RPB;
    RawPack<T> ndy[VPL], nx[VPL], nres[HAS_RES ? VPL : 1];
    float nmu = 0.0f, nrs = 0.0f;
    {
        const int64_t r = base + slot;
        const bool rv = r < rows;
        ln_load_row<T, LPR, VPL>(ndy, dy, r, rv, hidden, nv, sub);
        ln_load_row<T, LPR, VPL>(nx, x, r, rv, hidden, nv, sub);
        if constexpr (HAS_RES) ln_load_row<T, LPR, VPL>(nres, dres, r, rv, hidden, nv, sub);
        if (rv) { nmu = mean[r]; nrs = rstd[r]; }
    }
    for (; base < rows; base += gstride) {
        const int64_t r = base + slot;
        const bool rv = r < rows;
        const int64_t ro = r * hidden;
        RawPack<T> cdy[VPL], cx[VPL], cres[HAS_RES ? VPL : 1];
#pragma unroll
        for (int k = 0; k < VPL; ++k) { cdy[k] = ndy[k]; cx[k] = nx[k]; }
        if constexpr (HAS_RES) {
#pragma unroll
            for (int k = 0; k < VPL; ++k) cres[k] = nres[k];
        }
        const float mu = nmu, rs = nrs;
        if (base + gstride < rows) {          // prefetch the next row group
            const int64_t rn = r + gstride;
            const bool rnv = rn < rows;
            ln_load_row<T, LPR, VPL>(ndy, dy, rn, rnv, hidden, nv, sub);
            ln_load_row<T, LPR, VPL>(nx, x, rn, rnv, hidden, nv, sub);
            if constexpr (HAS_RES) ln_load_row<T, LPR, VPL>(nres, dres, rn, rnv, hidden, nv, sub);
            nmu = 0.0f; nrs = 0.0f;
            if (rnv) { nmu = mean[rn]; nrs = rstd[rn]; }
        }

        // pass 1 over registers: the two row sums and the column accumulators.  Absent packs
        // hold dy = 0, so they add nothing to any of the sums.  xhat = x*rstd - mean*rstd.
        const float nmr = -mu * rs;
        float s1 = 0.0f, s2 = 0.0f;
#pragma unroll
        for (int k = 0; k < VPL; ++k) {
            float gy[8], xv[8], g8[8];
            unpack<T>(cdy[k], gy);
            unpack<T>(cx[k], xv);
            unpack<T>(gm[k], g8);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float xhat = fmaf(xv[j], rs, nmr);
                if constexpr (kColsInRegs) {
                    dg[k][j] = fmaf(gy[j], xhat, dg[k][j]);
                    db[k][j] += gy[j];
                } else if constexpr (kColsInLds) {
                    if (sub + k * LPR < nv) {              // rows that do not exist hold dy = 0 and add nothing
                        float* a = colbuf + j * cstride + (sub + k * LPR);
                        a[0] = fmaf(gy[j], xhat, a[0]);
                        a[8 * cstride] += gy[j];
                    }
                }
                const float gg = gy[j] * g8[j];
                s1 += gg;
                s2 = fmaf(gg, xhat, s2);
            }
        }
        s1 = row_sum<LPR>(s1, lds);
        s2 = row_sum<LPR>(s2, lds);
        // dx = rstd*(g - (s1 + xhat*s2)/hidden) = g*rstd + xhat*c1 + c0
        const float c0 = -rs * s1 * inv_h, c1 = -rs * s2 * inv_h;
#pragma unroll
        for (int k = 0; k < VPL; ++k) {
            const int idx = sub + k * LPR;
            if (rv && idx < nv) {
                float o[8];
                if constexpr (HAS_RES) unpack<T>(cres[k], o);
                // xhat and gamma*dy are rebuilt from the packed row (a few flops) rather than kept
                // in 16 more registers per pack across the reduction
                opaque<T>(cdy[k]);
                opaque<T>(cx[k]);
                float gy[8], xv[8], g8[8];
                unpack<T>(cdy[k], gy);
                unpack<T>(cx[k], xv);
                unpack<T>(gm[k], g8);
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const float v = fmaf(gy[j] * g8[j], rs, fmaf(fmaf(xv[j], rs, nmr), c1, c0));
                    o[j] = HAS_RES ? o[j] + v : v;
                }
                pin_f32(o);               // the fused and the plain kernel round alike
                if constexpr (!FUSE) {
                    store8<T, kNT>(dx + ro + idx * kPack, o);
                } else {
                    const RawPack<T> hp = pack_raw<T>(o);
                    store_raw<T, kNT>(dx + ro + idx * kPack, hp);
                    float gq[8];
                    unpack<T>(hp, gq);
                    if constexpr (DROP) {
                        float kf[8];
                        dropout_factors8(fz.d, static_cast<uint64_t>(r) * nv + idx, kf);
#pragma unroll
                        for (int j = 0; j < 8; ++j) gq[j] *= kf[j];
                    }
                    pin_f32(gq);
                    store8<T, kNT>(fz.out + ro + idx * kPack, gq);
#pragma unroll
                    for (int j = 0; j < 8; ++j) dbi[k][j] += gq[j];
                }
            }
        }
    }

    if constexpr (!COLS) return;
    float* prow = partial + static_cast<int64_t>(blockIdx.x) * NACC * hidden;
    if constexpr (kColsInLds) {
#pragma unroll
        for (int k = 0; k < VPL; ++k) {
            const int idx = sub + k * LPR;
            if (idx < nv) {
                float a[8], b[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) { a[j] = colbuf[j * cstride + idx]; b[j] = colbuf[(8 + j) * cstride + idx]; }
                store8<float>(prow + idx * kPack, a);
                store8<float>(prow + hidden + idx * kPack, b);
            }
        }
    } else if constexpr (LPR >= 256) {        // every thread owns its columns: nothing to combine
#pragma unroll
        for (int k = 0; k < VPL; ++k) {
            const int idx = sub + k * LPR;
            if (idx < nv) {
                store8<float>(prow + idx * kPack, dg[k]);
                store8<float>(prow + hidden + idx * kPack, db[k]);
                if constexpr (FUSE) store8<float>(prow + 2 * hidden + idx * kPack, dbi[k]);
            }
        }
    } else {
        // Sum the RPB row slots in slot order through LDS.  Layout [dgamma|dbeta(|dbias)][j][pack] with
        // an odd pack stride: consecutive lanes (consecutive packs) fall in consecutive banks.  A
        // [column] layout would put the lanes of a wave 8 floats apart: a 16-way bank conflict.
        const int stride = nv | 1;
        if constexpr (ln_bwd_slots_parallel<LPR, VPL, THREADS, NACC>()) {
            // every slot has its own copy: all slots write at once, one barrier, then all threads
            // add the RPB copies of their columns in slot order (same sums as taking turns)
            const int per_slot = NACC * 8 * stride;
            float* mine = colbuf + slot * per_slot;
#pragma unroll
            for (int k = 0; k < VPL; ++k) {
                const int idx = sub + k * LPR;
                if (idx < nv) {
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        mine[j * stride + idx] = dg[k][j];
                        mine[8 * stride + j * stride + idx] = db[k][j];
                        if constexpr (FUSE) mine[16 * stride + j * stride + idx] = dbi[k][j];
                    }
                }
            }
            __syncthreads();
            for (int c = threadIdx.x; c < NACC * hidden; c += THREADS) {
                const int which = c / hidden;
                const int cc = c - which * hidden;
                const int off = which * 8 * stride + (cc & 7) * stride + (cc >> 3);
                float t = colbuf[off];
#pragma unroll
                for (int sl = 1; sl < RPB; ++sl) t += colbuf[sl * per_slot + off];
                prow[c] = t;
            }
        } else {
            float* cg = colbuf;
            float* cb = colbuf + 8 * stride;
            float* ci = colbuf + 16 * stride;      // FUSE only
            for (int turn = 0; turn < RPB; ++turn) {
                if (slot == turn) {
                    // all reads of the turn first, then the adds, then all writes: a read-add-write
                    // per element would pay one LDS round trip each, 48 in a row
                    if (turn > 0) {
#pragma unroll
                        for (int k = 0; k < VPL; ++k) {
                            const int idx = min(sub + k * LPR, nv - 1);
#pragma unroll
                            for (int j = 0; j < 8; ++j) {
                                dg[k][j] += cg[j * stride + idx];
                                db[k][j] += cb[j * stride + idx];
                                if constexpr (FUSE) dbi[k][j] += ci[j * stride + idx];
                            }
                        }
                    }
#pragma unroll
                    for (int k = 0; k < VPL; ++k) {
                        const int idx = sub + k * LPR;
                        if (idx < nv) {
#pragma unroll
                            for (int j = 0; j < 8; ++j) {
                                cg[j * stride + idx] = dg[k][j];
                                cb[j * stride + idx] = db[k][j];
                                if constexpr (FUSE) ci[j * stride + idx] = dbi[k][j];
                            }
                        }
                    }
                }
                __syncthreads();
            }
            for (int c = threadIdx.x; c < NACC * hidden; c += THREADS) {
                const int which = c / hidden;
                const int cc = c - which * hidden;
                prow[c] = colbuf[which * 8 * stride + (cc & 7) * stride + (cc >> 3)];
            }
        }
    }
}

// ---- generic path: any hidden; TH = 64 (one wave per row) or 256 lanes (one workgroup per row: rows beyond the
// register buckets), rows re-read from cache
// PACKS: the row is a whole number of packs (rows beyond 16384 columns), walked in 128-bit accesses.
template <typename T, int TH, bool PACKS>
__global__ __launch_bounds__(256) void ln_fwd_generic(T* __restrict__ y, float* __restrict__ mean,
                                                      float* __restrict__ rstd, const T* __restrict__ x,
                                                      const T* __restrict__ gamma, const T* __restrict__ beta,
                                                      int64_t rows, int hidden, float eps)
{
    __shared__ float lds[4];
    constexpr int W = PACKS ? kPack : 1;       // elements per access
    const int lane = threadIdx.x % TH;
    const int64_t r = static_cast<int64_t>(blockIdx.x) * (256 / TH) + threadIdx.x / TH;
    if (r >= rows) return;                     // whole waves (TH = 64) or the whole workgroup (TH = 256) leave together
    auto row_total = [&](float v) {
        if constexpr (TH == 64) return group_sum<64>(v);
        else return block_allreduce<4, OpSum>(v, lds);
    };
    auto get = [&](const T* p, float (&f)[W]) {
        if constexpr (PACKS) load8<T>(p, f);
        else f[0] = to_f32<T>(p[0]);
    };
    const T* xr = x + r * hidden;
    const float inv_h = 1.0f / static_cast<float>(hidden);
    float s = 0.0f;
    for (int i = lane * W; i < hidden; i += TH * W) {
        float v[W];
        get(xr + i, v);
#pragma unroll
        for (int j = 0; j < W; ++j) s += v[j];
    }
    const float mu = row_total(s) * inv_h;
    float q = 0.0f;
    for (int i = lane * W; i < hidden; i += TH * W) {
        float v[W];
        get(xr + i, v);
#pragma unroll
        for (int j = 0; j < W; ++j) { const float d = v[j] - mu; q = fmaf(d, d, q); }
    }
    const float rs = 1.0f / sqrtf(fmaf(row_total(q), inv_h, eps));
    if (lane == 0) { mean[r] = mu; rstd[r] = rs; }
    T* yr = y + r * hidden;
    for (int i = lane * W; i < hidden; i += TH * W) {
        float v[W], gm[W], bt[W];
        get(xr + i, v);
        get(gamma + i, gm);
        get(beta + i, bt);
#pragma unroll
        for (int j = 0; j < W; ++j) v[j] = fmaf((v[j] - mu) * rs, gm[j], bt[j]);
        if constexpr (PACKS) store8<T>(yr + i, v);
        else yr[i] = from_f32<T>(v[0]);
    }
}

template <typename T, int TH, bool PACKS>
__global__ __launch_bounds__(256) void ln_bwd_generic(T* dx, const T* dy, const T* __restrict__ x,
                                                      const T* __restrict__ gamma, const float* __restrict__ mean,
                                                      const float* __restrict__ rstd, const T* dres,
                                                      int64_t rows, int hidden)
{
    __shared__ float lds[4];
    constexpr int W = PACKS ? kPack : 1;
    const int lane = threadIdx.x % TH;
    const int64_t r = static_cast<int64_t>(blockIdx.x) * (256 / TH) + threadIdx.x / TH;
    if (r >= rows) return;
    auto row_total = [&](float v) {
        if constexpr (TH == 64) return group_sum<64>(v);
        else return block_allreduce<4, OpSum>(v, lds);
    };
    auto get = [&](const T* p, float (&f)[W]) {
        if constexpr (PACKS) load8<T>(p, f);
        else f[0] = to_f32<T>(p[0]);
    };
    const int64_t ro = r * hidden;
    const float mu = mean[r], rs = rstd[r];
    const float inv_h = 1.0f / static_cast<float>(hidden);
    float s1 = 0.0f, s2 = 0.0f;
    for (int i = lane * W; i < hidden; i += TH * W) {
        float gy[W], xv[W], gm[W];
        get(dy + ro + i, gy);
        get(x + ro + i, xv);
        get(gamma + i, gm);
#pragma unroll
        for (int j = 0; j < W; ++j) {
            const float gg = gy[j] * gm[j];
            s1 += gg;
            s2 = fmaf(gg, (xv[j] - mu) * rs, s2);
        }
    }
    const float a = row_total(s1) * inv_h, b = row_total(s2) * inv_h;
    for (int i = lane * W; i < hidden; i += TH * W) {
        float gy[W], xv[W], gm[W], rv[W];
        get(dy + ro + i, gy);
        get(x + ro + i, xv);
        get(gamma + i, gm);
        if (dres) get(dres + ro + i, rv);
#pragma unroll
        for (int j = 0; j < W; ++j) {
            const float gg = gy[j] * gm[j];
            const float xhat = (xv[j] - mu) * rs;
            float v = rs * (gg - fmaf(xhat, b, a));
            if (dres) v += rv[j];
            gy[j] = v;
        }
        if constexpr (PACKS) store8<T>(dx + ro + i, gy);
        else dx[ro + i] = from_f32<T>(gy[0]);
    }
}

// dgamma/dbeta for the generic path, first stage: one thread per column, gridDim.y row
// blocks that each walk every gridDim.y-th row (four rows in flight); partial[y] =
// [dgamma | dbeta] of block y, summed by colsum_finalize_kernel like the fast path's.
// Runs BEFORE ln_bwd_generic so that dx may alias dy.
template <typename T>
__global__ __launch_bounds__(256) void ln_dparams_generic(float* __restrict__ partial,
                                                          const T* __restrict__ dy, const T* __restrict__ x,
                                                          const float* __restrict__ mean, const float* __restrict__ rstd,
                                                          int64_t rows, int hidden)
{
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= hidden) return;
    float sg = 0.0f, sb = 0.0f;
    const int64_t stride = gridDim.y;
    for (int64_t r0 = blockIdx.y; r0 < rows; r0 += 4 * stride) {
        float gy[4], xv[4], mu[4], rs[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t r = r0 + u * stride;
            const bool ok = r < rows;
            gy[u] = ok ? to_f32<T>(dy[r * hidden + c]) : 0.0f;
            xv[u] = ok ? to_f32<T>(x[r * hidden + c]) : 0.0f;
            mu[u] = ok ? mean[r] : 0.0f;
            rs[u] = ok ? rstd[r] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            sg = fmaf(gy[u], (xv[u] - mu[u]) * rs[u], sg);
            sb += gy[u];
        }
    }
    float* prow = partial + static_cast<int64_t>(blockIdx.y) * 2 * hidden;
    prow[c] = sg;
    prow[hidden + c] = sb;
}

// The same first stage for rows of whole packs: one thread per PACK of 8 columns (128-bit
// loads), four rows in flight.  Serves the rows that are too wide for the column
// accumulators to stay in registers next to the row itself.
template <typename T>
__global__ __launch_bounds__(256) void ln_dparams_packed(float* __restrict__ partial,
                                                         const T* __restrict__ dy, const T* __restrict__ x,
                                                         const float* __restrict__ mean, const float* __restrict__ rstd,
                                                         int64_t rows, int hidden)
{
    const int idx = blockIdx.x * 256 + threadIdx.x;       // pack of the row
    if (idx >= hidden / kPack) return;
    float sg[8] = {0, 0, 0, 0, 0, 0, 0, 0}, sb[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    const int64_t stride = gridDim.y;
    for (int64_t r0 = blockIdx.y; r0 < rows; r0 += 4 * stride) {
        RawPack<T> gy[4], xv[4];
        float mu[4], rs[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t r = r0 + u * stride;
            const bool ok = r < rows;
            gy[u] = ok ? load_raw<T, false>(dy + r * hidden + idx * kPack) : zero_raw<T>();
            xv[u] = ok ? load_raw<T, false>(x + r * hidden + idx * kPack) : zero_raw<T>();
            mu[u] = ok ? mean[r] : 0.0f;
            rs[u] = ok ? rstd[r] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            float g8[8], x8[8];
            unpack<T>(gy[u], g8);
            unpack<T>(xv[u], x8);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                sg[j] = fmaf(g8[j], (x8[j] - mu[u]) * rs[u], sg[j]);
                sb[j] += g8[j];
            }
        }
    }
    float* prow = partial + static_cast<int64_t>(blockIdx.y) * 2 * hidden;
    store8<float>(prow + idx * kPack, sg);
    store8<float>(prow + hidden + idx * kPack, sb);
}

constexpr int kLnWideLpr = 1024, kLnWideVpl = 2;      // the bucket of rows with 1025..2048 packs

// ------------------------------------------------------------------ dispatch
// Shape buckets: lanes per row and packs per lane for a row of nv packs.
struct LnShape { int lpr, vpl; };

inline LnShape ln_shape(int hidden)
{
    if (hidden % kPack != 0) return {0, 0};
    const int nv = hidden / kPack;
    // rows of up to 384 packs: lanes of one wave, the shape with the fewest idle lane slots; among
    // equals 32 lanes (two rows per wave) before 64.  256..1536 columns in steps of 256 fit 32 x 1..6
    // exactly, 2560 and 3072 fit 64 x 5 and 64 x 6.  Measured forward at 8192 rows, 32 x 4 against
    // 64 x 2 at 1024 columns: 8.3 against 9.1 us (fused with bias+dropout+residual 13.9 against 15.7);
    // 32 x 2 against 64 x 1 at 512: 5.6 against 6.2; 32 x 6 against 64 x 3 at 1536: 11.6 against 12.3.
    // (32 x 8 at 2048 helps the plain forward, 14.3 against 16.8 us, but costs the fused one 2 us: not built.)
    static const LnShape wave_shapes[] = {{32, 1}, {32, 2}, {32, 3}, {32, 4}, {32, 5}, {32, 6}, {64, 1}, {64, 2}, {64, 3},
                                          {64, 4}, {64, 5}, {64, 6}, {16, 1}, {8, 1}};
    if (nv <= 384) {
        LnShape best{0, 0};
        for (const LnShape& c : wave_shapes)
            if (c.lpr * c.vpl >= nv && (best.lpr == 0 || c.lpr * c.vpl < best.lpr * best.vpl)) best = c;
        return best;
    }
    if (nv <= 512) return {256, 2};
    if (nv <= 768) return {256, 3};       // 5120 columns: 640 of 768 pack slots in use (of 1024 as 256 x 4); 6144 fit exactly
    if (nv <= 1024) return {256, 4};
    if (nv <= 2048) return {kLnWideLpr, kLnWideVpl};     // hidden up to 16384: one large workgroup per row
    return {0, 0};
}

// Backward keeps 2 (3 when fused) fp32 column accumulators per element of a lane next to the rows in
// flight and sums the row slots of a workgroup through LDS: from three packs per lane on, 64 lanes per
// row with an idle tail beat the exact fit on 32 (8192 rows: 1280 columns 18.9 against 20.7 us as 32 x 5,
// 1024 columns 16.9 against 20.0 us as 32 x 4); 512 columns stay on 32 x 2 (11.5 against 12.9 us as 64 x 1).
inline LnShape ln_bwd_shape(int hidden)
{
    const LnShape f = ln_shape(hidden);
    if (f.lpr != 32 || f.vpl <= 2) return f;
    return {64, (hidden / kPack + 63) / 64};
}

inline int ln_fwd_blocks(int64_t rows, int lpr)
{
    const int rpb = lpr > 256 ? 1 : 256 / lpr;
    int64_t b = ceil_div(rows, static_cast<int64_t>(rpb) * 2);   // two row groups per workgroup (one: 11.1, two: 9.2, four: 10.4 us at 8192 x 1280)
    if (b > 8192) b = 8192;
    if (b < 1) b = 1;
    return static_cast<int>(b);
}

#define LSQ_LN_CASES_COMMON(X) X(8, 1) X(16, 1) X(32, 1) X(64, 1) X(64, 2) X(64, 3) X(64, 4) X(64, 5) X(64, 6) X(256, 2) X(256, 3) X(256, 4)

// fuse != nullptr: x is the projection output and *fuse carries h / residual / bias / dropout
template <typename T>
static lsq_status ln_fwd_dispatch(void* y, float* mean, float* rstd, const void* x, const void* gamma, const void* beta,
                                  int64_t rows, int32_t hidden, float eps, hipStream_t s,
                                  const BdrFuse<T>* fuse = nullptr)
{
    T* yp = static_cast<T*>(y);
    const T* xp = static_cast<const T*>(x);
    const T* gp = static_cast<const T*>(gamma);
    const T* bp = static_cast<const T*>(beta);
    LnShape sh = ln_shape(hidden);
    // rows of 8193..16384 columns: the forward has the registers for 6 or 8 packs per lane of a 256-thread
    // workgroup (0.70 of peak at 12288 columns against 0.53 with the backward's 1024 lanes x 2 packs).  The fused
    // boundary follows (it would be 10 % faster on 1024 lanes, but then no longer bit-identical to the two calls).
    if (sh.lpr > 256) sh = hidden / kPack <= 1536 ? LnShape{256, 6} : LnShape{256, 8};
    if (sh.lpr == 0) {
        // rows too long for the register buckets come in small numbers: a whole workgroup per row
        if (hidden % kPack == 0)
            hipLaunchKernelGGL((ln_fwd_generic<T, 256, true>), dim3(static_cast<unsigned>(rows)), dim3(256), 0, s,
                               yp, mean, rstd, xp, gp, bp, rows, hidden, eps);
        else if (hidden > 2048)
            hipLaunchKernelGGL((ln_fwd_generic<T, 256, false>), dim3(static_cast<unsigned>(rows)), dim3(256), 0, s,
                               yp, mean, rstd, xp, gp, bp, rows, hidden, eps);
        else
            hipLaunchKernelGGL((ln_fwd_generic<T, 64, false>), dim3(static_cast<unsigned>(ceil_div(rows, 4))), dim3(256), 0, s,
                               yp, mean, rstd, xp, gp, bp, rows, hidden, eps);
        return launch_status();
    }
    const dim3 grid(ln_fwd_blocks(rows, sh.lpr)), block(sh.lpr > 256 ? sh.lpr : 256);
    const BdrFuse<T> none{};
#define X(L, V)                                                                                              \
    if (sh.lpr == L && sh.vpl == V) {                                                                        \
        if (!fuse) hipLaunchKernelGGL((ln_fwd_kernel<T, L, V>), grid, block, 0, s, yp, mean, rstd, xp, gp, bp, rows, hidden, eps, none); \
        else if (fuse->d.on) hipLaunchKernelGGL((ln_fwd_kernel<T, L, V, true, true>), grid, block, 0, s, yp, mean, rstd, xp, gp, bp, rows, hidden, eps, *fuse); \
        else hipLaunchKernelGGL((ln_fwd_kernel<T, L, V, true, false>), grid, block, 0, s, yp, mean, rstd, xp, gp, bp, rows, hidden, eps, *fuse); \
    }
    LSQ_LN_CASES_COMMON(X) X(32, 2) X(32, 3) X(32, 4) X(32, 5) X(32, 6) X(256, 6) X(256, 8)
#undef X
    return launch_status();
}

// Backward of rows with 1025..2048 packs: the column accumulators are thread-private LDS entries
// (up to 131 KB, above the 64 KiB a kernel gets by default: the limit is raised once per device).
template <typename T, int L, int V>
static lsq_status ln_bwd_wide(T* dxp, float* partial, const T* dyp, const T* xp, const T* gp, const float* mean,
                              const float* rstd, const T* rp, int64_t rows, int32_t hidden, int P, hipStream_t s)
{
    constexpr int TH = L >= 256 ? L : 256;
    const BdrFuse<T> nofuse{};
    const size_t shmem = sizeof(float) * 16 * ((hidden / kPack) | 1);
    auto* kres = &ln_bwd_kernel<T, L, V, true, TH, false, false, true>;
    auto* kplain = &ln_bwd_kernel<T, L, V, false, TH, false, false, true>;
    // once per residual variant and device (a host-side note, guarded for concurrent host threads)
    static std::mutex mu;
    static bool ready[2][64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return LSQ_LAUNCH_FAILED;
    const bool known = dev >= 0 && dev < 64;
    {
        std::lock_guard<std::mutex> lock(mu);
        if (!known || !ready[rp ? 1 : 0][dev]) {
            if (hipFuncSetAttribute(rp ? reinterpret_cast<const void*>(kres) : reinterpret_cast<const void*>(kplain),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 256) != hipSuccess)
                return LSQ_LAUNCH_FAILED;
            if (known) ready[rp ? 1 : 0][dev] = true;
        }
    }
    if (rp) hipLaunchKernelGGL(kres, dim3(P), dim3(TH), shmem, s, dxp, partial, dyp, xp, gp, mean, rstd, rp, rows, hidden, nofuse);
    else hipLaunchKernelGGL(kplain, dim3(P), dim3(TH), shmem, s, dxp, partial, dyp, xp, gp, mean, rstd, rp, rows, hidden, nofuse);
    return launch_status();
}

template <typename T>
static lsq_status ln_bwd_dispatch(void* dx, float* dgamma, float* dbeta, const void* dy, const void* x,
                                  const void* gamma, const float* mean, const float* rstd, const void* dres,
                                  void* workspace, int64_t rows, int32_t hidden, hipStream_t s,
                                  const BdrFuse<T>* fuse = nullptr, float* dbias = nullptr)
{
    T* dxp = static_cast<T*>(dx);
    const T* dyp = static_cast<const T*>(dy);
    const T* xp = static_cast<const T*>(x);
    const T* gp = static_cast<const T*>(gamma);
    const T* rp = static_cast<const T*>(dres);
    const LnShape sh = ln_bwd_shape(hidden);
    if (sh.lpr == 0) {
        const int Pg = ln_bwd_blocks(rows, hidden);
        float* gpartial = static_cast<float*>(workspace);
        if (hidden % kPack == 0)
            hipLaunchKernelGGL((ln_dparams_packed<T>), dim3(static_cast<unsigned>(ceil_div(hidden / kPack, 256)), static_cast<unsigned>(Pg)),
                               dim3(256), 0, s, gpartial, dyp, xp, mean, rstd, rows, hidden);
        else
            hipLaunchKernelGGL((ln_dparams_generic<T>), dim3(static_cast<unsigned>(ceil_div(hidden, 256)), static_cast<unsigned>(Pg)),
                               dim3(256), 0, s, gpartial, dyp, xp, mean, rstd, rows, hidden);
        launch_colsum_finalize(dgamma, dbeta, hidden, gpartial, Pg, 2 * hidden, s);
        if (hidden % kPack == 0)
            hipLaunchKernelGGL((ln_bwd_generic<T, 256, true>), dim3(static_cast<unsigned>(rows)), dim3(256), 0, s,
                               dxp, dyp, xp, gp, mean, rstd, rp, rows, hidden);
        else if (hidden > 2048)
            hipLaunchKernelGGL((ln_bwd_generic<T, 256, false>), dim3(static_cast<unsigned>(rows)), dim3(256), 0, s,
                               dxp, dyp, xp, gp, mean, rstd, rp, rows, hidden);
        else
            hipLaunchKernelGGL((ln_bwd_generic<T, 64, false>), dim3(static_cast<unsigned>(ceil_div(rows, 4))), dim3(256), 0, s,
                               dxp, dyp, xp, gp, mean, rstd, rp, rows, hidden);
        return launch_status();
    }
    const int P = ln_bwd_blocks(rows, hidden);
    float* partial = static_cast<float*>(workspace);
    if (sh.lpr > 256) {       // 8193..16384 columns (never fused: the entry point splits such rows into its two operators)
        lsq_status st;
        // (256 lanes x 6 or 8 packs with the same LDS accumulators: 200 us against 122 us at 8192 x 12288)
        st = ln_bwd_wide<T, kLnWideLpr, kLnWideVpl>(dxp, partial, dyp, xp, gp, mean, rstd, rp, rows, hidden, P, s);
        if (st != LSQ_OK) return st;
        launch_colsum_finalize(dgamma, dbeta, hidden, partial, P, 2 * hidden, s);
        return launch_status();
    }
    const int nacc = fuse ? 3 : 2;
    const size_t one_copy = sh.lpr >= 256 ? 0 : sizeof(float) * 8 * nacc * ((hidden / kPack) | 1);
    const BdrFuse<T> none{};
#define X(L, V)                                                                                              \
    if (sh.lpr == L && sh.vpl == V) {                                                                        \
        constexpr int TH = L >= 256 ? L : kLnBwdThreads;                                                   \
        const bool par = fuse ? ln_bwd_slots_parallel<L, V, TH, 3>() : ln_bwd_slots_parallel<L, V, TH, 2>(); \
        const size_t shmem = par ? one_copy * (TH / L) : one_copy;                                           \
        const dim3 grid(P), block(TH);                                                                       \
        if (!fuse) {                                                                                         \
            if (rp) hipLaunchKernelGGL((ln_bwd_kernel<T, L, V, true, TH>), grid, block, shmem, s, dxp, partial, dyp, xp, gp, mean, rstd, rp, rows, hidden, none); \
            else hipLaunchKernelGGL((ln_bwd_kernel<T, L, V, false, TH>), grid, block, shmem, s, dxp, partial, dyp, xp, gp, mean, rstd, rp, rows, hidden, none);   \
        } else if (fuse->d.on) {                                                                            \
            if (rp) hipLaunchKernelGGL((ln_bwd_kernel<T, L, V, true, TH, true, true>), grid, block, shmem, s, dxp, partial, dyp, xp, gp, mean, rstd, rp, rows, hidden, *fuse); \
            else hipLaunchKernelGGL((ln_bwd_kernel<T, L, V, false, TH, true, true>), grid, block, shmem, s, dxp, partial, dyp, xp, gp, mean, rstd, rp, rows, hidden, *fuse);   \
        } else {                                                                                             \
            if (rp) hipLaunchKernelGGL((ln_bwd_kernel<T, L, V, true, TH, true, false>), grid, block, shmem, s, dxp, partial, dyp, xp, gp, mean, rstd, rp, rows, hidden, *fuse); \
            else hipLaunchKernelGGL((ln_bwd_kernel<T, L, V, false, TH, true, false>), grid, block, shmem, s, dxp, partial, dyp, xp, gp, mean, rstd, rp, rows, hidden, *fuse);   \
        }                                                                                                    \
    }
    LSQ_LN_CASES_COMMON(X) X(32, 2)
#undef X
    if (fuse) launch_colsum_finalize(dgamma, dbeta, hidden, partial, P, 3 * hidden, s, dbias, 2 * hidden);
    else launch_colsum_finalize(dgamma, dbeta, hidden, partial, P, 2 * hidden, s);
    return launch_status();
}

}  // namespace lsq

extern "C" lsq_status lsq_layernorm_fwd(void* y, float* mean, float* rstd, const void* x, const void* gamma,
                                        const void* beta, int64_t rows, int32_t hidden, float eps, lsq_dtype dt,
                                        void* stream)
{
    using namespace lsq;
    LSQ_REQUIRE(rows >= 0 && hidden > 0 && eps >= 0.0f);
    if (!valid_dtype(dt)) return LSQ_UNSUPPORTED_DTYPE;
    if (rows == 0) return LSQ_OK;
    LSQ_REQUIRE(y && mean && rstd && x && gamma && beta);
    LSQ_ALIGNED(y); LSQ_ALIGNED(x); LSQ_ALIGNED(gamma); LSQ_ALIGNED(beta);
    LSQ_REQUIRE(rows <= 0x7FFFFFFF);
    hipStream_t s = static_cast<hipStream_t>(stream);
    switch (dt) {
        case LSQ_F16: return ln_fwd_dispatch<f16>(y, mean, rstd, x, gamma, beta, rows, hidden, eps, s);
        case LSQ_BF16: return ln_fwd_dispatch<bf16>(y, mean, rstd, x, gamma, beta, rows, hidden, eps, s);
        default: return ln_fwd_dispatch<float>(y, mean, rstd, x, gamma, beta, rows, hidden, eps, s);
    }
}

extern "C" lsq_status lsq_layernorm_bwd(void* dx, float* dgamma, float* dbeta, const void* dy, const void* x,
                                        const void* gamma, const float* mean, const float* rstd, const void* dres_in,
                                        void* workspace, size_t workspace_bytes, int64_t rows, int32_t hidden,
                                        lsq_dtype dt, void* stream)
{
    using namespace lsq;
    LSQ_REQUIRE(rows >= 0 && hidden > 0);
    if (!valid_dtype(dt)) return LSQ_UNSUPPORTED_DTYPE;
    LSQ_REQUIRE(dgamma && dbeta);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (rows == 0) {
        lsq_status st = zero_fill(dgamma, hidden, s);
        return st != LSQ_OK ? st : zero_fill(dbeta, hidden, s);
    }
    LSQ_REQUIRE(dx && dy && x && gamma && mean && rstd);
    LSQ_ALIGNED(dx); LSQ_ALIGNED(dy); LSQ_ALIGNED(x); LSQ_ALIGNED(gamma); LSQ_ALIGNED(dres_in); LSQ_ALIGNED(workspace);
    LSQ_REQUIRE(rows <= 0x7FFFFFFF);
    const size_t need = lsq_workspace_bytes(LSQ_OP_LAYERNORM_BWD, rows, hidden);
    if (need && (!workspace || workspace_bytes < need)) return LSQ_WORKSPACE_TOO_SMALL;
    switch (dt) {
        case LSQ_F16: return ln_bwd_dispatch<f16>(dx, dgamma, dbeta, dy, x, gamma, mean, rstd, dres_in, workspace, rows, hidden, s);
        case LSQ_BF16: return ln_bwd_dispatch<bf16>(dx, dgamma, dbeta, dy, x, gamma, mean, rstd, dres_in, workspace, rows, hidden, s);
        default: return ln_bwd_dispatch<float>(dx, dgamma, dbeta, dy, x, gamma, mean, rstd, dres_in, workspace, rows, hidden, s);
    }
}

// ---- LayerNorm backward for callers that may not allocate: the partial rows of the column sums go to
// device memory the library itself holds, one copy per GPU, for as long as the process lives.
namespace lsq {
constexpr size_t kLnScratchBytes = 8u << 20;
static __device__ __align__(256) unsigned char scratch[kLnScratchBytes];

// The array's address on the current device.  `scratch` itself is only a host-side handle: the
// address is asked for once per device (each GPU holds its own copy at its own address) and kept.
static void* ln_scratch_on_current_device()
{
    static std::mutex mu;
    static void* ptr[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        ptr[dev] = p;
    }
    return ptr[dev];
}
}  // namespace lsq

extern "C" lsq_status lsq_layernorm_bwd_noalloc(void* dx, float* dgamma, float* dbeta, const void* dy, const void* x,
                                                const void* gamma, const float* mean, const float* rstd,
                                                const void* dres_in, int64_t rows, int32_t hidden, lsq_dtype dt,
                                                void* stream)
{
    using namespace lsq;
    LSQ_REQUIRE(rows >= 0 && hidden > 0);
    if (lsq_workspace_bytes(LSQ_OP_LAYERNORM_BWD, rows, hidden) > kLnScratchBytes) return LSQ_WORKSPACE_TOO_SMALL;
    void* ws = nullptr;
    if (rows > 0) {
        ws = ln_scratch_on_current_device();
        if (!ws) return LSQ_LAUNCH_FAILED;
    }
    return lsq_layernorm_bwd(dx, dgamma, dbeta, dy, x, gamma, mean, rstd, dres_in, ws, kLnScratchBytes, rows, hidden, dt,
                             stream);
}

// ---- fused sub-layer boundary of a pre-LN Transformer
namespace lsq {
template <typename T>
static lsq_status bdr_ln_fwd_typed(void* h, void* y, float* mean, float* rstd, const void* x, const void* bias,
                                   const void* residual, const void* gamma, const void* beta, int64_t rows,
                                   int32_t hidden, float eps, const DropoutParams& d, hipStream_t s)
{
    const BdrFuse<T> fz{static_cast<T*>(h), static_cast<const T*>(residual), static_cast<const T*>(bias), d};
    return ln_fwd_dispatch<T>(y, mean, rstd, x, gamma, beta, rows, hidden, eps, s, &fz);
}

template <typename T>
static lsq_status bdr_ln_bwd_typed(void* dh, void* dx, float* dgamma, float* dbeta, float* dbias, const void* dy,
                                   const void* h, const void* gamma, const float* mean, const float* rstd,
                                   const void* dres_in, void* workspace, int64_t rows, int32_t hidden,
                                   const DropoutParams& d, hipStream_t s)
{
    const BdrFuse<T> fz{static_cast<T*>(dx), nullptr, nullptr, d};
    return ln_bwd_dispatch<T>(dh, dgamma, dbeta, dy, h, gamma, mean, rstd, dres_in, workspace, rows, hidden, s, &fz, dbias);
}
}  // namespace lsq

extern "C" lsq_status lsq_bdr_layernorm_fwd(void* h, void* y, float* mean, float* rstd, const void* x, const void* bias,
                                            const void* residual, const void* gamma, const void* beta, int64_t rows,
                                            int32_t hidden, float p, uint64_t seed, uint64_t offset, float eps,
                                            lsq_dtype dt, void* stream)
{
    using namespace lsq;
    LSQ_REQUIRE(rows >= 0 && hidden > 0 && eps >= 0.0f);
    if (!valid_dtype(dt)) return LSQ_UNSUPPORTED_DTYPE;
    DropoutParams d;
    LSQ_REQUIRE(make_dropout(p, seed, offset, &d));
    if (rows == 0) return LSQ_OK;
    LSQ_REQUIRE(h && y && mean && rstd && x && residual && gamma && beta);
    LSQ_ALIGNED(h); LSQ_ALIGNED(y); LSQ_ALIGNED(x); LSQ_ALIGNED(bias); LSQ_ALIGNED(residual); LSQ_ALIGNED(gamma); LSQ_ALIGNED(beta);
    LSQ_REQUIRE(ceil_div(rows * hidden, 256) <= 0x7FFFFFFF);
    if (ln_shape(hidden).lpr == 0) {      // no register bucket for this row length: the two operators back to back
        const lsq_status st = lsq_bias_dropout_residual_fwd(h, x, bias, residual, rows, hidden, p, seed, offset, dt, stream);
        return st != LSQ_OK ? st : lsq_layernorm_fwd(y, mean, rstd, h, gamma, beta, rows, hidden, eps, dt, stream);
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    switch (dt) {
        case LSQ_F16: return bdr_ln_fwd_typed<f16>(h, y, mean, rstd, x, bias, residual, gamma, beta, rows, hidden, eps, d, s);
        case LSQ_BF16: return bdr_ln_fwd_typed<bf16>(h, y, mean, rstd, x, bias, residual, gamma, beta, rows, hidden, eps, d, s);
        default: return bdr_ln_fwd_typed<float>(h, y, mean, rstd, x, bias, residual, gamma, beta, rows, hidden, eps, d, s);
    }
}

extern "C" lsq_status lsq_bdr_layernorm_bwd(void* dh, void* dx, float* dgamma, float* dbeta, float* dbias, const void* dy,
                                            const void* h, const void* gamma, const float* mean, const float* rstd,
                                            const void* dres_in, void* workspace, size_t workspace_bytes, int64_t rows,
                                            int32_t hidden, float p, uint64_t seed, uint64_t offset, lsq_dtype dt,
                                            void* stream)
{
    using namespace lsq;
    LSQ_REQUIRE(rows >= 0 && hidden > 0);
    if (!valid_dtype(dt)) return LSQ_UNSUPPORTED_DTYPE;
    DropoutParams d;
    LSQ_REQUIRE(make_dropout(p, seed, offset, &d));
    LSQ_REQUIRE(dgamma && dbeta && dbias);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (rows == 0) {
        lsq_status st = zero_fill(dgamma, hidden, s);
        if (st == LSQ_OK) st = zero_fill(dbeta, hidden, s);
        return st != LSQ_OK ? st : zero_fill(dbias, hidden, s);
    }
    LSQ_REQUIRE(dh && dx && dy && h && gamma && mean && rstd);
    LSQ_ALIGNED(dh); LSQ_ALIGNED(dx); LSQ_ALIGNED(dy); LSQ_ALIGNED(h); LSQ_ALIGNED(gamma); LSQ_ALIGNED(dres_in);
    LSQ_ALIGNED(workspace);
    LSQ_REQUIRE(ceil_div(rows * hidden, 256) <= 0x7FFFFFFF);
    const size_t need = lsq_workspace_bytes(LSQ_OP_BDR_LAYERNORM_BWD, rows, hidden);
    if (need && (!workspace || workspace_bytes < need)) return LSQ_WORKSPACE_TOO_SMALL;
    if (ln_shape(hidden).lpr == 0 || ln_shape(hidden).lpr > 256) {      // no fused bucket: the two operators back to back
        const lsq_status st = lsq_layernorm_bwd(dh, dgamma, dbeta, dy, h, gamma, mean, rstd, dres_in, workspace,
                                                workspace_bytes, rows, hidden, dt, stream);
        return st != LSQ_OK ? st : lsq_bias_dropout_residual_bwd(dx, dbias, dh, rows, hidden, p, seed, offset, workspace,
                                                                workspace_bytes, dt, stream);
    }
    switch (dt) {
        case LSQ_F16: return bdr_ln_bwd_typed<f16>(dh, dx, dgamma, dbeta, dbias, dy, h, gamma, mean, rstd, dres_in, workspace, rows, hidden, d, s);
        case LSQ_BF16: return bdr_ln_bwd_typed<bf16>(dh, dx, dgamma, dbeta, dbias, dy, h, gamma, mean, rstd, dres_in, workspace, rows, hidden, d, s);
        default: return bdr_ln_bwd_typed<float>(dh, dx, dgamma, dbeta, dbias, dy, h, gamma, mean, rstd, dres_in, workspace, rows, hidden, d, s);
    }
}
