// Streaming passes of a DA stage (Sec. 3.1): heat x' = e_x + c_m(i_m(x)), the new residue
// e_x = x' - c_m(i_m(x)), and the error of Eq. 1 (first line).  All are HBM-bound: every
// thread moves one float4 per row pass, a wave covers contiguous kilobytes, the K x D
// codebook (<= 1 MB) stays in L2.
#pragma once
#include "common.hpp"

namespace hclae {

constexpr int kStreamThreads = 256;    // heat / cool
constexpr int kStreamUnroll = 4;
constexpr int kFlatThreads = 256;      // flat float4 passes (copy, reduction, finish)

typedef float floatx4 __attribute__((ext_vector_type(4)));

// Geometry of heat / cool: a block is (1 << lcw) column threads by (kStreamThreads >> lcw) rows; column thread tx walks float4 columns tx, tx + cw, ...
struct RowGeom {
    int lcw;        // log2 of column threads per row
    int d4;         // D / 4
};

// residue_n (+|-)= C_m[codes[n][m]]  with optional by-products:
//   SIGN = +1 : heat.  Also saves column m of the codes (old_codes) and sums ||e_x||^2 of the input.
//   SIGN = -1 : cool.  Also sums ||e_x||^2 of the output and counts codes != old_codes.
// part_err[blockIdx.x], part_chg[blockIdx.x] receive this block's partial sums (fixed order).
template <int SIGN, bool STATS>
__global__ __launch_bounds__(kStreamThreads) void k_heat_cool(
    float *__restrict__ r, const uint8_t *__restrict__ codes, const float *__restrict__ Cm,
    int64_t N, int D, int M, int m, RowGeom g,
    uint8_t *__restrict__ old_codes, double *__restrict__ part_err, long long *__restrict__ part_chg)
{
    __shared__ double red[kStreamThreads / kWave];
    constexpr int U = kStreamUnroll;                       // independent rows per thread per pass
    const int cw = 1 << g.lcw;
    const int tx = threadIdx.x & (cw - 1);
    const int ty = threadIdx.x >> g.lcw;
    const int rows = kStreamThreads >> g.lcw;
    double err = 0.0;
    long long chg = 0;
    for (int64_t n0 = (int64_t)blockIdx.x * rows * U + ty; n0 < N; n0 += (int64_t)gridDim.x * rows * U) {
        int code[U];
        bool ok[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t n = n0 + (int64_t)u * rows;
            ok[u] = n < N;
            code[u] = ok[u] ? (int)codes[n * M + m] : 0;
        }
        if (STATS && tx == 0) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t n = n0 + (int64_t)u * rows;
                if (ok[u]) {
                    if (SIGN > 0) old_codes[n] = (uint8_t)code[u];
                    else chg += (old_codes[n] != (uint8_t)code[u]);
                }
            }
        }
        for (int j = tx; j < g.d4; j += cw) {
            floatx4 v[U], cv[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t n = n0 + (int64_t)u * rows;
                if (ok[u]) {
                    v[u] = __builtin_nontemporal_load(reinterpret_cast<const floatx4 *>(r + n * D) + j);
                    cv[u] = *(reinterpret_cast<const floatx4 *>(Cm + (size_t)code[u] * D) + j);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t n = n0 + (int64_t)u * rows;
                if (ok[u]) {
                    floatx4 w = v[u];
                    if (STATS && SIGN > 0)
                        err += (double)w.x * w.x + (double)w.y * w.y + (double)w.z * w.z + (double)w.w * w.w;
                    if (SIGN > 0) w = w + cv[u];
                    else w = w - cv[u];
                    if (STATS && SIGN < 0)
                        err += (double)w.x * w.x + (double)w.y * w.y + (double)w.z * w.z + (double)w.w * w.w;
                    __builtin_nontemporal_store(w, reinterpret_cast<floatx4 *>(r + n * D) + j);
                }
            }
        }
    }
    if (STATS) {
        const double e = block_sum(err, red);
        if (threadIdx.x == 0) part_err[blockIdx.x] = e;
        if (SIGN < 0) {
            // integer sum: any order gives the same value
            const double c = block_sum((double)chg, red);
            if (threadIdx.x == 0) part_chg[blockIdx.x] = (long long)c;
        }
    }
}

// Stage boundary inside a sweep, one pass instead of two: e_x = x' - c_m(i_m) (end of stage m) followed
// at once by x'' = e_x + c_j(i_j) (heat of the next stage j).  The intermediate e_x is rounded to fp32
// exactly as if it had been stored and reloaded, so the result equals cool(m) then heat(j) bit for bit.
// By-products: sum ||e_x||^2 (error after stage m = error before stage j), codes of stage m changed
// since its entry, and the code column of stage j saved for its own change count.
__global__ __launch_bounds__(kStreamThreads) void k_transition(
    float *__restrict__ r, const uint8_t *__restrict__ codes, const float *__restrict__ Cm, const float *__restrict__ Cj,
    int64_t N, int D, int M, int m, int j_stage, RowGeom g,
    uint8_t *__restrict__ old_codes, double *__restrict__ part_err, long long *__restrict__ part_chg)
{
    __shared__ double red[kStreamThreads / kWave];
    constexpr int U = kStreamUnroll;
    const int cw = 1 << g.lcw;
    const int tx = threadIdx.x & (cw - 1);
    const int ty = threadIdx.x >> g.lcw;
    const int rows = kStreamThreads >> g.lcw;
    double err = 0.0;
    long long chg = 0;
    for (int64_t n0 = (int64_t)blockIdx.x * rows * U + ty; n0 < N; n0 += (int64_t)gridDim.x * rows * U) {
        int cm[U], cj[U];
        bool ok[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t n = n0 + (int64_t)u * rows;
            ok[u] = n < N;
            cm[u] = ok[u] ? (int)codes[n * M + m] : 0;
            cj[u] = ok[u] ? (int)codes[n * M + j_stage] : 0;
        }
        if (tx == 0) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t n = n0 + (int64_t)u * rows;
                if (ok[u]) {
                    chg += (old_codes[n] != (uint8_t)cm[u]);
                    old_codes[n] = (uint8_t)cj[u];
                }
            }
        }
        for (int c4 = tx; c4 < g.d4; c4 += cw) {
            floatx4 v[U], a[U], b[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t n = n0 + (int64_t)u * rows;
                if (ok[u]) {
                    v[u] = __builtin_nontemporal_load(reinterpret_cast<const floatx4 *>(r + n * D) + c4);
                    a[u] = *(reinterpret_cast<const floatx4 *>(Cm + (size_t)cm[u] * D) + c4);
                    b[u] = *(reinterpret_cast<const floatx4 *>(Cj + (size_t)cj[u] * D) + c4);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t n = n0 + (int64_t)u * rows;
                if (ok[u]) {
                    floatx4 w = v[u] - a[u];
                    err += (double)w.x * w.x + (double)w.y * w.y + (double)w.z * w.z + (double)w.w * w.w;
                    w = w + b[u];
                    __builtin_nontemporal_store(w, reinterpret_cast<floatx4 *>(r + n * D) + c4);
                }
            }
        }
    }
    const double e = block_sum(err, red);
    if (threadIdx.x == 0) part_err[blockIdx.x] = e;
    const double c = block_sum((double)chg, red);
    if (threadIdx.x == 0) part_chg[blockIdx.x] = (long long)c;
}

// r <- X (first step of the greedy encoder): four float4 per thread in flight.
__global__ __launch_bounds__(kFlatThreads) void k_copy(
    floatx4 *__restrict__ dst, const floatx4 *__restrict__ src, int64_t n4)
{
    constexpr int U = 4;
    const int64_t stride = (int64_t)gridDim.x * kFlatThreads;
    for (int64_t i = (int64_t)blockIdx.x * kFlatThreads + threadIdx.x; i < n4; i += U * stride) {
        floatx4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (i + u * stride < n4) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (i + u * stride < n4) __builtin_nontemporal_store(v[u], dst + i + u * stride);
    }
}

// r <- float(X) for descriptors stored as bytes (online chunks): 16 bytes in, 64 bytes out per thread, over the
// flat array of `total` bytes (src 16-byte aligned); the last total % 16 bytes go one per thread.
__global__ __launch_bounds__(kFlatThreads) void k_convert_u8(
    float *__restrict__ dst, const uint8_t *__restrict__ src, int64_t total)
{
    typedef unsigned uintx4 __attribute__((ext_vector_type(4)));
    const int64_t n16 = total >> 4;
    if (blockIdx.x == 0 && 16 * n16 + threadIdx.x < total) dst[16 * n16 + threadIdx.x] = (float)src[16 * n16 + threadIdx.x];
    for (int64_t i = (int64_t)blockIdx.x * kFlatThreads + threadIdx.x; i < n16;
         i += (int64_t)gridDim.x * kFlatThreads) {
        const uintx4 w = __builtin_nontemporal_load(reinterpret_cast<const uintx4 *>(src) + i);
        floatx4 *o = reinterpret_cast<floatx4 *>(dst) + 4 * i;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const unsigned u = w[j];
            floatx4 f = {(float)(u & 255u), (float)((u >> 8) & 255u), (float)((u >> 16) & 255u), (float)(u >> 24)};
            __builtin_nontemporal_store(f, o + j);
        }
    }
}

// dst[n][m] = src[n][m] for one column m of the code matrix.
__global__ __launch_bounds__(kFlatThreads) void k_copy_column(
    uint8_t *__restrict__ dst, const uint8_t *__restrict__ src, int64_t N, int M, int m)
{
    for (int64_t n = (int64_t)blockIdx.x * kFlatThreads + threadIdx.x; n < N; n += (int64_t)gridDim.x * kFlatThreads)
        dst[n * M + m] = src[n * M + m];
}

// Partial sums of ||e_x||^2 (Eq. 1, first line), fp64 accumulation, four loads in flight.
__global__ __launch_bounds__(kFlatThreads) void k_sqnorm(
    const floatx4 *__restrict__ r, int64_t n4, double *__restrict__ part_err)
{
    __shared__ double red[kFlatThreads / kWave];
    constexpr int U = 4;
    const int64_t stride = (int64_t)gridDim.x * kFlatThreads;
    double err = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * kFlatThreads + threadIdx.x; i < n4; i += U * stride) {
        floatx4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            v[u] = (floatx4){0.f, 0.f, 0.f, 0.f};
            if (i + u * stride < n4) v[u] = __builtin_nontemporal_load(r + i + u * stride);
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            err += (double)v[u].x * v[u].x + (double)v[u].y * v[u].y + (double)v[u].z * v[u].z + (double)v[u].w * v[u].w;
    }
    const double e = block_sum(err, red);
    if (threadIdx.x == 0) part_err[blockIdx.x] = e;
}

// dmin_n = ||xp_n - C_m[codes[n][m]]||^2 in the direct form, one wave-row-group per row.
__global__ __launch_bounds__(kFlatThreads) void k_dist_to_code(
    const float *__restrict__ xp, const uint8_t *__restrict__ codes, const float *__restrict__ Cm,
    int64_t N, int D, int M, int m, float *__restrict__ dmin)
{
    const int lane = lane_id();
    const int wpb = kFlatThreads / kWave;
    for (int64_t n = (int64_t)blockIdx.x * wpb + (threadIdx.x >> 6); n < N; n += (int64_t)gridDim.x * wpb) {
        const float *x = xp + n * D;
        const float *c = Cm + (size_t)codes[n * M + m] * D;
        double s = 0.0;
        for (int d = lane; d < D; d += kWave) {
            const double t = (double)x[d] - (double)c[d];
            s += t * t;
        }
        s = wave_sum(s);
        if (lane == 0) dmin[n] = (float)s;
    }
}

// Device-side record of one stage's by-products; copied to the host only when asked for.
struct StageRecord {
    double sum_before;       // sum ||e_x||^2 at entry
    double sum_after;        // sum ||e_x||^2 at exit
    long long changed;
    long long refined;
    int empty;
    int pad;
};

// Final, fixed-order reduction of the per-block partials into a StageRecord (one block).
constexpr int kFinishThreads = 1024;
__global__ __launch_bounds__(kFinishThreads) void k_finish_stage(
    const double *__restrict__ part_before, const double *__restrict__ part_after,
    const long long *__restrict__ part_chg, int nparts,
    const int *__restrict__ nk, int K, const unsigned *__restrict__ refine_count,
    StageRecord *__restrict__ rec)
{
    __shared__ double red[kFinishThreads / kWave];
    double a = 0.0, b = 0.0, c = 0.0, e = 0.0;
    for (int i = threadIdx.x; i < nparts; i += kFinishThreads) {
        if (part_before) a += part_before[i];
        if (part_after) b += part_after[i];
        if (part_chg) c += (double)part_chg[i];
    }
    if (nk)
        for (int k = threadIdx.x; k < K; k += kFinishThreads) e += (nk[k] == 0);
    a = block_sum(a, red);
    b = block_sum(b, red);
    c = block_sum(c, red);
    e = block_sum(e, red);
    if (threadIdx.x == 0) {
        if (part_before) rec->sum_before = a;
        if (part_after) rec->sum_after = b;
        rec->changed = (long long)c;
        rec->empty = (int)e;
        rec->refined = refine_count ? (long long)*refine_count : 0;
        rec->pad = 0;
    }
}

// *out = (sum of the block partials) / N, the partials added in the order k_finish_stage adds them (N == 0: 0).
__global__ __launch_bounds__(kFinishThreads) void k_finish_mean(
    const double *__restrict__ part, int nparts, int64_t N, double *__restrict__ out)
{
    __shared__ double red[kFinishThreads / kWave];
    double b = 0.0;
    for (int i = threadIdx.x; i < nparts; i += kFinishThreads) b += part[i];
    b = block_sum(b, red);
    if (threadIdx.x == 0) *out = N > 0 ? b / (double)N : 0.0;
}

}  // namespace hclae
