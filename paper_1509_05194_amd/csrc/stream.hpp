// Streaming passes of a DA stage (Sec. 3.1): heat x' = e_x + c_m(i_m(x)), the new residue
// e_x = x' - c_m(i_m(x)), and the error of Eq. 1 (first line).  All are HBM-bound: every
// thread moves one float4 per row pass, a wave covers contiguous kilobytes, the K x D
// codebook (<= 1 MB) stays in L2.
#pragma once
#include "common.hpp"

namespace hclae {

constexpr int kStreamThreads = 512;    // heat / cool / stage boundary
constexpr int kStreamUnroll = 4;       // independent rows per thread per step
constexpr int kFlatThreads = 256;      // flat float4 passes (copy, reduction, finish)

typedef float floatx4 __attribute__((ext_vector_type(4)));

// Geometry of the row passes: a block is (1 << lcw) column threads by (kStreamThreads >> lcw) rows; column thread tx
// walks float4 columns tx, tx + cw, ...
struct RowGeom {
    int lcw;        // log2 of column threads per row
    int d4;         // D / 4
};

// max |x'| of a block merged into one of kAmaxSlots words (bits of a non-negative float: integer max is float max):
// one atomic per block, spread over the words so that thousands of blocks do not queue on one address; the reader
// (k_codeword_norms) takes the largest word and clears them.  scratch: kStreamThreads / kWave floats of LDS.
constexpr int kAmaxSlots = 64;
__device__ __forceinline__ void block_absmax(float amax, float *scratch, unsigned *__restrict__ slots)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) amax = fmaxf(amax, __shfl_xor(amax, o, kWave));
    __syncthreads();                                                // the scratch may still be read by a block_sum
    if (lane_id() == 0) scratch[threadIdx.x >> 6] = amax;
    __syncthreads();
    if (threadIdx.x == 0) {
        float mx = scratch[0];
        for (int w = 1; w < (int)(blockDim.x >> 6); ++w) mx = fmaxf(mx, scratch[w]);
        atomicMax(slots + (blockIdx.x & (kAmaxSlots - 1)), __float_as_uint(mx));
    }
}

// The in-place row passes of a stage (Sec. 3.1), one kernel body:
//   MODE +1  heat       r_n += C_m[i_m(n)]; by-products: column m of the codes saved (old_codes), sum ||e_x||^2 of the input
//   MODE -1  new residue r_n -= C_m[i_m(n)]; by-products: sum ||e_x||^2 of the output, codes that differ from old_codes
//   MODE  0  stage boundary inside a sweep, one pass instead of two: e_x = x' - c_m(i_m) (end of stage m) followed at
//            once by x'' = e_x + c_j(i_j) (heat of the next stage j).  The intermediate e_x is rounded to fp32 exactly
//            as if it had been stored and reloaded, so the result equals the two passes bit for bit.  By-products:
//            sum ||e_x||^2 (error after stage m = error before stage j), codes of stage m changed since its entry,
//            and the code column of stage j saved for its own change count.
// part_err[blockIdx.x], part_chg[blockIdx.x] receive this block's partial sums (fixed order); STATS false: no by-products.
//
// A thread works on kStreamUnroll rows at a time, one float4 column of each, in steps (row group, column chunk).
// The row loads of the NEXT step (and the code bytes of its rows) are issued before the codeword rows of the current
// step are gathered from L2: the HBM loads are then in flight all the time instead of half of it.  Measured on one
// MI355X at N = 1M, D = 128: stage boundary 213 us -> 176 us (5.9 TB/s; a device-to-device hipMemcpy of the same
// bytes takes 193 us); the launch shape (512 threads, 32 blocks per CU, about two steps per block) is the best of
// a sweep of shapes.  All three modes share the geometry, so a thread adds the same squares in the same order in
// the stage boundary as in the separate new-residue pass: the error sums are the same bits.
// DT: the row length as a compile-time constant (with the geometry row_geom gives it), or 0: taken from D and g.
// AMAX (MODE +1 and 0): max |x'| over everything written is merged into absmax_slot[0..kAmaxSlots) (block_absmax), for
// a stage whose first assignment does not read every row and so cannot provide it.
template <int MODE, bool STATS, int DT = 0, bool AMAX = false>
__global__ __launch_bounds__(kStreamThreads) void k_row_pass(
    float *__restrict__ r, const uint8_t *__restrict__ codes, const float *__restrict__ Cm, const float *__restrict__ Cj,
    int64_t N, int D_rt, int M, int m, int j_stage, RowGeom g_rt,
    uint8_t *__restrict__ old_codes, double *__restrict__ part_err, long long *__restrict__ part_chg,
    unsigned *__restrict__ absmax_slot = nullptr)
{
    __shared__ double red[kStreamThreads / kWave];
    constexpr int U = kStreamUnroll;
    const int D = DT ? DT : D_rt;
    RowGeom g = g_rt;
    if (DT) {
        g.d4 = DT / 4;
        g.lcw = DT >= 256 ? 6 : DT >= 128 ? 5 : DT >= 64 ? 4 : DT >= 32 ? 3 : DT >= 16 ? 2 : DT >= 8 ? 1 : 0;
    }
    const int cw = 1 << g.lcw;
    const int tx = threadIdx.x & (cw - 1);
    const int ty = threadIdx.x >> g.lcw;
    const int rows = kStreamThreads >> g.lcw;
    const int nchunks = (g.d4 + cw - 1) >> g.lcw;
    const int64_t stride = (int64_t)gridDim.x * rows * U;
    double err = 0.0;
    long long chg = 0;
    float amax = 0.f;

    // rows n0 + u * rows of a group; the loads of a step take rows clamped into range (never used beyond N)
    auto load_codes = [&](int64_t n0, int (&a)[U], int (&b)[U]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t n = n0 + (int64_t)u * rows;
            const int64_t nn = n < N ? n : N - 1;
            a[u] = codes[nn * M + m];
            if (MODE == 0) b[u] = codes[nn * M + j_stage];
        }
    };
    auto load_rows = [&](int64_t n0, int c4, floatx4 (&v)[U]) {
        const int cc = c4 < g.d4 ? c4 : g.d4 - 1;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t n = n0 + (int64_t)u * rows;
            const int64_t nn = n < N ? n : N - 1;
            v[u] = __builtin_nontemporal_load(reinterpret_cast<const floatx4 *>(r + nn * D) + cc);
        }
    };

    int64_t n0 = (int64_t)blockIdx.x * rows * U + ty;
    int chunk = 0;
    floatx4 v[U];
    int cm[U], cj[U];
    if (n0 < N) {
        load_codes(n0, cm, cj);
        load_rows(n0, tx, v);
    }
    while (n0 < N) {
        // the step after this one
        int chunk_next = chunk + 1;
        int64_t n0_next = n0;
        if (chunk_next == nchunks) { chunk_next = 0; n0_next = n0 + stride; }
        floatx4 vn[U];
        int cmn[U], cjn[U];
        if (n0_next < N) {
            if (chunk_next == 0) load_codes(n0_next, cmn, cjn);
            load_rows(n0_next, chunk_next * cw + tx, vn);
        }
        const int c4 = chunk * cw + tx;
        const bool live = c4 < g.d4;
        const int cc = live ? c4 : g.d4 - 1;
        floatx4 a[U], b[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            a[u] = *(reinterpret_cast<const floatx4 *>(Cm + (size_t)cm[u] * D) + cc);
            if (MODE == 0) b[u] = *(reinterpret_cast<const floatx4 *>(Cj + (size_t)cj[u] * D) + cc);
        }
        if (STATS && tx == 0 && chunk == 0) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t n = n0 + (int64_t)u * rows;
                if (n < N) {
                    if (MODE > 0) old_codes[n] = (uint8_t)cm[u];
                    if (MODE < 0) chg += (old_codes[n] != (uint8_t)cm[u]);
                    if (MODE == 0) {
                        chg += (old_codes[n] != (uint8_t)cm[u]);
                        old_codes[n] = (uint8_t)cj[u];
                    }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t n = n0 + (int64_t)u * rows;
            if (live && n < N) {
                floatx4 w = v[u];
                if (STATS && MODE > 0)
                    err += (double)w.x * w.x + (double)w.y * w.y + (double)w.z * w.z + (double)w.w * w.w;
                if (MODE > 0) w = w + a[u];
                else w = w - a[u];
                if (STATS && MODE <= 0)
                    err += (double)w.x * w.x + (double)w.y * w.y + (double)w.z * w.z + (double)w.w * w.w;
                if (MODE == 0) w = w + b[u];
                if (AMAX && MODE >= 0) {
                    amax = fmaxf(fmaxf(amax, fabsf(w.x)), fabsf(w.y));
                    amax = fmaxf(fmaxf(amax, fabsf(w.z)), fabsf(w.w));
                }
                __builtin_nontemporal_store(w, reinterpret_cast<floatx4 *>(r + n * D) + c4);
            }
        }
        if (chunk_next == 0) {
#pragma unroll
            for (int u = 0; u < U; ++u) { cm[u] = cmn[u]; cj[u] = cjn[u]; }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = vn[u];
        chunk = chunk_next;
        n0 = n0_next;
    }
    if (STATS) {
        const double e = block_sum(err, red);
        if (threadIdx.x == 0) part_err[blockIdx.x] = e;
        if (MODE <= 0) {
            // integer sum: any order gives the same value
            const double c = block_sum((double)chg, red);
            if (threadIdx.x == 0) part_chg[blockIdx.x] = (long long)c;
        }
    }
    if (AMAX && MODE >= 0) block_absmax(amax, reinterpret_cast<float *>(red), absmax_slot);
}

// The same passes for long rows (D >= kWideMinD): a wave owns whole rows.  Lane l takes float4 columns l, l + 64,
// l + 128, l + 192 of a group of 256 columns (one contiguous kilobyte of the row per wave-instruction, up to 4 KB of
// one row in flight), kWideRows rows per step, steps (row pair, column group) pipelined as in k_row_pass.  Measured at
// N = 1M, D = 960 (3.84 GB each way): stage boundary 1.39 ms against 1.51 ms for k_row_pass, new residue 1.36 ms
// against 1.43 ms.  Results are those of k_row_pass bit for bit (the same fp32 operations per element); the error
// sums differ in their order of additions, which is the same in all three modes here too.
constexpr int kWideMinD = 768;
constexpr int kWideRows = 2;
template <int MODE, bool STATS, bool AMAX = false>
__global__ __launch_bounds__(kStreamThreads) void k_row_pass_wide(
    float *__restrict__ r, const uint8_t *__restrict__ codes, const float *__restrict__ Cm, const float *__restrict__ Cj,
    int64_t N, int D, int M, int m, int j_stage,
    uint8_t *__restrict__ old_codes, double *__restrict__ part_err, long long *__restrict__ part_chg,
    unsigned *__restrict__ absmax_slot = nullptr)
{
    __shared__ double red[kStreamThreads / kWave];
    constexpr int U = 4, R = kWideRows;
    const int d4 = D >> 2;
    const int ngroups = (d4 + U * kWave - 1) / (U * kWave);
    const int lane = lane_id();
    const int64_t stride = (int64_t)gridDim.x * (kStreamThreads / kWave) * R;
    double err = 0.0;
    long long chg = 0;
    float amax = 0.f;

    auto load_codes = [&](int64_t n0, int (&a)[R], int (&b)[R]) {
#pragma unroll
        for (int q = 0; q < R; ++q) {
            const int64_t nn = n0 + q < N ? n0 + q : N - 1;
            a[q] = codes[nn * M + m];
            if (MODE == 0) b[q] = codes[nn * M + j_stage];
        }
    };
    auto load_rows = [&](int64_t n0, int group, floatx4 (&v)[R][U]) {
#pragma unroll
        for (int q = 0; q < R; ++q) {
            const int64_t nn = n0 + q < N ? n0 + q : N - 1;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int c = (group * U + u) * kWave + lane;
                v[q][u] = __builtin_nontemporal_load(reinterpret_cast<const floatx4 *>(r + nn * D) + (c < d4 ? c : d4 - 1));
            }
        }
    };

    int64_t n0 = ((int64_t)blockIdx.x * (kStreamThreads / kWave) + (threadIdx.x >> 6)) * R;
    int group = 0;
    floatx4 v[R][U];
    int cm[R], cj[R];
    if (n0 < N) {
        load_codes(n0, cm, cj);
        load_rows(n0, 0, v);
    }
    while (n0 < N) {
        int group_next = group + 1;
        int64_t n0_next = n0;
        if (group_next == ngroups) { group_next = 0; n0_next = n0 + stride; }
        floatx4 vn[R][U];
        int cmn[R], cjn[R];
        if (n0_next < N) {
            if (group_next == 0) load_codes(n0_next, cmn, cjn);
            load_rows(n0_next, group_next, vn);
        }
#pragma unroll
        for (int q = 0; q < R; ++q) {
            const int64_t n = n0 + q;
            floatx4 a[U], b[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int c = (group * U + u) * kWave + lane;
                const int cc = c < d4 ? c : d4 - 1;
                a[u] = *(reinterpret_cast<const floatx4 *>(Cm + (size_t)cm[q] * D) + cc);
                if (MODE == 0) b[u] = *(reinterpret_cast<const floatx4 *>(Cj + (size_t)cj[q] * D) + cc);
            }
            if (n < N) {
                if (STATS && lane == 0 && group == 0) {
                    if (MODE > 0) old_codes[n] = (uint8_t)cm[q];
                    if (MODE < 0) chg += (old_codes[n] != (uint8_t)cm[q]);
                    if (MODE == 0) {
                        chg += (old_codes[n] != (uint8_t)cm[q]);
                        old_codes[n] = (uint8_t)cj[q];
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int c = (group * U + u) * kWave + lane;
                    if (c < d4) {
                        floatx4 w = v[q][u];
                        if (STATS && MODE > 0)
                            err += (double)w.x * w.x + (double)w.y * w.y + (double)w.z * w.z + (double)w.w * w.w;
                        if (MODE > 0) w = w + a[u];
                        else w = w - a[u];
                        if (STATS && MODE <= 0)
                            err += (double)w.x * w.x + (double)w.y * w.y + (double)w.z * w.z + (double)w.w * w.w;
                        if (MODE == 0) w = w + b[u];
                        if (AMAX && MODE >= 0) {
                            amax = fmaxf(fmaxf(amax, fabsf(w.x)), fabsf(w.y));
                            amax = fmaxf(fmaxf(amax, fabsf(w.z)), fabsf(w.w));
                        }
                        __builtin_nontemporal_store(w, reinterpret_cast<floatx4 *>(r + n * D) + c);
                    }
                }
            }
        }
        if (group_next == 0) {
#pragma unroll
            for (int q = 0; q < R; ++q) { cm[q] = cmn[q]; cj[q] = cjn[q]; }
        }
#pragma unroll
        for (int q = 0; q < R; ++q)
#pragma unroll
            for (int u = 0; u < U; ++u) v[q][u] = vn[q][u];
        group = group_next;
        n0 = n0_next;
    }
    if (STATS) {
        const double e = block_sum(err, red);
        if (threadIdx.x == 0) part_err[blockIdx.x] = e;
        if (MODE <= 0) {
            const double c = block_sum((double)chg, red);
            if (threadIdx.x == 0) part_chg[blockIdx.x] = (long long)c;
        }
    }
    if (AMAX && MODE >= 0) block_absmax(amax, reinterpret_cast<float *>(red), absmax_slot);
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

// Partial sums of ||e_x||^2 (Eq. 1, first line), fp64 accumulation.  Every block reads one contiguous piece of the
// array, eight float4 per thread in flight: measured 79 us for 512 MB (6.5 TB/s) against 95 us when the blocks
// interleave their loads across the whole array.
constexpr int kSqUnroll = 8;
__host__ __device__ inline int64_t sqnorm_piece(int64_t n4, int blocks)
{
    const int64_t step = (int64_t)kSqUnroll * kFlatThreads;
    return ((n4 + blocks - 1) / blocks + step - 1) / step * step;
}
__global__ __launch_bounds__(kFlatThreads) void k_sqnorm(
    const floatx4 *__restrict__ r, int64_t n4, double *__restrict__ part_err)
{
    __shared__ double red[kFlatThreads / kWave];
    constexpr int U = kSqUnroll;
    const int64_t per = sqnorm_piece(n4, (int)gridDim.x);
    const int64_t lo = (int64_t)blockIdx.x * per;
    const int64_t hi = lo + per < n4 ? lo + per : n4;
    double err = 0.0;
    for (int64_t i = lo + threadIdx.x; i < hi; i += U * kFlatThreads) {
        floatx4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            v[u] = (floatx4){0.f, 0.f, 0.f, 0.f};
            if (i + u * kFlatThreads < hi) v[u] = __builtin_nontemporal_load(r + i + u * kFlatThreads);
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
