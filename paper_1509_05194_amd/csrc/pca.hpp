// Improved k-means for high-dimensional residues (Sec. 3.2): the pieces around the Lloyd kernels --
// second moments of {x'} for its PCA, and the projection x^r = R x' / C' = R C_m / C_m = R^T C'.
// Both are dense contractions and run on the fp32 matrix cores (v_mfma_f32_32x32x2_f32).
#pragma once
#include "assign.hpp"

namespace hclae {

// ---------------------------------------------------------------------------------------------
// out[n][o] = sum_j x[n][j] * R[o][j]  for o in [o0, o0 + 256), i.e. y = R x row by row.
// Same structure as k_assign_chunked: a block owns tiles of 8 x 32 vectors, walks the D axis in 64-dim
// chunks restaging that slice of (up to 256 rows of) R in LDS in MFMA operand order, keeps the 256
// outputs of a vector in accumulators, and stores them instead of taking an argmax.
// grid: (vector tiles, groups of 256 outputs).
__global__ __launch_bounds__(kAssignThreads) void k_project(
    const float *__restrict__ x, const float *__restrict__ R, int64_t N, int D, float *__restrict__ out)
{
    constexpr int KB = 8, S = 8;
    extern __shared__ float4 smem4[];
    float4 *lds_c = smem4;
    const int lane = lane_id();
    const int wave = threadIdx.x >> 6;
    const int h = lane >> 5;
    const int r = lane & 31;
    const int o0 = blockIdx.y * 32 * KB;
    const int rows = min(32 * KB, D - o0);                          // live rows of R in this group
    const float *Rg = R + (size_t)o0 * D;
    const int NC = (D + kChunkD - 1) / kChunkD;
    const int64_t nbt = (N + kTileVec * kAssignWaves - 1) / (kTileVec * kAssignWaves);
    for (int64_t bt = blockIdx.x; bt < nbt; bt += gridDim.x) {
        const int64_t n_raw = (bt * kAssignWaves + wave) * kTileVec + r;
        const int64_t n = n_raw < N ? n_raw : N - 1;
        const float *xrow = x + n * D;
        floatx16 acc[KB];
#pragma unroll
        for (int b = 0; b < KB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[b][v] = 0.f;
        float4 xc[8];
        float unused_sq = 0.f, unused_max = 0.f;
        for (int q = 0; q < NC; ++q) {
            load_x_chunk(xc, xrow, q, h, D);
            __syncthreads();
            for (int e = threadIdx.x; e < KB * S * kWave; e += blockDim.x) {
                const int l = e & 63;
                const int bs = e >> 6;
                const int s = bs & 7;
                const int b = bs >> 3;
                lds_c[e] = load_row_piece(Rg, 32 * b + (l & 31), kChunkD * q + 8 * s + 4 * (l >> 5), rows, D, D);
            }
            __syncthreads();
            mfma_chunk<KB>(acc, xc, lds_c, 0, S, lane, unused_sq, unused_max);
        }
        if (n_raw < N) {
            float *orow = out + n_raw * D + o0;
#pragma unroll
            for (int b = 0; b < KB; ++b)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int o = 32 * b + 8 * g + 4 * h;           // acc[b][4g..4g+3] are outputs o..o+3
                    if (o < rows)
                        *reinterpret_cast<float4 *>(orow + o) =
                            make_float4(acc[b][4 * g], acc[b][4 * g + 1], acc[b][4 * g + 2], acc[b][4 * g + 3]);
                }
        }
    }
}

// dst = src^T for a D x D matrix.
__global__ __launch_bounds__(256) void k_transpose(const float *__restrict__ src, int D, float *__restrict__ dst)
{
    for (int e = blockIdx.x * 256 + threadIdx.x; e < D * D; e += gridDim.x * 256) {
        const int i = e / D, j = e - i * D;
        dst[(size_t)j * D + i] = src[e];
    }
}

// ---------------------------------------------------------------------------------------------
// Column sums of x in fp64: part[blockIdx.x][d] over a contiguous range of rows.  A block is
// (1 << lcw) float4-column threads by (256 >> lcw) row groups; four rows per thread in flight; the row
// groups are combined through LDS in ascending order.
__global__ __launch_bounds__(256) void k_colsum(
    const float *__restrict__ x, int64_t N, int D, int64_t rows_per_block, int lcw, double *__restrict__ part)
{
    __shared__ double comb[256][4];
    const int cw = 1 << lcw, groups = 256 >> lcw;
    const int tx = threadIdx.x & (cw - 1), ty = threadIdx.x >> lcw;
    const int d4 = D >> 2;
    const int64_t r0 = (int64_t)blockIdx.x * rows_per_block;
    const int64_t r1 = (r0 + rows_per_block < N) ? r0 + rows_per_block : N;
    for (int c0 = 0; c0 < d4; c0 += cw) {
        const int c4 = c0 + tx;
        double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
        if (c4 < d4) {
            for (int64_t n = r0 + ty; n < r1; n += 4 * groups) {
                float4 v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int64_t row = n + (int64_t)u * groups;
                    v[u] = (row < r1) ? *(reinterpret_cast<const float4 *>(x + row * D) + c4) : make_float4(0.f, 0.f, 0.f, 0.f);
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) { s0 += (double)v[u].x; s1 += (double)v[u].y; s2 += (double)v[u].z; s3 += (double)v[u].w; }
            }
        }
        comb[threadIdx.x][0] = s0; comb[threadIdx.x][1] = s1; comb[threadIdx.x][2] = s2; comb[threadIdx.x][3] = s3;
        __syncthreads();
        if (ty == 0 && c4 < d4) {
            double t0 = 0.0, t1 = 0.0, t2 = 0.0, t3 = 0.0;
            for (int g = 0; g < groups; ++g) {
                const double *q = comb[g * cw + tx];
                t0 += q[0]; t1 += q[1]; t2 += q[2]; t3 += q[3];
            }
            double *o = part + (size_t)blockIdx.x * D + 4 * c4;
            o[0] = t0; o[1] = t1; o[2] = t2; o[3] = t3;
        }
        __syncthreads();
    }
}

// One 128 x 128 tile of the Gram matrix sum_n x_n x_n^T over a contiguous range of rows, fp32 MFMA.
// The contraction index is the row n: A = x[n][i0..], B = x[n][j0..].  Wave w owns 32 rows of the tile
// (i-block w & 3) and two 32-column blocks (2 (w >> 2), +1).  fp32 accumulation runs over 256 rows at
// a time and is then added to fp64 sums; the merge across ranges is in fp64 as well.
// grid: (row ranges, tiles along i, tiles along j); part: double [range][D][D].
__global__ __launch_bounds__(512) void k_gram_tile(
    const float *__restrict__ x, const float *__restrict__ mean32, int64_t N, int D, int64_t rows_per_block,
    double *__restrict__ part)
{
    const int lane = lane_id();
    const int wave = threadIdx.x >> 6;
    const int h = lane >> 5, c = lane & 31;
    const int i0 = blockIdx.y * 128 + 32 * (wave & 3);
    const int j0 = blockIdx.z * 128 + 64 * (wave >> 2);
    const int64_t r0 = (int64_t)blockIdx.x * rows_per_block;
    const int64_t r1 = (r0 + rows_per_block < N) ? r0 + rows_per_block : N;
    const bool ai = (i0 + c) < D, bj0 = (j0 + c) < D, bj1 = (j0 + 32 + c) < D;
    // the data are centred on the (fp32-rounded) mean before the products: no cancellation later
    const float ma = ai ? mean32[i0 + c] : 0.f, mb0 = bj0 ? mean32[j0 + c] : 0.f, mb1 = bj1 ? mean32[j0 + 32 + c] : 0.f;
    floatx16 acc0, acc1;
    double sum0[16], sum1[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) { acc0[v] = 0.f; acc1[v] = 0.f; sum0[v] = 0.0; sum1[v] = 0.0; }
    constexpr int U = 8;                                            // row pairs per batch
    constexpr int kFlush = 256 / (2 * U);                           // batches summed in fp32 before moving to fp64
    // Loads are unconditional (row and column clamped into range) and masked afterwards: guarded loads
    // would be serialised by the branches around them.
    const int ca = ai ? i0 + c : 0, cb0 = bj0 ? j0 + c : 0, cb1 = bj1 ? j0 + 32 + c : 0;
    const float *xa = x + ca, *xb0 = x + cb0, *xb1 = x + cb1;
    const float fa = ai ? 1.f : 0.f, fb0 = bj0 ? 1.f : 0.f, fb1 = bj1 ? 1.f : 0.f;
    auto fetch = [&](int64_t n, float (&a)[U], float (&b0)[U], float (&b1)[U]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t row = n + 2 * u + h;
            const bool ok = row < r1;
            const int64_t off = (ok ? row : r1 - 1) * D;
            const float va = xa[off], vb0 = xb0[off], vb1 = xb1[off];
            const float live = ok ? 1.f : 0.f;                      // a product keeps the loads unconditional
            a[u] = (va - ma) * (live * fa);
            b0[u] = (vb0 - mb0) * (live * fb0);
            b1[u] = (vb1 - mb1) * (live * fb1);
        }
    };
    auto contract = [&](const float (&a)[U], const float (&b0)[U], const float (&b1)[U]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u], b0[u], acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u], b1[u], acc1, 0, 0, 0);
        }
    };
    auto flush = [&]() {
        // the matrix cores' fp32 accumulation error grows with the number of terms: keep runs short
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            sum0[v] += (double)acc0[v]; sum1[v] += (double)acc1[v];
            acc0[v] = 0.f; acc1[v] = 0.f;
        }
    };
    // two register sets: the next batch of rows is in flight while the current one is contracted
    float a0[U], p0[U], q0[U], a1[U], p1[U], q1[U];
    fetch(r0, a0, p0, q0);
    int batch = 0;
    for (int64_t n = r0; n < r1; n += 4 * U) {
        fetch(n + 2 * U, a1, p1, q1);
        contract(a0, p0, q0);
        if (++batch % kFlush == 0) flush();
        fetch(n + 4 * U, a0, p0, q0);
        contract(a1, p1, q1);
        if (++batch % kFlush == 0) flush();
    }
    double *out = part + (size_t)blockIdx.x * D * D;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int i = i0 + 8 * (v >> 2) + 4 * h + (v & 3);
        if (i < D) {
            if (j0 + c < D) out[(size_t)i * D + j0 + c] = sum0[v] + (double)acc0[v];
            if (j0 + 32 + c < D) out[(size_t)i * D + j0 + 32 + c] = sum1[v] + (double)acc1[v];
        }
    }
}

// mean[d] = (sum of column partials) / N in fp64 (ascending range order) and its fp32 rounding.
__global__ __launch_bounds__(256) void k_mean_finish(
    const double *__restrict__ colpart, int ncol, int64_t N, int D, double *__restrict__ mean, float *__restrict__ mean32)
{
    for (int d = blockIdx.x * 256 + threadIdx.x; d < D; d += gridDim.x * 256) {
        double s = 0.0;
        for (int b = 0; b < ncol; ++b) s += colpart[(size_t)b * D + d];
        s /= (double)N;
        mean[d] = s;
        mean32[d] = (float)s;
    }
}

// cov[i][j] = (sum of the centred Gram partials)[i][j] / N - (mean - mean32)_i (mean - mean32)_j, in fp64,
// partials added in ascending range order.
__global__ __launch_bounds__(256) void k_cov_finish(
    const double *__restrict__ grampart, int ngram, int64_t N, int D,
    const double *__restrict__ mean, const float *__restrict__ mean32, double *__restrict__ cov)
{
    for (int e = blockIdx.x * 256 + threadIdx.x; e < D * D; e += gridDim.x * 256) {
        const int i = e / D, j = e - i * D;
        double g0 = 0.0, g1 = 0.0, g2 = 0.0, g3 = 0.0;
        int b = 0;
        for (; b + 3 < ngram; b += 4) {
            g0 += grampart[(size_t)b * D * D + e];
            g1 += grampart[(size_t)(b + 1) * D * D + e];
            g2 += grampart[(size_t)(b + 2) * D * D + e];
            g3 += grampart[(size_t)(b + 3) * D * D + e];
        }
        for (; b < ngram; ++b) g0 += grampart[(size_t)b * D * D + e];
        const double g = (g0 + g1) + (g2 + g3);
        cov[e] = g / (double)N - (mean[i] - (double)mean32[i]) * (mean[j] - (double)mean32[j]);
    }
}

}  // namespace hclae
