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
// Column sums of x in fp64: part[blockIdx.x][d] over a contiguous range of rows.
__global__ __launch_bounds__(256) void k_colsum(
    const float *__restrict__ x, int64_t N, int D, int64_t rows_per_block, double *__restrict__ part)
{
    const int64_t r0 = (int64_t)blockIdx.x * rows_per_block;
    const int64_t r1 = (r0 + rows_per_block < N) ? r0 + rows_per_block : N;
    for (int d = threadIdx.x; d < D; d += 256) {
        double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
        int64_t n = r0;
        for (; n + 3 < r1; n += 4) {
            s0 += (double)x[n * D + d];
            s1 += (double)x[(n + 1) * D + d];
            s2 += (double)x[(n + 2) * D + d];
            s3 += (double)x[(n + 3) * D + d];
        }
        for (; n < r1; ++n) s0 += (double)x[n * D + d];
        part[(size_t)blockIdx.x * D + d] = (s0 + s1) + (s2 + s3);
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
    constexpr int U = 8;                                            // row pairs in flight
    constexpr int kFlush = 256;                                     // rows summed in fp32 before moving to fp64
    for (int64_t n = r0; n < r1; n += 2 * U) {
        if (n > r0 && ((n - r0) % kFlush) == 0) {
            // the matrix cores' fp32 accumulation error grows with the number of terms: keep runs short
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                sum0[v] += (double)acc0[v]; sum1[v] += (double)acc1[v];
                acc0[v] = 0.f; acc1[v] = 0.f;
            }
        }
        float a[U], b0[U], b1[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t row = n + 2 * u + h;
            const bool ok = row < r1;
            const float *p = x + row * D;
            a[u] = (ok && ai) ? p[i0 + c] - ma : 0.f;
            b0[u] = (ok && bj0) ? p[j0 + c] - mb0 : 0.f;
            b1[u] = (ok && bj1) ? p[j0 + 32 + c] - mb1 : 0.f;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u], b0[u], acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u], b1[u], acc1, 0, 0, 0);
        }
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
        double g = 0.0;
        for (int b = 0; b < ngram; ++b) g += grampart[(size_t)b * D * D + e];
        cov[e] = g / (double)N - (mean[i] - (double)mean32[i]) * (mean[j] - (double)mean32[j]);
    }
}

}  // namespace hclae
