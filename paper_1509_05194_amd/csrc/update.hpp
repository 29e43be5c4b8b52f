// Centroid half of the k-means that cools a dictionary (Sec. 3.1/3.2): c_m(k) <- mean of the
// x' assigned to k; an empty cluster keeps its codeword.
//
// HBM-bound segmented sum.  Every block owns a contiguous range of vectors and a window of
// 128 dims; each of its 8 waves owns a 16-dim slice of that window and a private K x 16
// accumulator in LDS, which it alone updates with ds_add_f32 in program order -- so the sums do
// not depend on timing and two runs give identical bits.  Block partials go to scratch and a
// second kernel merges them in fp64 in block order, divides, and refreshes the codeword norms.
#pragma once
#include "common.hpp"

namespace hclae {

constexpr int kUpdThreads = 512;
constexpr int kUpdWaves = kUpdThreads / kWave;      // 8
constexpr int kUpdSlice = 16;                       // dims per wave
constexpr int kUpdWindow = kUpdWaves * kUpdSlice;   // 128 dims per block
constexpr int kUpdRows = 16;                        // rows per wave load (4 lanes x float4 per row)

// grid: (vector ranges, D windows).  partial: float [gridDim.x][K][D]; pcount: int [gridDim.x][K].
__global__ __launch_bounds__(kUpdThreads) void k_accumulate(
    const float *__restrict__ xp, const uint8_t *__restrict__ codes,
    int64_t N, int D, int K, int M, int m, int64_t rows_per_block,
    float *__restrict__ partial, int *__restrict__ pcount)
{
    extern __shared__ float4 smem4[];
    float *acc = reinterpret_cast<float *>(smem4);                   // [8 waves][K][16]
    int *cnt = reinterpret_cast<int *>(acc + kUpdWaves * K * kUpdSlice);   // [K]
    const int lane = lane_id();
    const int wave = threadIdx.x >> 6;
    const int rho = lane >> 2;                                       // row within the 16-row group
    const int dq = lane & 3;                                         // float4 within the slice
    const int d0 = blockIdx.y * kUpdWindow + wave * kUpdSlice + 4 * dq;
    const bool live = d0 < D;
    const bool counter = (blockIdx.y == 0) && (wave == 0) && (dq == 0);

    for (int e = threadIdx.x; e < kUpdWaves * K * kUpdSlice + K; e += kUpdThreads) acc[e] = 0.f;   // cnt too (bit pattern 0)
    __syncthreads();

    float *mine = acc + wave * K * kUpdSlice + 4 * dq;
    const int64_t row0 = (int64_t)blockIdx.x * rows_per_block;
    int64_t row1 = row0 + rows_per_block;
    if (row1 > N) row1 = N;
    constexpr int U = 4;                                             // row groups in flight
    for (int64_t base = row0; base < row1; base += U * kUpdRows) {
        float4 v[U];
        int code[U];
        bool ok[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t n = base + u * kUpdRows + rho;
            ok[u] = n < row1;
            code[u] = ok[u] ? codes[n * M + m] : 0;
            v[u] = (ok[u] && live) ? *reinterpret_cast<const float4 *>(xp + n * D + d0)
                                   : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (ok[u] && live) {
                float *a = mine + code[u] * kUpdSlice;
                atomicAdd(a + 0, v[u].x);
                atomicAdd(a + 1, v[u].y);
                atomicAdd(a + 2, v[u].z);
                atomicAdd(a + 3, v[u].w);
            }
            if (ok[u] && counter) atomicAdd(cnt + code[u], 1);
        }
    }
    __syncthreads();

    // partial[blockIdx.x][k][window dims]
    float *out = partial + (size_t)blockIdx.x * K * D;
    const int wd = min(kUpdWindow, D - blockIdx.y * kUpdWindow);     // live dims of this window
    for (int e = threadIdx.x; e < K * kUpdWindow; e += kUpdThreads) {
        const int k = e / kUpdWindow;
        const int d = e - k * kUpdWindow;                            // dim within window
        if (d < wd) {
            const int w = d / kUpdSlice;
            out[(size_t)k * D + blockIdx.y * kUpdWindow + d] = acc[(w * K + k) * kUpdSlice + (d - w * kUpdSlice)];
        }
    }
    if (blockIdx.y == 0)
        for (int k = threadIdx.x; k < K; k += kUpdThreads) pcount[blockIdx.x * K + k] = cnt[k];
}

// One block per codeword k: n_k = sum_b pcount[b][k];  C_m[k][d] = (sum_b partial[b][k][d]) / n_k
// with the sum over blocks in ascending b in fp64; untouched when n_k == 0.  Then
// hneg[k] = -||c_k||^2/2 for the next assignment, nk[k] = n_k, and the re-check counter is reset.
__global__ __launch_bounds__(256) void k_merge(
    const float *__restrict__ partial, const int *__restrict__ pcount, int nblk,
    int K, int D, float *__restrict__ Cm, float *__restrict__ hneg, int *__restrict__ nk,
    int *__restrict__ counts_out, unsigned *__restrict__ refine_count)
{
    __shared__ double red[256 / kWave];
    __shared__ int s_n;
    const int k = blockIdx.x;
    if (k == 0 && threadIdx.x == 0) *refine_count = 0u;
    if (threadIdx.x < kWave) {
        // integer sum: order-free
        long long c = 0;
        for (int b = threadIdx.x; b < nblk; b += kWave) c += pcount[b * K + k];
        c = wave_sum_ll(c);
        if (threadIdx.x == 0) s_n = (int)c;
    }
    __syncthreads();
    const int n = s_n;
    double sq = 0.0;
    for (int d = threadIdx.x; d < D; d += 256) {
        float c;
        if (n > 0) {
            double s = 0.0;
            for (int b = 0; b < nblk; ++b) s += (double)partial[((size_t)b * K + k) * D + d];
            c = (float)(s / (double)n);
            Cm[(size_t)k * D + d] = c;
        } else {
            c = Cm[(size_t)k * D + d];
        }
        sq += (double)c * (double)c;
    }
    sq = block_sum(sq, red);
    if (threadIdx.x == 0) {
        hneg[k] = -(float)(0.5 * sq);
        nk[k] = n;
        if (counts_out) counts_out[k] = n;
    }
}

// C_m[k] <- x'[idx[k]]: seeding of an all-zero dictionary (Sec. 3.1, learning from scratch).
__global__ __launch_bounds__(256) void k_seed(
    const float *__restrict__ xp, const int64_t *__restrict__ idx, int K, int D, float *__restrict__ Cm)
{
    const int k = blockIdx.x;
    const float *src = xp + idx[k] * (int64_t)D;
    for (int d = threadIdx.x; d < D; d += 256) Cm[(size_t)k * D + d] = src[d];
}

}  // namespace hclae
