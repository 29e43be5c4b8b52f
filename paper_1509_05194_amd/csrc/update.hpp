// Centroid half of the k-means that cools a dictionary (Sec. 3.1/3.2): c_m(k) <- mean of the
// x' assigned to k; an empty cluster keeps its codeword.
//
// HBM-bound segmented sum without floating-point atomics.  Every block owns a contiguous range
// of vectors and a window of 128 dims, with one K x 128 accumulator in LDS.  Wave w of the block
// owns the codewords k with k % 8 == w: it scans the codes of the range, fetches only the rows
// assigned to its codewords (one whole 512-byte row per load) and adds them to the LDS
// accumulator with a plain read-add-write.  No two waves ever touch the same accumulator row and
// a wave adds its rows in ascending vector order, so the sums are independent of timing: two
// runs give identical bits.  Block partials go to scratch; a second kernel merges them in
// fp64 in block order, divides, and refreshes the codeword norms.
#pragma once
#include "common.hpp"

namespace hclae {

constexpr int kUpdThreads = 512;
constexpr int kUpdWaves = kUpdThreads / kWave;      // 8 owners of codeword classes k % 8
constexpr int kUpdWindow = 128;                     // dims per block: two per lane
constexpr int kUpdDepth = 8;                        // row loads a wave keeps in flight

// grid: (vector ranges, D windows).  partial: float [gridDim.x][K][D]; pcount: int [gridDim.x][K].
__global__ __launch_bounds__(kUpdThreads) void k_accumulate(
    const float *__restrict__ xp, const uint8_t *__restrict__ codes,
    int64_t N, int D, int K, int M, int m, int64_t rows_per_block,
    float *__restrict__ partial, int *__restrict__ pcount)
{
    extern __shared__ float4 smem4[];
    float *acc = reinterpret_cast<float *>(smem4);                   // [K][128]
    int *cnt = reinterpret_cast<int *>(acc + K * kUpdWindow);        // [K]
    const int lane = lane_id();
    const int wave = threadIdx.x >> 6;
    const int d0 = blockIdx.y * kUpdWindow + 2 * lane;               // this lane's two dims
    const bool live = d0 < D;                                        // D % 4 == 0: both or neither

    for (int e = threadIdx.x; e < K * kUpdWindow + K; e += kUpdThreads) acc[e] = 0.f;   // cnt too (bit pattern 0)
    __syncthreads();

    float2 *mine = reinterpret_cast<float2 *>(acc) + lane;
    const int64_t row0 = (int64_t)blockIdx.x * rows_per_block;
    int64_t row1 = row0 + rows_per_block;
    if (row1 > N) row1 = N;
    for (int64_t base = row0; base < row1; base += kWave) {
        const int64_t n = base + lane;
        const int code = (n < row1) ? (int)codes[n * M + m] : -1;
        unsigned long long todo = __ballot(code >= 0 && (code & (kUpdWaves - 1)) == wave);
        while (todo) {
            float2 v[kUpdDepth];
            int c[kUpdDepth];
#pragma unroll
            for (int u = 0; u < kUpdDepth; ++u) {
                c[u] = -1;
                if (todo) {
                    const int bit = __builtin_ctzll(todo);
                    todo &= todo - 1;
                    c[u] = __builtin_amdgcn_readlane(code, bit);
                    v[u] = live ? *reinterpret_cast<const float2 *>(xp + (base + bit) * D + d0) : make_float2(0.f, 0.f);
                }
            }
#pragma unroll
            for (int u = 0; u < kUpdDepth; ++u) {
                if (c[u] >= 0) {
                    float2 *a = mine + c[u] * (kUpdWindow / 2);
                    float2 t = *a;
                    t.x += v[u].x;
                    t.y += v[u].y;
                    *a = t;
                    if (lane == 0) cnt[c[u]] += 1;
                }
            }
        }
    }
    __syncthreads();

    // partial[blockIdx.x][k][window dims]
    float *out = partial + (size_t)blockIdx.x * K * D;
    const int wd = min(kUpdWindow, D - blockIdx.y * kUpdWindow);     // live dims of this window
    for (int e = threadIdx.x; e < K * kUpdWindow; e += kUpdThreads) {
        const int k = e / kUpdWindow;
        const int d = e - k * kUpdWindow;
        if (d < wd) out[(size_t)k * D + blockIdx.y * kUpdWindow + d] = acc[e];
    }
    if (blockIdx.y == 0)
        for (int k = threadIdx.x; k < K; k += kUpdThreads) pcount[blockIdx.x * K + k] = cnt[k];
}

// One block per codeword k: n_k = sum_b pcount[b][k];  C_m[k][d] = (sum_b partial[b][k][d]) / n_k,
// summed in fp64 in a fixed order (8 groups of consecutive blocks, each in ascending b, then
// the groups in ascending order); untouched when n_k == 0.  Then hneg[k] = -||c_k||^2/2 for the
// next assignment, nk[k] = n_k, and the re-check counter is reset.
constexpr int kMergeGroups = 8;
__global__ __launch_bounds__(256) void k_merge(
    const float *__restrict__ partial, const int *__restrict__ pcount, int nblk,
    int K, int D, float *__restrict__ Cm, float *__restrict__ hneg, int *__restrict__ nk,
    int *__restrict__ counts_out, unsigned *__restrict__ refine_count)
{
    __shared__ double red[256 / kWave];
    __shared__ double comb[kMergeGroups][32][4];
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
    const int g = threadIdx.x >> 5;                    // block group
    const int l = threadIdx.x & 31;                    // float4 column within a pass
    const int d4 = D >> 2;
    const int per = (nblk + kMergeGroups - 1) / kMergeGroups;
    const int b0 = g * per, b1 = min(nblk, b0 + per);
    double sq = 0.0;
    for (int j0 = 0; j0 < d4; j0 += 32) {
        const int j = j0 + l;
        double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
        if (n > 0 && j < d4) {
            for (int b = b0; b < b1; ++b) {
                const float4 v = *reinterpret_cast<const float4 *>(partial + ((size_t)b * K + k) * D + 4 * j);
                s0 += (double)v.x; s1 += (double)v.y; s2 += (double)v.z; s3 += (double)v.w;
            }
        }
        comb[g][l][0] = s0; comb[g][l][1] = s1; comb[g][l][2] = s2; comb[g][l][3] = s3;
        __syncthreads();
        if (g == 0 && j < d4) {
            float4 c;
            float4 *dst = reinterpret_cast<float4 *>(Cm + (size_t)k * D + 4 * j);
            if (n > 0) {
                double t0 = 0.0, t1 = 0.0, t2 = 0.0, t3 = 0.0;
#pragma unroll
                for (int q = 0; q < kMergeGroups; ++q) {
                    t0 += comb[q][l][0]; t1 += comb[q][l][1]; t2 += comb[q][l][2]; t3 += comb[q][l][3];
                }
                const double inv = (double)n;
                c = make_float4((float)(t0 / inv), (float)(t1 / inv), (float)(t2 / inv), (float)(t3 / inv));
                *dst = c;
            } else {
                c = *dst;
            }
            sq += (double)c.x * c.x + (double)c.y * c.y + (double)c.z * c.z + (double)c.w * c.w;
        }
        __syncthreads();
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
