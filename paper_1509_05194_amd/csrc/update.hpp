// Centroid half of the k-means that cools a dictionary (Sec. 3.1/3.2): c_m(k) <- mean of the
// x' assigned to k; an empty cluster keeps its codeword.
//
// HBM-bound segmented sum without floating-point atomics.  Every block owns a contiguous range
// of vectors and a window of 128 dims, with one K x 128 accumulator in LDS.  Wave w of the block
// owns the codewords k with k % 8 == w.  The range is taken in segments of 4096 rows: the block
// first sorts the segment's rows by owner (a stable counting sort on the codes, in LDS), then
// every wave streams its own rows -- one whole 512-byte row per load, two chunks of 8 loads in
// flight -- and adds them to its accumulator rows with a plain LDS read-add-write.  No two waves
// ever touch the same accumulator row and a wave adds its rows in ascending vector order, so the
// sums do not depend on timing: two runs give identical bits.  Block partials go to scratch; a
// second kernel merges them in fp64 in block order, divides, and refreshes the codeword norms.
#pragma once
#include "common.hpp"

namespace hclae {

constexpr int kUpdThreads = 512;
constexpr int kUpdWaves = kUpdThreads / kWave;      // 8 owners of codeword classes k % 8
constexpr int kUpdWindow = 128;                     // dims per block: two per lane
constexpr int kUpdDepth = 16;                       // rows per chunk of loads
constexpr int kUpdSeg = 4096;                       // rows per segment (16-bit row index, 64 batches)
constexpr uint32_t kUpdNone = 0xffffffffu;

// LDS bytes of k_accumulate for K codewords.
constexpr size_t upd_lds_bytes(int K)
{
    return (size_t)K * kUpdWindow * sizeof(float)             // accumulator
           + (size_t)kUpdSeg * sizeof(uint32_t)               // row list of a segment
           + (size_t)(kUpdSeg / kWave) * kUpdWaves * sizeof(int)   // per batch, per owner offsets
           + 2 * kUpdWaves * sizeof(int);                     // owner bases and totals
}

// grid: (vector ranges, D windows).  partial: float [gridDim.x][K][D]; pcount: int [gridDim.x][K].
__global__ __launch_bounds__(kUpdThreads) void k_accumulate(
    const float *__restrict__ xp, const uint8_t *__restrict__ codes,
    int64_t N, int D, int K, int M, int m, int64_t rows_per_block,
    float *__restrict__ partial, int *__restrict__ pcount)
{
    extern __shared__ float4 smem4[];
    float *acc = reinterpret_cast<float *>(smem4);                   // [K][128]
    uint32_t *list = reinterpret_cast<uint32_t *>(acc + K * kUpdWindow);          // [kUpdSeg]: row | code << 16
    int *boff = reinterpret_cast<int *>(list + kUpdSeg);             // [64 batches][8 owners]
    int *wtotal = boff + (kUpdSeg / kWave) * kUpdWaves;              // [8]
    const int lane = lane_id();
    const int wave = threadIdx.x >> 6;
    const int d0 = blockIdx.y * kUpdWindow + 2 * lane;               // this lane's two dims
    const bool live = d0 < D;                                        // D % 4 == 0: both or neither

    for (int e = threadIdx.x; e < K * kUpdWindow / 4; e += kUpdThreads) smem4[e] = make_float4(0.f, 0.f, 0.f, 0.f);

    float2 *mine = reinterpret_cast<float2 *>(acc) + lane;
    const int64_t row0 = (int64_t)blockIdx.x * rows_per_block;
    int64_t row1 = row0 + rows_per_block;
    if (row1 > N) row1 = N;
    const unsigned long long lt = (1ull << lane) - 1ull;
    int own_cnt = 0;                                                 // members of codeword 8 * lane + wave (lane < 32)

    for (int64_t seg0 = row0; seg0 < row1; seg0 += kUpdSeg) {
        const int segn = (int)((row1 - seg0 < kUpdSeg) ? (row1 - seg0) : kUpdSeg);
        const int nbatch = (segn + kWave - 1) / kWave;
        // ---- stable counting sort of the segment's rows by owner wave ----
        int mycode[kUpdWaves];
#pragma unroll
        for (int i = 0; i < kUpdWaves; ++i) {
            const int b = wave + kUpdWaves * i;
            const int rloc = b * kWave + lane;
            mycode[i] = (rloc < segn) ? (int)codes[(seg0 + rloc) * M + m] : -1;
        }
#pragma unroll
        for (int i = 0; i < kUpdWaves; ++i) {
            const int b = wave + kUpdWaves * i;
            if (b < nbatch) {
                int mine_cnt = 0;
#pragma unroll
                for (int w = 0; w < kUpdWaves; ++w) {
                    const unsigned long long mk = __ballot(mycode[i] >= 0 && (mycode[i] & (kUpdWaves - 1)) == w);
                    if (lane == w) mine_cnt = __popcll(mk);
                }
                if (lane < kUpdWaves) boff[b * kUpdWaves + lane] = mine_cnt;
            }
        }
        __syncthreads();
        {
            // wave w turns the per-batch counts of owner w into exclusive offsets (lane = batch)
            const int c = (lane < nbatch) ? boff[lane * kUpdWaves + wave] : 0;
            int incl = c;
#pragma unroll
            for (int o = 1; o < kWave; o <<= 1) {
                const int t = __shfl_up(incl, o, kWave);
                if (lane >= o) incl += t;
            }
            if (lane < nbatch) boff[lane * kUpdWaves + wave] = incl - c;
            if (lane == kWave - 1) wtotal[wave] = incl;
        }
        __syncthreads();
        int obase[kUpdWaves];                                        // first list slot of every owner
        {
            int run = 0;
#pragma unroll
            for (int w = 0; w < kUpdWaves; ++w) { obase[w] = run; run += wtotal[w]; }
        }
#pragma unroll
        for (int i = 0; i < kUpdWaves; ++i) {
            const int b = wave + kUpdWaves * i;
            if (b < nbatch) {
                const int own = mycode[i] & (kUpdWaves - 1);
#pragma unroll
                for (int w = 0; w < kUpdWaves; ++w) {
                    const unsigned long long mk = __ballot(mycode[i] >= 0 && own == w);
                    if (mycode[i] >= 0 && own == w)
                        list[obase[w] + boff[b * kUpdWaves + w] + __popcll(mk & lt)] =
                            (uint32_t)(b * kWave + lane) | ((uint32_t)mycode[i] << 16);
                }
            }
        }
        __syncthreads();

        // ---- every wave streams its own rows, two chunks of loads in flight ----
        int my_base = 0;
#pragma unroll
        for (int w = 0; w < kUpdWaves; ++w) my_base = (w == wave) ? obase[w] : my_base;
        const uint32_t *L = list + my_base;
        const int n_own = wtotal[wave];
        const float *seg_x = xp + seg0 * D + d0;
        float2 va[kUpdDepth], vb[kUpdDepth];
        uint32_t ea, eb;
        auto fetch = [&](int i, float2 (&v)[kUpdDepth], uint32_t &e) {
            e = (lane < kUpdDepth && i + lane < n_own) ? L[i + lane] : kUpdNone;
#pragma unroll
            for (int u = 0; u < kUpdDepth; ++u) {
                const uint32_t ent = __builtin_amdgcn_readlane(e, u);
                v[u] = make_float2(0.f, 0.f);
                if (ent != kUpdNone && live)
                    v[u] = *reinterpret_cast<const float2 *>(seg_x + (size_t)(ent & 0xffffu) * D);
            }
        };
        auto rmw1 = [&](int c, const float2 &v) {
            float2 *a = mine + c * (kUpdWindow / 2);
            float2 t = *a;
            t.x += v.x;
            t.y += v.y;
            *a = t;
        };
        auto apply = [&](const float2 (&v)[kUpdDepth], uint32_t e) {
#pragma unroll
            for (int u = 0; u < kUpdDepth; u += 2) {
                const uint32_t e0 = __builtin_amdgcn_readlane(e, u);
                const uint32_t e1 = __builtin_amdgcn_readlane(e, u + 1);
                if (e0 == kUpdNone) break;
                const int c0 = (int)(e0 >> 16);
                own_cnt += (lane == (c0 >> 3));
                if (e1 == kUpdNone) { rmw1(c0, v[u]); break; }
                const int c1 = (int)(e1 >> 16);
                own_cnt += (lane == (c1 >> 3));
                if (c0 != c1) {
                    // distinct accumulator rows: overlap the two LDS round trips
                    float2 *a0 = mine + c0 * (kUpdWindow / 2);
                    float2 *a1 = mine + c1 * (kUpdWindow / 2);
                    float2 t0 = *a0, t1 = *a1;
                    t0.x += v[u].x; t0.y += v[u].y;
                    t1.x += v[u + 1].x; t1.y += v[u + 1].y;
                    *a0 = t0;
                    *a1 = t1;
                } else {
                    rmw1(c0, v[u]);
                    rmw1(c1, v[u + 1]);
                }
            }
        };
        fetch(0, va, ea);
        for (int i = 0; i < n_own; i += 2 * kUpdDepth) {
            fetch(i + kUpdDepth, vb, eb);
            apply(va, ea);
            fetch(i + 2 * kUpdDepth, va, ea);
            apply(vb, eb);
        }
        __syncthreads();
    }

    // partial[blockIdx.x][k][window dims]
    float *out = partial + (size_t)blockIdx.x * K * D;
    const int wd = min(kUpdWindow, D - blockIdx.y * kUpdWindow);     // live dims of this window
    for (int e = threadIdx.x; e < K * (kUpdWindow / 4); e += kUpdThreads) {
        const int k = e / (kUpdWindow / 4);
        const int d = 4 * (e - k * (kUpdWindow / 4));
        if (d < wd)
            *reinterpret_cast<float4 *>(out + (size_t)k * D + blockIdx.y * kUpdWindow + d) = smem4[e];
    }
    if (blockIdx.y == 0 && lane < 32 && kUpdWaves * lane + wave < K)
        pcount[blockIdx.x * K + kUpdWaves * lane + wave] = own_cnt;
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
