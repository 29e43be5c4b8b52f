// Centroid half of the k-means that cools a dictionary (Sec. 3.1/3.2): c_m(k) <- mean of the
// x' assigned to k; an empty cluster keeps its codeword.
//
// HBM-bound segmented sum in exact fixed point.  LDS float atomics run at about one lane per
// clock on this chip while integer LDS atomics keep up with HBM, and integer addition is
// associative, so the sums are taken on integers: every x' is scaled by a power of two chosen
// from max |x'| (published by the assign kernel that ran just before) so that |q| <= 2^30,
// rounded to an int32 q and added as int64 with ds_add_u64 into a K x 64 accumulator (2^30 times
// 2^31 rows cannot overflow).  The quantisation step is 2^-31..2^-30 of max |x'| -- finer than
// the fp32 spacing of every element within 2^-6 of the maximum -- and everything after it is
// exact, so the result does not depend on the order in which waves run: two runs give
// identical bits and no sort or ownership scheme is needed.  Rows are read once, fully
// coalesced (a wave-instruction covers one 256-byte half row), 16 rows per wave in flight.
#pragma once
#include "common.hpp"

namespace hclae {

constexpr int kUpdThreads = 1024;
constexpr int kUpdWaves = kUpdThreads / kWave;      // 16
constexpr int kUpdWindow = 64;                      // dims per block: one per lane
constexpr int kUpdDepth = 16;                       // rows a wave keeps in flight
constexpr int kUpdSeg = 8192;                       // rows per pointer rebase (keeps offsets in 32 bits)

// LDS bytes of k_accumulate for K codewords: int64 sums, counts.
constexpr size_t upd_lds_bytes(int K) { return (size_t)K * kUpdWindow * sizeof(long long) + (size_t)K * sizeof(int); }

// Power-of-two exponent s with max |x'| * 2^s in [2^29, 2^30): q = rint(x' * 2^s) fits int32.
__device__ __forceinline__ int fixed_point_shift(unsigned xmax_bits)
{
    const float mx = __uint_as_float(xmax_bits);
    if (!(mx > 0.f) || !(mx < __builtin_inff())) return 0;
    int e;
    (void)frexpf(mx, &e);                           // mx = f * 2^e, f in [0.5, 1)
    return 30 - e;
}

// grid: (vector ranges, 64-dim windows).  partial: int64 [gridDim.x][K][D] (sum of q); pcount: int [gridDim.x][K].
__global__ __launch_bounds__(kUpdThreads) void k_accumulate(
    const float *__restrict__ xp, const uint8_t *__restrict__ codes,
    int64_t N, int D, int K, int M, int m, int64_t rows_per_block, const unsigned *__restrict__ xmax_bits,
    long long *__restrict__ partial, int *__restrict__ pcount)
{
    extern __shared__ float4 smem4[];
    unsigned long long *acc = reinterpret_cast<unsigned long long *>(smem4);   // [K][64]
    unsigned *cnt = reinterpret_cast<unsigned *>(acc + K * kUpdWindow);        // [K]
    const int lane = lane_id();
    const int wave = threadIdx.x >> 6;
    const int d = blockIdx.y * kUpdWindow + lane;                    // this lane's dim
    const bool live = d < D;
    const bool counting = blockIdx.y == 0;
    const int shift = fixed_point_shift(*xmax_bits);

    for (int e = threadIdx.x; e < K * kUpdWindow; e += kUpdThreads) acc[e] = 0ull;
    for (int e = threadIdx.x; e < K; e += kUpdThreads) cnt[e] = 0u;
    __syncthreads();

    const int64_t row0 = (int64_t)blockIdx.x * rows_per_block;
    int64_t row1 = row0 + rows_per_block;
    if (row1 > N) row1 = N;
    unsigned own_cnt[4] = {0u, 0u, 0u, 0u};                          // rows seen with code 64 g + lane
    const int uwave = __builtin_amdgcn_readfirstlane(wave);          // wave-uniform copy for scalar address math
    unsigned long long *mine = acc + lane;
    for (int64_t seg0 = row0; seg0 < row1; seg0 += kUpdSeg) {
        const int segn = (int)((row1 - seg0 < kUpdSeg) ? (row1 - seg0) : kUpdSeg);
        const float *segx = xp + seg0 * D + (live ? d : 0);          // offsets below stay within 32 bits
        const uint8_t *segc = codes + seg0 * M + m;
        for (int r0 = uwave * kUpdDepth; r0 < segn; r0 += kUpdWaves * kUpdDepth) {
            const int nrow = min(kUpdDepth, segn - r0);              // uniform
            // lane u < nrow fetches the code of row r0 + u; values reach the scalar unit by readlane
            const int cvec = (lane < nrow) ? (int)segc[(unsigned)(r0 + lane) * (unsigned)M] : 0;
            float v[kUpdDepth];
#pragma unroll
            for (int u = 0; u < kUpdDepth; ++u) {
                v[u] = 0.f;
                if (u < nrow) v[u] = __builtin_nontemporal_load(segx + (unsigned)(r0 + u) * (unsigned)D);
            }
            unsigned packed = 0u;                                    // four 8-bit counters: codes 64 g + lane
#pragma unroll
            for (int u = 0; u < kUpdDepth; ++u) {
                if (u < nrow) {
                    const int cc = __builtin_amdgcn_readlane(cvec, u);
                    const int q = live ? (int)__builtin_rintf(ldexpf(v[u], shift)) : 0;
                    atomicAdd(mine + cc * kUpdWindow, (unsigned long long)(long long)q);
                    packed += (lane == (cc & 63)) ? (1u << ((cc >> 6) << 3)) : 0u;
                }
            }
            if (counting) {
#pragma unroll
                for (int g = 0; g < 4; ++g) own_cnt[g] += (packed >> (8 * g)) & 255u;
            }
        }
    }
    if (counting) {
#pragma unroll
        for (int g = 0; g < 4; ++g)
            if (64 * g + lane < K && own_cnt[g]) atomicAdd(cnt + 64 * g + lane, own_cnt[g]);
    }
    __syncthreads();

    long long *out = partial + (size_t)blockIdx.x * K * D;
    for (int e = threadIdx.x; e < K * kUpdWindow; e += kUpdThreads) {
        const int k = e / kUpdWindow, j = e - k * kUpdWindow;
        if (blockIdx.y * kUpdWindow + j < D) out[(size_t)k * D + blockIdx.y * kUpdWindow + j] = (long long)acc[e];
    }
    if (counting)
        for (int k = threadIdx.x; k < K; k += kUpdThreads) pcount[blockIdx.x * K + k] = (int)cnt[k];
}

// prev[n] = codes[n][m]: the column as the full centroid pass saw it.  (A kernel of its own: as a by-product of
// k_accumulate the byte stores sat in the row loop of the blocks of the first window and made those blocks, and with
// them the pass, 18 % slower at D = 960.)
__global__ __launch_bounds__(256) void k_save_column(
    const uint8_t *__restrict__ codes, int64_t N, int M, int m, uint8_t *__restrict__ prev)
{
    for (int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x; n < N; n += (int64_t)gridDim.x * 256)
        prev[n] = codes[n * M + m];
}

// Blocks (of the x dimension) that the pass over `total` moved vectors uses: 160 rows per block measured best
// on one MI355X (N = 1M, D = 128: the gather of the rows wants many blocks, the flush of 128 KB of partial sums
// per block and the merge that reads them want few).  The merge that follows computes the same number.
__device__ __forceinline__ int moved_blocks(unsigned total, int max_blocks)
{
    const unsigned want = (total + 159u) / 160u;
    return (int)(want < 1u ? 1u : (want > (unsigned)max_blocks ? (unsigned)max_blocks : want));
}

// k_accumulate over the moved vectors only: +q into the new cluster, -q out of the old one, counts likewise.
// Same grid roles, scale, rounding and partial layout as k_accumulate; the first moved_blocks(count)
// blocks stride over the list, the others leave at once.
__global__ __launch_bounds__(kUpdThreads) void k_accumulate_moved(
    const float *__restrict__ xp, const unsigned long long *__restrict__ list, const unsigned *__restrict__ count,
    int D, int K, const unsigned *__restrict__ xmax_bits, long long *__restrict__ partial, int *__restrict__ pcount)
{
    extern __shared__ float4 smem4[];
    unsigned long long *acc = reinterpret_cast<unsigned long long *>(smem4);   // [K][64]
    int *cnt = reinterpret_cast<int *>(acc + K * kUpdWindow);                  // [K]
    const int lane = lane_id();
    const int wave = threadIdx.x >> 6;
    const int d = blockIdx.y * kUpdWindow + lane;
    const bool live = d < D;
    const bool counting = blockIdx.y == 0;
    const int shift = fixed_point_shift(*xmax_bits);
    const unsigned total = *count;
    const int used = moved_blocks(total, (int)gridDim.x);
    if ((int)blockIdx.x >= used) return;

    for (int e = threadIdx.x; e < K * kUpdWindow; e += kUpdThreads) acc[e] = 0ull;
    for (int e = threadIdx.x; e < K; e += kUpdThreads) cnt[e] = 0;
    __syncthreads();

    unsigned long long *mine = acc + lane;
    const unsigned stride = (unsigned)used * kUpdWaves * kUpdDepth;
    for (unsigned e0 = (blockIdx.x * kUpdWaves + wave) * kUpdDepth; e0 < total; e0 += stride) {
        const int nent = (int)min((unsigned)kUpdDepth, total - e0);            // uniform
        const unsigned long long ent = (lane < nent) ? list[e0 + lane] : 0ull;
        const unsigned en = (unsigned)ent, eo = (unsigned)(ent >> 32) & 255u, ec = (unsigned)(ent >> 40) & 255u;
        float v[kUpdDepth];
#pragma unroll
        for (int u = 0; u < kUpdDepth; ++u) {
            v[u] = 0.f;
            if (u < nent) {
                const unsigned n = __builtin_amdgcn_readlane(en, u);
                v[u] = xp[(size_t)n * D + (live ? d : 0)];
            }
        }
#pragma unroll
        for (int u = 0; u < kUpdDepth; ++u) {
            if (u < nent) {
                const int ko = __builtin_amdgcn_readlane(eo, u), kn = __builtin_amdgcn_readlane(ec, u);
                const long long q = live ? (long long)(int)__builtin_rintf(ldexpf(v[u], shift)) : 0;
                atomicAdd(mine + kn * kUpdWindow, (unsigned long long)q);
                atomicAdd(mine + ko * kUpdWindow, (unsigned long long)(-q));
            }
        }
        if (counting && lane < nent) {
            atomicAdd(cnt + ec, 1);
            atomicAdd(cnt + eo, -1);
        }
    }
    __syncthreads();

    long long *out = partial + (size_t)blockIdx.x * K * D;
    for (int e = threadIdx.x; e < K * kUpdWindow; e += kUpdThreads) {
        const int k = e / kUpdWindow, j = e - k * kUpdWindow;
        if (blockIdx.y * kUpdWindow + j < D) out[(size_t)k * D + blockIdx.y * kUpdWindow + j] = (long long)acc[e];
    }
    if (counting)
        for (int k = threadIdx.x; k < K; k += kUpdThreads) pcount[blockIdx.x * K + k] = cnt[k];
}

// max |x'| over an array (bits of the float, see publish_absmax); used when the centroid update is
// called on its own, without the assign kernel that normally provides it.  *slot must start at 0.
__global__ __launch_bounds__(256) void k_absmax(const float4 *__restrict__ x, int64_t n4, unsigned *__restrict__ slot)
{
    float amax = 0.f;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (int64_t)gridDim.x * 256) {
        const float4 v = x[i];
        amax = fmaxf(fmaxf(amax, fmaxf(fabsf(v.x), fabsf(v.y))), fmaxf(fabsf(v.z), fabsf(v.w)));
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) amax = fmaxf(amax, __shfl_xor(amax, o, kWave));
    if (lane_id() == 0) atomicMax(slot, __float_as_uint(amax));
}

// Exact incremental form (tot_sum int64 [K][D], tot_cnt int [K]; both may be null): a full pass stores the
// integer sums and counts of the stage; while x' stays as it is, a later pass over only the vectors that
// changed cluster (listed by k_refine; k_accumulate_moved: +q into the new cluster, -q out of the old one) advances
// them with delta != 0.  Integer addition being exact, the totals -- and so the centroids -- are the very
// numbers a full pass would give.
//
// One block per codeword k: n_k = sum_b pcount[b][k];  C_m[k][d] = 2^-s * (sum_b partial[b][k][d]) / n_k
// with the integer sum exact (so its order is free: 4 groups of blocks in parallel) and the
// division in fp64; untouched when n_k == 0.  Then hneg[k] = -||c_k||^2/2 for the next
// assignment, nk[k] = n_k, and the re-check counter is reset (max |x'| stays: x' has not changed).
constexpr int kMergeGroups = 4;
constexpr int kMergePairs = 256 / kMergeGroups;     // dim pairs per pass
__global__ __launch_bounds__(256) void k_merge(
    const long long *__restrict__ partial, const int *__restrict__ pcount, int nblk,
    int K, int D, int dnorm, float *__restrict__ Cm, float *__restrict__ hneg, int *__restrict__ nk,
    int *__restrict__ counts_out, unsigned *__restrict__ refine_count,
    double *__restrict__ run_sum, long long *__restrict__ run_cnt,
    long long *__restrict__ tot_sum, int *__restrict__ tot_cnt, int delta, unsigned *__restrict__ moved_count,
    float *__restrict__ drift, float *__restrict__ img = nullptr, int S = 0)
{
    __shared__ double red[256 / kWave];
    __shared__ long long comb[kMergeGroups][kMergePairs][2];
    __shared__ int s_n;
    const int k = blockIdx.x;
    const int shift = fixed_point_shift(refine_count[1]);
    if (k == 0 && threadIdx.x == 0) refine_count[0] = 0u;
    // after a pass over the moved vectors only the blocks that pass used hold partials; the list counter is
    // handed back empty (every block reads it before the last one to arrive resets it)
    if (delta) nblk = moved_blocks(*moved_count, nblk);
    // moved_count[3]: the list counter of the pruning step that follows (k_bounds_step)
    if (moved_count) {
        __syncthreads();
        if (threadIdx.x == 0 && atomicAdd(moved_count + 1, 1u) == gridDim.x - 1) {
            moved_count[0] = 0u;
            moved_count[1] = 0u;
            moved_count[2] = 0u;
            moved_count[3] = 0u;
        }
    }
    if (threadIdx.x < kWave) {
        long long c = 0;
        for (int b = threadIdx.x; b < nblk; b += kWave) c += pcount[b * K + k];
        c = wave_sum_ll(c);
        if (threadIdx.x == 0) {
            // totals of the stage (tot_*): stored by a full pass, advanced by a pass over the moved vectors
            if (tot_cnt) {
                if (delta) c += tot_cnt[k];
                tot_cnt[k] = (int)c;
            }
            s_n = (int)c;
        }
    }
    __syncthreads();
    // online learning: the chunk's sums and counts join the running ones, which then define c_k
    const bool online = run_sum != nullptr;
    long long n_all = s_n;
    if (online) {
        n_all += run_cnt[k];
        __syncthreads();
        if (threadIdx.x == 0) run_cnt[k] = n_all;
    }
    const int n = online ? (n_all > 0 ? 1 : 0) : s_n;              // "has members" for the branches below
    const double denom = online ? (double)n_all : (double)s_n;
    const int g = threadIdx.x / kMergePairs;
    const int l = threadIdx.x - g * kMergePairs;
    const int per = (nblk + kMergeGroups - 1) / kMergeGroups;
    const int b0 = g * per, b1 = min(nblk, b0 + per);
    const int npairs = D >> 1;
    double sq = 0.0, moved2 = 0.0;                                  // ||c||^2 over dnorm dims; ||c_new - c_old||^2
    for (int p0 = 0; p0 < npairs; p0 += kMergePairs) {
        const int pr = p0 + l;
        long long s0 = 0, s1 = 0;
        if ((s_n > 0 || delta) && pr < npairs) {
            for (int b = b0; b < b1; ++b) {
                const longlong2 v = *reinterpret_cast<const longlong2 *>(partial + ((size_t)b * K + k) * D + 2 * pr);
                s0 += v.x;
                s1 += v.y;
            }
        }
        comb[g][l][0] = s0;
        comb[g][l][1] = s1;
        __syncthreads();
        if (g == 0 && pr < npairs) {
            float2 c;
            float2 *dst = reinterpret_cast<float2 *>(Cm + (size_t)k * D + 2 * pr);
            long long t0 = 0, t1 = 0;
#pragma unroll
            for (int q = 0; q < kMergeGroups; ++q) { t0 += comb[q][l][0]; t1 += comb[q][l][1]; }
            if (tot_sum) {
                longlong2 *ts = reinterpret_cast<longlong2 *>(tot_sum + (size_t)k * D + 2 * pr);
                if (delta) {
                    const longlong2 old = *ts;
                    t0 += old.x;
                    t1 += old.y;
                }
                *ts = make_longlong2(t0, t1);
            }
            if (n > 0) {
                double u0 = ldexp((double)t0, -shift), u1 = ldexp((double)t1, -shift);
                if (online) {
                    double *rs = run_sum + (size_t)k * D + 2 * pr;
                    u0 += rs[0];
                    u1 += rs[1];
                    rs[0] = u0;
                    rs[1] = u1;
                }
                c.x = (float)(u0 / denom);
                c.y = (float)(u1 / denom);
                if (drift) {
                    const float2 old = *dst;
                    const double e0 = (double)c.x - (double)old.x, e1 = (double)c.y - (double)old.y;
                    moved2 += e0 * e0 + e1 * e1;
                }
                *dst = c;
                // the copy in the LDS order of the assign kernel (k_codeword_norms): dims 2 pr, 2 pr + 1
                if (img) *reinterpret_cast<float2 *>(img + image_float(k, 2 * pr, S)) = c;
            } else {
                c = *dst;
            }
            // the next assignment may use only the first dnorm coordinates (improved k-means, Sec. 3.2)
            if (2 * pr < dnorm) sq += (double)c.x * c.x;
            if (2 * pr + 1 < dnorm) sq += (double)c.y * c.y;
        }
        __syncthreads();
    }
    sq = block_sum(sq, red);
    if (drift) {                                                    // how far the codeword moved, rounded up
        moved2 = block_sum(moved2, red);
        if (threadIdx.x == 0) drift[k] = (float)(sqrt(moved2) * 1.000001);
    }
    if (threadIdx.x == 0) {
        hneg[k] = -(float)(0.5 * sq);
        nk[k] = s_n;
        if (counts_out) counts_out[k] = s_n;
    }
}

// Running sums of the online mode from the current dictionaries: sum = c * n0 (n0 may be null: zeros).
__global__ __launch_bounds__(256) void k_online_begin(
    const float *__restrict__ C, const long long *__restrict__ n0, int64_t total, int D,
    double *__restrict__ run_sum, long long *__restrict__ run_cnt)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int64_t row = i / D;
        const long long w = n0 ? n0[row] : 0;
        run_sum[i] = (double)C[i] * (double)w;
        if (i == row * D) run_cnt[row] = w;
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
