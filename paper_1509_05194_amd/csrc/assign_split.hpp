// Nearest-codeword assignment with the distance contraction on the bf16 matrix cores
// (v_mfma_f32_32x32x16_bf16, 16x the rate of the fp32 MFMA on gfx950), fp32 operands split
// into two bf16 terms each:  x = xh + xl + dx,  c = ch + cl + dc  with |dx| <= 2^-16 |x|.
// The score x.c - ||c||^2/2 is accumulated in fp32 as  xh.ch + xh.cl + xl.ch  (three MFMAs per
// 16 dims); what is dropped, xl.cl + dx.c + x.dc, is bounded by norms the kernel has, and that
// bound joins the rounding bound of the accumulation in the margin of the decision: every codeword
// whose score is within the margin of the best goes to the same fp64 direct-form re-check
// (k_refine) as in the fp32 kernel.  The contraction only pre-selects candidates, so the codes
// are the same fp64 direct-form decisions whichever kernel ran.
//
// Accumulation error of one 32x32x16 bf16 MFMA, measured on gfx950 over 4.6e6 random sums with
// exponent spreads up to 2^+-16: at most 4.9 * 2^-24 * (|C| + sum |a_k b_k|).  The margin assumes
// 2^-21 (8 * 2^-24) per MFMA.
#pragma once
#include "assign.hpp"

namespace hclae {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

constexpr int kSplitStep = 16;                      // dims per bf16 MFMA

// (a, b) -> packed bf16 pairs hi = RNE(a, b), lo = RNE(a - hi_a, b - hi_b); element 0 in the low half.
__device__ __forceinline__ void split_pair(float a, float b, uint32_t &hi, uint32_t &lo)
{
    const floatx2 v = {a, b};
    hi = __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
    const float ha = __uint_as_float(hi << 16), hb = __uint_as_float(hi & 0xffff0000u);
    const floatx2 rem = {a - ha, b - hb};            // exact: hi keeps the leading 8 bits
    lo = __builtin_bit_cast(uint32_t, __builtin_convertvector(rem, bf16x2));
}

__device__ __forceinline__ void split8(const float4 &u, const float4 &v, uint4 &hi, uint4 &lo)
{
    split_pair(u.x, u.y, hi.x, lo.x);
    split_pair(u.z, u.w, hi.y, lo.y);
    split_pair(v.x, v.y, hi.z, lo.z);
    split_pair(v.z, v.w, hi.w, lo.w);
}

// Per-codeword constants of the split over the first D coordinates (row stride ld), as fp32 rounded up:
//   out[2k] = || cl_k ||  (low part),   out[2k + 1] = || c_k - ch_k - cl_k ||  (what two terms miss).
// One wave per codeword; the assign kernel takes the maxima over k.
// img (or nullptr; the grid then covers kpad rows): the split dictionary in the LDS order of k_assign_split (see
// stage_codebook_split), T steps of 16 dims and kb row blocks, so that the kernel fills its LDS with one copy.
__global__ __launch_bounds__(256) void k_split_norms(
    const float *__restrict__ Cm, int K, int D, int ld, float *__restrict__ out,
    uint4 *__restrict__ img = nullptr, int kb = 0, int T = 0)
{
    const int lane = lane_id();
    const int k = blockIdx.x * (256 / kWave) + (threadIdx.x >> 6);
    if (img && k < 32 * kb) {
        for (int j = lane; j < 2 * T; j += kWave) {                // piece (t, g): dims 16 t + 8 g .. + 7
            const int t = j >> 1, gg = j & 1, col = kSplitStep * t + 8 * gg;
            const float4 u = load_row_piece(Cm, k, col, K, D, ld);
            const float4 v = load_row_piece(Cm, k, col + 4, K, D, ld);
            uint4 hi, lo;
            split8(u, v, hi, lo);
            const size_t tb = (size_t)t * kb + (k >> 5);
            img[(tb * 2 + 0) * kWave + 32 * gg + (k & 31)] = hi;
            img[(tb * 2 + 1) * kWave + 32 * gg + (k & 31)] = lo;
        }
    }
    if (k >= K) return;
    const float *c = Cm + (size_t)k * ld;
    double sl = 0.0, sd = 0.0;
    for (int d = lane; d < D; d += kWave) {
        uint32_t hi, lo;
        split_pair(c[d], 0.f, hi, lo);
        const float ch = __uint_as_float(hi << 16), cl = __uint_as_float(lo << 16);
        const double dc = ((double)c[d] - (double)ch) - (double)cl;
        sl += (double)cl * (double)cl;
        sd += dc * dc;
    }
    sl = wave_sum(sl);
    sd = wave_sum(sd);
    if (lane == 0) {
        out[2 * k] = (float)(sqrt(sl) * 1.000001);
        out[2 * k + 1] = (float)(sqrt(sd) * 1.000001);
    }
}

// LDS image of the split codebook in MFMA operand order.  For step t (16 dims), row block b (32
// codewords), part p (0 = high, 1 = low) and lane l = 32 g + r, the uint4 at ((t*kb + b)*2 + p)*64 + l
// holds the bf16 values of C[32b + r][16t + 8g .. 16t + 8g + 7]: every operand read is one
// contiguous kilobyte, and the reads of one 64-dim chunk are one base address plus constants below 64 KB.
// Coordinates beyond D and rows beyond K are zero.
__device__ __forceinline__ void stage_codebook_split(
    uint4 *lds, const float *__restrict__ Cm, int K, int D, int ld, int kb, int T)
{
    const int total = kb * T * kWave;
    for (int e = threadIdx.x; e < total; e += blockDim.x) {
        const int l = e & 63;
        const int tb = e >> 6;
        const int b = tb % kb;
        const int t = tb / kb;
        const int row = 32 * b + (l & 31);
        const int col = kSplitStep * t + 8 * (l >> 5);
        const float4 u = load_row_piece(Cm, row, col, K, D, ld);
        const float4 v = load_row_piece(Cm, row, col + 4, K, D, ld);
        uint4 hi, lo;
        split8(u, v, hi, lo);
        lds[(size_t)(tb * 2 + 0) * kWave + l] = hi;
        lds[(size_t)(tb * 2 + 1) * kWave + l] = lo;
    }
}

// The 64-dim chunk q of a row in B-operand order: lane (g, r) gets, for step t = 0..3, the eight
// floats x'[row r][64q + 16t + 8g .. + 7] as x[2t], x[2t + 1].
__device__ __forceinline__ void load_x_chunk_split(
    float4 (&x)[8], const float *__restrict__ xrow, int q, int g, int D)
{
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int col = kChunkD * q + kSplitStep * t + 8 * g;
        x[2 * t] = (col < D) ? *reinterpret_cast<const float4 *>(xrow + col) : make_float4(0.f, 0.f, 0.f, 0.f);
        x[2 * t + 1] = (col + 4 < D) ? *reinterpret_cast<const float4 *>(xrow + col + 4) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
}

template <int KB>
__device__ __forceinline__ void mfma_chunk_split(
    floatx16 (&acc)[KB], const float4 (&x)[8], const uint4 *__restrict__ lds, int q, int T, int lane,
    float &xsq, float &amax)
{
    constexpr int GB = KB < 4 ? KB : 4;              // codeword blocks whose operands are in registers at once
    const uint4 *chunk = lds + (size_t)(4 * q) * KB * 2 * kWave + lane;
    (void)T;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const float4 u = x[2 * t], v = x[2 * t + 1];
        xsq = fmaf(u.x, u.x, xsq);
        xsq = fmaf(u.y, u.y, xsq);
        xsq = fmaf(u.z, u.z, xsq);
        xsq = fmaf(u.w, u.w, xsq);
        xsq = fmaf(v.x, v.x, xsq);
        xsq = fmaf(v.y, v.y, xsq);
        xsq = fmaf(v.z, v.z, xsq);
        xsq = fmaf(v.w, v.w, xsq);
        amax = fmaxf(fmaxf(amax, fabsf(u.x)), fabsf(u.y));      // one v_max3_f32 per two elements
        amax = fmaxf(fmaxf(amax, fabsf(u.z)), fabsf(u.w));
        amax = fmaxf(fmaxf(amax, fabsf(v.x)), fabsf(v.y));
        amax = fmaxf(fmaxf(amax, fabsf(v.z)), fabsf(v.w));
        uint4 xh4, xl4;
        split8(u, v, xh4, xl4);
        const bf16x8 xh = __builtin_bit_cast(bf16x8, xh4), xl = __builtin_bit_cast(bf16x8, xl4);
#pragma unroll
        for (int b0 = 0; b0 < KB; b0 += GB) {
            bf16x8 ch[GB], cl[GB];
#pragma unroll
            for (int b = 0; b < GB; ++b) {
                const uint4 *at = chunk + ((t * KB + b0 + b) * 2) * kWave;      // compile-time offset
                ch[b] = __builtin_bit_cast(bf16x8, at[0]);
                cl[b] = __builtin_bit_cast(bf16x8, at[kWave]);
            }
#pragma unroll
            for (int b = 0; b < GB; ++b) acc[b0 + b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cl[b], xh, acc[b0 + b], 0, 0, 0);
#pragma unroll
            for (int b = 0; b < GB; ++b) acc[b0 + b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ch[b], xl, acc[b0 + b], 0, 0, 0);
#pragma unroll
            for (int b = 0; b < GB; ++b) acc[b0 + b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ch[b], xh, acc[b0 + b], 0, 0, 0);
        }
    }
}

// Same tile schedule, register streaming and decision as k_assign_resident; only the contraction
// differs.  eps and cmax_eff fold the two bounds into the form the decision uses:
//   margin = eps * (hmax + ||x'|| * cmax_eff),  eps = 2 * (accumulation bound),
//   cmax_eff = 1.02 cmax + (split bound per unit ||x'||) / (accumulation bound)
// (1.02: the accumulated magnitudes are those of the split operands, ||xh|| ||ch|| + ||xh|| ||cl|| + ||xl|| ||ch||).
template <int KB, int PRUNE = 0>
__global__ __launch_bounds__(kAssignThreads) void k_assign_split(
    const float *__restrict__ xp, const float *__restrict__ Cm, const float *__restrict__ hneg,
    const float *__restrict__ split_norms,
    int64_t N, int D, int ld, int K, int M, int m, int NC, float acc_bound,
    uint8_t *__restrict__ codes, RefineItem *__restrict__ list, unsigned *__restrict__ refine_count,
    PruneArgs pa, const uint4 *__restrict__ img)
{
    extern __shared__ float4 smem4[];
    const int T = 4 * NC;                                                // 16-dim steps
    uint4 *lds_c = reinterpret_cast<uint4 *>(smem4);                     // KB * T * 2 * 64 uint4
    float *lds_h = reinterpret_cast<float *>(smem4 + (size_t)KB * T * 2 * kWave);
    const int lane = lane_id();
    const int wave = threadIdx.x >> 6;
    const int g = lane >> 5;
    const int r = lane & 31;

    {   // the split dictionary as k_split_norms has just laid it out: one contiguous copy
        constexpr int U = 8;
        const int total = KB * T * 2 * kWave;
        for (int e0 = threadIdx.x; e0 < total; e0 += U * blockDim.x) {
            uint4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int e = e0 + u * blockDim.x;
                v[u] = e < total ? img[e] : make_uint4(0u, 0u, 0u, 0u);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int e = e0 + u * blockDim.x;
                if (e < total) lds_c[e] = v[u];
            }
        }
    }
    for (int k = threadIdx.x; k < 32 * KB; k += blockDim.x) lds_h[k] = hneg[k];
    __syncthreads();
    float hmax = 0.f;
    for (int k = 0; k < K; ++k) hmax = fmaxf(hmax, -lds_h[k]);
    const float cmax = sqrtf(2.f * hmax) * 1.000001f;
    // dropped terms per unit ||x'||:  ||xl|| ||cl|| + ||dx|| ||c|| + ||x - dx|| ||dc||
    //   <= 2^-8 (1 + 2^-8) clmax + 2^-16 cmax + (1 + 2^-16) dcmax
    // maxima of the per-codeword split constants: first wave reduces, everyone reads the result from LDS
    if (wave == 0) {
        float a = 0.f, b = 0.f;
        for (int k = lane; k < K; k += kWave) {
            a = fmaxf(a, split_norms[2 * k]);
            b = fmaxf(b, split_norms[2 * k + 1]);
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            a = fmaxf(a, __shfl_xor(a, o, kWave));
            b = fmaxf(b, __shfl_xor(b, o, kWave));
        }
        if (lane == 0) { lds_h[32 * KB] = a; lds_h[32 * KB + 1] = b; }
    }
    __syncthreads();
    const float clmax = lds_h[32 * KB], dcmax = lds_h[32 * KB + 1];
    const float split_bound = (0.00390625f * 1.00391f) * clmax + 1.52587890625e-5f * cmax + 1.00002f * dcmax;
    const float eps = 2.f * acc_bound;
    const float cmax_eff = (cmax * 1.02f + split_bound / acc_bound) * 1.0001f;

    // rows of this launch: all N vectors, or the listed ones (PRUNE 2; see PruneArgs)
    const int64_t listed = PRUNE == 2 ? (int64_t)*pa.active_count : N;
    const bool gather = PRUNE == 2 && listed * 32 < N * 31;         // nearly all listed: all N in order
    const int64_t rows = gather ? listed : N;
    const int64_t ntiles = (rows + kTileVec - 1) / kTileVec;
    const int64_t nslots = (int64_t)gridDim.x * 4;
    const int64_t tstride = 2 * nslots;
    const int64_t t0 = (int64_t)blockIdx.x * 4 + (wave & 3) + nslots * (wave >> 2);
    if (t0 >= ntiles) return;
    const int64_t my_tiles = (ntiles - t0 + tstride - 1) / tstride;
    const int64_t G = my_tiles * NC;

    auto vec_of = [&](int64_t tile) -> int64_t {
        const int64_t i = tile * kTileVec + r;
        if (i >= rows) return N;
        return gather ? (int64_t)pa.active[i] : i;
    };
    auto row_ptr = [&](int64_t tile) {
        int64_t n = vec_of(tile);
        if (n >= N) n = gather ? (int64_t)pa.active[rows - 1] : N - 1;
        return xp + n * ld;
    };

    floatx16 acc[KB];
    float4 xa[8], xb[8];
    float xsq = 0.f, amax = 0.f;
    int64_t tile = t0;
    int q = 0;
    load_x_chunk_split(xa, row_ptr(tile), 0, g, D);
    for (int64_t s = 0; s < G; s += 2) {
        int64_t tile1 = tile;
        int q1 = q + 1;
        if (q1 == NC) { q1 = 0; tile1 = tile + tstride; }
        if (s + 1 < G) load_x_chunk_split(xb, row_ptr(tile1), q1, g, D);
        if (q == 0) { init_acc<KB>(acc, lds_h, g); xsq = 0.f; }
        mfma_chunk_split<KB>(acc, xa, lds_c, q, T, lane, xsq, amax);
        if (q == NC - 1)
            decide<KB, PRUNE>(acc, xsq, eps, hmax, cmax_eff, lane, vec_of(tile), N, M, m, codes, list, refine_count, pa);
        if (s + 1 >= G) break;
        int64_t tile2 = tile1;
        int q2 = q1 + 1;
        if (q2 == NC) { q2 = 0; tile2 = tile1 + tstride; }
        if (s + 2 < G) load_x_chunk_split(xa, row_ptr(tile2), q2, g, D);
        if (q1 == 0) { init_acc<KB>(acc, lds_h, g); xsq = 0.f; }
        mfma_chunk_split<KB>(acc, xb, lds_c, q1, T, lane, xsq, amax);
        if (q1 == NC - 1)
            decide<KB, PRUNE>(acc, xsq, eps, hmax, cmax_eff, lane, vec_of(tile1), N, M, m, codes, list, refine_count, pa);
        tile = tile2;
        q = q2;
    }
    publish_absmax(amax, refine_count + 1);
}

// ---- the same contraction for dimensions whose codebook does not fit LDS ---------------------------------

// Split codebook in the order the D-chunked split kernel stages it: the slice of 64-dim chunk q is KB * 512
// uint4 laid out as in stage_codebook_split with chunk-local steps t = 0..3 (element ((t*KB + b)*2 + p)*64 + l),
// slices one after the other.  Same size as the fp32 image of k_codebook_image.
__global__ __launch_bounds__(256) void k_codebook_image_split(
    const float *__restrict__ Cm, int K, int D, int ld, int kb, int NC, uint4 *__restrict__ img)
{
    const int total = NC * 4 * kb * kWave;                          // (q, t, b, l)
    for (int e = blockIdx.x * 256 + threadIdx.x; e < total; e += gridDim.x * 256) {
        const int l = e & 63;
        int tb = e >> 6;
        const int b = tb % kb;
        tb /= kb;
        const int t = tb & 3, q = tb >> 2;
        const int row = 32 * b + (l & 31);
        const int col = kChunkD * q + kSplitStep * t + 8 * (l >> 5);
        const float4 u = load_row_piece(Cm, row, col, K, D, ld);
        const float4 v = load_row_piece(Cm, row, col + 4, K, D, ld);
        uint4 hi, lo;
        split8(u, v, hi, lo);
        uint4 *dst = img + (size_t)q * kb * 8 * kWave + (size_t)((t * kb + b) * 2) * kWave + l;
        dst[0] = hi;
        dst[kWave] = lo;
    }
}

// One 64-dim chunk of the D-chunked split kernel (see mfma_chunk_refill): contracts x with the slice in `cur`
// while the next slice and the next chunk of x' arrive.  Each 16-dim step fetches its share of the thread's KB
// pieces of the next slice (src: its uint4 of piece 0; pieces are 8 * 64 uint4 apart) at its start and stores
// them to `nxt` late in the step; x[2t], x[2t+1] are refilled from xnext as soon as step t has them.
template <int KB>
__device__ __forceinline__ void mfma_chunk_split_refill(
    floatx16 (&acc)[KB], float4 (&x)[8], const uint4 *__restrict__ cur, uint4 *__restrict__ nxt,
    const uint4 *__restrict__ src, const float *__restrict__ xnext, int q, int qn, int D, int lane, int wave,
    float &xsq, float &amax)
{
    constexpr int GB = KB < 4 ? KB : 4;
    constexpr int PP = (KB + 3) / 4;                                // pieces fetched per step
    const int g = lane >> 5;
    const uint4 *chunk = cur + lane;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        // Fetched as relaxed atomics (two 64-bit halves) and fenced for the scheduler: an ordinary load would be
        // moved down next to its use, where its latency is no longer covered.
        unsigned long long piece[PP][2];
#pragma unroll
        for (int i = 0; i < PP; ++i)
            if (t * PP + i < KB) {
                const unsigned long long *s64 = reinterpret_cast<const unsigned long long *>(src + (t * PP + i) * 8 * kWave);
                piece[i][0] = __hip_atomic_load(s64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                piece[i][1] = __hip_atomic_load(s64 + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
        __builtin_amdgcn_sched_barrier(0x10f);
        float4 u = x[2 * t], v = x[2 * t + 1];
        {
            // columns past D are zeroed at use; the refill is unconditional, its address clamped into the row
            const int col = kChunkD * q + kSplitStep * t + 8 * g;
            if (col >= D) u = make_float4(0.f, 0.f, 0.f, 0.f);
            if (col + 4 >= D) v = make_float4(0.f, 0.f, 0.f, 0.f);
            const int coln = kChunkD * qn + kSplitStep * t + 8 * g;
            x[2 * t] = *reinterpret_cast<const float4 *>(xnext + min(coln, last_piece(D)));
            x[2 * t + 1] = *reinterpret_cast<const float4 *>(xnext + min(coln + 4, last_piece(D)));
        }
        xsq = fmaf(u.x, u.x, xsq);
        xsq = fmaf(u.y, u.y, xsq);
        xsq = fmaf(u.z, u.z, xsq);
        xsq = fmaf(u.w, u.w, xsq);
        xsq = fmaf(v.x, v.x, xsq);
        xsq = fmaf(v.y, v.y, xsq);
        xsq = fmaf(v.z, v.z, xsq);
        xsq = fmaf(v.w, v.w, xsq);
        amax = fmaxf(fmaxf(amax, fabsf(u.x)), fabsf(u.y));
        amax = fmaxf(fmaxf(amax, fabsf(u.z)), fabsf(u.w));
        amax = fmaxf(fmaxf(amax, fabsf(v.x)), fabsf(v.y));
        amax = fmaxf(fmaxf(amax, fabsf(v.z)), fabsf(v.w));
        uint4 xh4, xl4;
        split8(u, v, xh4, xl4);
        const bf16x8 xh = __builtin_bit_cast(bf16x8, xh4), xl = __builtin_bit_cast(bf16x8, xl4);
#pragma unroll
        for (int b0 = 0; b0 < KB; b0 += GB) {
            bf16x8 ch[GB], cl[GB];
#pragma unroll
            for (int b = 0; b < GB; ++b) {
                const uint4 *at = chunk + ((t * KB + b0 + b) * 2) * kWave;      // compile-time offset
                ch[b] = __builtin_bit_cast(bf16x8, at[0]);
                cl[b] = __builtin_bit_cast(bf16x8, at[kWave]);
            }
#pragma unroll
            for (int b = 0; b < GB; ++b) acc[b0 + b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cl[b], xh, acc[b0 + b], 0, 0, 0);
#pragma unroll
            for (int b = 0; b < GB; ++b) acc[b0 + b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ch[b], xl, acc[b0 + b], 0, 0, 0);
            if (b0 + GB >= KB) {
                // the stores (and the waits for their loads) stay behind most of the step's MFMAs
                __builtin_amdgcn_sched_barrier(0x10f);
#pragma unroll
                for (int i = 0; i < PP; ++i)
                    if (t * PP + i < KB) {
                        uint4 v4;
                        v4.x = (uint32_t)piece[i][0]; v4.y = (uint32_t)(piece[i][0] >> 32);
                        v4.z = (uint32_t)piece[i][1]; v4.w = (uint32_t)(piece[i][1] >> 32);
                        nxt[((t * PP + i) * 8 + wave) * kWave + lane] = v4;
                    }
            }
#pragma unroll
            for (int b = 0; b < GB; ++b) acc[b0 + b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ch[b], xh, acc[b0 + b], 0, 0, 0);
        }
    }
}

// k_assign_chunked with the split-bf16 contraction: tiles, slices, refills and decision as there; margin as
// in k_assign_split.  img = k_codebook_image_split of the codebook in use.
template <int KB, int PRUNE = 0>
__global__ __launch_bounds__(kAssignThreads) void k_assign_split_chunked(
    const float *__restrict__ xp, const uint4 *__restrict__ img, const float *__restrict__ hneg,
    const float *__restrict__ split_norms,
    int64_t N, int D, int ld, int K, int M, int m, int NC, float acc_bound,
    uint8_t *__restrict__ codes, RefineItem *__restrict__ list, unsigned *__restrict__ refine_count,
    PruneArgs pa)
{
    extern __shared__ float4 smem4[];
    constexpr int CH = KB * 8 * kWave;                              // uint4 per slice
    uint4 *buf0 = reinterpret_cast<uint4 *>(smem4), *buf1 = buf0 + CH;
    float *lds_h = reinterpret_cast<float *>(smem4 + 2 * CH);
    const int lane = lane_id();
    const int wave = threadIdx.x >> 6;
    const int g = lane >> 5;
    const int r = lane & 31;

    for (int k = threadIdx.x; k < 32 * KB; k += blockDim.x) lds_h[k] = hneg[k];
    const uint4 *mine = img + wave * kWave + lane;
#pragma unroll
    for (int p = 0; p < KB; ++p) buf0[(p * 8 + wave) * kWave + lane] = mine[p * 8 * kWave];
    __syncthreads();
    float hmax = 0.f;
    for (int k = 0; k < K; ++k) hmax = fmaxf(hmax, -lds_h[k]);
    const float cmax = sqrtf(2.f * hmax) * 1.000001f;
    if (wave == 0) {
        float a = 0.f, b = 0.f;
        for (int k = lane; k < K; k += kWave) {
            a = fmaxf(a, split_norms[2 * k]);
            b = fmaxf(b, split_norms[2 * k + 1]);
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            a = fmaxf(a, __shfl_xor(a, o, kWave));
            b = fmaxf(b, __shfl_xor(b, o, kWave));
        }
        if (lane == 0) { lds_h[32 * KB] = a; lds_h[32 * KB + 1] = b; }
    }
    __syncthreads();
    const float clmax = lds_h[32 * KB], dcmax = lds_h[32 * KB + 1];
    const float split_bound = (0.00390625f * 1.00391f) * clmax + 1.52587890625e-5f * cmax + 1.00002f * dcmax;
    const float eps = 2.f * acc_bound;
    const float cmax_eff = (cmax * 1.02f + split_bound / acc_bound) * 1.0001f;

    const int64_t listed = PRUNE == 2 ? (int64_t)*pa.active_count : N;
    const bool gather = PRUNE == 2 && listed * 32 < N * 31;         // nearly all listed: all N in order
    const int64_t rows = gather ? listed : N;
    const int64_t nbt = (rows + kTileVec * kAssignWaves - 1) / (kTileVec * kAssignWaves);
    float amax = 0.f;
    if ((int64_t)blockIdx.x < nbt) {
        auto tile_row = [&](int64_t bt, int64_t &vec) -> const float * {
            const int64_t i = (bt * kAssignWaves + wave) * kTileVec + r;
            const int64_t ic = i < rows ? i : rows - 1;
            const int64_t nrow = gather ? (int64_t)pa.active[ic] : ic;
            vec = i < rows ? nrow : N;
            return xp + nrow * ld;
        };
        int64_t vec;
        const float *xrow = tile_row(blockIdx.x, vec);
        float4 x[8];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            x[2 * t] = *reinterpret_cast<const float4 *>(xrow + min(kSplitStep * t + 8 * g, last_piece(D)));
            x[2 * t + 1] = *reinterpret_cast<const float4 *>(xrow + min(kSplitStep * t + 8 * g + 4, last_piece(D)));
        }
        int par = 0;
        for (int64_t bt = blockIdx.x; bt < nbt; bt += gridDim.x) {
            int64_t vec_next = vec;
            const float *xrow_next = xrow;
            if (bt + gridDim.x < nbt) xrow_next = tile_row(bt + gridDim.x, vec_next);
            floatx16 acc[KB];
            float xsq = 0.f;
            init_acc<KB>(acc, lds_h, g);
            for (int q = 0; q < NC; ++q) {
                const bool last = q + 1 == NC;
                const int qn = last ? 0 : q + 1;
                mfma_chunk_split_refill<KB>(acc, x, par ? buf1 : buf0, par ? buf0 : buf1, mine + (size_t)qn * CH,
                                            last ? xrow_next : xrow, q, qn, D, lane, wave, xsq, amax);
                __syncthreads();
                par ^= 1;
            }
            decide<KB, PRUNE>(acc, xsq, eps, hmax, cmax_eff, lane, vec, N, M, m, codes, list, refine_count, pa);
            xrow = xrow_next;
            vec = vec_next;
        }
    }
    publish_absmax(amax, refine_count + 1);
}

}  // namespace hclae
