// Multi-path encoding (Sec. 3.3, Eq. 3): for every vector keep the L best sums a_l of codewords
// of the dictionaries seen so far; for the next dictionary score all K * L sums a_l + c(k) by
// || x - a_l - c(k) ||^2 and keep the L smallest.
//
// The beam is stored as residuals r_l = x - a_l (fp32 rows), so a candidate's error is
// || r_l - c(k) ||^2 = e_l - 2 ( r_l . c(k) - ||c(k)||^2 / 2 ) and scoring a dictionary is the same
// codewords x vectors contraction as the nearest-codeword assignment, over N * L rows.  Two
// kernels per dictionary:
//   k_beam_score_*  fp32 matrix cores; per vector finds a threshold that at least L candidates
//                   reach and writes, per beam row, the bitmap of codewords that reach it minus
//                   twice the fp32 rounding bound (so the L best in exact arithmetic are in it);
//   k_beam_expand   evaluates the listed candidates in fp64 in the direct form, sorts them by
//                   (error, l, k), keeps the first L and writes their residuals, errors and
//                   code prefixes.
// The decision is therefore an fp64 direct-form decision, as in the assignment kernels.
#pragma once
#include "assign.hpp"
#include "assign_split.hpp"

namespace hclae {

constexpr int kBeamMaxL = 32;        // a vector's beam rows must fit one 32-column MFMA tile

// Candidate codewords of one beam row: bit p of w[h][i] is codeword 64 i + 8 (p >> 2) + 4 h + (p & 3).
struct BeamMask {
    uint32_t w[2][4];
};

// Threshold and bitmaps from a wave's scores.  Lane (h, r) holds the scores g = r_l.c - ||c||^2/2
// of beam row r of the tile against half of the codewords; a candidate's error is e_l - 2 g, so
// candidates are ranked by g - e_l / 2 (larger is better).
//   1. per lane, the maximum of each 16-score accumulator block (8 values, shifted by -e_l/2);
//   2. Ln rounds of "take the largest block maximum of the vector's group of lanes and strike it
//      out": the value taken in the last round is reached by at least Ln distinct candidates
//      (ties struck together only lower it);
//   3. every score within twice the rounding bound of that value is marked.
// gamma * (hmax + ||r|| cmax + ||r||^2) bounds the rounding error of a shifted score.
template <int KB>
__device__ __forceinline__ void beam_select(
    const floatx16 (&acc)[KB], float xsq, float e_l, float gamma, float hmax, float cmax,
    int lane, int gbase, int Lc, int Ln, bool valid, BeamMask *__restrict__ out)
{
    const int h = lane >> 5;
    const float ninf = -__builtin_inff();
    const float shift = 0.5f * e_l;
    float bm[KB];
#pragma unroll
    for (int b = 0; b < KB; ++b) {
        float t = acc[b][0];
#pragma unroll
        for (int v = 1; v < 16; ++v) t = fmaxf(t, acc[b][v]);
        bm[b] = valid ? t - shift : ninf;
    }
    const float x2 = xsq + __shfl_xor(xsq, 32, kWave);
    const float el = fmaxf(e_l, x2) * 1.00001f;
    const float bound = valid ? gamma * (hmax + sqrtf(el) * cmax + el) : 0.f;

    float tau = ninf;
    for (int it = 0; it < Ln; ++it) {
        float top = bm[0];
#pragma unroll
        for (int b = 1; b < KB; ++b) top = fmaxf(top, bm[b]);
        top = fmaxf(top, __shfl_xor(top, 32, kWave));
        float g = top;
        for (int j = 0; j < Lc; ++j) g = fmaxf(g, __shfl(top, gbase + j, kWave));
        tau = g;
#pragma unroll
        for (int b = 0; b < KB; ++b) bm[b] = (bm[b] == g) ? ninf : bm[b];
    }
    float gb = bound;
    for (int j = 0; j < Lc; ++j) gb = fmaxf(gb, __shfl(bound, gbase + j, kWave));
    const float thr = (tau - 2.f * gb) + shift;          // back to the lane's unshifted scores

    constexpr int NW = (KB + 1) / 2;
    uint32_t mk[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int b = 0; b < KB; ++b) {
        uint32_t below = 0u;                             // sign bits of acc - thr, shifted in (v_alignbit)
#pragma unroll
        for (int v = 15; v >= 0; --v)
            below = __builtin_amdgcn_alignbit(below, __float_as_uint(acc[b][v] - thr), 31);
        mk[b >> 1] |= (~below & 0xffffu) << ((b & 1) * 16);
    }
    (void)NW;
    if (valid) *reinterpret_cast<uint4 *>(&out->w[h][0]) = make_uint4(mk[0], mk[1], mk[2], mk[3]);
}

// Scoring with the whole padded codebook resident in LDS (same staging, operand order and
// two-register-set streaming as k_assign_resident).  A tile holds V = 32 / Lc whole vectors =
// V * Lc consecutive beam rows; the remaining columns idle.
template <int KB>
__global__ __launch_bounds__(kAssignThreads) void k_beam_score_resident(
    const float *__restrict__ rows, const double *__restrict__ err, const float *__restrict__ Cm,
    const float *__restrict__ hneg, int64_t N, int Lc, int Ln, int D, int ld, int K, int NC, float gamma,
    BeamMask *__restrict__ masks)
{
    extern __shared__ float4 smem4[];
    const int S = 8 * NC;
    float4 *lds_c = smem4;
    float *lds_h = reinterpret_cast<float *>(smem4 + KB * S * kWave);
    const int lane = lane_id();
    const int wave = threadIdx.x >> 6;
    const int h = lane >> 5;
    const int r = lane & 31;

    stage_codebook(lds_c, Cm, K, D, ld, KB, S);
    for (int k = threadIdx.x; k < 32 * KB; k += blockDim.x) lds_h[k] = hneg[k];
    __syncthreads();
    float hmax = 0.f;
    for (int k = 0; k < K; ++k) hmax = fmaxf(hmax, -lds_h[k]);
    const float cmax = sqrtf(2.f * hmax) * 1.000001f;

    const int V = kTileVec / Lc;                       // vectors per tile
    const int RT = V * Lc;                             // beam rows per tile
    const int gbase = (r < RT) ? (r / Lc) * Lc : 0;
    const int64_t nrows = N * Lc;
    const int64_t ntiles = (N + V - 1) / V;
    const int64_t nslots = (int64_t)gridDim.x * 4;
    const int64_t tstride = 2 * nslots;
    const int64_t t0 = (int64_t)blockIdx.x * 4 + (wave & 3) + nslots * (wave >> 2);
    if (t0 >= ntiles) return;
    const int64_t my_tiles = (ntiles - t0 + tstride - 1) / tstride;
    const int64_t G = my_tiles * NC;

    auto row_of = [&](int64_t tile) { return tile * RT + r; };
    auto row_ptr = [&](int64_t tile) {
        int64_t n = row_of(tile);
        if (r >= RT || n >= nrows) n = nrows - 1;      // idle columns re-read the last row
        return rows + n * ld;
    };
    auto e_of = [&](int64_t tile) {
        int64_t n = row_of(tile);
        if (r >= RT || n >= nrows) n = nrows - 1;
        return err ? (float)err[n] : 0.f;
    };

    floatx16 acc[KB];
    float4 xa[8], xb[8];
    float xsq = 0.f, amax = 0.f, e_l = 0.f;
    int64_t tile = t0;
    int q = 0;
    load_x_chunk(xa, row_ptr(tile), 0, h, D);
    for (int64_t g = 0; g < G; g += 2) {
        int64_t tile1 = tile;
        int q1 = q + 1;
        if (q1 == NC) { q1 = 0; tile1 = tile + tstride; }
        if (g + 1 < G) load_x_chunk(xb, row_ptr(tile1), q1, h, D);
        if (q == 0) { init_acc<KB>(acc, lds_h, h); xsq = 0.f; e_l = e_of(tile); }
        mfma_chunk<KB>(acc, xa, lds_c, q, S, lane, xsq, amax);
        if (q == NC - 1) {
            const int64_t row = row_of(tile);
            const bool valid = r < RT && row < nrows;
            beam_select<KB>(acc, xsq, e_l, gamma, hmax, cmax, lane, gbase, Lc, Ln, valid, masks + (valid ? row : 0));
        }
        if (g + 1 >= G) break;
        int64_t tile2 = tile1;
        int q2 = q1 + 1;
        if (q2 == NC) { q2 = 0; tile2 = tile1 + tstride; }
        if (g + 2 < G) load_x_chunk(xa, row_ptr(tile2), q2, h, D);
        if (q1 == 0) { init_acc<KB>(acc, lds_h, h); xsq = 0.f; e_l = e_of(tile1); }
        mfma_chunk<KB>(acc, xb, lds_c, q1, S, lane, xsq, amax);
        if (q1 == NC - 1) {
            const int64_t row = row_of(tile1);
            const bool valid = r < RT && row < nrows;
            beam_select<KB>(acc, xsq, e_l, gamma, hmax, cmax, lane, gbase, Lc, Ln, valid, masks + (valid ? row : 0));
        }
        tile = tile2;
        q = q2;
    }
}

// The same with the split-bf16 contraction of k_assign_split (operands as two bf16 terms, three bf16
// MFMAs per 16 dims).  gamma is then the accumulation bound and the bound on the dropped terms enters
// through the effective codeword norm, exactly as in k_assign_split.
template <int KB>
__global__ __launch_bounds__(kAssignThreads) void k_beam_score_split(
    const float *__restrict__ rows, const double *__restrict__ err, const float *__restrict__ Cm,
    const float *__restrict__ hneg, const float *__restrict__ split_norms,
    int64_t N, int Lc, int Ln, int D, int ld, int K, int NC, float gamma,
    BeamMask *__restrict__ masks)
{
    extern __shared__ float4 smem4[];
    const int T = 4 * NC;                                                // 16-dim steps
    uint4 *lds_c = reinterpret_cast<uint4 *>(smem4);                     // KB * T * 2 * 64 uint4
    float *lds_h = reinterpret_cast<float *>(smem4 + (size_t)KB * T * 2 * kWave);
    const int lane = lane_id();
    const int wave = threadIdx.x >> 6;
    const int h = lane >> 5;
    const int r = lane & 31;

    stage_codebook_split(lds_c, Cm, K, D, ld, KB, T);
    for (int k = threadIdx.x; k < 32 * KB; k += blockDim.x) lds_h[k] = hneg[k];
    __syncthreads();
    float hmax = 0.f;
    for (int k = 0; k < K; ++k) hmax = fmaxf(hmax, -lds_h[k]);
    float cmax = sqrtf(2.f * hmax) * 1.000001f;
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
    {   // dropped terms per unit ||r||, folded into the norm the margin multiplies (see k_assign_split)
        const float clmax = lds_h[32 * KB], dcmax = lds_h[32 * KB + 1];
        const float split_bound = (0.00390625f * 1.00391f) * clmax + 1.52587890625e-5f * cmax + 1.00002f * dcmax;
        cmax = (cmax * 1.02f + split_bound / gamma) * 1.0001f;
    }

    const int V = kTileVec / Lc;                       // vectors per tile
    const int RT = V * Lc;                             // beam rows per tile
    const int gbase = (r < RT) ? (r / Lc) * Lc : 0;
    const int64_t nrows = N * Lc;
    const int64_t ntiles = (N + V - 1) / V;
    const int64_t nslots = (int64_t)gridDim.x * 4;
    const int64_t tstride = 2 * nslots;
    const int64_t t0 = (int64_t)blockIdx.x * 4 + (wave & 3) + nslots * (wave >> 2);
    if (t0 >= ntiles) return;
    const int64_t my_tiles = (ntiles - t0 + tstride - 1) / tstride;
    const int64_t G = my_tiles * NC;

    auto row_of = [&](int64_t tile) { return tile * RT + r; };
    auto row_ptr = [&](int64_t tile) {
        int64_t n = row_of(tile);
        if (r >= RT || n >= nrows) n = nrows - 1;      // idle columns re-read the last row
        return rows + n * ld;
    };
    auto e_of = [&](int64_t tile) {
        int64_t n = row_of(tile);
        if (r >= RT || n >= nrows) n = nrows - 1;
        return err ? (float)err[n] : 0.f;
    };

    floatx16 acc[KB];
    float4 xa[8], xb[8];
    float xsq = 0.f, amax = 0.f, e_l = 0.f;
    int64_t tile = t0;
    int q = 0;
    load_x_chunk_split(xa, row_ptr(tile), 0, h, D);
    for (int64_t g = 0; g < G; g += 2) {
        int64_t tile1 = tile;
        int q1 = q + 1;
        if (q1 == NC) { q1 = 0; tile1 = tile + tstride; }
        if (g + 1 < G) load_x_chunk_split(xb, row_ptr(tile1), q1, h, D);
        if (q == 0) { init_acc<KB>(acc, lds_h, h); xsq = 0.f; e_l = e_of(tile); }
        mfma_chunk_split<KB>(acc, xa, lds_c, q, T, lane, xsq, amax);
        if (q == NC - 1) {
            const int64_t row = row_of(tile);
            const bool valid = r < RT && row < nrows;
            beam_select<KB>(acc, xsq, e_l, gamma, hmax, cmax, lane, gbase, Lc, Ln, valid, masks + (valid ? row : 0));
        }
        if (g + 1 >= G) break;
        int64_t tile2 = tile1;
        int q2 = q1 + 1;
        if (q2 == NC) { q2 = 0; tile2 = tile1 + tstride; }
        if (g + 2 < G) load_x_chunk_split(xa, row_ptr(tile2), q2, h, D);
        if (q1 == 0) { init_acc<KB>(acc, lds_h, h); xsq = 0.f; e_l = e_of(tile1); }
        mfma_chunk_split<KB>(acc, xb, lds_c, q1, T, lane, xsq, amax);
        if (q1 == NC - 1) {
            const int64_t row = row_of(tile1);
            const bool valid = r < RT && row < nrows;
            beam_select<KB>(acc, xsq, e_l, gamma, hmax, cmax, lane, gbase, Lc, Ln, valid, masks + (valid ? row : 0));
        }
        tile = tile2;
        q = q2;
    }
}

// Scoring for dimensions whose codebook does not fit LDS: as k_assign_chunked, the block walks the D axis in
// 64-dim slices of the codebook image (k_codebook_image), two LDS buffers alternating, the next slice and the
// next chunk of the residual rows arriving under the MFMAs (mfma_chunk_refill).
template <int KB>
__global__ __launch_bounds__(kAssignThreads) void k_beam_score_chunked(
    const float *__restrict__ rows, const double *__restrict__ err, const float4 *__restrict__ img,
    const float *__restrict__ hneg, int64_t N, int Lc, int Ln, int D, int ld, int K, int NC, float gamma,
    BeamMask *__restrict__ masks)
{
    extern __shared__ float4 smem4[];
    constexpr int CH = KB * 8 * kWave;                              // float4 per slice
    float4 *buf0 = smem4, *buf1 = smem4 + CH;
    float *lds_h = reinterpret_cast<float *>(smem4 + 2 * CH);
    const int lane = lane_id();
    const int wave = threadIdx.x >> 6;
    const int h = lane >> 5;
    const int r = lane & 31;

    for (int k = threadIdx.x; k < 32 * KB; k += blockDim.x) lds_h[k] = hneg[k];
    const float4 *mine = img + wave * kWave + lane;
#pragma unroll
    for (int p = 0; p < KB; ++p) buf0[(p * 8 + wave) * kWave + lane] = mine[p * 8 * kWave];
    __syncthreads();
    float hmax = 0.f;
    for (int k = 0; k < K; ++k) hmax = fmaxf(hmax, -lds_h[k]);
    const float cmax = sqrtf(2.f * hmax) * 1.000001f;

    const int V = kTileVec / Lc;
    const int RT = V * Lc;
    const int gbase = (r < RT) ? (r / Lc) * Lc : 0;
    const int64_t nrows = N * Lc;
    const int64_t ntiles = (N + V - 1) / V;
    const int64_t nbt = (ntiles + kAssignWaves - 1) / kAssignWaves;
    if ((int64_t)blockIdx.x >= nbt) return;
    // residual row this lane feeds for block tile bt (idle lanes and waves re-read the last row)
    auto tile_row = [&](int64_t bt, bool &valid) -> int64_t {
        const int64_t row = (bt * kAssignWaves + wave) * RT + r;
        valid = r < RT && row < nrows;
        return valid ? row : nrows - 1;
    };
    float amax = 0.f;
    bool valid;
    int64_t row = tile_row(blockIdx.x, valid);
    const float *xrow = rows + row * ld;
    float4 x[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) x[s] = *reinterpret_cast<const float4 *>(xrow + min(8 * s + 4 * h, last_piece(D)));
    int par = 0;
    for (int64_t bt = blockIdx.x; bt < nbt; bt += gridDim.x) {
        bool valid_next = valid;
        int64_t row_next = row;
        if (bt + gridDim.x < nbt) row_next = tile_row(bt + gridDim.x, valid_next);
        const float *xrow_next = rows + row_next * ld;
        const float e_l = err ? (float)err[row] : 0.f;
        floatx16 acc[KB];
        float xsq = 0.f;
        init_acc<KB>(acc, lds_h, h);
        for (int q = 0; q < NC; ++q) {
            const bool last = q + 1 == NC;
            const int qn = last ? 0 : q + 1;
            mfma_chunk_refill<KB>(acc, x, par ? buf1 : buf0, par ? buf0 : buf1, mine + (size_t)qn * CH,
                                  last ? xrow_next : xrow, q, qn, D, lane, wave, xsq, amax);
            __syncthreads();
            par ^= 1;
        }
        beam_select<KB>(acc, xsq, e_l, gamma, hmax, cmax, lane, gbase, Lc, Ln, valid, masks + (valid ? row : 0));
        row = row_next;
        valid = valid_next;
        xrow = xrow_next;
    }
}

// k_beam_score_chunked with the split-bf16 contraction (see k_assign_split_chunked and k_beam_score_split):
// img = k_codebook_image_split of the codebook in use; gamma is the accumulation bound.
template <int KB>
__global__ __launch_bounds__(kAssignThreads) void k_beam_score_split_chunked(
    const float *__restrict__ rows, const double *__restrict__ err, const uint4 *__restrict__ img,
    const float *__restrict__ hneg, const float *__restrict__ split_norms,
    int64_t N, int Lc, int Ln, int D, int ld, int K, int NC, float gamma,
    BeamMask *__restrict__ masks)
{
    extern __shared__ float4 smem4[];
    constexpr int CH = KB * 8 * kWave;                              // uint4 per slice
    uint4 *buf0 = reinterpret_cast<uint4 *>(smem4), *buf1 = buf0 + CH;
    float *lds_h = reinterpret_cast<float *>(smem4 + 2 * CH);
    const int lane = lane_id();
    const int wave = threadIdx.x >> 6;
    const int h = lane >> 5;
    const int r = lane & 31;

    for (int k = threadIdx.x; k < 32 * KB; k += blockDim.x) lds_h[k] = hneg[k];
    const uint4 *mine = img + wave * kWave + lane;
#pragma unroll
    for (int p = 0; p < KB; ++p) buf0[(p * 8 + wave) * kWave + lane] = mine[p * 8 * kWave];
    __syncthreads();
    float hmax = 0.f;
    for (int k = 0; k < K; ++k) hmax = fmaxf(hmax, -lds_h[k]);
    float cmax = sqrtf(2.f * hmax) * 1.000001f;
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
    {   // dropped terms per unit ||r||, folded into the norm the margin multiplies (see k_assign_split)
        const float clmax = lds_h[32 * KB], dcmax = lds_h[32 * KB + 1];
        const float split_bound = (0.00390625f * 1.00391f) * clmax + 1.52587890625e-5f * cmax + 1.00002f * dcmax;
        cmax = (cmax * 1.02f + split_bound / gamma) * 1.0001f;
    }

    const int V = kTileVec / Lc;
    const int RT = V * Lc;
    const int gbase = (r < RT) ? (r / Lc) * Lc : 0;
    const int64_t nrows = N * Lc;
    const int64_t ntiles = (N + V - 1) / V;
    const int64_t nbt = (ntiles + kAssignWaves - 1) / kAssignWaves;
    if ((int64_t)blockIdx.x >= nbt) return;
    auto tile_row = [&](int64_t bt, bool &valid) -> int64_t {
        const int64_t row = (bt * kAssignWaves + wave) * RT + r;
        valid = r < RT && row < nrows;
        return valid ? row : nrows - 1;
    };
    float amax = 0.f;
    bool valid;
    int64_t row = tile_row(blockIdx.x, valid);
    const float *xrow = rows + row * ld;
    float4 x[8];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        x[2 * t] = *reinterpret_cast<const float4 *>(xrow + min(kSplitStep * t + 8 * h, last_piece(D)));
        x[2 * t + 1] = *reinterpret_cast<const float4 *>(xrow + min(kSplitStep * t + 8 * h + 4, last_piece(D)));
    }
    int par = 0;
    for (int64_t bt = blockIdx.x; bt < nbt; bt += gridDim.x) {
        bool valid_next = valid;
        int64_t row_next = row;
        if (bt + gridDim.x < nbt) row_next = tile_row(bt + gridDim.x, valid_next);
        const float *xrow_next = rows + row_next * ld;
        const float e_l = err ? (float)err[row] : 0.f;
        floatx16 acc[KB];
        float xsq = 0.f;
        init_acc<KB>(acc, lds_h, h);
        for (int q = 0; q < NC; ++q) {
            const bool last = q + 1 == NC;
            const int qn = last ? 0 : q + 1;
            mfma_chunk_split_refill<KB>(acc, x, par ? buf1 : buf0, par ? buf0 : buf1, mine + (size_t)qn * CH,
                                        last ? xrow_next : xrow, q, qn, D, lane, wave, xsq, amax);
            __syncthreads();
            par ^= 1;
        }
        beam_select<KB>(acc, xsq, e_l, gamma, hmax, cmax, lane, gbase, Lc, Ln, valid, masks + (valid ? row : 0));
        row = row_next;
        valid = valid_next;
        xrow = xrow_next;
    }
}

constexpr int kExpandChunk = 32;     // candidates evaluated and ranked at a time
constexpr int kExpandList = 512;     // candidates listed in LDS at a time

// (error, id) order of the candidates: smaller error first, equal errors by id = (l << 8) | k.
__device__ __forceinline__ bool beam_before(double ea, int ia, double eb, int ib)
{
    return (ea < eb) || (ea == eb && ia < ib);
}

// Exact evaluation and selection for one dictionary; one wave (a 64-thread block) per vector.
// The vector's marked candidates are listed in LDS (kExpandList at a time).  kExpandChunk at a time they
// are evaluated in fp64 in the direct form, four lanes per candidate, and land one per lane in
// lanes 0..31; lanes 32..63 hold the best Ln found so far.  Every lane counts how many of the
// others come before it in (error, l, k) order: that rank is its position, and ranks below Ln are
// the new best list (kept in LDS).  After the last chunk the list is the next beam: residual rows
// r_l - c(k) rounded to fp32, their fp64 errors, and the parent's code prefix extended by k.
//   rows_c [N*Lc] stride ldc -> rows_n [N*Ln] stride ldn;  pre_c [N][Lc][M] -> pre_n [N][Ln][M]
//   (bytes 0..m-1 copied, byte m = k);  err_n, parent, code: [N*Ln], each may be null.
__global__ __launch_bounds__(kWave) void k_beam_expand(
    const float *__restrict__ rows_c, int ldc, const BeamMask *__restrict__ masks,
    const float *__restrict__ Cm, int K, int D, int64_t N, int Lc, int Ln,
    const uint8_t *__restrict__ pre_c, uint8_t *__restrict__ pre_n, int M, int m,
    float *__restrict__ rows_n, int ldn, double *__restrict__ err_n,
    uint8_t *__restrict__ parent, uint8_t *__restrict__ code)
{
    __shared__ uint16_t list[kExpandList];
    __shared__ double win_e[kBeamMaxL];
    __shared__ int win_id[kBeamMaxL];
    const int lane = lane_id();
    const int d4n = D >> 2;
    // words of a vector: j = 8 l + 4 h + i; a lane takes j = lane + 64 t, so (h, i) is fixed per lane
    const int wh = (lane >> 2) & 1, wi = lane & 3;
    uint32_t vm = 0u;                                   // bits of real codewords (k < K)
    for (int p = 0; p < 32; ++p)
        if (64 * wi + 8 * (p >> 2) + 4 * wh + (p & 3) < K) vm |= 1u << p;
    const uint32_t *mw = reinterpret_cast<const uint32_t *>(masks);
    const int nwords = 8 * Lc;
    const double inf = __builtin_inf();
    const int none = 0x7fffffff;

    uint32_t Wn[4];                                      // bitmap words of the next vector, fetched ahead
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int j = lane + 64 * t;
        Wn[t] = (j < nwords && (int64_t)blockIdx.x < N) ? mw[(size_t)blockIdx.x * nwords + j] : 0u;
    }
    for (int64_t n = blockIdx.x; n < N; n += gridDim.x) {
        uint32_t W[4];
        int cnt = 0;
        const int64_t nn = n + gridDim.x;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int j = lane + 64 * t;
            W[t] = Wn[t] & vm;
            cnt += __popc(W[t]);
            Wn[t] = (j < nwords && nn < N) ? mw[(size_t)nn * nwords + j] : 0u;
        }
        int incl = cnt;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) {
            const int y = __shfl_up(incl, o, kWave);
            if (lane >= o) incl += y;
        }
        const int total = __shfl(incl, kWave - 1, kWave);
        const int off = incl - cnt;                      // list position of the lane's first candidate
        if (lane < kBeamMaxL) { win_e[lane] = inf; win_id[lane] = none; }
        __syncthreads();

        int nwin = 0;                                    // entries of the best list so far
        for (int lbase = 0; lbase < total; lbase += kExpandList) {
        {   // list the candidates lbase .. lbase + kExpandList - 1 (any order: the ranking key is total)
            int at = off - lbase;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                uint32_t bits = W[t];
                const int l = (lane + 64 * t) >> 3;
                while (bits) {
                    const int p = __ffs(bits) - 1;
                    bits &= bits - 1;
                    if (at >= 0 && at < kExpandList)
                        list[at] = (uint16_t)((l << 8) | (64 * wi + 8 * (p >> 2) + 4 * wh + (p & 3)));
                    ++at;
                }
            }
        }
        __syncthreads();
        const int nl = min(kExpandList, total - lbase);
        for (int base = 0; base < nl; base += kExpandChunk) {
            const int nc = min(kExpandChunk, nl - base);
            // evaluate: pass p covers candidates base + 16 p + (lane >> 2), four lanes each
            double e_mine = inf;
            int id_mine = none;
#pragma unroll 1
            for (int p = 0; p < 2; ++p) {
                if (16 * p >= nc) break;                 // uniform
                const int c = 16 * p + (lane >> 2);
                const int ent = (c < nc) ? (int)list[base + c] : 0;
                const float4 *a = reinterpret_cast<const float4 *>(rows_c + ((size_t)n * Lc + (ent >> 8)) * ldc);
                const float4 *b = reinterpret_cast<const float4 *>(Cm + (size_t)(ent & 255) * D);
                double s0 = 0.0, s1 = 0.0;
                auto term = [&](const float4 &u, const float4 &v) {
                    const double t0 = (double)u.x - (double)v.x, t1 = (double)u.y - (double)v.y;
                    const double t2 = (double)u.z - (double)v.z, t3 = (double)u.w - (double)v.w;
                    s0 = fma(t0, t0, s0);
                    s1 = fma(t1, t1, s1);
                    s0 = fma(t2, t2, s0);
                    s1 = fma(t3, t3, s1);
                };
                int d = lane & 3;
                for (; d + 12 < d4n; d += 16) {          // four float4 pairs in flight per lane
                    const float4 u0 = a[d], u1 = a[d + 4], u2 = a[d + 8], u3 = a[d + 12];
                    const float4 v0 = b[d], v1 = b[d + 4], v2 = b[d + 8], v3 = b[d + 12];
                    term(u0, v0);
                    term(u1, v1);
                    term(u2, v2);
                    term(u3, v3);
                }
                for (; d < d4n; d += 4) term(a[d], b[d]);
                double s = s0 + s1;
                s += __shfl_xor(s, 1, kWave);
                s += __shfl_xor(s, 2, kWave);
                if (!(s == s)) s = inf;                  // non-finite input sorts last
                // candidate 16 p + q sits in lanes 4 q .. 4 q + 3; bring it to lane 16 p + q
                const double sq = __shfl(s, 4 * (lane & 15), kWave);
                const int iq = __shfl(ent, 4 * (lane & 15), kWave);
                if ((lane >> 4) == p && lane < nc) { e_mine = sq; id_mine = iq; }
            }
            if (lane >= 32) {                            // the best so far
                const int i = lane - 32;
                if (i < nwin) { e_mine = win_e[i]; id_mine = win_id[i]; }
            }
            __syncthreads();                             // win_* read before it is rewritten
            // rank among the nc new candidates and the nwin kept ones
            int rank = 0;
            for (int j = 0; j < nc; ++j) {
                const double ej = __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(e_mine), j),
                                                   __builtin_amdgcn_readlane(__double2loint(e_mine), j));
                const int ij = __builtin_amdgcn_readlane(id_mine, j);
                rank += beam_before(ej, ij, e_mine, id_mine) ? 1 : 0;
            }
            for (int j = 32; j < 32 + nwin; ++j) {
                const double ej = __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(e_mine), j),
                                                   __builtin_amdgcn_readlane(__double2loint(e_mine), j));
                const int ij = __builtin_amdgcn_readlane(id_mine, j);
                rank += beam_before(ej, ij, e_mine, id_mine) ? 1 : 0;
            }
            const bool live = (lane < nc) || (lane >= 32 && lane - 32 < nwin);
            if (live && rank < Ln) { win_e[rank] = e_mine; win_id[rank] = id_mine; }
            nwin = min(Ln, nwin + nc);
            __syncthreads();
        }
        }

        // the next beam: eight rows per pass, eight lanes each
        const int sub = lane & 7;
        for (int i0 = 0; i0 < Ln; i0 += 8) {
            const int i = i0 + (lane >> 3);
            if (i < Ln) {
                int id = win_id[i];
                if (id == none) id = 0;                  // fewer candidates than Ln: non-finite input only
                const int l = id >> 8, k = id & 255;
                const size_t src = (size_t)n * Lc + l, slot = (size_t)n * Ln + i;
                const float4 *a = reinterpret_cast<const float4 *>(rows_c + src * ldc);
                const float4 *b = reinterpret_cast<const float4 *>(Cm + (size_t)k * D);
                float4 *o = reinterpret_cast<float4 *>(rows_n + slot * ldn);
                int d = sub;
                for (; d + 24 < d4n; d += 32) {
                    const float4 u0 = a[d], u1 = a[d + 8], u2 = a[d + 16], u3 = a[d + 24];
                    const float4 v0 = b[d], v1 = b[d + 8], v2 = b[d + 16], v3 = b[d + 24];
                    o[d] = make_float4(u0.x - v0.x, u0.y - v0.y, u0.z - v0.z, u0.w - v0.w);
                    o[d + 8] = make_float4(u1.x - v1.x, u1.y - v1.y, u1.z - v1.z, u1.w - v1.w);
                    o[d + 16] = make_float4(u2.x - v2.x, u2.y - v2.y, u2.z - v2.z, u2.w - v2.w);
                    o[d + 24] = make_float4(u3.x - v3.x, u3.y - v3.y, u3.z - v3.z, u3.w - v3.w);
                }
                for (; d < d4n; d += 8) {
                    const float4 u = a[d], v = b[d];
                    o[d] = make_float4(u.x - v.x, u.y - v.y, u.z - v.z, u.w - v.w);
                }
                if (pre_n) {
                    for (int j = sub; j < m; j += 8) pre_n[slot * M + j] = pre_c[src * M + j];
                    if (sub == 0) pre_n[slot * M + m] = (uint8_t)k;
                }
                if (sub == 0) {
                    if (err_n) err_n[slot] = win_e[i];
                    if (parent) parent[slot] = (uint8_t)l;
                    if (code) code[slot] = (uint8_t)k;
                }
            }
        }
        __syncthreads();                                 // list and win_* are reused by the next vector
    }
}

}  // namespace hclae
