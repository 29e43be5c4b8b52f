// Nearest-codeword assignment (the assignment half of the k-means that cools a dictionary,
// Sec. 3.1/3.2; equally the per-dictionary step of Eq. 3 with one path).
//
// argmin_k ||x' - c_k||^2 = argmax_k ( x'.c_k - ||c_k||^2/2 ).  The right-hand score is a dense
// K x D by D x N contraction and runs on the fp32 matrix cores (v_mfma_f32_32x32x2_f32), with
// the accumulators started at -||c_k||^2/2.  The product is oriented codewords x vectors, so a
// lane ends up holding scores of many codewords for ONE vector and the argmax never leaves
// the wave (one exchange between lane l and lane l+32 at the end).
//
// fp32 rounding of the expanded form can reorder two codewords whose distances differ by less
// than the rounding error, which is far larger than the error of the direct form.  Each wave
// therefore bounds that error rigorously, collects every codeword whose score is within the
// bound of the best, and when more than one remains hands the vector to k_refine, which decides
// among the candidates with direct-form distances in fp64 (lowest index on exact ties).
#pragma once
#include "common.hpp"

namespace hclae {

constexpr int kAssignThreads = 512;                 // 8 waves: 2 per SIMD
constexpr int kAssignWaves = kAssignThreads / kWave;
constexpr int kTileVec = 32;                        // vectors per wave tile (N side of the MFMA)
constexpr int kChunkD = 64;                         // dims per register-resident chunk of x'

// One entry of the re-check list: the vector and the bitmap of its candidate codewords in the
// layout the wave produces it in.  Bit p of word mask[h][i] stands for codeword
// 64 i + 8 (p >> 2) + 4 h + (p & 3).
struct RefineItem {
    uint32_t n;
    uint32_t mask[2][4];
};

// Exact pruning of the assignments of one stage (x' fixed, only the dictionary moves).  For every vector
// the stage keeps an upper bound bu on the distance to its own codeword and a lower bound bl on the
// distance to every other one, both rigorous (they include the rounding bound of the scores).  When
// the dictionary moves, bu grows by the drift of the own codeword and bl shrinks by the largest drift
// of another one (triangle inequality); while bu < bl the own codeword is still the unique nearest
// and the vector is not recomputed.  The others are listed (k_bounds_step) and go through the same
// contraction, decision and fp64 re-check as before, which also renews their bounds.  The codes are
// therefore exactly those of full assignments.
//   PRUNE 0: plain assignment.  1: all vectors, and store their bounds.  2: only active[0..*active_count),
//   and store their bounds.
struct PruneArgs {
    float *bu, *bl;                    // [N]
    const uint32_t *active;            // [*active_count] vector indices (PRUNE 2)
    const unsigned *active_count;
    float slack;                       // rounding of ||x'||^2 and of the bound arithmetic, relative: grows with D
};
// Lower bound stored for a vector that goes to the fp64 re-check: no distance is negative, so the value
// keeps the vector listed and tells it from all others.
constexpr float kAmbiguousL = -2.f;

// Which vectors changed cluster since the last centroid update of the stage, found by the re-check kernel that
// follows a PRUNE 2 assignment (prev == nullptr: not wanted).  Only a vector that assignment recomputed can
// have changed code.  Entry = n | old code << 32 | new code << 40; order is free.
struct MovedArgs {
    uint8_t *prev;                     // [N] code column at the last update; brought up to date
    unsigned long long *list;
    unsigned *count;                   // zero on entry
    const uint32_t *cand;              // [*cand_count] the vectors the assignment recomputed
    const unsigned *cand_count;
    const float *bl;                   // [N] kAmbiguousL marks the ones on the re-check list
};

// -||c_k||^2 / 2 in fp32 (computed in fp64) over the first D coordinates of rows of stride ld, for
// k < K; -inf for the padding rows up to kpad.
// One wave per codeword.  Also resets the two counters the assign that follows will fill
// (refine_count[0]: re-check entries, refine_count[1]: bits of max |x'|).
// img (or nullptr): a copy of the dictionary in the LDS order of k_assign_resident (see stage_codebook), S = k-steps
// of a row; written here in full, zero beyond K and D, and kept up to date by k_merge, so that the assignments
// of a stage fill their LDS with one contiguous copy instead of a gather of 16-byte pieces.
// keep_absmax 2: max |x'| was left by the row pass that wrote x', spread over amax_parts[0..64) (block_absmax): the
// largest word becomes refine_count[1] and the words are cleared for the next such pass.
// entry_copy (or nullptr): receives the K x D dictionary as it is now (the carried bounds price a stage by how far
// it moves from here); zero_word (or nullptr): a counter cleared for the kernel that follows.
__global__ __launch_bounds__(256) void k_codeword_norms(
    const float *__restrict__ Cm, int K, int D, int ld, int kpad, float *__restrict__ hneg,
    unsigned *__restrict__ refine_count, int keep_absmax, float *__restrict__ img, int S,
    unsigned *__restrict__ amax_parts = nullptr, float *__restrict__ entry_copy = nullptr,
    unsigned *__restrict__ zero_word = nullptr)
{
    const int lane = lane_id();
    const int k = blockIdx.x * (256 / kWave) + (threadIdx.x >> 6);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        refine_count[0] = 0u;                      // re-check entries
        if (!keep_absmax) refine_count[1] = 0u;    // bits of max |x'|
        if (keep_absmax == 2) {
            unsigned mx = 0u;
            for (int i = 0; i < 64; ++i) {
                mx = max(mx, amax_parts[i]);
                amax_parts[i] = 0u;
            }
            refine_count[1] = mx;
        }
        if (zero_word) *zero_word = 0u;
    }
    if (k >= kpad) return;
    if (img)
        for (int d = lane; d < 8 * S; d += kWave) img[image_float(k, d, S)] = (k < K && d < D) ? Cm[(size_t)k * ld + d] : 0.f;
    if (k >= K) {
        if (lane == 0) hneg[k] = -__builtin_inff();
        return;
    }
    const float *c = Cm + (size_t)k * ld;
    double s = 0.0;
    for (int d = lane; d < D; d += kWave) {
        const float v = c[d];
        s += (double)v * (double)v;
        if (entry_copy) entry_copy[(size_t)k * D + d] = v;
    }
    s = wave_sum(s);
    if (lane == 0) hneg[k] = -(float)(0.5 * s);
}

// LDS image of the codebook in MFMA operand order.  For row block b (32 codewords), k-step s
// (8 dims) and lane l = 32*h + r, the float4 at index (b*S + s)*64 + l holds
// C[32b + r][8s + 4h .. 8s + 4h + 3]; a wave's ds_read_b128 of one (b, s) is one contiguous
// kilobyte (no bank conflicts), and component j of it is the A operand of the MFMA that
// contracts dims {8s + j, 8s + 4 + j}.
// Only the first D coordinates of each row (stride ld) enter; the rest of the image is zero, so
// whatever x' holds beyond D contributes nothing to the scores.
__device__ __forceinline__ float4 load_row_piece(const float *__restrict__ base, int row, int col, int K, int D, int ld)
{
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (row < K && col < D) {
        v = *reinterpret_cast<const float4 *>(base + (size_t)row * ld + col);
        if (col + 3 >= D) {                        // D need not be a multiple of 4
            if (col + 1 >= D) v.y = 0.f;
            if (col + 2 >= D) v.z = 0.f;
            v.w = 0.f;
        }
    }
    return v;
}

__device__ __forceinline__ void stage_codebook(
    float4 *lds, const float *__restrict__ Cm, int K, int D, int ld, int kb, int S)
{
    const int total = kb * S * kWave;
    constexpr int U = 8;                                   // gathers in flight per thread
    for (int e0 = threadIdx.x; e0 < total; e0 += U * blockDim.x) {
        float4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int e = e0 + u * blockDim.x;
            const int l = e & 63;
            const int bs = e >> 6;
            const int s = bs % S;
            const int b = bs / S;
            const int row = 32 * b + (l & 31);
            const int col = 8 * s + 4 * (l >> 5);
            v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (e < total) v[u] = load_row_piece(Cm, row, col, K, D, ld);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int e = e0 + u * blockDim.x;
            if (e < total) lds[e] = v[u];
        }
    }
}

// Loads the 64-dim chunk q of the wave's 32-vector tile into B-operand order:
// lane (h, r) gets x'[row r][64q + 8s + 4h .. +3] for s = 0..7.
// PREFIX: only the first `steps` 8-dim steps of the chunk are wanted (the others are not contracted either).
template <bool PREFIX = false>
__device__ __forceinline__ void load_x_chunk(
    float4 (&x)[8], const float *__restrict__ xrow, int q, int h, int D, int steps = 8)
{
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        const int col = kChunkD * q + 8 * s + 4 * h;
        x[s] = (col < D && (!PREFIX || s < steps)) ? *reinterpret_cast<const float4 *>(xrow + col)
                                                   : make_float4(0.f, 0.f, 0.f, 0.f);
    }
}

// max |x'| over everything the wave has read, merged into *slot (bit pattern of a non-negative
// float: integer max is float max, and an integer atomic is order-free).  The centroid-sum kernel
// that follows derives its fixed-point scale from it.
__device__ __forceinline__ void publish_absmax(float amax, unsigned *slot)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) amax = fmaxf(amax, __shfl_xor(amax, o, kWave));
    if (lane_id() == 0) atomicMax(slot, __float_as_uint(amax));
}

// PREFIX: the chunk ends after `steps` of its eight 8-dim steps (a short prefix of the coordinates counts;
// the codebook image is zero beyond it, so the steps left out would add nothing).
template <int KB, bool PREFIX = false>
__device__ __forceinline__ void mfma_chunk(
    floatx16 (&acc)[KB], const float4 (&x)[8], const float4 *__restrict__ lds, int q, int S, int lane,
    float &xsq, float &amax, int steps = 8)
{
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        if (PREFIX && s >= steps) break;
        float4 a[KB];
#pragma unroll
        for (int b = 0; b < KB; ++b) a[b] = lds[(b * S + 8 * q + s) * kWave + lane];
        const float4 xv = x[s];
        xsq = fmaf(xv.x, xv.x, xsq);
        xsq = fmaf(xv.y, xv.y, xsq);
        xsq = fmaf(xv.z, xv.z, xsq);
        xsq = fmaf(xv.w, xv.w, xsq);
        amax = fmaxf(fmaxf(amax, fabsf(xv.x)), fabsf(xv.y));      // one v_max3_f32 per two elements
        amax = fmaxf(fmaxf(amax, fabsf(xv.z)), fabsf(xv.w));
#pragma unroll
        for (int b = 0; b < KB; ++b) acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[b].x, xv.x, acc[b], 0, 0, 0);
#pragma unroll
        for (int b = 0; b < KB; ++b) acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[b].y, xv.y, acc[b], 0, 0, 0);
#pragma unroll
        for (int b = 0; b < KB; ++b) acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[b].z, xv.z, acc[b], 0, 0, 0);
#pragma unroll
        for (int b = 0; b < KB; ++b) acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[b].w, xv.w, acc[b], 0, 0, 0);
    }
}

// Accumulator start: element v of block b in lane (h, r) belongs to codeword
// 32b + 8(v/4) + 4h + v%4 (the 32x32 fp32 MFMA result layout).
template <int KB>
__device__ __forceinline__ void init_acc(floatx16 (&acc)[KB], const float *hneg_lds, int h)
{
#pragma unroll
    for (int b = 0; b < KB; ++b) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const float4 t = *reinterpret_cast<const float4 *>(hneg_lds + 32 * b + 8 * g + 4 * h);
            acc[b][4 * g + 0] = t.x;
            acc[b][4 * g + 1] = t.y;
            acc[b][4 * g + 2] = t.z;
            acc[b][4 * g + 3] = t.w;
        }
    }
}

// Per-vector decision from the wave's scores.  `eps` * (hmax + ||x'|| * cmax) bounds twice the
// rounding error of any score, so the true nearest codeword is among those within that
// margin of the best score.
template <int KB, int PRUNE = 0>
__device__ __forceinline__ void decide(
    const floatx16 (&acc)[KB], float xsq, float eps, float hmax, float cmax, int lane,
    int64_t n, int64_t N, int M, int m, uint8_t *__restrict__ codes,
    RefineItem *__restrict__ list, unsigned *__restrict__ refine_count, PruneArgs pa = PruneArgs())
{
    const int h = lane >> 5;
    float mx = -__builtin_inff(), m2 = -__builtin_inff();            // best and second best score
    if (PRUNE) {
        // top two per accumulator block (independent chains), then merged
        float bm[KB], b2[KB];
#pragma unroll
        for (int b = 0; b < KB; ++b) {
            bm[b] = acc[b][0];
            b2[b] = -__builtin_inff();
#pragma unroll
            for (int v = 1; v < 16; ++v) {
                b2[b] = __builtin_amdgcn_fmed3f(bm[b], b2[b], acc[b][v]);   // b2 <= bm always: the median is the new second
                bm[b] = fmaxf(bm[b], acc[b][v]);
            }
        }
#pragma unroll
        for (int b = 0; b < KB; ++b) {
            m2 = fmaxf(fminf(mx, bm[b]), fmaxf(m2, b2[b]));
            mx = fmaxf(mx, bm[b]);
        }
        const float mxo = __shfl_xor(mx, 32, kWave), m2o = __shfl_xor(m2, 32, kWave);
        m2 = fmaxf(fminf(mx, mxo), fmaxf(m2, m2o));
    } else {
#pragma unroll
        for (int b = 0; b < KB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) mx = fmaxf(mx, acc[b][v]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
    const float x2 = xsq + __shfl_xor(xsq, 32, kWave);
    const float margin = eps * (hmax + sqrtf(x2) * cmax);
    const float thr = mx - margin;

    // Candidate bitmaps without compare-and-select chains: the sign of acc - thr is shifted into a word
    // (v_alignbit), one subtraction and one shift-in per score; the 16 bits of a block end up "1 = below".
    constexpr int NW = (KB + 1) / 2;
    uint32_t mk[NW];
#pragma unroll
    for (int i = 0; i < NW; ++i) mk[i] = 0u;
#pragma unroll
    for (int b = 0; b < KB; ++b) {
        uint32_t below = 0u;
#pragma unroll
        for (int v = 15; v >= 0; --v)
            below = __builtin_amdgcn_alignbit(below, __float_as_uint(acc[b][v] - thr), 31);   // (below << 1) | sign
        mk[b >> 1] |= (~below & 0xffffu) << ((b & 1) * 16);
    }

    // bit p of word i is codeword 64 i + 8 (p >> 2) + 4 h + (p & 3): ascending in (i, p)
    int cnt = 0, lo = 0x7fffffff;
#pragma unroll
    for (int i = NW - 1; i >= 0; --i) {
        cnt += __popc(mk[i]);
        if (mk[i]) {
            const int p = __ffs(mk[i]) - 1;
            lo = 64 * i + 8 * (p >> 2) + 4 * h + (p & 3);
        }
    }
    cnt += __shfl_xor(cnt, 32, kWave);
    lo = min(lo, __shfl_xor(lo, 32, kWave));

    if (PRUNE) {
        // d^2 = ||x'||^2 - 2 score.  With E the rounding bound of a score (half the margin): the own codeword
        // has true score >= mx - E and every other one <= m2 + E.  A vector that goes to the re-check (or has
        // no candidate) gets bounds that keep it active.  slack covers the fp32 evaluation of these lines: x2 is a
        // chain of D/2 fused multiply-adds per lane (relative error <= (D/2 + 1) 2^-24, all terms positive) and the
        // few operations below add a handful of roundings of the magnitudes involved; pa.slack = (D/2 + 16) 2^-23.
        const float E = 0.5001f * margin;
        const float slack = pa.slack * (x2 + 2.f * fabsf(mx) + 2.f * fabsf(m2));
        float u = __builtin_inff(), l = cnt >= 2 ? kAmbiguousL : 0.f;
        if (cnt == 1) {
            u = sqrtf(fmaxf(0.f, (x2 - 2.f * (mx - E)) + slack)) * 1.00001f;
            l = sqrtf(fmaxf(0.f, (x2 - 2.f * (m2 + E)) - slack)) * 0.99999f;
        }
        if (h == 0 && n < N) {
            pa.bu[n] = u;
            pa.bl[n] = l;
        }
    }

    // provisional code: the lowest candidate (final when it is the only one)
    unsigned slot = 0;
    const bool amb = (cnt >= 2) && (n < N);
    if (h == 0 && n < N) {
        codes[n * M + m] = (uint8_t)(cnt == 0 ? 0 : lo);     // cnt == 0 only with non-finite input
        if (amb) slot = atomicAdd(refine_count, 1u);
    }
    slot = __shfl(slot, lane & 31, kWave);                    // the h = 1 partner learns the slot
    if (amb) {
        RefineItem *it = list + slot;
        if (h == 0) it->n = (uint32_t)n;
#pragma unroll
        for (int i = 0; i < 4; ++i) it->mask[h][i] = (i < NW) ? mk[i] : 0u;
    }
}

// Assignment with the whole (padded) codebook resident in LDS: D <= 64 * NC_max dims such that
// 32*KB * 64*NC floats fit.  Each wave owns tiles of 32 vectors, streams them from HBM straight
// into B-operand registers in 64-dim chunks (two register sets, the next chunk in flight while
// the current one is contracted) and keeps all 32*KB scores of a vector in accumulators.
// PREFIX (with PRUNE 0): the last 64-dim chunk stops after the 8-dim steps that hold coordinates below D
// (assignments on a short prefix of the coordinates, Sec. 3.2: D = 2 costs one step, not eight).
// IMG: the LDS is filled from the image of the dictionary in its own order (k_codeword_norms, k_merge).
template <int KB, int PRUNE = 0, bool PREFIX = false, bool IMG = false>
__global__ __launch_bounds__(kAssignThreads) void k_assign_resident(
    const float *__restrict__ xp, const float *__restrict__ Cm, const float *__restrict__ hneg,
    int64_t N, int D, int ld, int K, int M, int m, int NC, float eps,
    uint8_t *__restrict__ codes, RefineItem *__restrict__ list, unsigned *__restrict__ refine_count,
    PruneArgs pa, const float4 *__restrict__ img = nullptr)
{
    extern __shared__ float4 smem4[];
    const int S = 8 * NC;
    float4 *lds_c = smem4;                                          // KB * S * 64 float4
    float *lds_h = reinterpret_cast<float *>(smem4 + KB * S * kWave);   // 32*KB floats + 2
    const int lane = lane_id();
    const int wave = threadIdx.x >> 6;
    const int h = lane >> 5;
    const int r = lane & 31;

    if (IMG) {                                                      // the image kept by k_codeword_norms / k_merge
        // every block copies the same 16 * total bytes: each starts at a place of its own, so that the blocks of
        // an XCD do not all ask the same L2 channel at the same time
        constexpr int U = 8;
        const int total = KB * S * kWave;
        const int rot = (int)(blockIdx.x & 31u) * (total >> 5);
        for (int e0 = threadIdx.x; e0 < total; e0 += U * blockDim.x) {
            float4 v[U];
            int at[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int e = e0 + u * blockDim.x;
                at[u] = e + rot < total ? e + rot : e + rot - total;
                v[u] = e < total ? img[at[u]] : make_float4(0.f, 0.f, 0.f, 0.f);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int e = e0 + u * blockDim.x;
                if (e < total) lds_c[at[u]] = v[u];
            }
        }
    } else {
        stage_codebook(lds_c, Cm, K, D, ld, KB, S);
    }
    for (int k = threadIdx.x; k < 32 * KB; k += blockDim.x) lds_h[k] = hneg[k];
    __syncthreads();
    // largest ||c||^2/2 over the real codewords (every thread computes the same value)
    float hmax = 0.f;
    for (int k = 0; k < K; ++k) hmax = fmaxf(hmax, -lds_h[k]);
    const float cmax = sqrtf(2.f * hmax) * 1.000001f;

    // Static tile schedule balanced per SIMD: waves w and w + 4 of a block share a SIMD (and its
    // matrix pipe), so tiles are dealt round-robin to the gridDim.x * 4 SIMD slots and the two
    // waves of a slot take alternate ones; no SIMD gets more than one tile above the average.
    // rows of this launch: all N vectors, or the listed ones (PRUNE 2).  When nearly all are listed the launch
    // takes all N in order instead: streaming rows beats gathering them, and a settled vector that is
    // recomputed keeps its code (its bounds prove it) and gets fresh bounds.
    const int64_t listed = PRUNE == 2 ? (int64_t)*pa.active_count : N;
    const bool gather = PRUNE == 2 && listed * 32 < N * 31;
    const int64_t rows = gather ? listed : N;
    const int64_t ntiles = (rows + kTileVec - 1) / kTileVec;
    const int64_t nslots = (int64_t)gridDim.x * 4;
    const int64_t tstride = 2 * nslots;
    const int64_t t0 = (int64_t)blockIdx.x * 4 + (wave & 3) + nslots * (wave >> 2);
    if (t0 >= ntiles) return;
    const int64_t my_tiles = (ntiles - t0 + tstride - 1) / tstride;
    const int64_t G = my_tiles * NC;                                // (tile, chunk) steps of this wave

    // vector behind column r of a tile; N (= "none") for the columns of the ragged tail
    auto vec_of = [&](int64_t tile) -> int64_t {
        const int64_t i = tile * kTileVec + r;
        if (i >= rows) return N;
        return gather ? (int64_t)pa.active[i] : i;
    };
    auto row_ptr = [&](int64_t tile) {
        int64_t n = vec_of(tile);
        if (n >= N) n = gather ? (int64_t)pa.active[rows - 1] : N - 1;   // tail columns re-read the last row
        return xp + n * ld;
    };

    floatx16 acc[KB];
    float4 xa[8], xb[8];
    float xsq = 0.f, amax = 0.f;
    int64_t tile = t0;
    int q = 0;
    const int steps_last = PREFIX ? (D - kChunkD * (NC - 1) + 7) / 8 : 8;
    auto steps_of = [&](int qq) { return (PREFIX && qq == NC - 1) ? steps_last : 8; };
    load_x_chunk<PREFIX>(xa, row_ptr(tile), 0, h, D, steps_of(0));
    // Steps come in pairs so that the two register sets alternate with static names.
    for (int64_t g = 0; g < G; g += 2) {
        // ---- step g on xa; prefetch step g+1 into xb
        int64_t tile1 = tile;
        int q1 = q + 1;
        if (q1 == NC) { q1 = 0; tile1 = tile + tstride; }
        if (g + 1 < G) load_x_chunk<PREFIX>(xb, row_ptr(tile1), q1, h, D, steps_of(q1));
        if (q == 0) { init_acc<KB>(acc, lds_h, h); xsq = 0.f; }
        mfma_chunk<KB, PREFIX>(acc, xa, lds_c, q, S, lane, xsq, amax, steps_of(q));
        if (q == NC - 1)
            decide<KB, PRUNE>(acc, xsq, eps, hmax, cmax, lane, vec_of(tile), N, M, m, codes, list, refine_count, pa);
        if (g + 1 >= G) break;
        // ---- step g+1 on xb; prefetch step g+2 into xa
        int64_t tile2 = tile1;
        int q2 = q1 + 1;
        if (q2 == NC) { q2 = 0; tile2 = tile1 + tstride; }
        if (g + 2 < G) load_x_chunk<PREFIX>(xa, row_ptr(tile2), q2, h, D, steps_of(q2));
        if (q1 == 0) { init_acc<KB>(acc, lds_h, h); xsq = 0.f; }
        mfma_chunk<KB, PREFIX>(acc, xb, lds_c, q1, S, lane, xsq, amax, steps_of(q1));
        if (q1 == NC - 1)
            decide<KB, PRUNE>(acc, xsq, eps, hmax, cmax, lane, vec_of(tile1), N, M, m, codes, list, refine_count, pa);
        tile = tile2;
        q = q2;
    }
    publish_absmax(amax, refine_count + 1);
}

// Codebook in the order the D-chunked kernel stages it: float4 (q * KB * 8 + b * 8 + s) * 64 + l, l = 32 h + r,
// holds C[32 b + r][64 q + 8 s + 4 h .. + 3] (zero beyond K and D), so that the slice of 64-dim chunk q is one
// contiguous piece already in MFMA operand order (see stage_codebook).
__global__ __launch_bounds__(256) void k_codebook_image(
    const float *__restrict__ Cm, int K, int D, int ld, int kb, int NC, float4 *__restrict__ img)
{
    const int total = NC * kb * 8 * kWave;
    for (int e = blockIdx.x * 256 + threadIdx.x; e < total; e += gridDim.x * 256) {
        const int l = e & 63;
        int bs = e >> 6;
        const int s = bs & 7;
        bs >>= 3;
        const int b = bs % kb, q = bs / kb;
        img[e] = load_row_piece(Cm, 32 * b + (l & 31), kChunkD * q + 8 * s + 4 * (l >> 5), K, D, ld);
    }
}

// One 64-dim chunk of the D-chunked kernel: contracts x (the chunk in registers) with the slice in `cur`, and
// meanwhile brings in what the next chunk needs: k-step s refills x[s] from xnext (the same columns of the
// next chunk, or of the next tile's first one) as soon as it has used it, and fetches piece s of the next
// slice (src: this thread's float4 of piece 0; pieces are 8 * 64 float4 apart) at its start and stores it to
// `nxt` at its end, with the step's MFMAs between the load and its use.
template <int KB>
__device__ __forceinline__ void mfma_chunk_refill(
    floatx16 (&acc)[KB], float4 (&x)[8], const float4 *__restrict__ cur, float4 *__restrict__ nxt,
    const float4 *__restrict__ src, const float *__restrict__ xnext, int q, int qn, int D, int lane, int wave,
    float &xsq, float &amax)
{
    const int h = lane >> 5;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        float4 piece = make_float4(0.f, 0.f, 0.f, 0.f);
        if (s < KB) piece = src[s * 8 * kWave];
        float4 a[KB];
#pragma unroll
        for (int b = 0; b < KB; ++b) a[b] = cur[(b * 8 + s) * kWave + lane];
        // columns past D (last chunk only) are zeroed here, at use: the refill itself is unconditional (its
        // address clamped into the row), so that no branch hides from the compiler which loads are in flight
        float4 xv = x[s];
        if (kChunkD * q + 8 * s + 4 * h >= D) xv = make_float4(0.f, 0.f, 0.f, 0.f);
        x[s] = *reinterpret_cast<const float4 *>(xnext + min(kChunkD * qn + 8 * s + 4 * h, last_piece(D)));
        xsq = fmaf(xv.x, xv.x, xsq);
        xsq = fmaf(xv.y, xv.y, xsq);
        xsq = fmaf(xv.z, xv.z, xsq);
        xsq = fmaf(xv.w, xv.w, xsq);
        amax = fmaxf(fmaxf(amax, fabsf(xv.x)), fabsf(xv.y));
        amax = fmaxf(fmaxf(amax, fabsf(xv.z)), fabsf(xv.w));
#pragma unroll
        for (int b = 0; b < KB; ++b) acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[b].x, xv.x, acc[b], 0, 0, 0);
#pragma unroll
        for (int b = 0; b < KB; ++b) acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[b].y, xv.y, acc[b], 0, 0, 0);
#pragma unroll
        for (int b = 0; b < KB; ++b) acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[b].z, xv.z, acc[b], 0, 0, 0);
        // the store (and the wait for its load) stays behind three quarters of the step's MFMAs; arithmetic,
        // MFMAs and LDS reads of the next step may still move across
        __builtin_amdgcn_sched_barrier(0x10f);
        if (s < KB) nxt[(s * 8 + wave) * kWave + lane] = piece;
#pragma unroll
        for (int b = 0; b < KB; ++b) acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[b].w, xv.w, acc[b], 0, 0, 0);
    }
}

// Assignment for dimensions whose codebook does not fit LDS: the block walks the D axis in 64-dim chunks for
// every tile of 8 x 32 vectors, the accumulators persisting across chunks.  Two LDS buffers hold the slice in
// use and the one being brought in from the codebook image (k_codebook_image), one barrier per chunk; the
// refills run under the MFMAs (mfma_chunk_refill), across tile boundaries too.
template <int KB, int PRUNE = 0>
__global__ __launch_bounds__(kAssignThreads) void k_assign_chunked(
    const float *__restrict__ xp, const float4 *__restrict__ img, const float *__restrict__ hneg,
    int64_t N, int D, int ld, int K, int M, int m, int NC, float eps,
    uint8_t *__restrict__ codes, RefineItem *__restrict__ list, unsigned *__restrict__ refine_count,
    PruneArgs pa)
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
    // slice 0 (the same for every tile)
    const float4 *mine = img + wave * kWave + lane;
#pragma unroll
    for (int p = 0; p < KB; ++p) buf0[(p * 8 + wave) * kWave + lane] = mine[p * 8 * kWave];
    __syncthreads();
    float hmax = 0.f;
    for (int k = 0; k < K; ++k) hmax = fmaxf(hmax, -lds_h[k]);
    const float cmax = sqrtf(2.f * hmax) * 1.000001f;

    // rows of this launch: all N vectors, or the listed ones (PRUNE 2; see PruneArgs)
    // (nearly all listed: all N in order, as in k_assign_resident)
    const int64_t listed = PRUNE == 2 ? (int64_t)*pa.active_count : N;
    const bool gather = PRUNE == 2 && listed * 32 < N * 31;
    const int64_t rows = gather ? listed : N;
    const int64_t nbt = (rows + kTileVec * kAssignWaves - 1) / (kTileVec * kAssignWaves);   // block tiles
    float amax = 0.f;
    if ((int64_t)blockIdx.x < nbt) {
        // row of x' this lane feeds for block tile bt (tail columns re-read the last row); vec = N for "none"
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
        for (int s = 0; s < 8; ++s) x[s] = *reinterpret_cast<const float4 *>(xrow + min(8 * s + 4 * h, last_piece(D)));
        int par = 0;
        for (int64_t bt = blockIdx.x; bt < nbt; bt += gridDim.x) {
            int64_t vec_next = vec;
            const float *xrow_next = xrow;                          // the last tile refills with itself: unused
            if (bt + gridDim.x < nbt) xrow_next = tile_row(bt + gridDim.x, vec_next);
            floatx16 acc[KB];
            float xsq = 0.f;
            init_acc<KB>(acc, lds_h, h);
            for (int q = 0; q < NC; ++q) {
                const bool last = q + 1 == NC;
                const int qn = last ? 0 : q + 1;
                mfma_chunk_refill<KB>(acc, x, par ? buf1 : buf0, par ? buf0 : buf1, mine + (size_t)qn * CH,
                                      last ? xrow_next : xrow, q, qn, D, lane, wave, xsq, amax);
                __syncthreads();                                    // slice q consumed by all, slice qn complete
                par ^= 1;
            }
            decide<KB, PRUNE>(acc, xsq, eps, hmax, cmax, lane, vec, N, M, m, codes, list, refine_count, pa);
            xrow = xrow_next;
            vec = vec_next;
        }
    }
    publish_absmax(amax, refine_count + 1);
}

// Between two assignments of a stage: age the bounds by the drift of the dictionary (drift[k] >= the
// distance codeword k moved in the centroid update, 0 for a kept one) and list the vectors that have to be
// recomputed.  A block takes kBoundSpan consecutive vectors, stages its entries in LDS and claims its stretch
// of the list with one counter add (*count must be zero on entry; order is free).
//
// One codeword that moves far (a cluster of few members) costs every vector its lower bound.  When the
// largest drift stands out from the (kVolatile+1)-th, the block looks again at those of its unsettled vectors
// that the drift of the REST alone would leave settled (if they are many), with the kVolatile codewords that
// moved most treated apart: the lower bound ages by the largest drift of the rest, and the distance to each of
// those few is computed afresh from x' (expanded form in fp32 with its rounding bound) and joins the lower bound.
// Vectors that this settles get their aged bounds and leave the list.  Eight lanes share a vector.
// Dynamic LDS: kVolatile rows of D floats.
constexpr int kBoundSpan = 4096;
constexpr int kBoundThreads = 1024;
__global__ __launch_bounds__(kBoundThreads) void k_bounds_step(
    const uint8_t *__restrict__ codes, int64_t N, int M, int m, const float *__restrict__ drift, int K,
    float *__restrict__ bu, float *__restrict__ bl, uint32_t *__restrict__ list, unsigned *__restrict__ count,
    const float *__restrict__ xp, int D, const float *__restrict__ Cm)
{
    extern __shared__ float4 smem4[];
    float *vrow = reinterpret_cast<float *>(smem4);
    __shared__ uint32_t found[kBoundSpan], kept[kBoundSpan];
    __shared__ float sdrift[256];
    __shared__ unsigned nfound, nkept, base;
    __shared__ float s_vnorm[kVolatile], s_top[kVolatile + 1];
    __shared__ int s_tk[kVolatile + 1];
    if (threadIdx.x < 256) sdrift[threadIdx.x] = (int)threadIdx.x < K ? drift[threadIdx.x] : 0.f;
    if (threadIdx.x == 0) { nfound = 0u; nkept = 0u; }
    const int64_t n0 = (int64_t)blockIdx.x * kBoundSpan;
    constexpr int U = kBoundSpan / kBoundThreads;
    int c[U];
    float u[U], l[U];
#pragma unroll
    for (int j = 0; j < U; ++j) {                                   // all loads first: in flight during the ranking
        const int64_t n = n0 + j * kBoundThreads + threadIdx.x;
        const int64_t nn = n < N ? n : N - 1;
        c[j] = codes[nn * M + m];
        u[j] = bu[nn];
        l[j] = bl[nn];
    }
    __syncthreads();
    top_drifts(sdrift, K, s_top, s_tk);
    const float d1 = s_top[0], d2 = s_top[1], drest = s_top[kVolatile];
    const int k1 = s_tk[0];
    // The second look can only settle a vector whose upper bound stays below its lower bound aged by the drift
    // of the rest: the others are kept without it (found: worth the second look; kept: to recompute).
    const bool outlier = K > kVolatile + 1 && d1 > 3.0f * drest;
    {
#pragma unroll
        for (int j = 0; j < U; ++j) {
            const int64_t n = n0 + j * kBoundThreads + threadIdx.x;
            if (n < N) {
                const float un = (u[j] + sdrift[c[j]]) * 1.000001f;  // rounded up
                const float ln = (l[j] - ((c[j] == k1) ? d2 : d1)) * 0.999999f;   // rounded down while positive
                if (un < ln) {
                    bu[n] = un;
                    bl[n] = ln;
                } else if (outlier && un < (l[j] - drest) * 0.999999f) {
                    found[atomicAdd(&nfound, 1u)] = (uint32_t)n;      // its bounds stay as they were
                } else {
                    kept[atomicAdd(&nkept, 1u)] = (uint32_t)n;        // likewise
                }
            }
        }
    }
    __syncthreads();
    const unsigned nf = nfound;
    // worth a gather of those rows of x'?
    const bool apart = nf * 8u > (unsigned)kBoundSpan;
    if (!apart) {
        const unsigned nk0 = nkept;
        if (threadIdx.x == 0 && nf + nk0) base = atomicAdd(count, nf + nk0);
        __syncthreads();
        for (unsigned i = threadIdx.x; i < nk0; i += kBoundThreads) list[base + i] = kept[i];
        for (unsigned i = threadIdx.x; i < nf; i += kBoundThreads) list[base + nk0 + i] = found[i];
        return;
    }
    for (int e = threadIdx.x; e < kVolatile * D; e += kBoundThreads) {
        const int j = e / D;
        vrow[e] = s_tk[j] >= 0 ? Cm[(size_t)s_tk[j] * D + (e - j * D)] : 0.f;
    }
    __syncthreads();
    {
        const int w = threadIdx.x >> 6;                             // the first kVolatile waves, one row each
        if (w < kVolatile) {
            double q = 0.0;
            for (int d = lane_id(); d < D; d += kWave) q += (double)vrow[w * D + d] * (double)vrow[w * D + d];
            q = wave_sum(q);
            if (lane_id() == 0) s_vnorm[w] = (float)q;
        }
    }
    __syncthreads();
    const int sub = threadIdx.x & 7;
    const int d4n = D >> 2;
    // fp32 rounding of ||x'||^2 - 2 x'.c + ||c||^2 (D/8 chained fmas per lane, three shuffle adds, the final
    // sums) as a fraction of ||x'||^2 + 2|x'.c| + ||c||^2
    const float slack = (float)(D / 8 + 8) * 1.2e-7f;
    for (unsigned i0 = 0; i0 < nf; i0 += kBoundThreads / 8) {
        const unsigned e = i0 + (threadIdx.x >> 3);
        const bool ok = e < nf;
        const int64_t n = found[ok ? e : nf - 1];
        const float4 *row = reinterpret_cast<const float4 *>(xp + n * D);
        float x2 = 0.f, dot[kVolatile];
#pragma unroll
        for (int j = 0; j < kVolatile; ++j) dot[j] = 0.f;
#pragma unroll 4
        for (int q = sub; q < d4n; q += 8) {
            const float4 x = row[q];
            x2 = fmaf(x.x, x.x, fmaf(x.y, x.y, fmaf(x.z, x.z, fmaf(x.w, x.w, x2))));
#pragma unroll
            for (int j = 0; j < kVolatile; ++j) {
                const float4 c = *reinterpret_cast<const float4 *>(vrow + j * D + 4 * q);
                dot[j] = fmaf(x.x, c.x, fmaf(x.y, c.y, fmaf(x.z, c.z, fmaf(x.w, c.w, dot[j]))));
            }
        }
#pragma unroll
        for (int o = 1; o < 8; o <<= 1) {
            x2 += __shfl_xor(x2, o, kWave);
#pragma unroll
            for (int j = 0; j < kVolatile; ++j) dot[j] += __shfl_xor(dot[j], o, kWave);
        }
        if (ok && sub == 0) {
            const int c = codes[n * M + m];
            const float u = (bu[n] + sdrift[c]) * 1.000001f;
            float l = (bl[n] - drest) * 0.999999f;                   // the rest moved by at most drest
#pragma unroll
            for (int j = 0; j < kVolatile; ++j) {
                if (s_tk[j] >= 0 && s_tk[j] != c) {
                    const float mag = x2 + 2.f * fabsf(dot[j]) + s_vnorm[j];
                    const float dj2 = (x2 - 2.f * dot[j] + s_vnorm[j]) - slack * mag;
                    l = fminf(l, sqrtf(fmaxf(dj2, 0.f)) * 0.999999f);
                }
            }
            if (u < l) {
                bu[n] = u;
                bl[n] = l;
            } else {
                kept[atomicAdd(&nkept, 1u)] = (uint32_t)n;
            }
        }
    }
    __syncthreads();
    const unsigned nk = nkept;
    if (threadIdx.x == 0 && nk) base = atomicAdd(count, nk);
    __syncthreads();
    for (unsigned i = threadIdx.x; i < nk; i += kBoundThreads) list[base + i] = kept[i];
}

// ---- Distance bounds carried from one sweep to the next (several sweeps in one call, plain Lloyd cool-down) ----
// When a sweep comes back to stage m, C_m and column m of the codes are as the stage's last visit left them
// (Sec. 3.1: a stage changes its own dictionary and code only); x' alone has moved, in exact arithmetic by
//   x'_new - x'_old = - sum over the stages j visited in between of d_j,   d_j = c_j,new(i_j,new) - c_j,old(i_j,old),
// the change of stage j's part of the reconstruction.  The bounds the last visit ended with therefore still hold
// once the upper one has grown and the lower one has shrunk by delta >= ||x'_new - x'_old||, and a vector they still
// settle keeps its code without being assigned again.  delta is taken per vector as the sum of ||d_j|| (triangle
// inequality), read from a K x K table per stage, plus a bound on the fp32 roundings of the passes in between:
// 2M results of magnitude <= 2A per coordinate (A = largest |x'| or |codeword| coordinate seen), each off by at
// most 2^-24 of itself, i.e. at most 3M 2^-24 sqrt(D) A in norm; (8M + 16) 2^-24 sqrt(D) A is used.

// T[a][b] = ||C_now[b] - C_entry[a]||, rounded up: how far the reconstruction part of a vector moved whose code went
// from a (dictionary as the stage found it) to b (as it leaves it).  One block per a; dynamic LDS: D floats.
__global__ __launch_bounds__(256) void k_pair_table(
    const float *__restrict__ Centry, const float *__restrict__ Cm, int K, int D, float *__restrict__ T)
{
    extern __shared__ float4 smem4[];
    const int a = blockIdx.x;
    const int d4 = D >> 2;
    for (int d = threadIdx.x; d < d4; d += 256) smem4[d] = reinterpret_cast<const float4 *>(Centry + (size_t)a * D)[d];
    __syncthreads();
    // a thread per b: its row of the dictionary against the row in LDS (every lane reads the same LDS address)
    for (int b = threadIdx.x; b < K; b += 256) {
        const float4 *cb = reinterpret_cast<const float4 *>(Cm + (size_t)b * D);
        double s0 = 0.0, s1 = 0.0;
#pragma unroll 4
        for (int d = 0; d < d4; ++d) {
            const float4 x = cb[d], y = smem4[d];
            const double t0 = (double)x.x - (double)y.x, t1 = (double)x.y - (double)y.y;
            const double t2 = (double)x.z - (double)y.z, t3 = (double)x.w - (double)y.w;
            s0 += t0 * t0 + t2 * t2;
            s1 += t1 * t1 + t3 * t3;
        }
        T[(size_t)a * K + b] = (float)(sqrt(s0 + s1) * 1.000001);
    }
}

// End of stage m: path[n] += T[code at entry][code now]; snap[n] = path[n] (the stage's mark on the running path
// length: when it is visited again, path - snap is the sum of ||d_j|| over the stages in between).  Also folds the
// stage's max |x'| (refine_count[1]) into the running maximum.
__global__ __launch_bounds__(256) void k_path_step(
    const uint8_t *__restrict__ entry, const uint8_t *__restrict__ codes, int64_t N, int M, int m,
    const float *__restrict__ T, int K, double *__restrict__ path, double *__restrict__ snap,
    unsigned *__restrict__ refine_count, unsigned *__restrict__ amax_run)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        const unsigned a = refine_count[1];
        if (a > *amax_run) *amax_run = a;
    }
    for (int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x; n < N; n += (int64_t)gridDim.x * 256) {
        const double s = path[n] + (double)T[(size_t)entry[n] * K + codes[n * M + m]];
        path[n] = s;
        snap[n] = s;
    }
}

// Entry of a stage whose bounds were kept: widen them by delta and list the vectors they no longer settle
// (*count must be zero on entry; order is free), as k_bounds_step does after a centroid update.
__global__ __launch_bounds__(kBoundThreads) void k_bounds_carry(
    const double *__restrict__ path, const double *__restrict__ snap, int64_t N, double slack_unit,
    const unsigned *__restrict__ amax_run, const unsigned *__restrict__ amax_now,
    float *__restrict__ bu, float *__restrict__ bl, uint32_t *__restrict__ list, unsigned *__restrict__ count)
{
    __shared__ uint32_t kept[kBoundSpan];
    __shared__ unsigned nkept, base;
    if (threadIdx.x == 0) nkept = 0u;
    __syncthreads();
    const unsigned abits = max(*amax_run, *amax_now);
    const double slack = slack_unit * (double)__uint_as_float(abits);
    const int64_t n0 = (int64_t)blockIdx.x * kBoundSpan;
    constexpr int U = kBoundSpan / kBoundThreads;
#pragma unroll
    for (int j = 0; j < U; ++j) {
        const int64_t n = n0 + j * kBoundThreads + threadIdx.x;
        if (n < N) {
            const double delta = (path[n] - snap[n]) * (1.0 + 1e-9) + slack;
            const float un = (float)((double)bu[n] + delta) * 1.000001f;    // rounded up
            const float ln = (float)((double)bl[n] - delta) * 0.999999f;    // rounded down while positive
            if (un < ln) {
                bu[n] = un;
                bl[n] = ln;
            } else {
                kept[atomicAdd(&nkept, 1u)] = (uint32_t)n;                  // its bounds stay; the assignment renews them
            }
        }
    }
    __syncthreads();
    const unsigned nk = nkept;
    if (threadIdx.x == 0 && nk) base = atomicAdd(count, nk);
    __syncthreads();
    for (unsigned i = threadIdx.x; i < nk; i += kBoundThreads) list[base + i] = kept[i];
}

__global__ void k_zero_words(unsigned *__restrict__ p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

constexpr int kMovedSpan = 1024;
// fp64 re-check of the vectors whose fp32 scores were too close to call: direct-form squared
// distances summed in ascending dimension order, smallest wins, exact ties go to the lowest
// index.  A group of kRefineLanes lanes takes one list entry and gives each candidate its own lane (most
// entries have two or three candidates; more take further rounds).
constexpr int kRefineLanes = 4;
__global__ __launch_bounds__(256) void k_refine(
    const float *__restrict__ xp, const float *__restrict__ Cm, int D, int ld, int M, int m,
    uint8_t *__restrict__ codes, const RefineItem *__restrict__ list,
    const unsigned *__restrict__ refine_count, MovedArgs mv,
    unsigned long long *__restrict__ work, unsigned long long rows, const unsigned *__restrict__ rows_listed)
{
    __shared__ unsigned long long found[kMovedSpan];
    __shared__ unsigned nfound, base;
    const unsigned count = *refine_count;
    // Work counters of the ctx (read by hclae_work_counters): assignments run, vectors they recomputed, vectors that
    // went to this re-check.  Launches on one stream follow one another, so one thread may add without atomics.
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        work[0] += 1ull;
        work[1] += rows_listed ? (unsigned long long)*rows_listed : rows;
        work[2] += count;
    }
    // With the moved-vector list wanted, the two jobs run side by side: the first half of the blocks re-checks,
    // the second half scans the other recomputed vectors (below).
    const unsigned nr = mv.prev ? gridDim.x / 2 : gridDim.x;        // blocks that re-check
    const bool scans = blockIdx.x >= nr;
    // re-checked vectors that changed cluster are staged in LDS like the others while a block's share fits
    const bool staged = count <= nr * (unsigned)kMovedSpan;
    if (mv.prev) {
        if (threadIdx.x == 0) nfound = 0u;
        __syncthreads();
    }
    const int l16 = threadIdx.x & (kRefineLanes - 1);
    const unsigned groups = nr * (256 / kRefineLanes);
    const int d4 = D >> 2;
    for (unsigned e = scans ? count : blockIdx.x * (256 / kRefineLanes) + threadIdx.x / kRefineLanes; e < count;
         e += groups) {
        const RefineItem it = list[e];
        int total = 0;
#pragma unroll
        for (int w = 0; w < 8; ++w) total += __popc(it.mask[w >> 2][w & 3]);
        const float4 *x = reinterpret_cast<const float4 *>(xp + (size_t)it.n * ld);
        double best = __builtin_inf();
        int kbest = 0x7fffffff;
        for (int first = 0; first < total; first += kRefineLanes) {
            int j = first + l16;
            if (j < total) {
                // codeword of the j-th set bit
                int k = 0;
#pragma unroll
                for (int w = 0; w < 8; ++w) {
                    uint32_t bits = it.mask[w >> 2][w & 3];
                    const int c = __popc(bits);
                    if (j >= 0 && j < c) {
                        for (int q = 0; q < j; ++q) bits &= bits - 1;
                        const int p = __ffs(bits) - 1;
                        k = 64 * (w & 3) + 8 * (p >> 2) + 4 * (w >> 2) + (p & 3);
                        j = -1;
                    } else if (j >= 0) {
                        j -= c;
                    }
                }
                const float4 *c4 = reinterpret_cast<const float4 *>(Cm + (size_t)k * ld);
                double s = 0.0;
                // unrolled so that eight rounds of loads are in flight; the additions keep their order
#pragma unroll 8
                for (int d = 0; d < d4; ++d) {
                    const float4 a = x[d], b = c4[d];
                    const double t0 = (double)a.x - (double)b.x, t1 = (double)a.y - (double)b.y;
                    const double t2 = (double)a.z - (double)b.z, t3 = (double)a.w - (double)b.w;
                    s += t0 * t0;
                    s += t1 * t1;
                    s += t2 * t2;
                    s += t3 * t3;
                }
                for (int d = 4 * d4; d < D; ++d) {                  // D need not be a multiple of 4
                    const double t = (double)reinterpret_cast<const float *>(x)[d] - (double)reinterpret_cast<const float *>(c4)[d];
                    s += t * t;
                }
                if (s < best || (s == best && k < kbest)) { best = s; kbest = k; }
            }
        }
#pragma unroll
        for (int o = kRefineLanes / 2; o > 0; o >>= 1) {
            const double ob = __shfl_xor(best, o, kWave);
            const int ok = __shfl_xor(kbest, o, kWave);
            if (ob < best || (ob == best && ok < kbest)) { best = ob; kbest = ok; }
        }
        if (l16 == 0) {
            codes[(size_t)it.n * M + m] = (uint8_t)kbest;
            if (mv.prev) {
                const unsigned co = mv.prev[it.n];
                if (co != (unsigned)kbest) {
                    mv.prev[it.n] = (uint8_t)kbest;
                    const unsigned long long ent =
                        (unsigned long long)it.n | ((unsigned long long)co << 32) | ((unsigned long long)kbest << 40);
                    if (staged) found[atomicAdd(&nfound, 1u)] = ent;
                    else mv.list[atomicAdd(mv.count, 1u)] = ent;
                }
            }
        }
    }
    if (!mv.prev) return;
    if (!scans) {
        __syncthreads();
        if (threadIdx.x == 0 && nfound) base = atomicAdd(mv.count, nfound);
        __syncthreads();
        for (unsigned i = threadIdx.x; i < nfound; i += 256) mv.list[base + i] = found[i];
        return;
    }
    // The other recomputed vectors have their final code already.  A block takes kMovedSpan list entries at a
    // time, stages what it finds in LDS and claims its stretch of the output with one counter add.
    const int64_t total = (int64_t)*mv.cand_count;
    const int64_t ns = gridDim.x - nr;                              // blocks that scan
    for (int64_t i0 = (int64_t)(blockIdx.x - nr) * kMovedSpan; i0 < total; i0 += ns * kMovedSpan) {
        if (threadIdx.x == 0) nfound = 0u;
        __syncthreads();
#pragma unroll
        for (int i = threadIdx.x; i < kMovedSpan; i += 256) {
            const int64_t j = i0 + i;
            if (j < total) {
                const int64_t n = mv.cand[j];
                if (mv.bl[n] != kAmbiguousL) {
                    const unsigned cn = codes[n * M + m], co = mv.prev[n];
                    if (cn != co) {
                        mv.prev[n] = (uint8_t)cn;
                        found[atomicAdd(&nfound, 1u)] =
                            (unsigned long long)(uint32_t)n | ((unsigned long long)co << 32) | ((unsigned long long)cn << 40);
                    }
                }
            }
        }
        __syncthreads();
        if (threadIdx.x == 0 && nfound) base = atomicAdd(mv.count, nfound);
        __syncthreads();
        for (unsigned i = threadIdx.x; i < nfound; i += 256) mv.list[base + i] = found[i];
        __syncthreads();
    }
}

}  // namespace hclae
