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

// -||c_k||^2 / 2 in fp32 (computed in fp64) over the first D coordinates of rows of stride ld, for
// k < K; -inf for the padding rows up to kpad.
// One wave per codeword.  Also resets the two counters the assign that follows will fill
// (refine_count[0]: re-check entries, refine_count[1]: bits of max |x'|).
__global__ __launch_bounds__(256) void k_codeword_norms(
    const float *__restrict__ Cm, int K, int D, int ld, int kpad, float *__restrict__ hneg,
    unsigned *__restrict__ refine_count, int keep_absmax)
{
    const int lane = lane_id();
    const int k = blockIdx.x * (256 / kWave) + (threadIdx.x >> 6);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        refine_count[0] = 0u;                      // re-check entries
        if (!keep_absmax) refine_count[1] = 0u;    // bits of max |x'|
    }
    if (k >= kpad) return;
    if (k >= K) {
        if (lane == 0) hneg[k] = -__builtin_inff();
        return;
    }
    const float *c = Cm + (size_t)k * ld;
    double s = 0.0;
    for (int d = lane; d < D; d += kWave) s += (double)c[d] * (double)c[d];
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
__device__ __forceinline__ void load_x_chunk(
    float4 (&x)[8], const float *__restrict__ xrow, int q, int h, int D)
{
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        const int col = kChunkD * q + 8 * s + 4 * h;
        x[s] = (col < D) ? *reinterpret_cast<const float4 *>(xrow + col) : make_float4(0.f, 0.f, 0.f, 0.f);
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

template <int KB>
__device__ __forceinline__ void mfma_chunk(
    floatx16 (&acc)[KB], const float4 (&x)[8], const float4 *__restrict__ lds, int q, int S, int lane,
    float &xsq, float &amax)
{
#pragma unroll
    for (int s = 0; s < 8; ++s) {
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
template <int KB>
__device__ __forceinline__ void decide(
    const floatx16 (&acc)[KB], float xsq, float eps, float hmax, float cmax, int lane,
    int64_t n, int64_t N, int M, int m, uint8_t *__restrict__ codes,
    RefineItem *__restrict__ list, unsigned *__restrict__ refine_count)
{
    const int h = lane >> 5;
    float mx = -__builtin_inff();
#pragma unroll
    for (int b = 0; b < KB; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) mx = fmaxf(mx, acc[b][v]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
    const float x2 = xsq + __shfl_xor(xsq, 32, kWave);
    const float thr = mx - eps * (hmax + sqrtf(x2) * cmax);

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
template <int KB>
__global__ __launch_bounds__(kAssignThreads) void k_assign_resident(
    const float *__restrict__ xp, const float *__restrict__ Cm, const float *__restrict__ hneg,
    int64_t N, int D, int ld, int K, int M, int m, int NC, float eps,
    uint8_t *__restrict__ codes, RefineItem *__restrict__ list, unsigned *__restrict__ refine_count)
{
    extern __shared__ float4 smem4[];
    const int S = 8 * NC;
    float4 *lds_c = smem4;                                          // KB * S * 64 float4
    float *lds_h = reinterpret_cast<float *>(smem4 + KB * S * kWave);   // 32*KB floats + 2
    const int lane = lane_id();
    const int wave = threadIdx.x >> 6;
    const int h = lane >> 5;
    const int r = lane & 31;

    stage_codebook(lds_c, Cm, K, D, ld, KB, S);
    for (int k = threadIdx.x; k < 32 * KB; k += blockDim.x) lds_h[k] = hneg[k];
    __syncthreads();
    // largest ||c||^2/2 over the real codewords (every thread computes the same value)
    float hmax = 0.f;
    for (int k = 0; k < K; ++k) hmax = fmaxf(hmax, -lds_h[k]);
    const float cmax = sqrtf(2.f * hmax) * 1.000001f;

    // Static tile schedule balanced per SIMD: waves w and w + 4 of a block share a SIMD (and its
    // matrix pipe), so tiles are dealt round-robin to the gridDim.x * 4 SIMD slots and the two
    // waves of a slot take alternate ones; no SIMD gets more than one tile above the average.
    const int64_t ntiles = (N + kTileVec - 1) / kTileVec;
    const int64_t nslots = (int64_t)gridDim.x * 4;
    const int64_t tstride = 2 * nslots;
    const int64_t t0 = (int64_t)blockIdx.x * 4 + (wave & 3) + nslots * (wave >> 2);
    if (t0 >= ntiles) return;
    const int64_t my_tiles = (ntiles - t0 + tstride - 1) / tstride;
    const int64_t G = my_tiles * NC;                                // (tile, chunk) steps of this wave

    auto row_ptr = [&](int64_t tile) {
        int64_t n = tile * kTileVec + r;
        if (n >= N) n = N - 1;                                      // tail rows re-read the last vector
        return xp + n * ld;
    };

    floatx16 acc[KB];
    float4 xa[8], xb[8];
    float xsq = 0.f, amax = 0.f;
    int64_t tile = t0;
    int q = 0;
    load_x_chunk(xa, row_ptr(tile), 0, h, D);
    // Steps come in pairs so that the two register sets alternate with static names.
    for (int64_t g = 0; g < G; g += 2) {
        // ---- step g on xa; prefetch step g+1 into xb
        int64_t tile1 = tile;
        int q1 = q + 1;
        if (q1 == NC) { q1 = 0; tile1 = tile + tstride; }
        if (g + 1 < G) load_x_chunk(xb, row_ptr(tile1), q1, h, D);
        if (q == 0) { init_acc<KB>(acc, lds_h, h); xsq = 0.f; }
        mfma_chunk<KB>(acc, xa, lds_c, q, S, lane, xsq, amax);
        if (q == NC - 1)
            decide<KB>(acc, xsq, eps, hmax, cmax, lane, tile * kTileVec + r, N, M, m, codes, list, refine_count);
        if (g + 1 >= G) break;
        // ---- step g+1 on xb; prefetch step g+2 into xa
        int64_t tile2 = tile1;
        int q2 = q1 + 1;
        if (q2 == NC) { q2 = 0; tile2 = tile1 + tstride; }
        if (g + 2 < G) load_x_chunk(xa, row_ptr(tile2), q2, h, D);
        if (q1 == 0) { init_acc<KB>(acc, lds_h, h); xsq = 0.f; }
        mfma_chunk<KB>(acc, xb, lds_c, q1, S, lane, xsq, amax);
        if (q1 == NC - 1)
            decide<KB>(acc, xsq, eps, hmax, cmax, lane, tile1 * kTileVec + r, N, M, m, codes, list, refine_count);
        tile = tile2;
        q = q2;
    }
    publish_absmax(amax, refine_count + 1);
}

// Assignment for dimensions whose codebook does not fit LDS: the block walks the D axis in
// 64-dim chunks, restaging that slice of the codebook for every tile of 8 x 32 vectors; the
// accumulators persist across chunks.
template <int KB>
__global__ __launch_bounds__(kAssignThreads) void k_assign_chunked(
    const float *__restrict__ xp, const float *__restrict__ Cm, const float *__restrict__ hneg,
    int64_t N, int D, int ld, int K, int M, int m, int NC, float eps,
    uint8_t *__restrict__ codes, RefineItem *__restrict__ list, unsigned *__restrict__ refine_count)
{
    extern __shared__ float4 smem4[];
    constexpr int S = 8;                                            // one chunk resident
    float4 *lds_c = smem4;                                          // KB * 8 * 64 float4
    float *lds_h = reinterpret_cast<float *>(smem4 + KB * S * kWave);
    const int lane = lane_id();
    const int wave = threadIdx.x >> 6;
    const int h = lane >> 5;
    const int r = lane & 31;

    for (int k = threadIdx.x; k < 32 * KB; k += blockDim.x) lds_h[k] = hneg[k];
    __syncthreads();
    float hmax = 0.f;
    for (int k = 0; k < K; ++k) hmax = fmaxf(hmax, -lds_h[k]);
    const float cmax = sqrtf(2.f * hmax) * 1.000001f;

    const int64_t nbt = (N + kTileVec * kAssignWaves - 1) / (kTileVec * kAssignWaves);   // block tiles
    float amax = 0.f;
    for (int64_t bt = blockIdx.x; bt < nbt; bt += gridDim.x) {
        const int64_t n_raw = (bt * kAssignWaves + wave) * kTileVec + r;
        const int64_t n = n_raw < N ? n_raw : N - 1;
        const float *xrow = xp + n * ld;
        floatx16 acc[KB];
        float4 x[8];
        float xsq = 0.f;
        init_acc<KB>(acc, lds_h, h);
        for (int q = 0; q < NC; ++q) {
            load_x_chunk(x, xrow, q, h, D);
            __syncthreads();                                        // previous chunk fully consumed
            // slice [64q, 64q+64) of the codebook, as chunk 0 of an S = 8 image
            for (int e = threadIdx.x; e < KB * S * kWave; e += blockDim.x) {
                const int l = e & 63;
                const int bs = e >> 6;
                const int s = bs & 7;
                const int b = bs >> 3;
                const int row = 32 * b + (l & 31);
                const int col = kChunkD * q + 8 * s + 4 * (l >> 5);
                lds_c[e] = load_row_piece(Cm, row, col, K, D, ld);
            }
            __syncthreads();
            mfma_chunk<KB>(acc, x, lds_c, 0, S, lane, xsq, amax);
        }
        decide<KB>(acc, xsq, eps, hmax, cmax, lane, n_raw, N, M, m, codes, list, refine_count);
    }
    publish_absmax(amax, refine_count + 1);
}

// fp64 re-check of the vectors whose fp32 scores were too close to call: direct-form squared
// distances summed in ascending dimension order, smallest wins, exact ties go to the lowest
// index.  A group of 16 lanes takes one list entry and gives each candidate its own lane.
__global__ __launch_bounds__(256) void k_refine(
    const float *__restrict__ xp, const float *__restrict__ Cm, int D, int ld, int M, int m,
    uint8_t *__restrict__ codes, const RefineItem *__restrict__ list,
    const unsigned *__restrict__ refine_count)
{
    const unsigned count = *refine_count;
    const int l16 = threadIdx.x & 15;
    const unsigned groups = gridDim.x * (256 / 16);
    const int d4 = D >> 2;
    for (unsigned e = blockIdx.x * (256 / 16) + (threadIdx.x >> 4); e < count; e += groups) {
        const RefineItem it = list[e];
        int total = 0;
#pragma unroll
        for (int w = 0; w < 8; ++w) total += __popc(it.mask[w >> 2][w & 3]);
        const float4 *x = reinterpret_cast<const float4 *>(xp + (size_t)it.n * ld);
        double best = __builtin_inf();
        int kbest = 0x7fffffff;
        for (int base = 0; base < total; base += 16) {
            int j = base + l16;
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
        for (int o = 8; o > 0; o >>= 1) {
            const double ob = __shfl_xor(best, o, kWave);
            const int ok = __shfl_xor(kbest, o, kWave);
            if (ob < best || (ob == best && ok < kbest)) { best = ob; kbest = ok; }
        }
        if (l16 == 0) codes[(size_t)it.n * M + m] = (uint8_t)kbest;
    }
}

}  // namespace hclae
