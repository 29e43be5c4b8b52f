// Shared device helpers for the DA kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hclae {

constexpr int kWave = 64;

typedef float floatx16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

// Butterfly sum over the 64 lanes of a wave; every lane ends with the same value
// (each step adds the same two operands on both partners, so the result is lane-independent).
__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

__device__ __forceinline__ long long wave_sum_ll(long long v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

// Block sum in a fixed order: wave butterflies, then wave 0 adds the per-wave values
// in ascending wave order.  `scratch` holds >= blockDim.x/64 doubles.  Result valid in thread 0.
__device__ __forceinline__ double block_sum(double v, double *scratch)
{
    v = wave_sum(v);
    const int w = threadIdx.x >> 6;
    if (lane_id() == 0) scratch[w] = v;
    __syncthreads();
    double t = 0.0;
    if (threadIdx.x == 0) {
        const int nw = (blockDim.x + kWave - 1) >> 6;
        for (int i = 0; i < nw; ++i) t += scratch[i];
    }
    __syncthreads();
    return t;
}

// Float index of coordinate d of codeword k in the LDS order of the resident assign kernels: for row block b = k / 32,
// k-step s = d / 8 (S steps a row) and lane l = 32 * (d / 4 % 2) + k % 32, the float4 at (b * S + s) * 64 + l holds
// C[k][8 s + 4 h .. + 3].
__device__ __forceinline__ size_t image_float(int k, int d, int S)
{
    return 4 * ((size_t)((k >> 5) * S + (d >> 3)) * kWave + 32 * ((d >> 2) & 1) + (k & 31)) + (d & 3);
}

// First column of the last 4-float piece of a row that starts below D: the clamp for unconditional row loads
// whose out-of-range columns are zeroed at use.  D itself need not be a multiple of 4 (a prefix of the
// coordinates); the row it lies in is, so the piece is inside the row.
__device__ __forceinline__ int last_piece(int D) { return ((D + 3) & ~3) - 4; }

// The kVolatile + 1 largest entries of drift[0..K) (K <= 256), descending, with their indices; computed by
// the first wave of the block into LDS (top[], tk[]; unused slots 0 / -1).  Ends with a barrier.
constexpr int kVolatile = 4;
__device__ __forceinline__ void top_drifts(const float *sdrift, int K, float *top, int *tk)
{
    if (threadIdx.x < kWave) {
        const int lane = threadIdx.x;
        float v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = (lane + kWave * j < K) ? sdrift[lane + kWave * j] : -1.f;
        for (int i = 0; i <= kVolatile; ++i) {
            float best = v[0];
            int at = lane;
#pragma unroll
            for (int j = 1; j < 4; ++j)
                if (v[j] > best) { best = v[j]; at = lane + kWave * j; }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) {
                const float ob = __shfl_xor(best, o, kWave);
                const int oa = __shfl_xor(at, o, kWave);
                if (ob > best || (ob == best && oa < at)) { best = ob; at = oa; }
            }
            if (lane == 0) { top[i] = best > 0.f ? best : 0.f; tk[i] = best > 0.f ? at : -1; }
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (at == lane + kWave * j) v[j] = -1.f;             // struck out
        }
    }
    __syncthreads();
}

}  // namespace hclae
