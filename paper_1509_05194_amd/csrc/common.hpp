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

}  // namespace hclae
