// Dictionary ordering and code statistics (Sec. 3.3: dictionaries in descending order of the variance of
// their elements; Sec. 2.2: self-information H(I_m) and mutual information of the code parts).
// Small integer / fp64 kernels; none is on the hot path.
#pragma once
#include "common.hpp"

namespace hclae {

// var[m] = (1/K) sum_k || c_m(k) - mean_k c_m ||^2, fp64, one block per dictionary.
__global__ __launch_bounds__(256) void k_dictionary_variance(
    const float *__restrict__ C, int K, int D, double *__restrict__ var)
{
    __shared__ double red[256 / kWave];
    const float *Cm = C + (size_t)blockIdx.x * K * D;
    double acc = 0.0;
    for (int d = threadIdx.x; d < D; d += 256) {
        double s = 0.0;
        for (int k = 0; k < K; ++k) s += (double)Cm[(size_t)k * D + d];
        const double mu = s / (double)K;
        double q = 0.0;
        for (int k = 0; k < K; ++k) {
            const double t = (double)Cm[(size_t)k * D + d] - mu;
            q += t * t;
        }
        acc += q;
    }
    acc = block_sum(acc, red);
    if (threadIdx.x == 0) var[blockIdx.x] = acc / (double)K;
}

// dst[j] = src[order[j]] for whole dictionaries (K*D floats each).
__global__ __launch_bounds__(256) void k_permute_dictionaries(
    const float *__restrict__ src, const int *__restrict__ order, int M, size_t per, float *__restrict__ dst)
{
    const size_t total = (size_t)M * per;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const size_t j = i / per;
        dst[i] = src[(size_t)order[j] * per + (i - j * per)];
    }
}

// codes[n][j] <- codes[n][order[j]] in place, one thread per row (M <= 256 bytes per row).
__global__ __launch_bounds__(256) void k_permute_code_columns(
    uint8_t *__restrict__ codes, const int *__restrict__ order, int64_t N, int M)
{
    for (int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x; n < N; n += (int64_t)gridDim.x * 256) {
        uint8_t *row = codes + n * M;
        uint8_t tmp[256];
        for (int j = 0; j < M; ++j) tmp[j] = row[order[j]];
        for (int j = 0; j < M; ++j) row[j] = tmp[j];
    }
}

__global__ __launch_bounds__(256) void k_zero_u64(unsigned long long *p, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) p[i] = 0ull;
}

// hist[m][k] += 1 for every code; joint[ka][kb] += 1 for the pair of columns (a, b) when joint != null.
// Integer atomics: the result does not depend on the order.
__global__ __launch_bounds__(256) void k_code_histograms(
    const uint8_t *__restrict__ codes, int64_t N, int M, int K, int a, int b,
    unsigned long long *__restrict__ hist, unsigned long long *__restrict__ joint)
{
    for (int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x; n < N; n += (int64_t)gridDim.x * 256) {
        const uint8_t *row = codes + n * M;
        for (int m = 0; m < M; ++m) atomicAdd(hist + (size_t)m * K + row[m], 1ull);
        if (joint) atomicAdd(joint + (size_t)row[a] * K + row[b], 1ull);
    }
}

}  // namespace hclae
