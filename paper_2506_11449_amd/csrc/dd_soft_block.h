// Soft TopK weights of one score vector by one workgroup of 256 threads (Sec. 3.2, Eq. 5), shared by the kernel
// that computes only them and by the selection kernel that also emits them.
#pragma once
#include "dd_common.h"

namespace dd {

constexpr int kSoftThreads = 256;

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v = fmaxf(v, __shfl_xor(v, d, 64));
    return v;
}
// all-reduce over the 256 threads of a workgroup; every thread gets the result
template <bool MAX>
__device__ __forceinline__ float block_reduce(float v, float *scratch /* [4] */)
{
    v = MAX ? wave_max(v) : wave_sum(v);
    __syncthreads();  // scratch may still be read from a previous reduction
    if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = v;
    __syncthreads();
    const float a = scratch[0], b = scratch[1], c = scratch[2], d = scratch[3];
    return MAX ? fmaxf(fmaxf(a, b), fmaxf(c, d)) : (a + b) + (c + d);
}

// alpha_tilde_i = min(K * exp((a_i - max) / temp) / sum_j exp((a_j - max) / temp), 1)
__device__ __forceinline__ void soft_topk_block(int D, float k_over_1, float inv_temp, const float *__restrict__ a,
                                                float *__restrict__ out)
{
    __shared__ float scratch[4];
    float m = -INFINITY;
    for (int i = threadIdx.x; i < D; i += kSoftThreads) m = fmaxf(m, a[i]);
    m = block_reduce<true>(m, scratch);
    float s = 0.f;
    for (int i = threadIdx.x; i < D; i += kSoftThreads) s += expf((a[i] - m) * inv_temp);
    s = block_reduce<false>(s, scratch);
    const float scale = k_over_1 / s;
    for (int i = threadIdx.x; i < D; i += kSoftThreads) out[i] = fminf(scale * expf((a[i] - m) * inv_temp), 1.f);
}

}  // namespace dd
