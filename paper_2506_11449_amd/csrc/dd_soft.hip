// Soft TopK weights of the candidate diagonals and the scaling of the active diagonals by them
// (Sec. 3.2, Eq. 4 and Eq. 5), forward and backward.  O(D) and O(K*L) element-wise work with block
// reductions: launch-bound, one workgroup per score vector / per diagonal, fixed reduction order.
#include "dd_common.h"
#include "dd_launch.h"
#include "dd_soft_block.h"

namespace dd {

__global__ __launch_bounds__(kSoftThreads) void soft_topk_kernel(int D, float k_over_1, float inv_temp,
                                                                 const float *__restrict__ scores,
                                                                 float *__restrict__ alpha_tilde)
{
    soft_topk_block(D, k_over_1, inv_temp, scores + size_t(blockIdx.x) * D, alpha_tilde + size_t(blockIdx.x) * D);
}

// d a_i = (K / temp) * s_i * (m_i g_i - sum_j m_j g_j s_j),  m_j = [K s_j < 1]
__global__ __launch_bounds__(kSoftThreads) void soft_topk_bwd_kernel(int D, float k_over_1, float inv_temp,
                                                                     const float *__restrict__ scores,
                                                                     const float *__restrict__ g,
                                                                     float *__restrict__ dscores)
{
    __shared__ float scratch[4];
    const float *a = scores + size_t(blockIdx.x) * D, *gb = g + size_t(blockIdx.x) * D;
    float *out = dscores + size_t(blockIdx.x) * D;
    float m = -INFINITY;
    for (int i = threadIdx.x; i < D; i += kSoftThreads) m = fmaxf(m, a[i]);
    m = block_reduce<true>(m, scratch);
    float s = 0.f;
    for (int i = threadIdx.x; i < D; i += kSoftThreads) s += expf((a[i] - m) * inv_temp);
    s = block_reduce<false>(s, scratch);
    const float inv_s = 1.f / s;
    float dot = 0.f;
    for (int i = threadIdx.x; i < D; i += kSoftThreads) {
        const float si = expf((a[i] - m) * inv_temp) * inv_s;
        if (k_over_1 * si < 1.f) dot += gb[i] * si;
    }
    dot = block_reduce<false>(dot, scratch);
    for (int i = threadIdx.x; i < D; i += kSoftThreads) {
        const float si = expf((a[i] - m) * inv_temp) * inv_s;
        const float mg = k_over_1 * si < 1.f ? gb[i] : 0.f;
        out[i] = k_over_1 * inv_temp * si * (mg - dot);
    }
}

// values_eff[k][p] = alpha_tilde[o_k] * V[k][p]
template <class S>
__global__ __launch_bounds__(kSoftThreads) void scale_values_kernel(int L, int D, const int *__restrict__ offsets,
                                                                    const float *__restrict__ alpha_tilde,
                                                                    const typename S::storage *__restrict__ V,
                                                                    typename S::storage *__restrict__ out)
{
    const int k = blockIdx.y, p = blockIdx.x * kSoftThreads + threadIdx.x;
    if (p >= L) return;
    const float a = alpha_tilde[canonical_offset(offsets[k], D)];
    S::store(out + size_t(k) * L + p, a * S::load(V + size_t(k) * L + p));
}

// dV[k][p] = alpha_tilde[o_k] * dValues[k][p];  dots[k] = <dValues[k], V[k]>
template <class S>
__global__ __launch_bounds__(kSoftThreads) void scale_values_bwd_kernel(int L, int D, const int *__restrict__ offsets,
                                                                        const float *__restrict__ alpha_tilde,
                                                                        const typename S::storage *__restrict__ V,
                                                                        const float *__restrict__ dValues,
                                                                        float *__restrict__ dV,
                                                                        float *__restrict__ dots)
{
    __shared__ float scratch[4];
    const int k = blockIdx.x;
    const float a = alpha_tilde[canonical_offset(offsets[k], D)];
    float dot = 0.f;
    for (int p = threadIdx.x; p < L; p += kSoftThreads) {
        const float g = dValues[size_t(k) * L + p];
        dV[size_t(k) * L + p] = a * g;
        dot = fmaf(g, S::load(V + size_t(k) * L + p), dot);
    }
    dot = block_reduce<false>(dot, scratch);
    if (threadIdx.x == 0) dots[k] = dot;
}

// dalpha_tilde[i] = sum over the diagonals k with offset i, in index order, of dots[k]
__global__ __launch_bounds__(kSoftThreads) void scatter_alpha_grad_kernel(int D, int K, const int *__restrict__ offsets,
                                                                          const float *__restrict__ dots,
                                                                          float *__restrict__ dalpha)
{
    const int i = blockIdx.x * kSoftThreads + threadIdx.x;
    if (i >= D) return;
    float acc = 0.f;
    for (int k = 0; k < K; ++k)
        if (canonical_offset(offsets[k], D) == i) acc += dots[k];
    dalpha[i] = acc;
}

hipError_t launch_soft_topk(int batch, int D, int K, float temperature, const float *scores, float *alpha_tilde,
                            hipStream_t stream)
{
    hipLaunchKernelGGL(soft_topk_kernel, dim3(batch), dim3(kSoftThreads), 0, stream, D, float(K), 1.f / temperature,
                       scores, alpha_tilde);
    return hipGetLastError();
}

hipError_t launch_soft_topk_bwd(int batch, int D, int K, float temperature, const float *scores, const float *g,
                                float *dscores, hipStream_t stream)
{
    hipLaunchKernelGGL(soft_topk_bwd_kernel, dim3(batch), dim3(kSoftThreads), 0, stream, D, float(K),
                       1.f / temperature, scores, g, dscores);
    return hipGetLastError();
}

hipError_t launch_scale_values(int K, int L, int D, bool bf16, const int *offsets, const float *alpha_tilde,
                               const void *V, void *out, hipStream_t stream)
{
    dim3 grid((L + kSoftThreads - 1) / kSoftThreads, K);
    if (bf16)
        hipLaunchKernelGGL(scale_values_kernel<BF16>, grid, dim3(kSoftThreads), 0, stream, L, D, offsets, alpha_tilde,
                           static_cast<const uint16_t *>(V), static_cast<uint16_t *>(out));
    else
        hipLaunchKernelGGL(scale_values_kernel<F32>, grid, dim3(kSoftThreads), 0, stream, L, D, offsets, alpha_tilde,
                           static_cast<const float *>(V), static_cast<float *>(out));
    return hipGetLastError();
}

hipError_t launch_scale_values_bwd(int K, int L, int D, bool bf16, const int *offsets, const float *alpha_tilde,
                                   const void *V, const float *dValues, float *dV, float *dalpha, float *dots,
                                   hipStream_t stream)
{
    if (bf16)
        hipLaunchKernelGGL(scale_values_bwd_kernel<BF16>, dim3(K), dim3(kSoftThreads), 0, stream, L, D, offsets,
                           alpha_tilde, static_cast<const uint16_t *>(V), dValues, dV, dots);
    else
        hipLaunchKernelGGL(scale_values_bwd_kernel<F32>, dim3(K), dim3(kSoftThreads), 0, stream, L, D, offsets,
                           alpha_tilde, static_cast<const float *>(V), dValues, dV, dots);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(scatter_alpha_grad_kernel, dim3((D + kSoftThreads - 1) / kSoftThreads), dim3(kSoftThreads), 0,
                       stream, D, K, offsets, dots, dalpha);
    return hipGetLastError();
}

}  // namespace dd
