// Hard TopK re-selection of active diagonals (Sec. 3.2, Eq. 4): which K of the D importance
// scores are kept.  One workgroup per score vector, integer comparisons only, so the result
// is the same on every run and on every device.
// The method itself is in dd_select_block.h.
#include "dd_common.h"
#include "dd_launch.h"
#include "dd_select_block.h"
#include "dd_soft_block.h"

namespace dd {

template <bool KEYS_IN_LDS>
__global__ __launch_bounds__(kSelectThreads) void select_topk_kernel(
    int D, int K, const float *__restrict__ scores, int *__restrict__ out)
{
    extern __shared__ uint32_t s_keys[];  // [D] when KEYS_IN_LDS
    select_topk_block<KEYS_IN_LDS>(D, K, scores + size_t(blockIdx.x) * D, s_keys, out + size_t(blockIdx.x) * K);
}

// The selection and, in the same launch, the soft TopK weights of the same scores (Eq. 4 picks the diagonals, Eq. 5
// weighs them): the workgroup that has just ranked a score vector also normalises it.
template <bool KEYS_IN_LDS>
__global__ __launch_bounds__(kSelectThreads) void select_soft_kernel(int D, int K, float inv_temp,
                                                                     const float *__restrict__ scores,
                                                                     int *__restrict__ out,
                                                                     float *__restrict__ alpha_tilde)
{
    extern __shared__ uint32_t s_keys[];  // [D] when KEYS_IN_LDS
    static_assert(kSelectThreads == kSoftThreads, "one workgroup serves both routines");
    select_topk_block<KEYS_IN_LDS>(D, K, scores + size_t(blockIdx.x) * D, s_keys, out + size_t(blockIdx.x) * K);
    soft_topk_block(D, float(K), inv_temp, scores + size_t(blockIdx.x) * D, alpha_tilde + size_t(blockIdx.x) * D);
}

hipError_t launch_select_soft(int batch, int D, int K, float temperature, const float *scores, int *out,
                              float *alpha_tilde, hipStream_t stream)
{
    if (D <= kSelectLdsKeys) {
        static std::atomic<uint64_t> lds_allowed{0};  // one bit per device
        if (hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(&select_soft_kernel<true>), kSelectLdsKeys * int(sizeof(uint32_t)), lds_allowed)) return e;
        hipLaunchKernelGGL(select_soft_kernel<true>, dim3(batch), dim3(kSelectThreads), size_t(D) * sizeof(uint32_t),
                           stream, D, K, 1.f / temperature, scores, out, alpha_tilde);
    } else {
        hipLaunchKernelGGL(select_soft_kernel<false>, dim3(batch), dim3(kSelectThreads), 0, stream, D, K,
                           1.f / temperature, scores, out, alpha_tilde);
    }
    return hipGetLastError();
}

hipError_t launch_select(int batch, int D, int K, const float *scores, int *out, hipStream_t stream)
{
    if (D <= kSelectLdsKeys) {
        static std::atomic<uint64_t> lds_allowed{0};  // one bit per device
        if (hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(&select_topk_kernel<true>), kSelectLdsKeys * int(sizeof(uint32_t)), lds_allowed)) return e;
        hipLaunchKernelGGL(select_topk_kernel<true>, dim3(batch), dim3(kSelectThreads), size_t(D) * sizeof(uint32_t),
                           stream, D, K, scores, out);
    } else {
        hipLaunchKernelGGL(select_topk_kernel<false>, dim3(batch), dim3(kSelectThreads), 0, stream, D, K, scores, out);
    }
    return hipGetLastError();
}

}  // namespace dd
