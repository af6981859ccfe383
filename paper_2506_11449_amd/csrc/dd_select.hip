// Hard TopK re-selection of active diagonals (Sec. 3.2, Eq. 4): which K of the D importance
// scores are kept.  One workgroup per score vector, integer comparisons only, so the result
// is the same on every run and on every device.
//
// Method: scores are mapped to 32-bit keys whose unsigned order is the required total order
// (NaN lowest, -0 == +0).  A four-pass byte-wise radix search finds the K-th largest key tau
// and how many of the keys equal to tau still belong to the selection (the lowest-indexed
// ones).  A last pass walks the indices in ascending order and compacts the chosen ones with
// a workgroup prefix sum, which also yields them already sorted by index.
#include "dd_common.h"
#include "dd_launch.h"

namespace dd {

constexpr int kSelectThreads = 256;

__device__ __forceinline__ uint32_t score_key(float s)
{
    if (s != s) return 0u;             // NaN: below every number
    uint32_t u = __float_as_uint(s + 0.0f);  // -0 + 0 = +0
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__global__ __launch_bounds__(kSelectThreads) void select_topk_kernel(
    int D, int K, const float *__restrict__ scores, int *__restrict__ out)
{
    __shared__ unsigned hist[256];
    __shared__ unsigned s_prefix, s_remaining;
    __shared__ unsigned scan_gt[kSelectThreads], scan_eq[kSelectThreads];

    const int tid = threadIdx.x;
    const float *row = scores + size_t(blockIdx.x) * D;
    int *dst = out + size_t(blockIdx.x) * K;

    if (tid == 0) { s_prefix = 0u; s_remaining = unsigned(K); }
    unsigned mask = 0u;
    for (int shift = 24; shift >= 0; shift -= 8) {
        hist[tid] = 0u;
        __syncthreads();
        const unsigned prefix = s_prefix;
        for (int i = tid; i < D; i += kSelectThreads) {
            const uint32_t key = score_key(row[i]);
            if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
        }
        __syncthreads();
        if (tid == 0) {
            unsigned remaining = s_remaining, above = 0u;
            int bin = 255;
            for (; bin > 0; --bin) {
                if (above + hist[bin] >= remaining) break;
                above += hist[bin];
            }
            s_remaining = remaining - above;  // still to take inside this bin
            s_prefix = prefix | (unsigned(bin) << shift);
        }
        mask |= 255u << shift;
        __syncthreads();
    }
    const uint32_t tau = s_prefix;          // the K-th largest key
    const unsigned take_eq = s_remaining;   // how many keys equal to tau are selected (>= 1)

    // contiguous chunk of indices per thread, so that a prefix sum keeps ascending order
    const int chunk = (D + kSelectThreads - 1) / kSelectThreads;
    const int lo = min(tid * chunk, D), hi = min(lo + chunk, D);
    unsigned n_gt = 0u, n_eq = 0u;
    for (int i = lo; i < hi; ++i) {
        const uint32_t key = score_key(row[i]);
        n_gt += key > tau;
        n_eq += key == tau;
    }
    scan_gt[tid] = n_gt;
    scan_eq[tid] = n_eq;
    __syncthreads();
    for (int d = 1; d < kSelectThreads; d <<= 1) {  // inclusive Hillis-Steele scan
        unsigned a = 0u, b = 0u;
        if (tid >= d) { a = scan_gt[tid - d]; b = scan_eq[tid - d]; }
        __syncthreads();
        scan_gt[tid] += a;
        scan_eq[tid] += b;
        __syncthreads();
    }
    unsigned eq_rank = scan_eq[tid] - n_eq;                      // equal keys before this chunk
    unsigned pos = (scan_gt[tid] - n_gt) + min(eq_rank, take_eq);  // selected before this chunk
    for (int i = lo; i < hi; ++i) {
        const uint32_t key = score_key(row[i]);
        if (key > tau) {
            dst[pos++] = i;
        } else if (key == tau) {
            if (eq_rank < take_eq) dst[pos++] = i;
            ++eq_rank;
        }
    }
}

hipError_t launch_select(int batch, int D, int K, const float *scores, int *out, hipStream_t stream)
{
    hipLaunchKernelGGL(select_topk_kernel, dim3(batch), dim3(kSelectThreads), 0, stream, D, K, scores, out);
    return hipGetLastError();
}

}  // namespace dd
