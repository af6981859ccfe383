// Heuristic update of the set of active diagonals (DiagHeur, appendix "Details of the Heuristics-Based
// Method"): the diagonals of lowest magnitude leave, as many inactive candidates enter at random.  The random
// scores are an input, so the result is a pure function of its arguments.
//
// The update is two hard TopK selections on score vectors over the D candidates, and runs on the selection
// kernel of Sec. 3.2 (dd_select.hip) without leaving the device:
//   1. scores_1[i] = magnitude of the active diagonal with offset i (a NaN magnitude counts as -1, below
//      every true magnitude, which is a sum of absolute values), -inf where no diagonal is active;
//      keep = TopK(scores_1, K - n_drop)                     the diagonals that stay
//   2. scores_2[i] = +inf for i in keep, random[i] for i that was not active (finite by contract; NaN
//      counts as -inf), NaN -- the lowest rank there is -- for the diagonals that have just left;
//      new = TopK(scores_2, K)                               the K - n_drop kept ones and the n_drop grown ones
// Both selections order equal scores by lower index and NaN lowest, and emit ascending indices.
#include "dd_common.h"
#include "dd_launch.h"

#include <float.h>
#include <math.h>

namespace dd {

constexpr int kHeurThreads = 256;

// magnitudes[k] = sum_p |values[k][p]|: one workgroup per diagonal, fixed-order tree reduction
template <typename Tr>
__global__ __launch_bounds__(kHeurThreads) void diag_magnitude_kernel(int L, const typename Tr::storage *__restrict__ values,
                                                                      float *__restrict__ magnitudes)
{
    __shared__ float part[kHeurThreads];
    const typename Tr::storage *row = values + size_t(blockIdx.x) * L;
    float s = 0.f;
    for (int p = threadIdx.x; p < L; p += kHeurThreads) s += fabsf(Tr::load(row + p));
    part[threadIdx.x] = s;
    __syncthreads();
    for (int w = kHeurThreads / 2; w > 0; w >>= 1) {
        if (threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) magnitudes[blockIdx.x] = part[0];
}

// scores_1 and the table offset -> position in `offsets` (-1: not active); one workgroup
__global__ __launch_bounds__(1024) void heur_scatter_kernel(int D, int K, const int *__restrict__ offsets,
                                                            const float *__restrict__ magnitudes,
                                                            float *__restrict__ scores, int *__restrict__ slot)
{
    for (int i = threadIdx.x; i < D; i += 1024) {
        scores[i] = -INFINITY;
        slot[i] = -1;
    }
    __syncthreads();  // one workgroup: its own global writes above are ordered before those below
    for (int k = threadIdx.x; k < K; k += 1024) {
        const int o = canonical_offset(offsets[k], D);
        const float m = magnitudes[k];
        scores[o] = m != m ? -1.f : m;
        slot[o] = k;
    }
}

// scores_2 from the table, the random scores and the kept offsets; one workgroup
__global__ __launch_bounds__(1024) void heur_combine_kernel(int D, int n_keep, const int *__restrict__ slot,
                                                            const float *__restrict__ random,
                                                            const int *__restrict__ keep, float *__restrict__ scores)
{
    for (int i = threadIdx.x; i < D; i += 1024) {
        const float r = random[i];
        scores[i] = slot[i] >= 0 ? NAN : (r != r ? -INFINITY : r);
    }
    __syncthreads();
    for (int j = threadIdx.x; j < n_keep; j += 1024) scores[keep[j]] = INFINITY;
}

// source[j] = position in the old arrays of new diagonal j, -1 for a grown one
__global__ __launch_bounds__(kHeurThreads) void heur_source_kernel(int K, const int *__restrict__ slot,
                                                                   const int *__restrict__ new_offsets,
                                                                   int *__restrict__ source)
{
    const int j = blockIdx.x * kHeurThreads + threadIdx.x;
    if (j < K) source[j] = slot[new_offsets[j]];
}

hipError_t launch_diag_magnitude(int K, int L, bool bf16, const void *values, float *magnitudes, hipStream_t stream)
{
    if (bf16)
        hipLaunchKernelGGL(diag_magnitude_kernel<BF16>, dim3(K), dim3(kHeurThreads), 0, stream, L,
                           static_cast<const uint16_t *>(values), magnitudes);
    else
        hipLaunchKernelGGL(diag_magnitude_kernel<F32>, dim3(K), dim3(kHeurThreads), 0, stream, L,
                           static_cast<const float *>(values), magnitudes);
    return hipGetLastError();
}

size_t diagheur_ws_bytes(int D, int K)
{
    // scores [D] float, slot [D] int, keep [K] int; each part a multiple of 256 bytes
    auto up = [](size_t b) { return (b + 255) / 256 * 256; };
    return 2 * up(size_t(D) * 4) + up(size_t(K) * 4);
}

hipError_t launch_diagheur_update(int D, int K, int n_drop, const int *offsets, const float *magnitudes,
                                  const float *random, int *new_offsets, int *source, void *ws, hipStream_t stream)
{
    auto up = [](size_t b) { return (b + 255) / 256 * 256; };
    unsigned char *base = static_cast<unsigned char *>(ws);
    float *scores = reinterpret_cast<float *>(base);
    int *slot = reinterpret_cast<int *>(base + up(size_t(D) * 4));
    int *keep = reinterpret_cast<int *>(base + 2 * up(size_t(D) * 4));
    const int n_keep = K - n_drop;
    hipLaunchKernelGGL(heur_scatter_kernel, dim3(1), dim3(1024), 0, stream, D, K, offsets, magnitudes, scores, slot);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (n_keep > 0) {
        e = launch_select(1, D, n_keep, scores, keep, stream);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(heur_combine_kernel, dim3(1), dim3(1024), 0, stream, D, n_keep, slot, random, keep, scores);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    e = launch_select(1, D, K, scores, new_offsets, stream);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(heur_source_kernel, dim3((K + kHeurThreads - 1) / kHeurThreads), dim3(kHeurThreads), 0, stream,
                       K, slot, new_offsets, source);
    return hipGetLastError();
}

}  // namespace dd
