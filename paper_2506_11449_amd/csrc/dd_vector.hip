// Direct diagonal kernels on the vector ALUs: every multiply-add of the K*L stored weights
// is done once per token (Sec. 3.1 Eq. 3 applied diagonal by diagonal, no dense blocks).
#include "dd_common.h"
#include "dd_launch.h"

namespace dd {

constexpr int kProdThreads = 256;
constexpr int kMaxKShared = 4096;  // canonical offsets cached per workgroup, in slices of this size

// dst[t, p] = sum_k src[t, (p + o_k) mod D] * v_k[p]
template <class S>
__global__ __launch_bounds__(kProdThreads) void gather_kernel(
    int D, int L, int K, const typename S::storage *__restrict__ src, const int *__restrict__ offsets,
    const typename S::storage *__restrict__ values, typename S::storage *__restrict__ dst)
{
    __shared__ int s_off[kMaxKShared];
    const int p = blockIdx.x * kProdThreads + threadIdx.x;
    const size_t t = blockIdx.y;
    const typename S::storage *row = src + t * size_t(D);
    float acc = 0.f;
    for (int k0 = 0; k0 < K; k0 += kMaxKShared) {
        const int kn = min(K - k0, kMaxKShared);
        __syncthreads();
        for (int k = threadIdx.x; k < kn; k += kProdThreads) s_off[k] = canonical_offset(offsets[k0 + k], D);
        __syncthreads();
        if (p < L) {
            for (int k = 0; k < kn; ++k) {
                int q = p + s_off[k];
                if (q >= D) q -= D;
                acc = fmaf(S::load(row + q), S::load(values + size_t(k0 + k) * L + p), acc);
            }
        }
    }
    if (p < L) S::store(dst + t * size_t(L) + p, acc);
}

// dst[t, q] = sum over k with c = (q - o_k) mod D < L of src[t, c] * v_k[c]
template <class S>
__global__ __launch_bounds__(kProdThreads) void masked_gather_kernel(
    int D, int L, int K, const typename S::storage *__restrict__ src, const int *__restrict__ offsets,
    const typename S::storage *__restrict__ values, typename S::storage *__restrict__ dst)
{
    __shared__ int s_off[kMaxKShared];
    const int q = blockIdx.x * kProdThreads + threadIdx.x;
    const size_t t = blockIdx.y;
    const typename S::storage *row = src + t * size_t(L);
    float acc = 0.f;
    for (int k0 = 0; k0 < K; k0 += kMaxKShared) {
        const int kn = min(K - k0, kMaxKShared);
        __syncthreads();
        for (int k = threadIdx.x; k < kn; k += kProdThreads) s_off[k] = canonical_offset(offsets[k0 + k], D);
        __syncthreads();
        if (q < D) {
            for (int k = 0; k < kn; ++k) {
                int c = q - s_off[k];
                if (c < 0) c += D;
                if (c < L) acc = fmaf(S::load(row + c), S::load(values + size_t(k0 + k) * L + c), acc);
            }
        }
    }
    if (q < D) S::store(dst + t * size_t(D) + q, acc);
}

template <class S>
static hipError_t launch_product_t(const ProductArgs &a, hipStream_t stream)
{
    using st = typename S::storage;
    const int cols = a.masked ? a.D : a.L;
    // grid.y carries the token index; split calls so that it stays within the 65535 limit
    const int64_t max_rows = 65535;
    for (int64_t t0 = 0; t0 < a.T; t0 += max_rows) {
        const int64_t rows = a.T - t0 < max_rows ? a.T - t0 : max_rows;
        dim3 grid((cols + kProdThreads - 1) / kProdThreads, unsigned(rows));
        const st *src = static_cast<const st *>(a.src) + t0 * (a.masked ? a.L : a.D);
        st *dst = static_cast<st *>(a.dst) + t0 * cols;
        if (a.masked)
            hipLaunchKernelGGL(masked_gather_kernel<S>, grid, dim3(kProdThreads), 0, stream, a.D, a.L, a.K, src,
                               a.offsets, static_cast<const st *>(a.values), dst);
        else
            hipLaunchKernelGGL(gather_kernel<S>, grid, dim3(kProdThreads), 0, stream, a.D, a.L, a.K, src,
                               a.offsets, static_cast<const st *>(a.values), dst);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_product_vector(const ProductArgs &a, hipStream_t stream)
{
    return a.bf16 ? launch_product_t<BF16>(a, stream) : launch_product_t<F32>(a, stream);
}

// ---- gradient of the values: a sum over tokens per (diagonal, position) ----

constexpr int kWgThreads = 256;
constexpr int kWgTokensPerSplit = 1024;
constexpr int kWgMaxSplits = 64;

static int weight_grad_splits(int64_t T)
{
    int64_t s = (T + kWgTokensPerSplit - 1) / kWgTokensPerSplit;
    if (s < 1) s = 1;
    if (s > kWgMaxSplits) s = kWgMaxSplits;
    return int(s);
}

size_t weight_grad_vector_ws_bytes(int64_t T, int D, int L, int K)
{
    (void)D;
    return size_t(weight_grad_splits(T)) * size_t(K) * size_t(L) * sizeof(float);
}

// partial[s][k][p] = sum over the tokens of split s of A[t, p] * B[t, (p + o_k) mod D]
template <class S>
__global__ __launch_bounds__(kWgThreads) void weight_grad_partial_kernel(
    int64_t T, int D, int L, int K, int splits, const typename S::storage *__restrict__ A,
    const typename S::storage *__restrict__ B, const int *__restrict__ offsets, float *__restrict__ partial)
{
    const int p = blockIdx.x * kWgThreads + threadIdx.x;
    const int k = blockIdx.y;
    const int s = blockIdx.z;
    if (p >= L) return;
    const int64_t per = (T + splits - 1) / splits;
    const int64_t t0 = s * per, t1 = min(t0 + per, T);
    int q = p + canonical_offset(offsets[k], D);
    if (q >= D) q -= D;
    float acc = 0.f;
    for (int64_t t = t0; t < t1; ++t)
        acc = fmaf(S::load(A + t * L + p), S::load(B + t * D + q), acc);
    partial[(size_t(s) * K + k) * L + p] = acc;
}

// dV[i] = partial[0][i] + partial[1][i] + ... in that order
__global__ __launch_bounds__(256) void weight_grad_reduce_kernel(size_t n, int splits, const float *__restrict__ partial,
                                                                float *__restrict__ dV)
{
    const size_t i = size_t(blockIdx.x) * 256 + threadIdx.x;
    if (i >= n) return;
    float acc = 0.f;
    for (int s = 0; s < splits; ++s) acc += partial[size_t(s) * n + i];
    dV[i] = acc;
}

template <class S>
static hipError_t launch_weight_grad_t(const WeightGradArgs &a, hipStream_t stream)
{
    using st = typename S::storage;
    const int splits = weight_grad_splits(a.T);
    const size_t n = size_t(a.K) * a.L;
    float *partial = static_cast<float *>(a.ws);
    // K can exceed the grid.y limit only beyond 65535 diagonals, which the ABI rejects
    dim3 grid((a.L + kWgThreads - 1) / kWgThreads, a.K, splits);
    hipLaunchKernelGGL(weight_grad_partial_kernel<S>, grid, dim3(kWgThreads), 0, stream, a.T, a.D, a.L, a.K, splits,
                       static_cast<const st *>(a.A), static_cast<const st *>(a.B), a.offsets, partial);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(weight_grad_reduce_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, n, splits, partial,
                       a.dValues);
    return hipGetLastError();
}

hipError_t launch_weight_grad_vector(const WeightGradArgs &a, hipStream_t stream)
{
    return a.bf16 ? launch_weight_grad_t<BF16>(a, stream) : launch_weight_grad_t<F32>(a, stream);
}

}  // namespace dd
