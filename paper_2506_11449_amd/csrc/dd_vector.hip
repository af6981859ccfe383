// Direct diagonal kernels on the vector ALUs: every multiply-add of the K*L stored weights
// is done once per token (Sec. 3.1 Eq. 3 applied diagonal by diagonal, no dense blocks).
// Serves fp32 storage, feature counts the matrix-core kernels do not cover, and very low densities.
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

// ---- tiled variant: the source tile of TT tokens sits in LDS, every shifted read comes from there ----
//
// Layout: tile[c][TT + 4] fp32 (column-major, tokens minor).  A lane owns one destination column and TT
// tokens: per diagonal it computes its source column once and fetches its TT tokens with TT/4 16-byte
// reads at fixed offsets; the 4-float pad makes neighbouring columns start 16 bytes apart modulo the
// 256-byte bank row, so the eight lanes served per clock never share a bank.  The weight of the
// (column, diagonal) pair is read once and used for all TT tokens.
typedef float f32x4v __attribute__((ext_vector_type(4)));

template <class S, int TT, bool MASKED>
__global__ __launch_bounds__(kProdThreads) void product_tiled_kernel(
    int64_t T, int D, int L, int K, const typename S::storage *__restrict__ src, const int *__restrict__ offsets,
    const typename S::storage *__restrict__ values, typename S::storage *__restrict__ dst)
{
    constexpr int STRIDE = TT + 4;
    extern __shared__ __align__(16) float smem[];
    const int src_cols = MASKED ? L : D, dst_cols = MASKED ? D : L;
    float *tile = smem;
    int *s_off = reinterpret_cast<int *>(smem + size_t(src_cols) * STRIDE);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t t0 = int64_t(blockIdx.x) * TT;

    for (int k = tid; k < K; k += kProdThreads) s_off[k] = canonical_offset(offsets[k], D);
#pragma unroll 4
    for (int t = 0; t < TT; ++t) {
        const int64_t tg = t0 + t;
        const typename S::storage *row = src + tg * src_cols;
        const typename S::storage *safe = tg < T ? row : src;  // rows past the end read row 0 and store zeros
        for (int c = tid; c < src_cols; c += kProdThreads) {
            const float x = S::load(safe + c);
            tile[c * STRIDE + t] = tg < T ? x : 0.f;
        }
    }
    __syncthreads();

    for (int jb = wave * 64; jb < dst_cols; jb += 4 * 64) {
        const int j = jb + lane;
        const bool active = j < dst_cols;
        float acc[TT];
#pragma unroll
        for (int t = 0; t < TT; ++t) acc[t] = 0.f;
        // Diagonals are taken eight at a time; the weights of the next eight are requested from memory
        // (L2) before the current eight are multiplied, which hides that latency at two waves per SIMD.
        constexpr int KB = 8;
        float w_cur[KB], w_nxt[KB];
        int c_cur[KB], c_nxt[KB];
        auto fetch = [&](int k0, float (&w)[KB], int (&cc)[KB]) {
            // lane u of this vector holds the offset of diagonal k0 + u; broadcast by lane index below
            const int off_vec = s_off[min(k0 + (lane & (KB - 1)), K - 1)];
#pragma unroll
            for (int u = 0; u < KB; ++u) {
                const int k = k0 + u;
                const int o = __builtin_amdgcn_readlane(off_vec, u);
                int c;
                bool valid = active && k < K;
                unsigned widx;  // K * L < 2^32: both are below 65536
                if (MASKED) {
                    c = j - o;
                    if (c < 0) c += D;
                    valid = valid && c < L;
                    widx = unsigned(k) * unsigned(L) + unsigned(c);
                } else {
                    c = j + o;
                    if (c >= D) c -= D;
                    widx = unsigned(k) * unsigned(L) + unsigned(j);
                }
                // the load itself is unconditional (entry 0 stands in) so that eight of them stay in flight
                const float wv = S::load(values + (valid ? widx : 0u));
                w[u] = valid ? wv : 0.f;
                cc[u] = valid ? c : 0;
            }
        };
        fetch(0, w_cur, c_cur);
        for (int k0 = 0; k0 < K; k0 += KB) {
            fetch(k0 + KB, w_nxt, c_nxt);
#pragma unroll
            for (int u = 0; u < KB; ++u) {
                const float *col = tile + c_cur[u] * STRIDE;
#pragma unroll
                for (int q = 0; q < TT / 4; ++q) {
                    const f32x4v x = *reinterpret_cast<const f32x4v *>(col + 4 * q);
#pragma unroll
                    for (int i = 0; i < 4; ++i) acc[4 * q + i] = fmaf(x[i], w_cur[u], acc[4 * q + i]);
                }
            }
#pragma unroll
            for (int u = 0; u < KB; ++u) { w_cur[u] = w_nxt[u]; c_cur[u] = c_nxt[u]; }
        }
        if (active) {
#pragma unroll
            for (int t = 0; t < TT; ++t)
                if (t0 + t < T) S::store(dst + (t0 + t) * dst_cols + j, acc[t]);
        }
    }
}

template <class S, int TT>
static hipError_t launch_tiled(const ProductArgs &a, hipStream_t stream, size_t lds)
{
    using st = typename S::storage;
    const unsigned grid = unsigned((a.T + TT - 1) / TT);
    const st *src = static_cast<const st *>(a.src), *values = static_cast<const st *>(a.values);
    st *dst = static_cast<st *>(a.dst);
    if (a.masked) {
        static std::atomic<uint64_t> lds_allowed{0};  // one bit per device
        if (hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(&product_tiled_kernel<S, TT, true>), 160 * 1024, lds_allowed)) return e;
        hipLaunchKernelGGL((product_tiled_kernel<S, TT, true>), dim3(grid), dim3(kProdThreads), lds, stream, a.T, a.D,
                           a.L, a.K, src, a.offsets, values, dst);
    } else {
        static std::atomic<uint64_t> lds_allowed{0};  // one bit per device
        if (hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(&product_tiled_kernel<S, TT, false>), 160 * 1024, lds_allowed)) return e;
        hipLaunchKernelGGL((product_tiled_kernel<S, TT, false>), dim3(grid), dim3(kProdThreads), lds, stream, a.T, a.D,
                           a.L, a.K, src, a.offsets, values, dst);
    }
    return hipGetLastError();
}

template <class S>
static hipError_t launch_product_t(const ProductArgs &a, hipStream_t stream)
{
    using st = typename S::storage;
    const int cols = a.masked ? a.D : a.L;
    // the tiled kernel needs the source tile (and the K offsets) in LDS and a 32-bit workgroup count
    const size_t src_cols = a.masked ? a.L : a.D;
    const size_t lds_limit = 160 * 1024;
    auto lds_for = [&](int tt) { return (src_cols * size_t(tt + 4) + size_t(a.K)) * 4; };
    if (a.T / 4 < (int64_t(1) << 31) - 1) {
        if (lds_for(16) <= lds_limit) return launch_tiled<S, 16>(a, stream, lds_for(16));
        if (lds_for(8) <= lds_limit) return launch_tiled<S, 8>(a, stream, lds_for(8));
        if (lds_for(4) <= lds_limit) return launch_tiled<S, 4>(a, stream, lds_for(4));
    }
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

size_t weight_grad_vector_ws_bytes(int64_t T, int D, int L, int K, bool bf16)
{
    // whichever kernel runs (the choice also depends on pointer alignment, unknown here) must fit
    const size_t plain = size_t(weight_grad_splits(T)) * size_t(K) * size_t(L) * sizeof(float);
    const size_t dot2 = bf16 && weight_grad_dot2_supported(T, D, L, K) ? weight_grad_dot2_ws_bytes(T, D, L, K) : 0;
    return plain > dot2 ? plain : dot2;
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
    const bool aligned = reinterpret_cast<uintptr_t>(a.A) % 16 == 0 && reinterpret_cast<uintptr_t>(a.B) % 16 == 0;
    if (a.bf16 && aligned && weight_grad_dot2_supported(a.T, a.D, a.L, a.K)) {
        hipError_t e = launch_weight_grad_dot2_partials(a, stream);
        if (e != hipSuccess) return e;
        const size_t n = size_t(a.K) * a.L;
        hipLaunchKernelGGL(weight_grad_reduce_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, n,
                           weight_grad_dot2_chunks(a.T, a.D, a.L, a.K), static_cast<const float *>(a.ws), a.dValues);
        return hipGetLastError();
    }
    return a.bf16 ? launch_weight_grad_t<BF16>(a, stream) : launch_weight_grad_t<F32>(a, stream);
}

}  // namespace dd
