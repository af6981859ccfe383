// Host-side launchers, one per kernel family.  Arguments are already validated by the C ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

namespace dd {

// Raises a kernel's limit of dynamic LDS, once per device: the attribute belongs to the kernel as loaded on the
// current device, so a flag per process would leave every device but the first at the default limit.
// `done` is a bit set of device ordinals, one per kernel (a function-local static at the call site).
// Host threads may launch at the same time: the bits are set atomically, and two threads that both find a bit
// clear merely set the same attribute twice.  Devices past ordinal 63 are not remembered (the attribute is set
// on every launch there).
inline hipError_t allow_dynamic_lds(const void *kernel, int bytes, std::atomic<uint64_t> &done)
{
    int device = 0;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess) return e;
    const uint64_t bit = device < 64 ? uint64_t(1) << device : 0;
    if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) done.fetch_or(bit, std::memory_order_release);
    return e;
}

// The two product shapes every forward / backward-input call reduces to
// (D = long side, L = short side, offsets taken modulo D):
//   gather:        dst[t, p] = sum_k src[t, (p + o_k) mod D] * v_k[p]              src [T x D], dst [T x L]
//   masked gather: dst[t, q] = sum_{k : c < L} src[t, c] * v_k[c], c = (q - o_k) mod D   src [T x L], dst [T x D]
struct ProductArgs {
    int64_t T;
    int D, L, K;
    bool bf16;
    bool masked;          // false: gather, true: masked gather
    const void *src;
    const int32_t *offsets;
    const void *values;   // [K x L]
    void *dst;
    void *ws;             // scratch of the size the chosen kernel family asks for
    bool prepared = false;  // matrix family: ws already holds the dense operand of this product
    // Matrix family, prepared operands only: a group of equally shaped layers that share their input.
    // dst_sets > 1: dst is that many [T x cols] matrices one after the other, one per set (the forward product);
    // src_sets > 1: src likewise, and the sets' products are summed into the one dst (the backward-input product).
    int src_sets = 1, dst_sets = 1;
};

// dV[k][p] = sum_t A[t, p] * B[t, (p + o_k) mod D];  A [T x L] (short side), B [T x D] (long side)
struct WeightGradArgs {
    int64_t T;
    int D, L, K;
    bool bf16;
    const void *A;
    const void *B;
    const int32_t *offsets;
    float *dValues;       // [K x L]
    void *ws;
};

hipError_t launch_product_vector(const ProductArgs &a, hipStream_t stream);
// vector kernels for a handful of diagonals (K <= 16, bf16 storage, feature counts multiples of 128, long side <= 8192,
// 16-byte aligned matrices): bound by reading the input and writing the output once
bool product_lowk_supported(int64_t T, int D, int L, int K, bool bf16, bool masked);
hipError_t launch_product_lowk(const ProductArgs &a, hipStream_t stream);
// the weight gradient of the same family: partial sums per workgroup, then an ordered sum over them
bool weight_grad_lowk_supported(int64_t T, int D, int L, int K, bool bf16);
size_t weight_grad_lowk_ws_bytes(int64_t T, int D, int L, int K);
hipError_t launch_weight_grad_lowk(const WeightGradArgs &a, hipStream_t stream);

// matrix-core family (bf16 only, feature counts multiples of 128)
bool product_matrix_supported(int64_t T, int D, int L, bool bf16);
size_t product_matrix_ws_bytes(int D, int L);
hipError_t launch_product_matrix(const ProductArgs &a, hipStream_t stream);
// The same product on prepared operands, skipping the 32 x 16 operand blocks that no diagonal crosses (a.offsets says
// which); one layer at a time (no groups), long side <= 8192.
bool product_blocks_supported(int64_t T, int D, int L, bool bf16);
hipError_t launch_product_blocks(const ProductArgs &a, hipStream_t stream);
// Both dense operands of `sets` equally shaped layers (offsets [sets x K], values [sets x K x L]) in one launch:
// the forward operands side by side at `forward_operand`, the backward-input operands stacked along the
// contraction at `backward_operand`, sets * D * L elements each.
// alpha (or null): importance weights of the D candidates; diagonal k enters as bf16(alpha[o_k] * values[k]).
hipError_t launch_prepare_matrix(int D, int L, int K, int sets, bool expanding, const int32_t *offsets,
                                 const void *values, void *forward_operand, void *backward_operand,
                                 hipStream_t stream, const float *alpha = nullptr);
// The operands of `layers` independent layers of one shape in one launch (offsets [layers x K], values
// [layers x K x L]): layer i's block, laid out as launch_prepare_matrix lays out a single layer (forward operand,
// then backward-input operand), starts 2 * D * L elements after layer i-1's.
hipError_t launch_prepare_matrix_batched(int D, int L, int K, int layers, bool expanding, const int32_t *offsets,
                                         const void *values, void *prepared, hipStream_t stream);
// Selection of the K diagonals from `scores` [D] and both dense operands from them in one launch (small layers
// only: ask select_prepare_fused first).  offsets_out [K] receives the chosen offsets, ascending.
bool select_prepare_fused(int D, int L, int K);
hipError_t launch_select_prepare(int D, int L, int K, bool expanding, const float *scores, const void *values,
                                 int32_t *offsets_out, void *forward_operand, void *backward_operand,
                                 hipStream_t stream);
size_t weight_grad_vector_ws_bytes(int64_t T, int D, int L, int K, bool bf16);
hipError_t launch_weight_grad_vector(const WeightGradArgs &a, hipStream_t stream);
// bf16 dot-product kernel of the vector family (feature counts multiples of 8, long side <= 2304)
bool weight_grad_dot2_supported(int64_t T, int D, int L, int K);
size_t weight_grad_dot2_ws_bytes(int64_t T, int D, int L, int K);
int weight_grad_dot2_chunks(int64_t T, int D, int L, int K);
hipError_t launch_weight_grad_dot2_partials(const WeightGradArgs &a, hipStream_t stream);

// matrix-core family (bf16 only, both feature counts multiples of 192 or both multiples of 128)
bool weight_grad_matrix_supported(int64_t T, int D, int L, bool bf16);
size_t weight_grad_matrix_ws_bytes(int64_t T, int D, int L, int K);
hipError_t launch_weight_grad_matrix(const WeightGradArgs &a, hipStream_t stream);
// The same with the adjoint of the scaling by the importance weights (Sec. 3.2 Eq. 4) as the epilogue of the ordered
// sum over the token chunks: dV[k][p] = alpha[o_k] * dValues[k][p] (to a.dValues) and dalpha[i] = sum over the
// diagonals with offset i of <dValues[k], V[k]>.  tail: scratch behind the partial sums, weight_grad_scaled_tail_bytes.
size_t weight_grad_scaled_tail_bytes(int L, int K);
hipError_t launch_weight_grad_matrix_scaled(const WeightGradArgs &a, const float *alpha, const void *V, float *dalpha,
                                            void *tail, hipStream_t stream);

hipError_t launch_select(int batch, int D, int K, const float *scores, int *out, hipStream_t stream);
// selection and soft TopK weights of the same score vectors in one launch
hipError_t launch_select_soft(int batch, int D, int K, float temperature, const float *scores, int *out,
                              float *alpha_tilde, hipStream_t stream);

// soft TopK weights and the scaling of the diagonals by them
hipError_t launch_soft_topk(int batch, int D, int K, float temperature, const float *scores, float *alpha_tilde,
                            hipStream_t stream);
hipError_t launch_soft_topk_bwd(int batch, int D, int K, float temperature, const float *scores, const float *g,
                                float *dscores, hipStream_t stream);
hipError_t launch_scale_values(int K, int L, int D, bool bf16, const int *offsets, const float *alpha_tilde,
                               const void *V, void *out, hipStream_t stream);
hipError_t launch_scale_values_bwd(int K, int L, int D, bool bf16, const int *offsets, const float *alpha_tilde,
                                   const void *V, const float *dValues, float *dV, float *dalpha, float *dots,
                                   hipStream_t stream);

// DiagHeur: magnitude of each diagonal, and the update of the active set built on launch_select
hipError_t launch_diag_magnitude(int K, int L, bool bf16, const void *values, float *magnitudes, hipStream_t stream);
size_t diagheur_ws_bytes(int D, int K);
hipError_t launch_diagheur_update(int D, int K, int n_drop, const int *offsets, const float *magnitudes,
                                  const float *random, int *new_offsets, int *source, void *ws, hipStream_t stream);

}  // namespace dd
