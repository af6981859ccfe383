// C ABI of the diagonally-sparse layer: argument checks, reduction of the four products to the
// two gather shapes (Appendix A: the transpose of a diagonal-sparse matrix is diagonal-sparse
// with the same starts, so forward and backward-input share kernels), and kernel dispatch.
#include "../../include/dynadiag.h"

#include "dd_launch.h"

#include <atomic>

namespace {

constexpr int kMaxFeatures = 65535;
constexpr size_t kWsAlign = 256;

struct Shape {
    int D, L;
    bool expanding;  // M <= N (square included): the diagonal position p is the row of W
};

dd_status check_layer(const dd_layer *l, Shape *s)
{
    if (!l) return DD_ERR_INVALID_ARG;
    if (l->tokens < 0 || l->in_features < 1 || l->out_features < 1 || l->K < 1) return DD_ERR_INVALID_ARG;
    if (l->dtype != DD_F32 && l->dtype != DD_BF16) return DD_ERR_INVALID_ARG;
    if (l->algo != DD_ALGO_AUTO && l->algo != DD_ALGO_VECTOR && l->algo != DD_ALGO_MATRIX &&
        l->algo != DD_ALGO_PREPARED && l->algo != DD_ALGO_BLOCKS)
        return DD_ERR_INVALID_ARG;
    const int D = l->in_features > l->out_features ? l->in_features : l->out_features;
    const int L = l->in_features < l->out_features ? l->in_features : l->out_features;
    if (l->K > D) return DD_ERR_INVALID_ARG;
    if (D > kMaxFeatures) return DD_ERR_UNSUPPORTED;
    s->D = D;
    s->L = L;
    s->expanding = l->in_features <= l->out_features;
    return DD_OK;
}

dd_status check_ws(const void *ws, size_t ws_bytes, size_t need)
{
    if (need == 0) return DD_OK;
    if (!ws || ws_bytes < need) return DD_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(ws) % kWsAlign) return DD_ERR_WORKSPACE;
    return DD_OK;
}

size_t select_ws_bytes(int32_t, int32_t, int32_t) { return 0; }

bool aligned16(const void *p) { return reinterpret_cast<uintptr_t>(p) % 16 == 0; }

// Does the shape allow the matrix-core kernels?  Then every request but DD_ALGO_VECTOR may run them.  The dense
// contraction costs the same whatever K is and the general vector kernels cost in proportion to K, but measured over
// K = 1 ... D/8 (`bench.py --k-sweep`) the matrix cores are ahead of those at every density, so between the two there
// is no density threshold; the kernels for a handful of diagonals (wants_lowk) are asked first.
bool wants_matrix(const dd_layer *l, const Shape &s)
{
    if (l->algo == DD_ALGO_VECTOR) return false;
    // (a call without tokens launches nothing, whatever the family)
    if (!dd::product_matrix_supported(l->tokens > 0 ? l->tokens : 1, s.D, s.L, l->dtype == DD_BF16)) return false;
    return true;
}

// A handful of diagonals given as offsets and values: the kernels that visit only the stored weights and are bound by
// reading the input and writing the output once.  DD_ALGO_VECTOR takes them wherever they apply (up to 16 diagonals);
// DD_ALGO_AUTO where they are ahead of the dense contraction.  Their time grows with K times the width of the side the
// lanes own, the dense contraction's with D * L, and the measured crossings (`bench.py --k-sweep`: 768^2, 1024^2,
// 768 <-> 3072) sit at K * width = D * L / 96 for the products and at K = D / 192 for the weight gradient.
bool wants_lowk(const dd_layer *l, const Shape &s, bool masked)
{
    if (l->algo != DD_ALGO_VECTOR && l->algo != DD_ALGO_AUTO) return false;
    if (l->algo == DD_ALGO_AUTO && int64_t(l->K) * (masked ? s.D : s.L) * 96 > int64_t(s.D) * s.L) return false;
    return dd::product_lowk_supported(l->tokens, s.D, s.L, l->K, l->dtype == DD_BF16, masked);
}
bool wants_lowk_wgrad(const dd_layer *l, const Shape &s)
{
    if (l->algo != DD_ALGO_VECTOR && l->algo != DD_ALGO_AUTO) return false;
    if (l->algo == DD_ALGO_AUTO && int64_t(l->K) * 192 > s.D) return false;
    return dd::weight_grad_lowk_supported(l->tokens, s.D, s.L, l->K, l->dtype == DD_BF16);
}

// the block dd_prepare fills: the operand of the forward product, then the one of the backward-input product
size_t prepared_bytes(const Shape &s) { return 2 * dd::product_matrix_ws_bytes(s.D, s.L); }

bool wants_matrix_wgrad(const dd_layer *l, const Shape &s)
{
    if (l->algo == DD_ALGO_VECTOR) return false;
    if (!dd::weight_grad_matrix_supported(l->tokens, s.D, s.L, l->dtype == DD_BF16)) return false;
    return true;
}

// Scratch of dd_bwd_weight.  A forced matrix-core call runs those kernels or fails, so it needs their partial
// sums only.  Under DD_ALGO_AUTO the family is settled at the call, once the alignment of X and dY is known, and
// the two families cut the tokens into different numbers of chunks: the size covers whichever of them runs.
size_t weight_grad_ws_bytes(const dd_layer *l, const Shape &s)
{
    size_t vector = dd::weight_grad_vector_ws_bytes(l->tokens, s.D, s.L, l->K, l->dtype == DD_BF16);
    if (wants_lowk_wgrad(l, s)) {
        const size_t lowk = dd::weight_grad_lowk_ws_bytes(l->tokens, s.D, s.L, l->K);
        vector = lowk > vector ? lowk : vector;
    }
    if (!wants_matrix_wgrad(l, s)) return vector;
    const size_t matrix = dd::weight_grad_matrix_ws_bytes(l->tokens, s.D, s.L, l->K);
    if (l->algo != DD_ALGO_AUTO) return matrix;
    return matrix > vector ? matrix : vector;
}

constexpr int kMaxSets = 8;

// `sets` > 1: a group of equally shaped layers sharing their input, operands prepared by dd_prepare_shared
dd_status product(const dd_layer *l, const Shape &s, bool transposed, const void *src, const int32_t *offsets,
                  const void *values, void *dst, void *ws, size_t ws_bytes, void *stream, int sets = 1)
{
    const bool blocks = l->algo == DD_ALGO_BLOCKS;  // prepared operands, and the offsets to tell which blocks are empty
    const bool prepared = l->algo == DD_ALGO_PREPARED || blocks;
    if (!prepared && (!offsets || !values)) return DD_ERR_INVALID_ARG;
    if (blocks && (!offsets || sets != 1)) return DD_ERR_INVALID_ARG;
    if (l->tokens > 0 && (!src || !dst)) return DD_ERR_INVALID_ARG;
    bool matrix = wants_matrix(l, s);
    if (prepared && !matrix) return DD_ERR_UNSUPPORTED;
    const size_t need = dd_workspace_bytes(transposed ? DD_OP_BWD_INPUT : DD_OP_FWD, l, 0) * size_t(sets);
    if (dd_status st = check_ws(ws, ws_bytes, need)) return st;
    if (l->tokens == 0) return DD_OK;
    if (matrix && !(aligned16(src) && aligned16(dst))) matrix = false;  // 16-byte vector accesses
    if ((l->algo == DD_ALGO_MATRIX || prepared) && !matrix) return DD_ERR_UNSUPPORTED;
    if (blocks && !dd::product_blocks_supported(l->tokens, s.D, s.L, l->dtype == DD_BF16)) return DD_ERR_UNSUPPORTED;
    dd::ProductArgs a;
    a.T = l->tokens;
    a.D = s.D;
    a.L = s.L;
    a.K = l->K;
    a.bf16 = l->dtype == DD_BF16;
    // forward reads the short side when the layer expands; backward-input is the mirror image
    a.masked = transposed ? !s.expanding : s.expanding;
    a.src = src;
    a.offsets = offsets;
    a.values = values;
    a.dst = dst;
    a.ws = ws;
    if (prepared) {
        a.prepared = true;
        if (transposed) a.ws = static_cast<unsigned char *>(ws) + dd::product_matrix_ws_bytes(s.D, s.L) * size_t(sets);
        (transposed ? a.src_sets : a.dst_sets) = sets;
    }
    const bool lowk = !prepared && wants_lowk(l, s, a.masked) && aligned16(src) && aligned16(dst);
    const hipError_t e = blocks   ? dd::launch_product_blocks(a, static_cast<hipStream_t>(stream))
                         : lowk   ? dd::launch_product_lowk(a, static_cast<hipStream_t>(stream))
                         : matrix ? dd::launch_product_matrix(a, static_cast<hipStream_t>(stream))
                                  : dd::launch_product_vector(a, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? DD_OK : DD_ERR_HIP;
}

// ---- the backward pass as one call (dd_bwd): the two products back to back, sharing one scratch ----
size_t bwd_ws_bytes(const dd_layer *l)
{
    dd_layer plain = *l;
    if (plain.algo == DD_ALGO_PREPARED) plain.algo = DD_ALGO_MATRIX;  // the prepared block is passed beside the scratch
    const size_t a = l->algo == DD_ALGO_PREPARED ? 0 : dd_workspace_bytes(DD_OP_BWD_INPUT, &plain, 0);
    const size_t b = dd_workspace_bytes(DD_OP_BWD_WEIGHT, &plain, 0);
    return a > b ? a : b;
}

}  // namespace

extern "C" {

size_t dd_workspace_bytes(int op, const dd_layer *layer, int32_t batch)
{
    if (op == DD_OP_SELECT) {
        if (!layer) return 0;
        return select_ws_bytes(batch, layer->in_features, layer->K);
    }
    if (op == DD_OP_DIAGHEUR) {
        if (!layer || layer->in_features < 1 || layer->K < 1 || layer->K > layer->in_features) return 0;
        return dd::diagheur_ws_bytes(layer->in_features, layer->K);
    }
    if (op == DD_OP_SCALE_VALUES_BWD) {
        if (!layer || layer->K < 1) return 0;
        return (size_t(layer->K) * sizeof(float) + kWsAlign - 1) / kWsAlign * kWsAlign;
    }
    Shape s;
    if (check_layer(layer, &s) != DD_OK) return 0;
    switch (op) {
    case DD_OP_FWD:
    case DD_OP_BWD_INPUT:
        if (layer->algo == DD_ALGO_PREPARED || layer->algo == DD_ALGO_BLOCKS)
            return wants_matrix(layer, s) ? prepared_bytes(s) : 0;
        return wants_matrix(layer, s) ? dd::product_matrix_ws_bytes(s.D, s.L) : 0;
    case DD_OP_PREPARE:
        return dd::product_matrix_supported(1, s.D, s.L, layer->dtype == DD_BF16) ? prepared_bytes(s) : 0;
    case DD_OP_BWD_WEIGHT:
        return weight_grad_ws_bytes(layer, s);
    case DD_OP_BWD:
        return layer->algo == DD_ALGO_BLOCKS ? 0 : bwd_ws_bytes(layer);
    case DD_OP_BWD_WEIGHT_SCALED: {
        if (layer->algo == DD_ALGO_VECTOR || !wants_matrix_wgrad(layer, s)) return 0;
        const size_t partials = dd::weight_grad_matrix_ws_bytes(layer->tokens, s.D, s.L, layer->K);
        return (partials + kWsAlign - 1) / kWsAlign * kWsAlign + dd::weight_grad_scaled_tail_bytes(s.L, layer->K);
    }
    default:
        return 0;
    }
}

dd_status dd_fwd(const dd_layer *layer, const void *X, const int32_t *offsets, const void *values, void *Y, void *ws,
                 size_t ws_bytes, void *hip_stream)
{
    Shape s;
    if (dd_status st = check_layer(layer, &s)) return st;
    return product(layer, s, false, X, offsets, values, Y, ws, ws_bytes, hip_stream);
}

dd_status dd_prepare(const dd_layer *layer, const int32_t *offsets, const void *values, void *prepared,
                     size_t prepared_bytes_given, void *hip_stream)
{
    Shape s;
    if (dd_status st = check_layer(layer, &s)) return st;
    if (!offsets || !values) return DD_ERR_INVALID_ARG;
    if (layer->algo == DD_ALGO_VECTOR) return DD_ERR_UNSUPPORTED;
    if (!dd::product_matrix_supported(1, s.D, s.L, layer->dtype == DD_BF16)) return DD_ERR_UNSUPPORTED;
    if (dd_status st = check_ws(prepared, prepared_bytes_given, prepared_bytes(s))) return st;
    unsigned char *first = static_cast<unsigned char *>(prepared);
    const hipError_t e = dd::launch_prepare_matrix(s.D, s.L, layer->K, 1, s.expanding, offsets, values, first,
                                                   first + dd::product_matrix_ws_bytes(s.D, s.L),
                                                   static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? DD_OK : DD_ERR_HIP;
}

dd_status dd_prepare_batched(const dd_layer *layer, int32_t n_layers, const int32_t *offsets, const void *values,
                             void *prepared, size_t prepared_bytes_given, void *hip_stream)
{
    Shape s;
    if (dd_status st = check_layer(layer, &s)) return st;
    if (n_layers < 0) return DD_ERR_INVALID_ARG;
    if (n_layers == 0) return DD_OK;
    if (!offsets || !values) return DD_ERR_INVALID_ARG;
    if (n_layers > 65535 || layer->algo == DD_ALGO_VECTOR) return DD_ERR_UNSUPPORTED;
    if (!dd::product_matrix_supported(1, s.D, s.L, layer->dtype == DD_BF16)) return DD_ERR_UNSUPPORTED;
    if (dd_status st = check_ws(prepared, prepared_bytes_given, prepared_bytes(s) * size_t(n_layers))) return st;
    const hipError_t e = dd::launch_prepare_matrix_batched(s.D, s.L, layer->K, n_layers, s.expanding, offsets, values,
                                                           prepared, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? DD_OK : DD_ERR_HIP;
}

dd_status dd_select_prepare(const dd_layer *layer, const float *scores, const void *values, int32_t *offsets_out,
                            void *prepared, size_t prepared_bytes_given, void *hip_stream)
{
    Shape s;
    if (dd_status st = check_layer(layer, &s)) return st;
    if (!scores || !values || !offsets_out) return DD_ERR_INVALID_ARG;
    if (layer->algo == DD_ALGO_VECTOR) return DD_ERR_UNSUPPORTED;
    if (!dd::product_matrix_supported(1, s.D, s.L, layer->dtype == DD_BF16)) return DD_ERR_UNSUPPORTED;
    if (dd_status st = check_ws(prepared, prepared_bytes_given, prepared_bytes(s))) return st;
    unsigned char *first = static_cast<unsigned char *>(prepared);
    unsigned char *second = first + dd::product_matrix_ws_bytes(s.D, s.L);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipError_t e;
    if (dd::select_prepare_fused(s.D, s.L, layer->K)) {
        e = dd::launch_select_prepare(s.D, s.L, layer->K, s.expanding, scores, values, offsets_out, first, second, stream);
    } else {  // larger layers: the two steps one after the other, same results
        e = dd::launch_select(1, s.D, layer->K, scores, offsets_out, stream);
        if (e == hipSuccess)
            e = dd::launch_prepare_matrix(s.D, s.L, layer->K, 1, s.expanding, offsets_out, values, first, second, stream);
    }
    return e == hipSuccess ? DD_OK : DD_ERR_HIP;
}

dd_status dd_prepare_shared(const dd_layer *layer, int32_t n_sets, const int32_t *offsets, const void *values,
                            void *prepared, size_t prepared_bytes_given, void *hip_stream)
{
    Shape s;
    if (dd_status st = check_layer(layer, &s)) return st;
    if (n_sets < 1 || !offsets || !values) return DD_ERR_INVALID_ARG;
    if (n_sets > kMaxSets || layer->algo == DD_ALGO_VECTOR) return DD_ERR_UNSUPPORTED;
    if (!dd::product_matrix_supported(1, s.D, s.L, layer->dtype == DD_BF16)) return DD_ERR_UNSUPPORTED;
    if (dd_status st = check_ws(prepared, prepared_bytes_given, prepared_bytes(s) * size_t(n_sets))) return st;
    unsigned char *first = static_cast<unsigned char *>(prepared);
    const hipError_t e = dd::launch_prepare_matrix(s.D, s.L, layer->K, n_sets, s.expanding, offsets, values, first,
                                                   first + dd::product_matrix_ws_bytes(s.D, s.L) * size_t(n_sets),
                                                   static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? DD_OK : DD_ERR_HIP;
}

static dd_status product_shared(const dd_layer *layer, int32_t n_sets, bool transposed, const void *src,
                                const void *prepared, size_t prepared_bytes_given, void *dst, void *hip_stream)
{
    Shape s;
    if (dd_status st = check_layer(layer, &s)) return st;
    if (n_sets < 1) return DD_ERR_INVALID_ARG;
    if (n_sets > kMaxSets) return DD_ERR_UNSUPPORTED;
    dd_layer l = *layer;
    l.algo = DD_ALGO_PREPARED;
    return product(&l, s, transposed, src, nullptr, nullptr, dst, const_cast<void *>(prepared), prepared_bytes_given,
                   hip_stream, n_sets);
}

dd_status dd_fwd_shared(const dd_layer *layer, int32_t n_sets, const void *X, const void *prepared,
                        size_t prepared_bytes_given, void *Y, void *hip_stream)
{
    return product_shared(layer, n_sets, false, X, prepared, prepared_bytes_given, Y, hip_stream);
}

dd_status dd_bwd_input_shared(const dd_layer *layer, int32_t n_sets, const void *dY, const void *prepared,
                              size_t prepared_bytes_given, void *dX, void *hip_stream)
{
    return product_shared(layer, n_sets, true, dY, prepared, prepared_bytes_given, dX, hip_stream);
}

dd_status dd_bwd_input(const dd_layer *layer, const void *dY, const int32_t *offsets, const void *values, void *dX,
                       void *ws, size_t ws_bytes, void *hip_stream)
{
    Shape s;
    if (dd_status st = check_layer(layer, &s)) return st;
    return product(layer, s, true, dY, offsets, values, dX, ws, ws_bytes, hip_stream);
}

dd_status dd_bwd_weight(const dd_layer *layer, const void *X, const void *dY, const int32_t *offsets, float *dValues,
                        void *ws, size_t ws_bytes, void *hip_stream)
{
    Shape s;
    if (dd_status st = check_layer(layer, &s)) return st;
    if (!offsets || !dValues) return DD_ERR_INVALID_ARG;
    if (layer->tokens > 0 && (!X || !dY)) return DD_ERR_INVALID_ARG;
    if (dd_status st = check_ws(ws, ws_bytes, dd_workspace_bytes(DD_OP_BWD_WEIGHT, layer, 0))) return st;
    const bool aligned = aligned16(X) && aligned16(dY);  // 16-byte transfers
    const bool lowk = layer->tokens > 0 && aligned && wants_lowk_wgrad(layer, s);
    const bool matrix = !lowk && aligned && wants_matrix_wgrad(layer, s);
    if (layer->algo != DD_ALGO_AUTO && layer->algo != DD_ALGO_VECTOR && !matrix) return DD_ERR_UNSUPPORTED;
    // the family that runs must fit the scratch that was checked (the families cut the tokens differently)
    const size_t runs_in = lowk     ? dd::weight_grad_lowk_ws_bytes(layer->tokens, s.D, s.L, layer->K)
                           : matrix ? dd::weight_grad_matrix_ws_bytes(layer->tokens, s.D, s.L, layer->K)
                                    : dd::weight_grad_vector_ws_bytes(layer->tokens, s.D, s.L, layer->K,
                                                                      layer->dtype == DD_BF16);
    if (ws_bytes < runs_in) return DD_ERR_WORKSPACE;
    dd::WeightGradArgs a;
    a.T = layer->tokens;
    a.D = s.D;
    a.L = s.L;
    a.K = layer->K;
    a.bf16 = layer->dtype == DD_BF16;
    // the short side supplies the unshifted operand, the long side the shifted one
    a.A = s.expanding ? X : dY;
    a.B = s.expanding ? dY : X;
    a.offsets = offsets;
    a.dValues = dValues;
    a.ws = ws;
    const hipError_t e = lowk     ? dd::launch_weight_grad_lowk(a, static_cast<hipStream_t>(hip_stream))
                         : matrix ? dd::launch_weight_grad_matrix(a, static_cast<hipStream_t>(hip_stream))
                                  : dd::launch_weight_grad_vector(a, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? DD_OK : DD_ERR_HIP;
}

dd_status dd_bwd(const dd_layer *layer, const void *X, const void *dY, const int32_t *offsets, const void *values,
                 const void *prepared, size_t prepared_bytes_given, void *dX, float *dValues, void *ws, size_t ws_bytes,
                 void *hip_stream)
{
    Shape s;
    if (dd_status st = check_layer(layer, &s)) return st;
    if (layer->algo == DD_ALGO_BLOCKS) return DD_ERR_UNSUPPORTED;
    const bool have_prepared = layer->algo == DD_ALGO_PREPARED;
    if (have_prepared && !prepared) return DD_ERR_INVALID_ARG;
    if (dd_status st = check_ws(ws, ws_bytes, bwd_ws_bytes(layer))) return st;
    // The input gradient first: the weight gradient, issued right behind it, then finds in the memory-side cache
    // whatever of dY that cache could keep.  Both take their scratch from the same block, one after the other.
    if (dd_status st = dd_bwd_input(layer, dY, offsets, values, dX, have_prepared ? const_cast<void *>(prepared) : ws,
                                    have_prepared ? prepared_bytes_given : ws_bytes, hip_stream))
        return st;
    dd_layer second = *layer;
    if (have_prepared) second.algo = DD_ALGO_MATRIX;
    return dd_bwd_weight(&second, X, dY, offsets, dValues, ws, ws_bytes, hip_stream);
}

dd_status dd_select_soft(int32_t batch, int32_t D, int32_t K, float temperature, const float *scores,
                         int32_t *offsets_out, float *alpha_tilde, void *hip_stream)
{
    if (batch < 0 || D < 1 || K < 1 || K > D || !(temperature > 0.f)) return DD_ERR_INVALID_ARG;
    if (D > 65536) return DD_ERR_UNSUPPORTED;
    if (batch == 0) return DD_OK;
    if (!scores || !offsets_out || !alpha_tilde) return DD_ERR_INVALID_ARG;
    return dd::launch_select_soft(batch, D, K, temperature, scores, offsets_out, alpha_tilde,
                                  static_cast<hipStream_t>(hip_stream)) == hipSuccess
               ? DD_OK
               : DD_ERR_HIP;
}

dd_status dd_prepare_scaled(const dd_layer *layer, const int32_t *offsets, const float *alpha_tilde, const void *V,
                            void *prepared, size_t prepared_bytes_given, void *hip_stream)
{
    Shape s;
    if (dd_status st = check_layer(layer, &s)) return st;
    if (!offsets || !alpha_tilde || !V) return DD_ERR_INVALID_ARG;
    if (layer->algo == DD_ALGO_VECTOR) return DD_ERR_UNSUPPORTED;
    if (!dd::product_matrix_supported(1, s.D, s.L, layer->dtype == DD_BF16)) return DD_ERR_UNSUPPORTED;
    if (dd_status st = check_ws(prepared, prepared_bytes_given, prepared_bytes(s))) return st;
    unsigned char *first = static_cast<unsigned char *>(prepared);
    const hipError_t e = dd::launch_prepare_matrix(s.D, s.L, layer->K, 1, s.expanding, offsets, V, first,
                                                   first + dd::product_matrix_ws_bytes(s.D, s.L),
                                                   static_cast<hipStream_t>(hip_stream), alpha_tilde);
    return e == hipSuccess ? DD_OK : DD_ERR_HIP;
}

dd_status dd_bwd_weight_scaled(const dd_layer *layer, const void *X, const void *dY, const int32_t *offsets,
                               const float *alpha_tilde, const void *V, float *dV, float *d_alpha_tilde, void *ws,
                               size_t ws_bytes, void *hip_stream)
{
    Shape s;
    if (dd_status st = check_layer(layer, &s)) return st;
    if (!offsets || !alpha_tilde || !V || !dV || !d_alpha_tilde) return DD_ERR_INVALID_ARG;
    if (layer->tokens < 1 || !X || !dY) return DD_ERR_INVALID_ARG;
    if (layer->algo == DD_ALGO_VECTOR || !wants_matrix_wgrad(layer, s) || !(aligned16(X) && aligned16(dY)))
        return DD_ERR_UNSUPPORTED;  // elsewhere: dd_bwd_weight, then dd_scale_values_bwd
    const size_t partials = dd::weight_grad_matrix_ws_bytes(layer->tokens, s.D, s.L, layer->K);
    const size_t partials_padded = (partials + kWsAlign - 1) / kWsAlign * kWsAlign;
    if (dd_status st = check_ws(ws, ws_bytes, partials_padded + dd::weight_grad_scaled_tail_bytes(s.L, layer->K))) return st;
    dd::WeightGradArgs a;
    a.T = layer->tokens;
    a.D = s.D;
    a.L = s.L;
    a.K = layer->K;
    a.bf16 = true;
    a.A = s.expanding ? X : dY;
    a.B = s.expanding ? dY : X;
    a.offsets = offsets;
    a.dValues = dV;
    a.ws = ws;
    const hipError_t e = dd::launch_weight_grad_matrix_scaled(a, alpha_tilde, V, d_alpha_tilde,
                                                              static_cast<unsigned char *>(ws) + partials_padded,
                                                              static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? DD_OK : DD_ERR_HIP;
}

dd_status dd_select_diagonals(int32_t batch, int32_t D, int32_t K, const float *scores, int32_t *offsets_out, void *ws,
                              size_t ws_bytes, void *hip_stream)
{
    (void)ws;
    (void)ws_bytes;
    if (batch < 0 || D < 1 || K < 1 || K > D) return DD_ERR_INVALID_ARG;
    if (D > 65536) return DD_ERR_UNSUPPORTED;
    if (batch == 0) return DD_OK;
    if (!scores || !offsets_out) return DD_ERR_INVALID_ARG;
    return dd::launch_select(batch, D, K, scores, offsets_out, static_cast<hipStream_t>(hip_stream)) == hipSuccess
               ? DD_OK
               : DD_ERR_HIP;
}

dd_status dd_soft_topk(int32_t batch, int32_t D, int32_t K, float temperature, const float *scores,
                       float *alpha_tilde, void *hip_stream)
{
    if (batch < 0 || D < 1 || K < 1 || K > D || !(temperature > 0.f)) return DD_ERR_INVALID_ARG;
    if (batch == 0) return DD_OK;
    if (!scores || !alpha_tilde) return DD_ERR_INVALID_ARG;
    return dd::launch_soft_topk(batch, D, K, temperature, scores, alpha_tilde, static_cast<hipStream_t>(hip_stream)) ==
                   hipSuccess
               ? DD_OK
               : DD_ERR_HIP;
}

dd_status dd_soft_topk_bwd(int32_t batch, int32_t D, int32_t K, float temperature, const float *scores,
                           const float *d_alpha_tilde, float *d_scores, void *hip_stream)
{
    if (batch < 0 || D < 1 || K < 1 || K > D || !(temperature > 0.f)) return DD_ERR_INVALID_ARG;
    if (batch == 0) return DD_OK;
    if (!scores || !d_alpha_tilde || !d_scores) return DD_ERR_INVALID_ARG;
    return dd::launch_soft_topk_bwd(batch, D, K, temperature, scores, d_alpha_tilde, d_scores,
                                    static_cast<hipStream_t>(hip_stream)) == hipSuccess
               ? DD_OK
               : DD_ERR_HIP;
}

dd_status dd_scale_values(int32_t K, int32_t L, int32_t D, int32_t dtype, const int32_t *offsets,
                          const float *alpha_tilde, const void *V, void *values_eff, void *hip_stream)
{
    if (K < 1 || L < 1 || D < L || K > D || (dtype != DD_F32 && dtype != DD_BF16)) return DD_ERR_INVALID_ARG;
    if (D > kMaxFeatures) return DD_ERR_UNSUPPORTED;
    if (!offsets || !alpha_tilde || !V || !values_eff) return DD_ERR_INVALID_ARG;
    return dd::launch_scale_values(K, L, D, dtype == DD_BF16, offsets, alpha_tilde, V, values_eff,
                                   static_cast<hipStream_t>(hip_stream)) == hipSuccess
               ? DD_OK
               : DD_ERR_HIP;
}

dd_status dd_scale_values_bwd(int32_t K, int32_t L, int32_t D, int32_t dtype, const int32_t *offsets,
                              const float *alpha_tilde, const void *V, const float *dValues, float *dV,
                              float *d_alpha_tilde, void *ws, size_t ws_bytes, void *hip_stream)
{
    if (K < 1 || L < 1 || D < L || K > D || (dtype != DD_F32 && dtype != DD_BF16)) return DD_ERR_INVALID_ARG;
    if (D > kMaxFeatures) return DD_ERR_UNSUPPORTED;
    if (!offsets || !alpha_tilde || !V || !dValues || !dV || !d_alpha_tilde) return DD_ERR_INVALID_ARG;
    const size_t need = (size_t(K) * sizeof(float) + kWsAlign - 1) / kWsAlign * kWsAlign;
    if (dd_status st = check_ws(ws, ws_bytes, need)) return st;
    return dd::launch_scale_values_bwd(K, L, D, dtype == DD_BF16, offsets, alpha_tilde, V, dValues, dV, d_alpha_tilde,
                                       static_cast<float *>(ws), static_cast<hipStream_t>(hip_stream)) == hipSuccess
               ? DD_OK
               : DD_ERR_HIP;
}

dd_status dd_diag_magnitude(int32_t K, int32_t L, int32_t dtype, const void *values, float *magnitudes,
                            void *hip_stream)
{
    if (K < 1 || L < 1 || (dtype != DD_F32 && dtype != DD_BF16)) return DD_ERR_INVALID_ARG;
    if (!values || !magnitudes) return DD_ERR_INVALID_ARG;
    return dd::launch_diag_magnitude(K, L, dtype == DD_BF16, values, magnitudes,
                                     static_cast<hipStream_t>(hip_stream)) == hipSuccess
               ? DD_OK
               : DD_ERR_HIP;
}

dd_status dd_diagheur_update(int32_t D, int32_t K, int32_t n_drop, const int32_t *offsets, const float *magnitudes,
                             const float *random, int32_t *new_offsets, int32_t *source, void *ws, size_t ws_bytes,
                             void *hip_stream)
{
    if (D < 1 || K < 1 || K > D || n_drop < 0 || n_drop > K || n_drop > D - K) return DD_ERR_INVALID_ARG;
    if (D > 65536) return DD_ERR_UNSUPPORTED;
    if (!offsets || !magnitudes || !random || !new_offsets || !source) return DD_ERR_INVALID_ARG;
    if (dd_status st = check_ws(ws, ws_bytes, dd::diagheur_ws_bytes(D, K))) return st;
    return dd::launch_diagheur_update(D, K, n_drop, offsets, magnitudes, random, new_offsets, source, ws,
                                      static_cast<hipStream_t>(hip_stream)) == hipSuccess
               ? DD_OK
               : DD_ERR_HIP;
}

// ---------------------------------------------------------------------------------------------
// dd_bwd_weight for callers that cannot allocate: the partial sums of the token chunks live in an array of
// this library's own instead of a workspace of the caller's.
// ---------------------------------------------------------------------------------------------
}  // extern "C"

namespace {

constexpr size_t kStaticScratchBytes = size_t(32) << 20;
// One copy per GPU, at an address of its own on each; host code must not use the name as an address.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::atomic<void *> scratch_ptr[kMaxDevices];  // the array's address on each device, asked for once

// The array's address on the current device (hipGetSymbolAddress answers for the device that is current).
hipError_t static_scratch(void **ptr)
{
    int device = 0;
    if (hipError_t e = hipGetDevice(&device)) return e;
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    void *p = scratch_ptr[device].load(std::memory_order_acquire);
    if (!p) {
        if (hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch))) return e;
        if (!p) return hipErrorInvalidSymbol;
        scratch_ptr[device].store(p, std::memory_order_release);  // two threads racing here store the same address
    }
    *ptr = p;
    return hipSuccess;
}

}  // namespace

extern "C" {

size_t dd_static_scratch_bytes(void) { return kStaticScratchBytes; }

dd_status dd_bwd_weight_static(const dd_layer *layer, const void *X, const void *dY, const int32_t *offsets,
                               float *dValues, void *hip_stream)
{
    Shape s;
    if (dd_status st = check_layer(layer, &s)) return st;
    // beyond the array: refused before anything is launched or looked up
    if (weight_grad_ws_bytes(layer, s) > kStaticScratchBytes) return DD_ERR_WORKSPACE;
    void *ptr = nullptr;
    if (static_scratch(&ptr) != hipSuccess) return DD_ERR_HIP;
    // The kernels overwrite every partial sum they later read, so what the last call left behind needs no clearing.
    return dd_bwd_weight(layer, X, dY, offsets, dValues, ptr, kStaticScratchBytes, hip_stream);
}

const char *dd_status_string(dd_status status)
{
    switch (status) {
    case DD_OK: return "ok";
    case DD_ERR_INVALID_ARG: return "invalid argument";
    case DD_ERR_UNSUPPORTED: return "unsupported size or algorithm";
    case DD_ERR_WORKSPACE: return "workspace too small or misaligned";
    case DD_ERR_HIP: return "HIP launch failed";
    }
    return "unknown status";
}

}  // extern "C"
