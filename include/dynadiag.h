/*
 * dynadiag.h -- C ABI of the diagonally-sparse linear layer for AMD MI355X (gfx950).
 *
 * The layer is the one of "Dynamic Sparse Training of Diagonally Sparse Networks"
 * (DynaDiag, arxiv 2506.11449): a weight matrix W [in_features x out_features] that holds
 * only K wrapped diagonals, each stored as an (offset, value-vector) pair (Sec. 3.1, Eq. 1-3).
 *
 * Index convention (Sec. 3.1 Eq. 1 and Appendix A; M = in_features, N = out_features):
 *   D = max(M, N) is the number of candidate diagonals and the wrap modulus,
 *   L = min(M, N) is the length of every diagonal.
 *   Position p in [0, L) of diagonal k lies at long-side index q = (p + o_k) mod D, and
 *     M <= N :  W[p, q] += values[k][p]        (Appendix A, case m < n; Eq. 1 for squares)
 *     M >  N :  W[q, p] += values[k][p]        (Appendix A, case m >= n)
 *   o_k = offsets[k] reduced modulo D into [0, D); any int32 is accepted, a negative offset
 *   is a diagonal below the main one.  Repeated offsets are legal and add (Eq. 3 is a sum).
 *   The importance weight of Eq. 4 is not an argument: the caller passes the effective
 *   values alpha_k * V_k.
 *
 * Common rules for every entry point
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library never
 *     allocates, frees or keeps device memory; scratch comes from the caller's `ws`
 *     (size from dd_workspace_bytes, 256-byte aligned; may be NULL when that size is 0).
 *   - All matrices are row-major and contiguous.  Inputs and outputs must not overlap.
 *   - Outputs are overwritten.  Work is enqueued on `hip_stream` (a hipStream_t passed as
 *     void*, NULL = the default stream) and the call returns without waiting for it.  The
 *     stream's device must be the current device of the calling thread.
 *   - Errors are reported by the return value; nothing is thrown and nothing aborts.
 *     DD_ERR_INVALID_ARG: null pointer, tokens < 0, features < 1, K < 1, K > D, unknown
 *     dtype or algo.  DD_ERR_WORKSPACE: ws_bytes below dd_workspace_bytes or ws misaligned.
 *     DD_ERR_UNSUPPORTED: a size the kernels do not cover (stated per function); for the three
 *     products: max(M, N) > 65535, or DD_ALGO_MATRIX / DD_ALGO_PREPARED forced where the matrix-core
 *     kernels do not apply.  They cover bf16 storage, 16-byte aligned matrices and M, N both multiples
 *     of 128 (dd_bwd_weight: both multiples of 192, or both of 128), max(M, N) <= 8192; DD_ALGO_AUTO
 *     takes them there at every density but the extreme one -- for a handful of diagonals (K <= 16 and, for a
 *     product whose output is W columns wide, K * W <= D * L / 96; for dd_bwd_weight K <= D / 192; Sec. 4.4's
 *     regime of >= 99 % sparsity) it takes vector kernels built for that case, whose time follows K down to
 *     the cost of reading the input and writing the output once -- and the vector kernels everywhere else,
 *     also for a matrix that is not 16-byte aligned (a view that starts at an odd element): such a call is legal under DD_ALGO_AUTO
 *     and several times slower; DD_ALGO_MATRIX / DD_ALGO_PREPARED report it as DD_ERR_UNSUPPORTED instead.
 *     DD_ERR_HIP: the launch itself failed.
 *   - tokens == 0 is legal: fwd / bwd_input return DD_OK without a launch; bwd_weight
 *     writes zeros.
 */
#ifndef DYNADIAG_H
#define DYNADIAG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DD_OK = 0,
    DD_ERR_INVALID_ARG = 1,
    DD_ERR_UNSUPPORTED = 2,
    DD_ERR_WORKSPACE = 3,
    DD_ERR_HIP = 4
} dd_status;

/* Storage type of X, dY, Y, dX and values.  Accumulation is always fp32. */
typedef enum { DD_F32 = 0, DD_BF16 = 1 } dd_dtype;

/* Which kernel family runs the product.  DD_ALGO_AUTO picks by shape and density. */
typedef enum {
    DD_ALGO_AUTO = 0,
    DD_ALGO_VECTOR = 1, /* direct diagonal kernels on the vector ALUs: work ~ tokens*K*L (K <= 16, bf16, M and N
                           multiples of 128: the kernels built for a handful of diagonals) */
    DD_ALGO_MATRIX = 2, /* the diagonals rebuilt as a dense operand in scratch, product on the matrix cores */
    DD_ALGO_PREPARED = 3, /* as DD_ALGO_MATRIX, with the dense operands already built by dd_prepare */
    DD_ALGO_BLOCKS = 4    /* as DD_ALGO_PREPARED, and the product skips every 32 x 16 block of the operand that no
                             diagonal crosses; it also reads `offsets` (to tell which blocks those are).  For active
                             sets that lie in runs of adjacent diagonals (Sec. 3.3: the learned masks cluster): with
                             offsets spread uniformly nearly every block is crossed and DD_ALGO_PREPARED is faster.
                             dd_fwd / dd_bwd_input only; max(M, N) <= 8192; dd_bwd_weight treats it as DD_ALGO_MATRIX. */
} dd_algo;

typedef enum {
    DD_OP_FWD = 0,
    DD_OP_BWD_INPUT = 1,
    DD_OP_BWD_WEIGHT = 2,
    DD_OP_SELECT = 3,
    DD_OP_SCALE_VALUES_BWD = 4, /* layer->K diagonals: scratch of dd_scale_values_bwd */
    DD_OP_PREPARE = 5,          /* the block dd_prepare fills and DD_ALGO_PREPARED calls read */
    DD_OP_DIAGHEUR = 6,         /* layer->in_features candidates, layer->K diagonals: scratch of dd_diagheur_update */
    DD_OP_BWD_WEIGHT_SCALED = 7, /* scratch of dd_bwd_weight_scaled (0 where it returns DD_ERR_UNSUPPORTED) */
    DD_OP_BWD = 8               /* scratch of dd_bwd */
} dd_op;

typedef struct {
    int64_t tokens;       /* T: rows of X / dY                                   */
    int32_t in_features;  /* M: columns of X, rows of W                          */
    int32_t out_features; /* N: columns of Y, columns of W                       */
    int32_t K;            /* number of active diagonals, 1 <= K <= max(M, N)     */
    int32_t dtype;        /* dd_dtype                                            */
    int32_t algo;         /* dd_algo                                             */
} dd_layer;

/*
 * Bytes of device scratch that `op` needs for this layer (for DD_OP_SELECT: layer->in_features
 * is read as D, layer->K as K, and `batch` is the number of score vectors; otherwise `batch`
 * is ignored).  Returns 0 for arguments the op would reject.
 */
size_t dd_workspace_bytes(int op, const dd_layer *layer, int32_t batch);

/*
 * Forward product Y = X . W_K  (Sec. 3.1 Eq. 3; Fig. 3 b-e).
 *   X       [tokens x M]  dtype          in
 *   offsets [K]           int32          in   one offset per diagonal, any order
 *   values  [K x L]       dtype          in   values[k][p] belongs to offsets[k]
 *   Y       [tokens x N]  dtype          out  rounded to nearest-even from the fp32 sum
 */
dd_status dd_fwd(const dd_layer *layer, const void *X, const int32_t *offsets, const void *values,
                 void *Y, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Builds once what dd_fwd and dd_bwd_input would otherwise rebuild on every call of the matrix-core path:
 * the K diagonals of (offsets, values) laid out as the two dense bf16 operands (W_K for the forward
 * product, its transpose for the backward one; Sec. 3.1 Eq. 1-3, Appendix A).  Meant for weights that
 * serve several products: inference, where they never change, and training, where forward and backward
 * of one step share them.
 *   prepared: dd_workspace_bytes(DD_OP_PREPARE, layer, 0) bytes, 256-byte aligned, owned by the caller and
 *   left alone by every other call; valid until offsets or values change.
 * Afterwards dd_fwd / dd_bwd_input take layer->algo = DD_ALGO_PREPARED with ws = prepared (their offsets
 * and values arguments are then not read).  dd_bwd_weight treats DD_ALGO_PREPARED exactly like DD_ALGO_MATRIX
 * (DD_ERR_UNSUPPORTED where the matrix-core kernels do not apply) and needs its own scratch.  layer->tokens is not used here.
 * DD_ERR_UNSUPPORTED where DD_ALGO_MATRIX would be (dtype other than bf16, feature counts that are not
 * multiples of 128).
 */
dd_status dd_prepare(const dd_layer *layer, const int32_t *offsets, const void *values, void *prepared,
                     size_t prepared_bytes, void *hip_stream);

/*
 * dd_prepare for n_layers independent layers of one shape (M -> N, K diagonals each) in one launch, as a training
 * step over a stack of equal layers needs it after re-selecting every layer's diagonals (Sec. 3.2 Eq. 4 per layer).
 *   offsets  [n_layers x K] int32, values [n_layers x K x L] dtype   in   (row i belongs to layer i; the offsets
 *            are exactly what dd_select_diagonals writes for a batch of n_layers score vectors)
 *   prepared n_layers * dd_workspace_bytes(DD_OP_PREPARE, layer, 0) bytes, 256-byte aligned: layer i's block is
 *            the i-th piece of that size, bit for bit what dd_prepare builds for layer i, and is handed to
 *            dd_fwd / dd_bwd_input (DD_ALGO_PREPARED) by itself.
 * n_layers = 0 is legal (nothing is launched); more than 65535 layers: DD_ERR_UNSUPPORTED; other errors as dd_prepare.
 */
dd_status dd_prepare_batched(const dd_layer *layer, int32_t n_layers, const int32_t *offsets, const void *values,
                             void *prepared, size_t prepared_bytes, void *hip_stream);

/*
 * dd_select_diagonals for one score vector followed by dd_prepare on the diagonals it chose, as one call (one
 * launch for layers of up to 1024 candidate diagonals, where the launches are most of what the two steps cost;
 * two launches beyond).  The results are those of the two calls, bit for bit.
 *   scores      [D]      fp32   in    importance of the D = max(M, N) candidate diagonals (Sec. 3.2 Eq. 4)
 *   values      [K x L]  dtype  in    values[k] belongs to the k-th chosen diagonal in ascending order of offset
 *   offsets_out [K]      int32  out   the chosen offsets, ascending (for dd_bwd_weight and the caller)
 *   prepared                    out   as for dd_prepare
 * Errors as for dd_prepare.
 */
dd_status dd_select_prepare(const dd_layer *layer, const float *scores, const void *values, int32_t *offsets_out,
                            void *prepared, size_t prepared_bytes, void *hip_stream);

/*
 * Backward product with respect to the input, dX = dY . W_K^T, over the same diagonals
 * (Sec. 3.3: the transposed matrix is again diagonal-sparse with the same starts, Appendix A).
 *   dY [tokens x N] in,  dX [tokens x M] out;  offsets / values exactly as given to dd_fwd.
 */
dd_status dd_bwd_input(const dd_layer *layer, const void *dY, const int32_t *offsets,
                       const void *values, void *dX, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * A group of n_sets diagonally sparse layers of one shape (M -> N, K diagonals each) that read the same input,
 * such as the query, key and value projections of an attention block where those are sparse (Sec. 4.3: GPT-2
 * with attention and MLP layers sparse).  Set s is the layer of Sec. 3.1 Eq. 3 with its own offsets and values:
 *   dd_fwd_shared        Y_s = X . W_s for every set, X read once;               Y  [n_sets][tokens x N] out
 *   dd_bwd_input_shared  dX = sum_s dY_s . W_s^T, summed in fp32 in one contraction and rounded once
 *                        (the gradient of the shared input);                     dY [n_sets][tokens x N] in
 * The n_sets output (gradient) matrices lie one after the other, each row-major and contiguous, so each is a
 * valid argument of dd_bwd_weight for its set.
 *   dd_prepare_shared    offsets [n_sets x K], values [n_sets x K x L] in; builds the dense operands of both
 *                        products for all sets into `prepared`: n_sets * dd_workspace_bytes(DD_OP_PREPARE, layer, 0)
 *                        bytes, 256-byte aligned, owned by the caller, valid until offsets or values change.
 *                        With n_sets = 1 the block equals the one dd_prepare fills.
 * layer->algo is not read by the two products (they always take the prepared operands); n_sets is 1..8.
 * DD_ERR_UNSUPPORTED where dd_prepare returns it, DD_ERR_WORKSPACE for a block that is too small or misaligned.
 * On other shapes or dtypes call dd_fwd / dd_bwd_input once per set.
 */
dd_status dd_prepare_shared(const dd_layer *layer, int32_t n_sets, const int32_t *offsets, const void *values,
                            void *prepared, size_t prepared_bytes, void *hip_stream);
dd_status dd_fwd_shared(const dd_layer *layer, int32_t n_sets, const void *X, const void *prepared,
                        size_t prepared_bytes, void *Y, void *hip_stream);
dd_status dd_bwd_input_shared(const dd_layer *layer, int32_t n_sets, const void *dY, const void *prepared,
                              size_t prepared_bytes, void *dX, void *hip_stream);

/*
 * Backward product with respect to the values on the K diagonals (Fig. 3 h, i): the dense
 * gradient X^T . dY restricted to the entries each diagonal owns, i.e. a sum over tokens,
 *   dValues[k][p] = sum_t X[t, row(k,p)] * dY[t, col(k,p)].
 *   X [tokens x M] in, dY [tokens x N] in, dValues [K x L] fp32 out (always fp32).
 * The sum over tokens is split into fixed chunks that are added in a fixed order: two calls
 * on the same inputs give bit-identical results.
 */
dd_status dd_bwd_weight(const dd_layer *layer, const void *X, const void *dY, const int32_t *offsets,
                        float *dValues, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * The backward pass of the layer as one call (Fig. 3 g-i; Sec. 3.3): dX exactly as dd_bwd_input and dValues exactly as
 * dd_bwd_weight compute them (bit for bit), issued back to back on one scratch block, input gradient first, so that
 * the weight gradient finds in the 256 MB memory-side cache whatever of dY that cache kept.  On the matrix cores the
 * two products are different contractions (over features, over tokens) whose tiles share neither registers nor
 * LDS; a schedule that takes the tokens in runs small enough for dY to stay cached between the two was built and
 * measured slower than this one at every benchmark shape (more launches and partial sums than the cached read saves).
 *   X [tokens x M], dY [tokens x N] in;  dX [tokens x M] out;  dValues [K x L] fp32 out.
 *   layer->algo = DD_ALGO_PREPARED: `prepared` is the block dd_prepare filled (values is not read); any other
 *   algo: prepared is not read.  DD_ALGO_BLOCKS: DD_ERR_UNSUPPORTED.
 *   ws: dd_workspace_bytes(DD_OP_BWD, layer, 0).  Errors as for the two calls.
 */
dd_status dd_bwd(const dd_layer *layer, const void *X, const void *dY, const int32_t *offsets, const void *values,
                 const void *prepared, size_t prepared_bytes, void *dX, float *dValues, void *ws, size_t ws_bytes,
                 void *hip_stream);

/*
 * dd_bwd_weight for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without `ws`, same kernels,
 * same results bit for bit; the partial sums of the token chunks go to an array inside the library,
 * dd_static_scratch_bytes() bytes (32 MiB) per GPU, which every GPU the library runs on holds from the first such
 * call until the process ends.  The call allocates and frees nothing.
 *   DD_ERR_WORKSPACE  dd_workspace_bytes(DD_OP_BWD_WEIGHT, layer, 0) exceeds dd_static_scratch_bytes(); nothing is
 *                     launched.  (Under DD_ALGO_AUTO that size covers both kernel families; where it is too large,
 *                     DD_ALGO_MATRIX, which needs less, may still fit.)
 * Every call on one GPU uses that GPU's one array: calls that overlap in time on one GPU (two streams, two
 * threads) race and give wrong sums; calls in stream order, or on different GPUs, are safe.  Nothing has to be
 * cleared between calls: the kernels write every partial sum before they read it.
 */
size_t dd_static_scratch_bytes(void);
dd_status dd_bwd_weight_static(const dd_layer *layer, const void *X, const void *dY, const int32_t *offsets,
                               float *dValues, void *hip_stream);

/*
 * Hard TopK re-selection of the active diagonals (Sec. 3.2, Eq. 4): for each of `batch`
 * score vectors alpha [D], the indices of the K largest scores.
 *   Order between scores: larger first; equal scores (and -0 / +0) by lower index; NaN ranks
 *   below every number.  The K chosen indices are written in ascending order, so the output
 *   row can be handed to dd_fwd / dd_bwd_* as `offsets` without leaving the device.
 *   scores      [batch x D] fp32   in
 *   offsets_out [batch x K] int32  out
 * DD_ERR_UNSUPPORTED if D > 65536.
 */
dd_status dd_select_diagonals(int32_t batch, int32_t D, int32_t K, const float *scores,
                              int32_t *offsets_out, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Soft TopK weights of the D candidate diagonals (Sec. 3.2, Eq. 5; the printed denominator is read as
 * a softmax over the candidates):
 *   alpha_tilde[b][i] = min(K * exp(scores[b][i] / temperature) / sum_j exp(scores[b][j] / temperature), 1).
 *   scores [batch x D] fp32 in, alpha_tilde [batch x D] fp32 out, temperature > 0 (else INVALID_ARG).
 * The index set of the K active diagonals is still chosen by dd_select_diagonals on the raw scores
 * (Eq. 5 is monotone in the score, so both orders agree); these weights only scale them (Eq. 4).
 */
dd_status dd_soft_topk(int32_t batch, int32_t D, int32_t K, float temperature, const float *scores,
                       float *alpha_tilde, void *hip_stream);

/*
 * The differentiable selection of Sec. 3.2 with its steps folded into the launches of the layer's own path (the
 * four calls above and below remain for callers that want the steps one by one; results agree as stated):
 *
 * dd_select_soft       dd_select_diagonals and dd_soft_topk on the same score vectors in one launch (Eq. 4 picks the K
 *                      diagonals, Eq. 5 weighs the D candidates).  offsets_out [batch x K] and alpha_tilde [batch x D]
 *                      are bit for bit those of the two calls.  Errors as for the two calls.
 * dd_prepare_scaled    dd_prepare on the effective values alpha_tilde[o_k] * V[k] (Eq. 4), formed while the dense
 *                      operands are built: no values_eff array is written or read.  alpha_tilde [D] fp32, V [K x L]
 *                      dtype; the block is bit for bit what dd_scale_values followed by dd_prepare builds.
 * dd_bwd_weight_scaled dd_bwd_weight followed by dd_scale_values_bwd, the adjoint of the scaling being the epilogue of
 *                      the weight gradient's ordered sum over the token chunks (no dValues array in between, three
 *                      launches instead of four):  dV[k][p] = alpha_tilde[o_k] * dValues[k][p]  [K x L] fp32 (bit for
 *                      bit as the two calls), d_alpha_tilde[i] = sum over the diagonals with o_k = i of
 *                      <dValues[k], V[k]>  [D] fp32 (0 elsewhere; within 1e-5, the dot products are summed in another
 *                      order).  An offset given three times or more: the order of those fp32 additions is unspecified.
 *                      ws: dd_workspace_bytes(DD_OP_BWD_WEIGHT_SCALED, layer, 0).  Matrix-core kernels only:
 *                      DD_ERR_UNSUPPORTED for fp32 storage, shapes dd_bwd_weight's matrix-core kernels do not cover,
 *                      X or dY not 16-byte aligned, DD_ALGO_VECTOR, tokens = 0 -- call the two steps there.
 */
dd_status dd_select_soft(int32_t batch, int32_t D, int32_t K, float temperature, const float *scores,
                         int32_t *offsets_out, float *alpha_tilde, void *hip_stream);
dd_status dd_prepare_scaled(const dd_layer *layer, const int32_t *offsets, const float *alpha_tilde, const void *V,
                            void *prepared, size_t prepared_bytes, void *hip_stream);
dd_status dd_bwd_weight_scaled(const dd_layer *layer, const void *X, const void *dY, const int32_t *offsets,
                               const float *alpha_tilde, const void *V, float *dV, float *d_alpha_tilde, void *ws,
                               size_t ws_bytes, void *hip_stream);

/*
 * Derivative of dd_soft_topk: d_scores [batch x D] from d_alpha_tilde [batch x D] (both fp32); entries
 * clamped to 1 pass no gradient.
 */
dd_status dd_soft_topk_bwd(int32_t batch, int32_t D, int32_t K, float temperature, const float *scores,
                           const float *d_alpha_tilde, float *d_scores, void *hip_stream);

/*
 * The values the products see (Sec. 3.2, Eq. 4): values_eff[k][p] = alpha_tilde[offsets[k] mod D] * V[k][p].
 *   offsets [K] int32, alpha_tilde [D] fp32, V and values_eff [K x L] of `dtype` (dd_dtype).
 */
dd_status dd_scale_values(int32_t K, int32_t L, int32_t D, int32_t dtype, const int32_t *offsets,
                          const float *alpha_tilde, const void *V, void *values_eff, void *hip_stream);

/*
 * Adjoint of dd_scale_values, applied to the output of dd_bwd_weight:
 *   dV[k][p] = alpha_tilde[o_k] * dValues[k][p]                          [K x L] fp32 out
 *   d_alpha_tilde[i] = sum over diagonals k with o_k = i of <dValues[k], V[k]>   [D] fp32 out (0 elsewhere)
 * Sums run in a fixed order.  ws: dd_workspace_bytes(DD_OP_SCALE_VALUES_BWD, layer with K set, 0) bytes.
 */
dd_status dd_scale_values_bwd(int32_t K, int32_t L, int32_t D, int32_t dtype, const int32_t *offsets,
                              const float *alpha_tilde, const void *V, const float *dValues, float *dV,
                              float *d_alpha_tilde, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Magnitude of each diagonal, the quantity the heuristic variant of the method (DiagHeur, appendix "Details
 * of the Heuristics-Based Method") ranks diagonals by.  The appendix names no norm; as in RigL, which it
 * follows, absolute values are summed:  magnitudes[k] = sum_p |values[k][p]|   (fp32, fixed summation order).
 *   values [K x L] of `dtype` in, magnitudes [K] fp32 out.
 */
dd_status dd_diag_magnitude(int32_t K, int32_t L, int32_t dtype, const void *values, float *magnitudes,
                            void *hip_stream);

/*
 * One DiagHeur update of the active set: the n_drop active diagonals of lowest magnitude leave and the n_drop
 * candidates with the largest `random` score among those that were not active enter (a diagonal that has just
 * left cannot return in the same update).  Order in both choices: larger first, equal values by lower offset,
 * NaN lowest.  The caller draws the random scores, so the update is a pure function of its arguments.
 *   offsets     [K] int32  in   the active diagonals, distinct modulo D (as dd_select_diagonals emits them)
 *   magnitudes  [K] fp32   in   non-negative, +inf or NaN (as dd_diag_magnitude emits them)
 *   random      [D] fp32   in   finite or NaN
 *   new_offsets [K] int32  out  the new active set, ascending
 *   source      [K] int32  out  for new diagonal j the position in `offsets` whose values it keeps, or -1
 *                               for a grown one (RigL starts grown weights at zero; that is the caller's move)
 * DD_ERR_INVALID_ARG unless 0 <= n_drop <= min(K, D - K).  DD_ERR_UNSUPPORTED if D > 65536.
 * ws: dd_workspace_bytes(DD_OP_DIAGHEUR, layer with in_features = D and K set, 0) bytes.
 */
dd_status dd_diagheur_update(int32_t D, int32_t K, int32_t n_drop, const int32_t *offsets, const float *magnitudes,
                             const float *random, int32_t *new_offsets, int32_t *source, void *ws, size_t ws_bytes,
                             void *hip_stream);

const char *dd_status_string(dd_status status);

#ifdef __cplusplus
}
#endif
#endif /* DYNADIAG_H */
