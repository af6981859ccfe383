/*
 * CPU oracle for the diagonally-sparse linear layer (DynaDiag, arxiv 2506.11449).
 *
 * TEST INFRASTRUCTURE ONLY.  Slow, plain, fp64.  Nothing in the product path may
 * call this file; it shares no code, header, table or helper with the HIP library.
 *
 * What it computes, and where the paper defines it:
 *   - the weight matrix W_K as a sum of K wrapped diagonals            (Sec. 3.1, Eq. 1-3)
 *   - rectangular orientation of a diagonal and of its transpose        (Appendix A, both cases)
 *   - forward  Y  = X  . W_K                                            (Fig. 3 b-e)
 *   - backward dX = dY . W_K^T over the same diagonals                  (Sec. 3.3; Fig. 3 g)
 *   - backward dV: the gradient restricted to the K diagonals           (Fig. 3 h, i)
 *   - hard TopK choice of K of the D candidate diagonals                (Sec. 3.2, Eq. 4)
 *   - soft TopK weights, their derivative, and the scaling of the
 *     diagonals by them with its adjoint                                (Sec. 3.2, Eq. 4 and Eq. 5)
 *   - the heuristic update of the active set (DiagHeur): magnitude of
 *     each diagonal, drop the weakest, grow as many at random           (Appendix "Details of the
 *                                                                        Heuristics-Based Method")
 *
 * Reading of the rectangular convention (the paper states it in two incompatible
 * ways; this is the one under which the K-from-sparsity footnote of Sec. 3.1, the
 * size of alpha in Sec. 3.2, Lemma 1 of Appendix B and all of Appendix A agree):
 *   D = max(M, N) candidate diagonals, each of length L = min(M, N), wrap modulus D.
 *   Position p in [0, L) along diagonal k sits at long-side index q = (p + o_k) mod D.
 *   M <= N (square included): entry (row, col) = (p, q)     -- Appendix A, case m < n, and Eq. 1
 *   M >  N                  : entry (row, col) = (q, p)     -- Appendix A, case m >= n
 *   The value vector v_k has L entries and is indexed by p.
 *   Offsets may be any integer; they are taken modulo D (a negative offset is a
 *   diagonal below the main one, Sec. 3.1).  Repeated offsets add (Eq. 3 is a sum).
 *
 * All matrices are row-major and contiguous.  All floating point is double; callers
 * widen fp32 / bf16 inputs exactly before calling.
 *
 * Every function is pinned by tests/test_oracle_pins.py against hand-enumerated
 * index lists, closed forms (identity, cyclic shift), numpy's dense matmul on a
 * brute-force scatter, adjoint identities, finite differences and numpy's stable
 * argsort.  Parity is pinned for every function in this file.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* number of threads the row loops will use */
int ddo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static int64_t canon(int64_t off, int64_t D)
{
    int64_t r = off % D;
    if (r < 0) r += D;
    return r;
}

/* Sec. 3.1 Eq. 1-3 with the Appendix A orientation: W[M x N] = sum_k P_k diag(v_k). */
void ddo_materialize(int M, int N, int K, const int32_t *offsets, const double *values, double *W)
{
    const int64_t D = M > N ? M : N;
    const int64_t L = M < N ? M : N;
    memset(W, 0, sizeof(double) * (size_t)M * (size_t)N);
    for (int k = 0; k < K; ++k) {
        const int64_t o = canon(offsets[k], D);
        for (int64_t p = 0; p < L; ++p) {
            const int64_t q = (p + o) % D;
            int64_t row, col;
            if (M <= N) { row = p; col = q; } else { row = q; col = p; }
            W[row * N + col] += values[(int64_t)k * L + p];
        }
    }
}

/* Y[T x N] = X[T x M] . W : the plain definition, one token row at a time. */
static void dense_fwd(int64_t T, int M, int N, const double *W, const double *X, double *Y)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        double *y = Y + t * N;
        const double *x = X + t * M;
        for (int j = 0; j < N; ++j) y[j] = 0.0;
        for (int i = 0; i < M; ++i) {
            const double xi = x[i];
            const double *w = W + (int64_t)i * N;
            for (int j = 0; j < N; ++j) y[j] += xi * w[j];
        }
    }
}

/* dX[T x M] = dY[T x N] . W^T */
static void dense_bwd_input(int64_t T, int M, int N, const double *W, const double *dY, double *dX)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        const double *g = dY + t * N;
        double *dx = dX + t * M;
        for (int i = 0; i < M; ++i) {
            const double *w = W + (int64_t)i * N;
            double s = 0.0;
            for (int j = 0; j < N; ++j) s += g[j] * w[j];
            dx[i] = s;
        }
    }
}

int ddo_fwd(int64_t T, int M, int N, int K, const int32_t *offsets, const double *values,
            const double *X, double *Y)
{
    double *W = (double *)malloc(sizeof(double) * (size_t)M * (size_t)N);
    if (!W) return 1;
    ddo_materialize(M, N, K, offsets, values, W);
    dense_fwd(T, M, N, W, X, Y);
    free(W);
    return 0;
}

int ddo_bwd_input(int64_t T, int M, int N, int K, const int32_t *offsets, const double *values,
                  const double *dY, double *dX)
{
    double *W = (double *)malloc(sizeof(double) * (size_t)M * (size_t)N);
    if (!W) return 1;
    ddo_materialize(M, N, K, offsets, values, W);
    dense_bwd_input(T, M, N, W, dY, dX);
    free(W);
    return 0;
}

/* Row and column of position p on diagonal with raw offset off (same rule as ddo_materialize). */
static void entry_of(int M, int N, int32_t off, int64_t p, int64_t *row, int64_t *col)
{
    const int64_t D = M > N ? M : N;
    const int64_t q = (p + canon(off, D)) % D;
    if (M <= N) { *row = p; *col = q; } else { *row = q; *col = p; }
}

/*
 * Gradient of the loss with respect to the values on the K diagonals (Fig. 3 h, i):
 * the dense gradient G = X^T . dY [M x N], read back at the entries each diagonal owns.
 */
int ddo_bwd_weight(int64_t T, int M, int N, int K, const int32_t *offsets,
                   const double *X, const double *dY, double *dValues)
{
    const int64_t L = M < N ? M : N;
    double *G = (double *)calloc((size_t)M * (size_t)N, sizeof(double));
    if (!G) return 1;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < M; ++i) {
        double *g = G + (int64_t)i * N;
        for (int64_t t = 0; t < T; ++t) {
            const double xi = X[t * M + i];
            const double *dy = dY + t * N;
            for (int j = 0; j < N; ++j) g[j] += xi * dy[j];
        }
    }
    for (int k = 0; k < K; ++k)
        for (int64_t p = 0; p < L; ++p) {
            int64_t row, col;
            entry_of(M, N, offsets[k], p, &row, &col);
            dValues[(int64_t)k * L + p] = G[row * N + col];
        }
    free(G);
    return 0;
}

/*
 * The same gradient, but only for a list of (diagonal, position) samples, each computed
 * from the definition G[row, col] = sum_t X[t, row] dY[t, col].  For sizes at which the
 * full dense G would take minutes.
 */
void ddo_bwd_weight_sampled(int64_t T, int M, int N, const int32_t *offsets,
                            const double *X, const double *dY,
                            int64_t n_samples, const int32_t *sample_k, const int32_t *sample_p,
                            double *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t s = 0; s < n_samples; ++s) {
        int64_t row, col;
        entry_of(M, N, offsets[sample_k[s]], sample_p[s], &row, &col);
        double acc = 0.0;
        for (int64_t t = 0; t < T; ++t) acc += X[t * M + row] * dY[t * N + col];
        out[s] = acc;
    }
}

/* ---- hard TopK of the importance scores (Sec. 3.2, Eq. 4) ---- */

typedef struct { float score; int32_t index; } scored;

/* Total order: larger score first; NaN ranks below every number; -0 equals +0; ties by smaller index. */
static int scored_cmp(const void *pa, const void *pb)
{
    const scored *a = (const scored *)pa, *b = (const scored *)pb;
    const int an = isnan(a->score), bn = isnan(b->score);
    if (an != bn) return an ? 1 : -1;
    if (!an) {
        if (a->score > b->score) return -1;
        if (a->score < b->score) return 1;
    }
    return (a->index > b->index) - (a->index < b->index);
}

static int int32_cmp(const void *pa, const void *pb)
{
    const int32_t a = *(const int32_t *)pa, b = *(const int32_t *)pb;
    return (a > b) - (a < b);
}

/*
 * For each of `batch` score vectors of length D: full sort by the total order above,
 * keep the first K indices, emit them in ascending index order.
 */
int ddo_select(int batch, int D, int K, const float *scores, int32_t *offsets_out)
{
    scored *buf = (scored *)malloc(sizeof(scored) * (size_t)D);
    if (!buf) return 1;
    for (int b = 0; b < batch; ++b) {
        for (int i = 0; i < D; ++i) { buf[i].score = scores[(int64_t)b * D + i]; buf[i].index = i; }
        qsort(buf, (size_t)D, sizeof(scored), scored_cmp);
        int32_t *out = offsets_out + (int64_t)b * K;
        for (int i = 0; i < K; ++i) out[i] = buf[i].index;
        qsort(out, (size_t)K, sizeof(int32_t), int32_cmp);
    }
    free(buf);
    return 0;
}

/* ---- soft TopK weights and the scaling of the diagonals by them (Sec. 3.2, Eq. 4 and Eq. 5) ---- */

/*
 * Eq. 5: alpha_tilde_i = min(K * exp(alpha_i / temp) / sum_j exp(alpha_j / temp), 1).
 * (The printed denominator carries the index i; it is read as the sum over j, i.e. a softmax.)
 * The maximum is subtracted before exponentiation, which leaves the quotient unchanged.
 */
void ddo_soft_topk(int batch, int D, int K, double temp, const double *scores, double *alpha_tilde)
{
    for (int b = 0; b < batch; ++b) {
        const double *a = scores + (int64_t)b * D;
        double *out = alpha_tilde + (int64_t)b * D;
        double amax = a[0];
        for (int i = 1; i < D; ++i) if (a[i] > amax) amax = a[i];
        double sum = 0.0;
        for (int i = 0; i < D; ++i) sum += exp((a[i] - amax) / temp);
        for (int i = 0; i < D; ++i) {
            const double v = (double)K * exp((a[i] - amax) / temp) / sum;
            out[i] = v < 1.0 ? v : 1.0;
        }
    }
}

/*
 * Derivative of Eq. 5: with s = softmax(alpha / temp) and m_j = 1 where K s_j < 1 (not clamped), else 0,
 *   dalpha_i = (K / temp) * s_i * (m_i g_i - sum_j m_j g_j s_j),   g = dL/dalpha_tilde.
 */
void ddo_soft_topk_bwd(int batch, int D, int K, double temp, const double *scores, const double *g,
                       double *dscores)
{
    double *s = (double *)malloc(sizeof(double) * (size_t)D);
    for (int b = 0; b < batch; ++b) {
        const double *a = scores + (int64_t)b * D, *gb = g + (int64_t)b * D;
        double *out = dscores + (int64_t)b * D;
        double amax = a[0];
        for (int i = 1; i < D; ++i) if (a[i] > amax) amax = a[i];
        double sum = 0.0;
        for (int i = 0; i < D; ++i) { s[i] = exp((a[i] - amax) / temp); sum += s[i]; }
        double dot = 0.0;
        for (int i = 0; i < D; ++i) {
            s[i] /= sum;
            if ((double)K * s[i] < 1.0) dot += gb[i] * s[i];
        }
        for (int i = 0; i < D; ++i) {
            const double mi = (double)K * s[i] < 1.0 ? 1.0 : 0.0;
            out[i] = (double)K / temp * s[i] * (mi * gb[i] - dot);
        }
    }
    free(s);
}

/* Eq. 4: the values the products see, values_eff[k][p] = alpha_tilde[o_k mod D] * V[k][p]. */
void ddo_scale_values(int K, int L, int D, const int32_t *offsets, const double *alpha_tilde, const double *V,
                      double *values_eff)
{
    for (int k = 0; k < K; ++k) {
        const double a = alpha_tilde[canon(offsets[k], D)];
        for (int p = 0; p < L; ++p) values_eff[(int64_t)k * L + p] = a * V[(int64_t)k * L + p];
    }
}

/*
 * Its adjoint: given dValues = dL/dvalues_eff,
 *   dV[k][p] = alpha_tilde[o_k] * dValues[k][p],   dalpha_tilde[i] = sum_{k: o_k = i} <dValues[k], V[k]>.
 */
void ddo_scale_values_bwd(int K, int L, int D, const int32_t *offsets, const double *alpha_tilde, const double *V,
                          const double *dValues, double *dV, double *dalpha_tilde)
{
    for (int i = 0; i < D; ++i) dalpha_tilde[i] = 0.0;
    for (int k = 0; k < K; ++k) {
        const int64_t o = canon(offsets[k], D);
        double dot = 0.0;
        for (int p = 0; p < L; ++p) {
            dV[(int64_t)k * L + p] = alpha_tilde[o] * dValues[(int64_t)k * L + p];
            dot += dValues[(int64_t)k * L + p] * V[(int64_t)k * L + p];
        }
        dalpha_tilde[o] += dot;
    }
}

/* ---- DiagHeur: prune the diagonals of lowest magnitude, grow as many at random (Appendix, heuristics) ---- */

/*
 * Magnitude of a diagonal.  The appendix says "lowest magnitudes" without naming a norm; RigL, which it
 * follows, ranks single weights by |w|, so the sum of |v_k[p]| over the diagonal is read (all diagonals
 * have the same length, so sum and mean rank alike).
 */
void ddo_diag_magnitude(int K, int L, const double *values, double *magnitudes)
{
    for (int k = 0; k < K; ++k) {
        double s = 0.0;
        for (int p = 0; p < L; ++p) s += fabs(values[(int64_t)k * L + p]);
        magnitudes[k] = s;
    }
}

/*
 * One update of the active set.  offsets [K]: the active diagonals, distinct modulo D.  Of them the
 * n_drop with the lowest magnitude leave (order: larger magnitude first, equal magnitudes by lower offset,
 * NaN lowest; the first K - n_drop stay).  Of the D - K candidates that were not active, the n_drop with
 * the largest `random` score enter (same order, by candidate index); a diagonal that has just left is not
 * a candidate, as in RigL.  new_offsets [K]: the new set, ascending.  source [K]: for each new diagonal the
 * position in `offsets` whose values it keeps, or -1 if it was grown (RigL starts grown weights at zero).
 * Returns 1 if the arguments do not allow the update (n_drop > K or n_drop > D - K), 2 on allocation failure.
 */
int ddo_diagheur_update(int D, int K, int n_drop, const int32_t *offsets, const float *magnitudes,
                        const float *random, int32_t *new_offsets, int32_t *source)
{
    if (n_drop < 0 || n_drop > K || n_drop > D - K) return 1;
    int32_t *slot = (int32_t *)malloc(sizeof(int32_t) * (size_t)D);
    scored *act = (scored *)malloc(sizeof(scored) * (size_t)K);
    scored *cand = (scored *)malloc(sizeof(scored) * (size_t)(D - K > 0 ? D - K : 1));
    if (!slot || !act || !cand) { free(slot); free(act); free(cand); return 2; }
    for (int i = 0; i < D; ++i) slot[i] = -1;
    for (int k = 0; k < K; ++k) {
        const int o = (int)((((int64_t)offsets[k] % D) + D) % D);
        slot[o] = k;
        act[k].score = magnitudes[k];
        act[k].index = o;
    }
    qsort(act, (size_t)K, sizeof(scored), scored_cmp);
    int n = 0;
    for (int i = 0; i < K - n_drop; ++i) new_offsets[n++] = act[i].index;
    int c = 0;
    for (int i = 0; i < D; ++i)
        if (slot[i] < 0) { cand[c].score = random[i]; cand[c].index = i; ++c; }
    qsort(cand, (size_t)c, sizeof(scored), scored_cmp);
    for (int i = 0; i < n_drop; ++i) new_offsets[n++] = cand[i].index;
    qsort(new_offsets, (size_t)K, sizeof(int32_t), int32_cmp);
    for (int j = 0; j < K; ++j) {
        const int k = slot[new_offsets[j]];
        /* a diagonal that has just left cannot come back in the same update, so slot >= 0 means kept */
        source[j] = k;
    }
    free(slot); free(act); free(cand);
    return 0;
}
