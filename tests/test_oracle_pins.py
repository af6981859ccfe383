"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU).

The oracle is the yardstick for the HIP kernels, so it is itself tied down here by things
that are not the oracle: index lists enumerated by hand from Sec. 3.1 Eq. 1 and Appendix A,
closed forms (identity, cyclic shift, truncation), the transposition theorem of Appendix A,
the coverage lemma of Appendix B, numpy's dense matmul on a matrix scattered in this file,
adjoint identities, finite differences, and numpy's stable sort for the selection.
"""
import os

import numpy as np
import pytest

from oracle import dd_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "diagonal_entries.txt")


def _golden_rows():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            head, tail = line.split("|")
            M, N, off = (int(x) for x in head.split())
            entries = [tuple(int(v) for v in e.split(",")) for e in tail.split()]
            rows.append((M, N, off, entries))
    return rows


@pytest.mark.parametrize("M,N,off,entries", _golden_rows())
def test_single_diagonal_matches_hand_enumeration(M, N, off, entries):
    L = min(M, N)
    assert len(entries) == L
    values = np.arange(1, L + 1, dtype=np.float64)[None, :]  # v[p] = p + 1 marks the position
    W = orc.materialize(M, N, [off], values)
    expect = np.zeros((M, N))
    for p, (r, c) in enumerate(entries):
        expect[r, c] = p + 1
    np.testing.assert_array_equal(W, expect)


def _scatter(M, N, offsets, values):
    """Dense W written out entry by entry from the two cases of Appendix A."""
    D, L = max(M, N), min(M, N)
    W = np.zeros((M, N))
    for k, s in enumerate(offsets):
        s = int(s) % D  # Python's % is already non-negative
        if M > N:
            for c in range(N):
                W[(s + c) % M, c] += values[k][c]
        else:
            for r in range(M):
                W[r, (s + r) % N] += values[k][r]
    assert L == values.shape[1]
    return W


SHAPES = [(4, 4), (7, 7), (5, 12), (12, 5), (6, 4), (4, 6), (1, 9), (9, 1), (16, 16), (3, 10)]


@pytest.mark.parametrize("M,N", SHAPES)
def test_materialize_matches_scatter_and_counts(M, N):
    rng = np.random.default_rng(100 * M + N)
    D, L = max(M, N), min(M, N)
    K = max(1, D // 3)
    offsets = rng.permutation(D)[:K].astype(np.int32)
    values = rng.uniform(0.5, 1.5, size=(K, L))  # strictly positive: no cancellation in nnz
    W = orc.materialize(M, N, offsets, values)
    np.testing.assert_array_equal(W, _scatter(M, N, offsets, values))
    # K diagonals of length min(M,N) hold (1-S) M N non-zeros (Sec. 3.1)
    assert np.count_nonzero(W) == K * L
    # each diagonal meets every short-side index exactly once (Appendix B, Lemma 1)
    per_short = np.count_nonzero(W, axis=1 if M <= N else 0)
    np.testing.assert_array_equal(per_short, np.full(L, K))


@pytest.mark.parametrize("M,N", SHAPES)
def test_transpose_is_the_swapped_case_with_the_same_start(M, N):
    """Appendix A: the transpose of a start-s diagonal is a start-s diagonal of the other case."""
    rng = np.random.default_rng(7 + 31 * M + N)
    D, L = max(M, N), min(M, N)
    K = min(D, 4)
    offsets = rng.integers(-2 * D, 2 * D, size=K).astype(np.int32)
    values = rng.standard_normal((K, L))
    W = orc.materialize(M, N, offsets, values)
    Wt = orc.materialize(N, M, offsets, values)
    if M != N:
        np.testing.assert_array_equal(W.T, Wt)
    else:
        # a square transposes into the opposite offsets, read at the shifted position
        neg = orc.materialize(M, N, -offsets, np.stack(
            [np.roll(values[k], int(offsets[k]) % D) for k in range(K)]))
        np.testing.assert_allclose(W.T, neg, rtol=0, atol=0)


def test_identity_shift_and_truncation_closed_forms():
    rng = np.random.default_rng(3)
    X = rng.standard_normal((5, 8))
    ones = np.ones((1, 8))
    np.testing.assert_array_equal(orc.fwd(X, [0], ones, 8), X)
    for o in (1, 3, 7, -1, 8 + 2):
        np.testing.assert_array_equal(orc.fwd(X, [o], ones, 8), np.roll(X, o, axis=1))
        # dY . W^T undoes the shift
        np.testing.assert_array_equal(orc.bwd_input(X, [o], ones, 8), np.roll(X, -o, axis=1))
    # expanding layer, offset 0, all ones: the input lands in the first M outputs
    Y = orc.fwd(X, [0], ones, 12)
    np.testing.assert_array_equal(Y[:, :8], X)
    np.testing.assert_array_equal(Y[:, 8:], 0)
    # contracting layer, offset 0, all ones: the first N inputs pass through
    Xw = rng.standard_normal((5, 12))
    np.testing.assert_array_equal(orc.fwd(Xw, [0], ones, 8), Xw[:, :8])
    # contracting layer, offset s: output c reads input (s + c) mod M
    np.testing.assert_array_equal(orc.fwd(Xw, [5], ones, 8), np.roll(Xw, -5, axis=1)[:, :8])


@pytest.mark.parametrize("M,N", SHAPES)
def test_products_match_numpy_on_the_scattered_matrix(M, N):
    rng = np.random.default_rng(1000 + 17 * M + N)
    D, L = max(M, N), min(M, N)
    T = 9
    K = max(1, D // 2)
    offsets = rng.permutation(D)[:K].astype(np.int32)
    offsets[0] -= D  # one negative offset
    values = rng.standard_normal((K, L))
    X = rng.standard_normal((T, M))
    dY = rng.standard_normal((T, N))
    W = _scatter(M, N, offsets, values)
    np.testing.assert_allclose(orc.fwd(X, offsets, values, N), X @ W, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(orc.bwd_input(dY, offsets, values, M), dY @ W.T, rtol=1e-13, atol=1e-13)
    G = X.T @ dY
    dV = orc.bwd_weight(X, dY, offsets)
    expect = np.empty((K, L))
    for k in range(K):
        mask = _scatter(M, N, offsets[k:k + 1], np.arange(1, L + 1, dtype=np.float64)[None, :])
        for p in range(L):
            r, c = np.argwhere(mask == p + 1)[0]
            expect[k, p] = G[r, c]
    np.testing.assert_allclose(dV, expect, rtol=1e-13, atol=1e-13)


def test_all_diagonals_is_a_dense_layer():
    """K = D with every offset once: W has no structural zero and the layer is dense."""
    rng = np.random.default_rng(5)
    for M, N in ((6, 6), (4, 10), (10, 4)):
        D, L = max(M, N), min(M, N)
        values = rng.uniform(1.0, 2.0, size=(D, L))
        W = orc.materialize(M, N, np.arange(D), values)
        assert np.count_nonzero(W) == M * N
        X = rng.standard_normal((3, M))
        np.testing.assert_allclose(orc.fwd(X, np.arange(D), values, N), X @ W, rtol=1e-13)
        # and every dense matrix is reachable: dValues is then the whole dense gradient
        dY = rng.standard_normal((3, N))
        dV = orc.bwd_weight(X, dY, np.arange(D))
        np.testing.assert_allclose(np.sort(dV.ravel()), np.sort((X.T @ dY).ravel()), rtol=1e-13)


def test_duplicate_offsets_add():
    rng = np.random.default_rng(6)
    values = rng.standard_normal((2, 8))
    X = rng.standard_normal((4, 8))
    both = orc.fwd(X, [3, 3], values, 8)
    once = orc.fwd(X, [3], values.sum(axis=0, keepdims=True), 8)
    np.testing.assert_allclose(both, once, rtol=1e-14, atol=1e-14)
    dY = rng.standard_normal((4, 8))
    dV = orc.bwd_weight(X, dY, [3, 3])
    np.testing.assert_array_equal(dV[0], dV[1])


@pytest.mark.parametrize("M,N", [(16, 16), (8, 24), (24, 8)])
def test_adjoint_identities(M, N):
    """<dY, fwd(X)> = <bwd_input(dY), X> = <bwd_weight(X, dY), values>: Y is bilinear in (X, values)."""
    rng = np.random.default_rng(11 + M)
    D, L = max(M, N), min(M, N)
    K = D // 4
    offsets = rng.permutation(D)[:K]
    values = rng.standard_normal((K, L))
    X = rng.standard_normal((13, M))
    dY = rng.standard_normal((13, N))
    a = np.sum(dY * orc.fwd(X, offsets, values, N))
    b = np.sum(orc.bwd_input(dY, offsets, values, M) * X)
    c = np.sum(orc.bwd_weight(X, dY, offsets) * values)
    assert abs(a - b) <= 1e-12 * abs(a)
    assert abs(a - c) <= 1e-12 * abs(a)


@pytest.mark.parametrize("M,N", [(6, 6), (4, 9), (9, 4)])
def test_gradients_match_finite_differences(M, N):
    rng = np.random.default_rng(13 + N)
    D, L = max(M, N), min(M, N)
    K = 3
    offsets = rng.permutation(D)[:K]
    values = rng.standard_normal((K, L))
    X = rng.standard_normal((5, M))
    dY = rng.standard_normal((5, N))

    def loss(Xa, va):
        return np.sum(orc.fwd(Xa, offsets, va, N) * dY)

    dX = orc.bwd_input(dY, offsets, values, M)
    dV = orc.bwd_weight(X, dY, offsets)
    h = 1e-3  # the loss is linear in each argument: central differences are exact up to rounding
    for (t, i) in [(0, 0), (2, M - 1), (4, M // 2)]:
        E = np.zeros_like(X)
        E[t, i] = h
        fd = (loss(X + E, values) - loss(X - E, values)) / (2 * h)
        assert abs(fd - dX[t, i]) <= 1e-9 * max(1.0, abs(fd))
    for (k, p) in [(0, 0), (1, L - 1), (2, L // 2)]:
        E = np.zeros_like(values)
        E[k, p] = h
        fd = (loss(X, values + E) - loss(X, values - E)) / (2 * h)
        assert abs(fd - dV[k, p]) <= 1e-9 * max(1.0, abs(fd))


def test_fwd_is_linear_in_x_and_in_values():
    rng = np.random.default_rng(17)
    M, N, K = 10, 14, 5
    offsets = rng.permutation(N)[:K]
    v1, v2 = rng.standard_normal((2, K, M))
    x1, x2 = rng.standard_normal((2, 4, M))
    f = lambda x, v: orc.fwd(x, offsets, v, N)
    np.testing.assert_allclose(f(2 * x1 - 3 * x2, v1), 2 * f(x1, v1) - 3 * f(x2, v1), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(f(x1, v1 + 0.5 * v2), f(x1, v1) + 0.5 * f(x1, v2), rtol=1e-12, atol=1e-12)


def test_sampled_weight_gradient_equals_full():
    rng = np.random.default_rng(19)
    for M, N in ((12, 12), (6, 20), (20, 6)):
        D, L = max(M, N), min(M, N)
        offsets = rng.permutation(D)[:4]
        X = rng.standard_normal((7, M))
        dY = rng.standard_normal((7, N))
        full = orc.bwd_weight(X, dY, offsets)
        ks = rng.integers(0, 4, size=30)
        ps = rng.integers(0, L, size=30)
        np.testing.assert_allclose(orc.bwd_weight_sampled(X, dY, offsets, ks, ps), full[ks, ps],
                                   rtol=1e-13, atol=1e-13)


# ---- selection (Sec. 3.2, Eq. 4: which K of the D importance scores are kept) ----

def _select_numpy(scores, K):
    s = np.array(scores, dtype=np.float32)
    s = np.where(np.isnan(s), -np.inf, s) + np.float32(0.0)  # -0 + 0 = +0
    nan_rank = np.isnan(np.asarray(scores, dtype=np.float32))
    order = np.lexsort((np.arange(s.size), -s.astype(np.float64), nan_rank))
    return np.sort(order[:K]).astype(np.int32)


def test_select_matches_numpy_sort():
    rng = np.random.default_rng(23)
    for D, K in ((64, 8), (768, 77), (1000, 1), (100, 100), (3072, 307)):
        scores = rng.standard_normal((3, D)).astype(np.float32)
        got = orc.select(scores, K)
        for b in range(3):
            np.testing.assert_array_equal(got[b], _select_numpy(scores[b], K))


def test_select_special_cases():
    rng = np.random.default_rng(29)
    s = rng.standard_normal(50).astype(np.float32)
    np.testing.assert_array_equal(orc.select(s, 50)[0], np.arange(50))
    assert orc.select(s, 1)[0, 0] == int(np.argmax(s))
    # ties go to the lower index
    np.testing.assert_array_equal(orc.select(np.array([1, 5, 5, 5, 0], np.float32), 2)[0], [1, 2])
    np.testing.assert_array_equal(orc.select(np.zeros(9, np.float32), 4)[0], [0, 1, 2, 3])
    # -0 equals +0, NaN ranks below everything, -inf is an ordinary number
    np.testing.assert_array_equal(orc.select(np.array([-0.0, 0.0, -1.0], np.float32), 2)[0], [0, 1])
    np.testing.assert_array_equal(
        orc.select(np.array([np.nan, -np.inf, np.nan, 2.0], np.float32), 3)[0], [0, 1, 3])
    # a strictly increasing transform of the scores keeps the choice (Eq. 5 is monotone in alpha)
    q = np.round(s * 4) / 4  # tie-heavy
    np.testing.assert_array_equal(orc.select(q, 13), orc.select(np.exp(q.astype(np.float64)).astype(np.float32), 13))
    np.testing.assert_array_equal(orc.select(q, 13)[0], _select_numpy(q, 13))


# ---- soft TopK weights (Sec. 3.2, Eq. 5) and the scaling of the diagonals by them (Eq. 4) ----

def test_soft_topk_closed_forms():
    # two candidates, K = 1: the softmax is a logistic function of the score difference
    for a0, a1, T in ((0.3, -1.1, 0.7), (2.0, 2.0, 1.0), (-4.0, 1.0, 2.5)):
        got = orc.soft_topk(np.array([a0, a1]), 1, T)[0]
        s0 = 1.0 / (1.0 + np.exp((a1 - a0) / T))
        np.testing.assert_allclose(got, [s0, 1.0 - s0], rtol=1e-14)
    rng = np.random.default_rng(31)
    a = rng.standard_normal(40)
    # before the clamp the weights sum to K; the clamp only ever lowers them
    for K, T in ((1, 1.0), (5, 0.5), (5, 50.0), (40, 3.0)):
        at = orc.soft_topk(a, K, T)[0]
        s = np.exp(a / T) / np.exp(a / T).sum()
        np.testing.assert_allclose(at, np.minimum(K * s, 1.0), rtol=1e-13)
        assert np.all(at <= 1.0) and np.all(at > 0.0)
    # a constant added to every score changes nothing; a hot temperature flattens to K / D
    np.testing.assert_allclose(orc.soft_topk(a + 123.0, 7, 0.9), orc.soft_topk(a, 7, 0.9), rtol=1e-10)
    np.testing.assert_allclose(orc.soft_topk(a, 8, 1e9)[0], np.full(40, 8 / 40), rtol=1e-6)
    # a cold temperature puts everything on the largest score
    cold = orc.soft_topk(a, 3, 1e-3)[0]
    assert cold[np.argmax(a)] == 1.0 and np.sum(cold) < 1.0 + 1e-9
    # monotone in the score: sorting by alpha_tilde never contradicts sorting by alpha
    at = orc.soft_topk(a, 6, 0.8)[0]
    order = np.argsort(a)
    assert np.all(np.diff(at[order]) >= 0)
    # rows are independent
    two = orc.soft_topk(np.stack([a, -a]), 6, 0.8)
    np.testing.assert_array_equal(two[0], at)
    np.testing.assert_array_equal(two[1], orc.soft_topk(-a, 6, 0.8)[0])


def test_soft_topk_gradient_matches_finite_differences():
    rng = np.random.default_rng(37)
    D, K, T = 12, 4, 0.6
    a = rng.standard_normal(D)
    at = orc.soft_topk(a, K, T)[0]
    assert np.any(at == 1.0) and np.any(at < 1.0)  # both branches of the min are exercised
    assert np.min(np.abs(K * np.exp(a / T) / np.exp(a / T).sum() - 1.0)) > 1e-3  # no score sits on the kink
    g = rng.standard_normal(D)
    got = orc.soft_topk_bwd(a, K, T, g)[0]
    h = 1e-6
    for i in range(D):
        e = np.zeros(D)
        e[i] = h
        fd = np.dot(g, orc.soft_topk(a + e, K, T)[0] - orc.soft_topk(a - e, K, T)[0]) / (2 * h)
        assert abs(fd - got[i]) <= 1e-7 * max(1.0, abs(fd))


def test_scale_values_and_its_adjoint():
    rng = np.random.default_rng(41)
    D, L, K = 10, 6, 4
    offsets = np.array([3, -1, 13, 3])  # -1 -> 9, 13 -> 3: offset 3 is held three times
    alpha = rng.uniform(0.1, 1.0, D)
    V = rng.standard_normal((K, L))
    eff = orc.scale_values(offsets, alpha, V)
    np.testing.assert_allclose(eff, alpha[[3, 9, 3, 3]][:, None] * V, rtol=1e-15)
    dValues = rng.standard_normal((K, L))
    dV, dalpha = orc.scale_values_bwd(offsets, alpha, V, dValues)
    # <dValues, alpha * V> is bilinear in (alpha, V): both gradients reproduce it
    ref = np.sum(dValues * eff)
    assert abs(np.sum(dV * V) - ref) <= 1e-12 * abs(ref)
    assert abs(np.dot(dalpha, alpha) - ref) <= 1e-12 * abs(ref)
    # entries of alpha no diagonal points at get no gradient; repeated offsets add
    assert np.count_nonzero(dalpha) == 2
    np.testing.assert_allclose(dalpha[3], np.sum(dValues[[0, 2, 3]] * V[[0, 2, 3]]), rtol=1e-13)
    np.testing.assert_allclose(dalpha[9], np.sum(dValues[1] * V[1]), rtol=1e-13)
    # chained with the layer: the loss <dY, fwd(X; alpha * V)> differentiated with respect to one alpha
    M = N = D
    X = rng.standard_normal((5, M))
    dY = rng.standard_normal((5, N))
    Vs = rng.standard_normal((K, M))
    loss = lambda al: np.sum(dY * orc.fwd(X, offsets, orc.scale_values(offsets, al, Vs), N))
    dValues = orc.bwd_weight(X, dY, offsets)
    _, dalpha = orc.scale_values_bwd(offsets, alpha, Vs, dValues)
    for i in (3, 9, 0):
        e = np.zeros(D)
        e[i] = 1e-4
        fd = (loss(alpha + e) - loss(alpha - e)) / 2e-4
        assert abs(fd - dalpha[i]) <= 1e-8 * max(1.0, abs(fd))


# ---- DiagHeur: drop the weakest diagonals, grow as many at random (appendix on the heuristics-based method) ----

def test_diag_magnitude_is_the_sum_of_absolute_values():
    rng = np.random.default_rng(5)
    V = rng.standard_normal((7, 33))
    np.testing.assert_allclose(orc.diag_magnitude(V), np.abs(V).sum(axis=1), rtol=1e-14)
    # closed forms: sign does not matter, scaling is homogeneous, a zero diagonal has magnitude zero
    np.testing.assert_allclose(orc.diag_magnitude(-3.0 * V), 3.0 * orc.diag_magnitude(V), rtol=1e-14)
    assert orc.diag_magnitude(np.zeros((2, 5))).tolist() == [0.0, 0.0]
    assert orc.diag_magnitude(np.array([[1.0, -2.0, 3.0], [0.0, 0.0, -0.5]])).tolist() == [6.0, 0.5]


def test_diagheur_update_worked_example():
    # active {1, 3, 6} with magnitudes {5, 1, 3}: offset 3 is the weakest and leaves; of the inactive
    # candidates {0, 2, 4, 5, 7} number 7 carries the largest random score and enters
    new, src = orc.diagheur_update(8, [1, 3, 6], [5.0, 1.0, 3.0], [0.1, 0.9, 0.8, 0.7, 0.6, 0.5, 0.4, 0.95], 1)
    assert new.tolist() == [1, 6, 7] and src.tolist() == [0, 2, -1]
    # unsorted input, two leave: the kept one is found wherever it stands
    new, src = orc.diagheur_update(8, [6, 1, 3], [3.0, 5.0, 1.0], [0.1, 0.9, 0.8, 0.7, 0.6, 0.5, 0.4, 0.95], 2)
    assert new.tolist() == [1, 2, 7] and src.tolist() == [1, -1, -1]
    # nothing leaves: the same set, ascending, every diagonal keeps its values
    new, src = orc.diagheur_update(8, [6, 1, 3], [3.0, 5.0, 1.0], np.zeros(8), 0)
    assert new.tolist() == [1, 3, 6] and src.tolist() == [1, 2, 0]
    # offsets are taken modulo D; equal magnitudes leave by higher offset first, equal scores enter by lower index
    new, src = orc.diagheur_update(6, [-1, 8], [2.0, 2.0], np.zeros(6), 1)   # offsets 5 and 2
    assert new.tolist() == [0, 2] and src.tolist() == [-1, 1]
    for bad in (3, -1):
        with pytest.raises(ValueError):
            orc.diagheur_update(5, [0, 1, 2], [1.0, 1.0, 1.0], np.zeros(5), bad)  # only two candidates to grow


def _diagheur_by_numpy(D, offsets, mags, rnd, n_drop):
    """The same update written with numpy's stable lexsort: keys (NaN last, value descending, index ascending)."""
    offsets = np.mod(np.asarray(offsets, dtype=np.int64), D)
    K = len(offsets)

    def order(values, index):
        values = np.asarray(values, dtype=np.float32)
        nan = np.isnan(values)
        return np.lexsort((index, -np.where(nan, 0, values), nan))

    kept = offsets[order(mags, offsets)[:K - n_drop]]
    inactive = np.setdiff1d(np.arange(D), offsets)
    grown = inactive[order(np.asarray(rnd)[inactive], inactive)[:n_drop]]
    new = np.sort(np.concatenate([kept, grown]))
    slot = {int(o): k for k, o in enumerate(offsets)}
    return new, np.array([slot[int(o)] if int(o) in set(kept.tolist()) else -1 for o in new])


@pytest.mark.parametrize("D,K,n_drop,seed", [(16, 5, 2, 0), (64, 8, 8, 1), (64, 50, 14, 2), (768, 77, 23, 3),
                                             (100, 100, 0, 4), (33, 1, 1, 5), (257, 128, 64, 6)])
def test_diagheur_update_against_numpy_and_invariants(D, K, n_drop, seed):
    rng = np.random.default_rng(seed)
    offsets = rng.permutation(D)[:K].astype(np.int32)
    # few distinct values so that ties occur, some NaN, signed zeros
    mags = rng.integers(0, 4, K).astype(np.float32)
    rnd = (rng.integers(0, 5, D) / 4).astype(np.float32)
    if K > 3:
        mags[1] = np.nan
    if D > 10:
        rnd[[2, 7]] = np.nan
        rnd[5] = -0.0
    new, src = orc.diagheur_update(D, offsets, mags, rnd, n_drop)
    ref_new, ref_src = _diagheur_by_numpy(D, offsets, mags, rnd, n_drop)
    assert new.tolist() == ref_new.tolist() and src.tolist() == ref_src.tolist()
    # invariants: K distinct diagonals, ascending; the kept ones were active and keep their own values,
    # the grown ones were not active; as many enter as leave
    assert len(set(new.tolist())) == K and np.all(np.diff(new) > 0)
    old = set(offsets.tolist())
    assert sum(o not in old for o in new.tolist()) == n_drop == int(np.sum(src < 0))
    for o, k in zip(new.tolist(), src.tolist()):
        assert (k >= 0 and offsets[k] == o) or (k < 0 and o not in old)
    # no dropped diagonal outranks a kept one
    key = lambda m: -np.inf if np.isnan(m) else m
    kept_slots = [k for k in src.tolist() if k >= 0]
    dropped = [k for k in range(K) if k not in kept_slots]
    if kept_slots and dropped:
        assert max(key(mags[k]) for k in dropped) <= min(key(mags[k]) for k in kept_slots)
