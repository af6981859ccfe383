"""GPU parity of the shared-input group (dd_prepare_shared, dd_fwd_shared, dd_bwd_input_shared): several
diagonally sparse layers of one shape that read the same input.  The oracle has no entry of its own for a
group: by definition set s is the plain layer with its own (offsets, values), so Y_s = fwd(X, set s) and the
gradient of the shared input is the sum over the sets of bwd_input(dY_s, set s), summed here in fp64."""
import numpy as np
import pytest
import torch

import paper_2506_11449_amd as dd
from oracle import dd_oracle as orc
from paper_2506_11449_amd import synth
from tests.parity_util import TOL, TOL_DV, rel_err, to_dev, to_host

pytestmark = pytest.mark.gpu


def group_case(M, N, K, T, S, seed):
    rng = np.random.default_rng(seed)
    D, L = max(M, N), min(M, N)
    offsets = np.stack([np.sort(rng.permutation(D)[:K]) for _ in range(S)]).astype(np.int32)
    values = synth.round_to_bf16((rng.standard_normal((S, K, L)) * 0.02).astype(np.float32))
    X = synth.round_to_bf16(rng.standard_normal((T, M)).astype(np.float32))
    dY = synth.round_to_bf16(rng.standard_normal((S, T, N)).astype(np.float32))
    return offsets, values, X, dY


def oracle_group(offsets, values, X, dY, M, N, rows=None):
    S = offsets.shape[0]
    if rows is not None:
        X, dY = X[rows], dY[:, rows]
    Y = np.stack([orc.fwd(X, offsets[s], values[s], N) for s in range(S)])
    dX = sum(orc.bwd_input(np.ascontiguousarray(dY[s]), offsets[s], values[s], M) for s in range(S))
    return Y, dX


# (M, N, K, T, S): square, expanding and contracting layers; set widths of 128 and 384, so that 256-column result
# tiles hold two sets or straddle a set boundary and the contraction changes matrix every 2 or 6 k-slices; one
# token; the largest group; results of 128-wide column tiles (3 x 128).
GROUPS = [
    (768, 768, 77, 300, 3),
    (128, 384, 40, 415, 2),
    (384, 128, 30, 200, 4),
    (256, 128, 26, 161, 3),
    (128, 128, 13, 1, 8),
    (128, 128, 13, 333, 3),
    (1024, 1024, 51, 257, 2),
    (128, 256, 26, 90, 1),
]


@pytest.mark.parametrize("M,N,K,T,S", GROUPS)
def test_group_against_oracle(M, N, K, T, S):
    offsets, values, X, dY = group_case(M, N, K, T, S, seed=31 * M + 7 * N + S)
    d_X, d_dY = to_dev(X, "bf16"), to_dev(dY, "bf16")
    prepared = None
    for round_ in range(2):
        if round_ == 1:  # refill the same block for other diagonals: repeated and negative offsets among them
            offsets = offsets.copy()
            offsets[:, 0] = offsets[:, -1]
            offsets[S - 1, K // 2] = offsets[S - 1, -1] - max(M, N)
        d_off, d_val = torch.from_numpy(offsets).cuda(), to_dev(values, "bf16")
        prepared = dd.dd_prepare_shared(d_off, d_val, M, N, prepared=prepared)
        Y = dd.dd_fwd_shared(d_X, prepared)
        dX = dd.dd_bwd_input_shared(d_dY, prepared)
        torch.cuda.synchronize()
        assert Y.shape == (S, T, N) and dX.shape == (T, M)
        ref_Y, ref_dX = oracle_group(offsets, values, X, dY, M, N)
        for s in range(S):
            assert rel_err(to_host(Y[s]), ref_Y[s]) <= TOL["bf16"], f"set {s}"
        assert rel_err(to_host(dX), ref_dX) <= TOL["bf16"]
        # every set's forward result is the one the plain prepared call gives, bit for bit (same contraction order)
        for s in range(S):
            one = dd.dd_prepare(d_off[s], d_val[s], M, N)
            Y1 = dd.dd_fwd(d_X, None, None, N, prepared=one)
            assert torch.equal(Y[s].view(torch.int16), Y1.view(torch.int16)), f"set {s}"
            if S == 1:
                assert torch.equal(one.buf, prepared.buf)
                dX1 = dd.dd_bwd_input(d_dY[0], None, None, M, prepared=one)
                assert torch.equal(dX.view(torch.int16), dX1.view(torch.int16))
        # each slice of the stacked gradient is a valid operand of the weight gradient of its set
        s = S - 1
        dV = dd.dd_bwd_weight(d_X, d_dY[s], d_off[s])
        assert rel_err(to_host(dV), orc.bwd_weight(X, np.ascontiguousarray(dY[s]), offsets[s])) <= TOL_DV


@pytest.mark.parametrize("M,N,K,T,S", [(512, 512, 50, 7000, 3), (2048, 128, 40, 5300, 3), (128, 384, 40, 14000, 2)])
def test_group_with_more_tiles_than_cus(M, N, K, T, S):
    """Results with more than 256 tiles go through the kernel in which a workgroup walks several tiles: the forward
    product of the first and the last case, the backward-input product of the second."""
    offsets, values, X, dY = group_case(M, N, K, T, S, seed=M + N + T)
    prepared = dd.dd_prepare_shared(torch.from_numpy(offsets).cuda(), to_dev(values, "bf16"), M, N)
    Y = dd.dd_fwd_shared(to_dev(X, "bf16"), prepared)
    dX = dd.dd_bwd_input_shared(to_dev(dY, "bf16"), prepared)
    ref_Y, ref_dX = oracle_group(offsets, values, X, dY, M, N)
    for s in range(S):
        assert rel_err(to_host(Y[s]), ref_Y[s]) <= TOL["bf16"], f"set {s}"
    assert rel_err(to_host(dX), ref_dX) <= TOL["bf16"]


def test_qkv_of_the_vitb_attention_block_sampled():
    """Three 768 -> 768 layers at 90 % sparsity over the 12608 tokens of the benchmark: sampled token rows (rows are
    independent, so the oracle on a subset of rows gives those rows of the full result)."""
    layer = synth.WORKLOADS["vitb_attn_proj"][0]
    M, N, K, T, S = layer.in_features, layer.out_features, layer.K, layer.tokens, 3
    offsets, values, X, dY = group_case(M, N, K, T, S, seed=2506)
    prepared = dd.dd_prepare_shared(torch.from_numpy(offsets).cuda(), to_dev(values, "bf16"), M, N)
    Y = to_host(dd.dd_fwd_shared(to_dev(X, "bf16"), prepared))
    dX = to_host(dd.dd_bwd_input_shared(to_dev(dY, "bf16"), prepared))
    rng = np.random.default_rng(2506)
    rows = np.unique(np.concatenate([[0, T - 1], rng.integers(0, T, 64)]))
    ref_Y, ref_dX = oracle_group(offsets, values, X, dY, M, N, rows=rows)
    assert rel_err(Y[:, rows], ref_Y) <= TOL["bf16"]
    assert rel_err(dX[rows], ref_dX) <= TOL["bf16"]
    assert np.all(np.isfinite(Y)) and np.all(np.isfinite(dX))


def test_group_rules():
    off = torch.zeros((3, 4), dtype=torch.int32, device="cuda")
    for M, N, dtype in ((100, 768, torch.bfloat16), (768, 768, torch.float32)):
        val = torch.zeros((3, 4, min(M, N)), dtype=dtype, device="cuda")
        with pytest.raises(dd.DynaDiagError) as e:
            dd.dd_prepare_shared(off, val, M, N)
        assert e.value.status == 2
    val = torch.zeros((3, 4, 128), dtype=torch.bfloat16, device="cuda")
    prepared = dd.dd_prepare_shared(off, val, 128, 256)
    with pytest.raises(ValueError):
        dd.dd_fwd_shared(torch.zeros((5, 256), dtype=torch.bfloat16, device="cuda"), prepared)  # M is 128
    with pytest.raises(ValueError):
        dd.dd_bwd_input_shared(torch.zeros((2, 5, 256), dtype=torch.bfloat16, device="cuda"), prepared)  # 3 sets
    with pytest.raises(ValueError):
        dd.dd_prepare_shared(off[:2], val[:2], 128, 256, prepared=prepared)
    # no tokens: nothing is launched, empty results come back
    assert dd.dd_fwd_shared(torch.zeros((0, 128), dtype=torch.bfloat16, device="cuda"), prepared).shape == (3, 0, 256)
    assert dd.dd_bwd_input_shared(torch.zeros((3, 0, 256), dtype=torch.bfloat16, device="cuda"), prepared).shape == (0, 128)


@pytest.mark.parametrize("seed", range(12))
def test_random_groups(seed):
    """Seeded random shapes (feature counts multiples of 128 up to 1024, any K, any token count up to 2000, one to
    four sets): the group calls, the plain prepared calls and the self-contained calls against the oracle."""
    rng = np.random.default_rng(9000 + seed)
    M, N = (int(rng.integers(1, 9)) * 128 for _ in range(2))
    D = max(M, N)
    K = int(rng.integers(1, D + 1)) if seed % 3 == 0 else int(rng.integers(1, D // 8 + 2))
    T = int(rng.integers(1, 2001))
    S = int(rng.integers(1, 5))
    offsets, values, X, dY = group_case(M, N, K, T, S, seed=seed)
    d_off, d_val = torch.from_numpy(offsets).cuda(), to_dev(values, "bf16")
    d_X, d_dY = to_dev(X, "bf16"), to_dev(dY, "bf16")
    prepared = dd.dd_prepare_shared(d_off, d_val, M, N)
    Y = dd.dd_fwd_shared(d_X, prepared)
    dX = dd.dd_bwd_input_shared(d_dY, prepared)
    ref_Y, ref_dX = oracle_group(offsets, values, X, dY, M, N)
    for s in range(S):
        assert rel_err(to_host(Y[s]), ref_Y[s]) <= TOL["bf16"], (M, N, K, T, S, s)
    assert rel_err(to_host(dX), ref_dX) <= TOL["bf16"], (M, N, K, T, S)
    s = int(rng.integers(0, S))
    Y1 = dd.dd_fwd(d_X, d_off[s], d_val[s], N)                       # kernel family by shape and density
    dX1 = dd.dd_bwd_input(d_dY[s], d_off[s], d_val[s], M)
    dV1 = dd.dd_bwd_weight(d_X, d_dY[s], d_off[s])
    assert rel_err(to_host(Y1), ref_Y[s]) <= TOL["bf16"], (M, N, K, T, S, s)
    assert rel_err(to_host(dX1), orc.bwd_input(np.ascontiguousarray(dY[s]), offsets[s], values[s], M)) <= TOL["bf16"]
    assert rel_err(to_host(dV1), orc.bwd_weight(X, np.ascontiguousarray(dY[s]), offsets[s])) <= TOL_DV
