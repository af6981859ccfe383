"""dd_bwd, the backward pass as one call (input gradient, then weight gradient, on one scratch block), against the CPU
oracle and, bit for bit, against the two plain calls."""
import numpy as np
import pytest
import torch

import paper_2506_11449_amd as dd
from oracle import dd_oracle as orc
from paper_2506_11449_amd import synth
from tests.parity_util import TOL, TOL_DV, random_case, rel_err, to_dev, to_host

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("prepared", [False, True])
@pytest.mark.parametrize("M,N,K,T", [(768, 768, 77, 300), (768, 3072, 307, 430), (3072, 768, 307, 130), (128, 384, 40, 4150),
                                     (1024, 1024, 51, 257), (256, 128, 26, 1)])
def test_equals_the_two_calls(M, N, K, T, prepared):
    offsets, values, X, dY = random_case(M, N, K, T, "bf16", seed=M + N + K + T)
    d_off, d_val = torch.from_numpy(offsets).cuda(), to_dev(values, "bf16")
    d_X, d_dY = to_dev(X, "bf16"), to_dev(dY, "bf16")
    prep = dd.dd_prepare(d_off, d_val, M, N) if prepared else None
    dX, dV = dd.dd_bwd(d_X, d_dY, d_off, d_val, prepared=prep)
    assert rel_err(to_host(dX), orc.bwd_input(dY, offsets, values, M)) <= TOL["bf16"]
    assert rel_err(to_host(dV), orc.bwd_weight(X, dY, offsets)) <= TOL_DV
    assert torch.equal(dX.view(torch.int16), dd.dd_bwd_input(d_dY, d_off, d_val, M, algo=dd.DD_ALGO_MATRIX).view(torch.int16))
    assert torch.equal(dV, dd.dd_bwd_weight(d_X, d_dY, d_off, algo=dd.DD_ALGO_MATRIX))


@pytest.mark.parametrize("M,N,K,T", [(128, 8192, 100, 8300), (256, 8192, 60, 8193)])
def test_large_output_gradient_every_element(M, N, K, T):
    """dY of more than 128 MB (more than the memory-side cache keeps between the two products)."""
    offsets, values, X, dY = random_case(M, N, K, T, "bf16", seed=T)
    d_off, d_val = torch.from_numpy(offsets).cuda(), to_dev(values, "bf16")
    d_X, d_dY = to_dev(X, "bf16"), to_dev(dY, "bf16")
    dX, dV = dd.dd_bwd(d_X, d_dY, d_off, d_val)
    dX, dV = dX.clone(), dV.clone()
    assert rel_err(to_host(dX), orc.bwd_input(dY, offsets, values, M)) <= TOL["bf16"]
    assert rel_err(to_host(dV), orc.bwd_weight(X, dY, offsets)) <= TOL_DV
    assert torch.equal(dX.view(torch.int16), dd.dd_bwd_input(d_dY, d_off, d_val, M, algo=dd.DD_ALGO_MATRIX).view(torch.int16))
    assert torch.equal(dV, dd.dd_bwd_weight(d_X, d_dY, d_off, algo=dd.DD_ALGO_MATRIX))


def test_stack_fc1_at_full_size_sampled():
    """768 -> 3072 at 50432 tokens (dY = 310 MB), operands prepared, as bench.py times it."""
    layer = synth.WORKLOADS["vitb_stack"][4]
    M, N, K = layer.in_features, layer.out_features, layer.K
    offsets, values, X, dY = synth.layer_inputs(layer, seed=77)
    d_off, d_val = torch.from_numpy(offsets).cuda(), to_dev(values, "bf16")
    d_X, d_dY = to_dev(X, "bf16"), to_dev(dY, "bf16")
    prep = dd.dd_prepare(d_off, d_val, M, N)
    dX, dV = dd.dd_bwd(d_X, d_dY, d_off, None, prepared=prep)
    assert torch.equal(dX.view(torch.int16), dd.dd_bwd_input(d_dY, None, None, M, prepared=prep).view(torch.int16))
    rng = np.random.default_rng(9)
    rows = np.unique(np.concatenate([[0, layer.tokens - 1, 13599, 13600], rng.integers(0, layer.tokens, 12)]))
    assert rel_err(to_host(dX[rows]), orc.bwd_input(dY[rows], offsets, values, M)) <= TOL["bf16"]
    ks, ps = rng.integers(0, K, 96), rng.integers(0, layer.L, 96)
    got = to_host(dV)
    assert np.all(np.isfinite(got))
    assert rel_err(got[ks, ps], orc.bwd_weight_sampled(X, dY, offsets, ks, ps)) <= TOL_DV


def test_shapes_and_types_outside_the_matrix_cores_and_no_tokens():
    for M, N, K, T, dtype in ((100, 260, 31, 129, "bf16"), (64, 64, 8, 16, "f32"), (768, 768, 77, 70, "f32")):
        offsets, values, X, dY = random_case(M, N, K, T, dtype, seed=M + T)
        d_off, d_val = torch.from_numpy(offsets).cuda(), to_dev(values, dtype)
        dX, dV = dd.dd_bwd(to_dev(X, dtype), to_dev(dY, dtype), d_off, d_val)
        assert rel_err(to_host(dX), orc.bwd_input(dY, offsets, values, M)) <= TOL[dtype]
        assert rel_err(to_host(dV), orc.bwd_weight(X, dY, offsets)) <= TOL_DV
        with pytest.raises(dd.DynaDiagError) as e:
            dd.dd_bwd(to_dev(X, dtype), to_dev(dY, dtype), d_off, d_val, algo=dd.DD_ALGO_MATRIX)
        assert e.value.status == 2
    off = torch.tensor([1, 5], dtype=torch.int32, device="cuda")
    val = torch.ones((2, 128), device="cuda", dtype=torch.bfloat16)
    empty = torch.empty((0, 128), device="cuda", dtype=torch.bfloat16)
    dX, dV = dd.dd_bwd(empty, empty, off, val)
    assert dX.shape == (0, 128) and torch.count_nonzero(dV).item() == 0
