"""dd_bwd_weight_static -- the weight gradient for callers that cannot allocate -- against dd_bwd_weight, through the
C ABI: bit-identical results (same kernels, scratch in the library's own array instead of the caller's workspace)
and within 1e-5 of the oracle, on two calls in a row, the second with a smaller input, in both kernel families."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2506_11449_amd as dd
from oracle import dd_oracle as orc
from tests.parity_util import TOL_DV, random_case, rel_err, to_dev, to_host

pytestmark = pytest.mark.gpu


def _both(M, N, K, T, dtype, algo, seed):
    offsets, values, X, dY = random_case(M, N, K, T, dtype, seed=seed)
    d_off = torch.from_numpy(offsets).cuda()
    d_X, d_dY = to_dev(X, dtype), to_dev(dY, dtype)
    ref = dd.dd_bwd_weight(d_X, d_dY, d_off, algo=algo).clone()
    out = torch.full((K, min(M, N)), float("nan"), dtype=torch.float32, device="cuda")
    before = torch.cuda.memory_allocated()
    dd.dd_bwd_weight_static(d_X, d_dY, d_off, out, algo=algo)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(out, ref), "the static-scratch call differs from dd_bwd_weight"
    assert rel_err(to_host(out), orc.bwd_weight(X, dY, offsets)) <= TOL_DV


@pytest.mark.parametrize("algo", ["matrix", "vector"])
def test_two_calls_in_a_row_the_second_smaller(algo):
    a = {"matrix": dd.DD_ALGO_MATRIX, "vector": dd.DD_ALGO_VECTOR}[algo]
    # 768 x 768 over several token chunks with a ragged tail, then a smaller layer with fewer tokens: the second
    # call finds the first one's partial sums in the array and must not read any of them
    _both(768, 768, 77, 4133, "bf16", a, seed=1)
    _both(256, 384, 38, 517, "bf16", a, seed=2)
    _both(768, 768, 77, 4133, "bf16", a, seed=3)


def test_a_handful_of_diagonals():
    """K <= 16 takes kernels of its own with partial sums per token chunk: every chunk the reduction reads must have
    been written by this call, whatever a larger call left in the array."""
    _both(768, 768, 4, 9000, "bf16", dd.DD_ALGO_VECTOR, seed=6)
    _both(256, 1024, 3, 333, "bf16", dd.DD_ALGO_AUTO, seed=7)
    _both(768, 768, 16, 1200, "bf16", dd.DD_ALGO_VECTOR, seed=8)


def test_fp32_storage_and_auto():
    _both(100, 260, 31, 1290, "f32", dd.DD_ALGO_AUTO, seed=4)
    _both(64, 64, 8, 16, "f32", dd.DD_ALGO_AUTO, seed=5)


def test_sizes_beyond_the_array_are_refused():
    lib = dd.load_library()
    limit = dd.dd_static_scratch_bytes()
    assert limit == 32 << 20
    T, M, N, K = 25216, 1024, 4096, 819
    l = dd.make_layer(T, M, N, K, torch.bfloat16, dd.DD_ALGO_AUTO)
    assert dd.dd_workspace_bytes(dd.DD_OP_BWD_WEIGHT, l) > limit
    one = ctypes.c_void_p(256)  # never dereferenced: the size check comes first
    assert lib.dd_bwd_weight_static(ctypes.byref(l), one, one, one, one, None) == 3
    # the same layer forced onto the matrix cores fits, and runs
    lm = dd.make_layer(T, M, N, K, torch.bfloat16, dd.DD_ALGO_MATRIX)
    assert 0 < dd.dd_workspace_bytes(dd.DD_OP_BWD_WEIGHT, lm) <= limit
