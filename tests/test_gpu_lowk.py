"""GPU parity of the kernels for a handful of diagonals (K <= 16, the regime of extreme sparsity, Sec. 4.4): the three
products against the CPU oracle, element by element on small cases that span several tiles, slabs and a ragged tail, and
on sampled outputs at benchmark sizes; the guard behind the weight gradient's scratch; what DD_ALGO_AUTO hands to them."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2506_11449_amd as dd
from oracle import dd_oracle as orc
from paper_2506_11449_amd import synth
from tests.parity_util import ALGOS, TOL, TOL_DV, random_case, rel_err, to_dev, to_host

pytestmark = pytest.mark.gpu

# (M, N, K, T): every unrolled diagonal count, squares and both rectangular orientations, one to four column pairs
# per lane, slabs shared by several waves (narrow outputs) and several workgroups side by side (wide ones), the widest
# long side, token counts of one row, less than a tile and many tiles with a ragged last one.
LOWK = [
    (128, 128, 1, 5),
    (128, 128, 16, 70),
    (256, 128, 7, 161),
    (128, 384, 9, 415),
    (512, 512, 3, 700),
    (768, 768, 8, 300),
    (768, 768, 2, 1),
    (768, 3072, 16, 130),
    (3072, 768, 16, 130),
    (640, 128, 2, 77),
    (128, 640, 2, 77),
    (1024, 1024, 12, 257),
    (1024, 1024, 4, 2049),
    (384, 1152, 5, 333),
    (1152, 384, 6, 333),
    (8192, 128, 4, 40),
    (128, 8192, 4, 40),
    (4096, 4096, 3, 19),
    (2048, 2048, 16, 100),
    (1536, 1536, 1, 64),
    (4096, 1024, 10, 90),
    (1024, 4096, 11, 90),
]


def _run(offsets, values, X, dY, algo):
    M, N = X.shape[1], dY.shape[1]
    d_off = torch.from_numpy(np.asarray(offsets, dtype=np.int32)).cuda()
    d_val, d_X, d_dY = to_dev(values, "bf16"), to_dev(X, "bf16"), to_dev(dY, "bf16")
    Y = dd.dd_fwd(d_X, d_off, d_val, N, algo=algo)
    dX = dd.dd_bwd_input(d_dY, d_off, d_val, M, algo=algo)
    dV = dd.dd_bwd_weight(d_X, d_dY, d_off, algo=algo)
    dV2 = dd.dd_bwd_weight(d_X, d_dY, d_off, algo=algo)
    torch.cuda.synchronize()
    assert torch.equal(dV, dV2), "the weight gradient is not reproducible"
    return to_host(Y), to_host(dX), to_host(dV)


@pytest.mark.parametrize("algo", ["vector", "auto"])
@pytest.mark.parametrize("M,N,K,T", LOWK)
def test_few_diagonals_elementwise(M, N, K, T, algo):
    """Offsets include a repeated diagonal written as a negative offset (contributions add, both copies get the same
    gradient row) wherever K >= 2."""
    offsets, values, X, dY = random_case(M, N, K, T, "bf16", seed=M + 3 * N + K)
    if K >= 2:
        offsets = offsets.copy()
        offsets[1] = offsets[0] - max(M, N)
    Y, dX, dV = _run(offsets, values, X, dY, ALGOS[algo])
    assert rel_err(Y, orc.fwd(X, offsets, values, N)) <= TOL["bf16"]
    assert rel_err(dX, orc.bwd_input(dY, offsets, values, M)) <= TOL["bf16"]
    assert rel_err(dV, orc.bwd_weight(X, dY, offsets)) <= TOL_DV
    if K >= 2:
        assert np.array_equal(dV[0], dV[1])


@pytest.mark.parametrize("M,N", [(768, 768), (768, 3072), (3072, 768)])
def test_single_diagonal_closed_forms(M, N):
    """One diagonal of ones at offset o: a cyclic shift of the columns (truncated or zero-padded when the layer is
    rectangular), exact in bf16; its gradient row is the plain column-wise inner product of X and shifted dY."""
    D, L, T, o = max(M, N), min(M, N), 37, 129
    rng = np.random.default_rng(M + N)
    X = synth.round_to_bf16(rng.standard_normal((T, M)).astype(np.float32))
    dY = synth.round_to_bf16(rng.standard_normal((T, N)).astype(np.float32))
    offsets = np.array([o], dtype=np.int32)
    values = np.ones((1, L), dtype=np.float32)
    Y, dX, dV = _run(offsets, values, X, dY, dd.DD_ALGO_VECTOR)
    p = np.arange(L)
    q = (p + o) % D
    want_Y = np.zeros((T, N))
    want_dX = np.zeros((T, M))
    if M <= N:   # W[p, q] = 1
        want_Y[:, q] = X[:, p]
        want_dX[:, p] = dY[:, q]
        want_dV = np.einsum("tp,tp->p", X[:, p].astype(np.float64), dY[:, q].astype(np.float64))
    else:        # W[q, p] = 1
        want_Y[:, p] = X[:, q]
        want_dX[:, q] = dY[:, p]
        want_dV = np.einsum("tp,tp->p", X[:, q].astype(np.float64), dY[:, p].astype(np.float64))
    assert np.array_equal(Y, want_Y)
    assert np.array_equal(dX, want_dX)
    assert rel_err(dV[0], want_dV) <= TOL_DV


@pytest.mark.parametrize("algo", ["vector", "auto"])
@pytest.mark.parametrize("M,N,K,T", [(768, 768, 4, 50432), (768, 3072, 8, 25216), (3072, 768, 3, 25216),
                                     (1024, 1024, 16, 25216)])
def test_few_diagonals_at_benchmark_sizes_sampled(M, N, K, T, algo):
    """Full token counts of the ViT workloads in the launch configuration the K sweep of bench.py times: sampled token
    rows of Y and dX (rows are independent) and sampled gradient entries against the oracle."""
    layer = synth.Layer("fewdiag", T, M, N, K, "bf16")
    offsets, values, X, dY = synth.layer_inputs(layer, seed=11)
    Y, dX, dV = _run(offsets, values, X, dY, ALGOS[algo])
    rng = np.random.default_rng(5)
    rows = np.unique(np.concatenate([[0, T - 1], rng.integers(0, T, 48)]))
    assert rel_err(Y[rows], orc.fwd(X[rows], offsets, values, N)) <= TOL["bf16"]
    assert rel_err(dX[rows], orc.bwd_input(dY[rows], offsets, values, M)) <= TOL["bf16"]
    assert np.all(np.isfinite(Y)) and np.all(np.isfinite(dX)) and np.all(np.isfinite(dV))
    ks, ps = rng.integers(0, K, 128), rng.integers(0, min(M, N), 128)
    ks[:2], ps[:2] = [0, K - 1], [0, min(M, N) - 1]
    assert rel_err(dV[ks, ps], orc.bwd_weight_sampled(X, dY, offsets, ks, ps)) <= TOL_DV


@pytest.mark.parametrize("algo", ["vector", "auto"])
@pytest.mark.parametrize("M,N,K,T", [(768, 768, 4, 12608), (128, 8192, 16, 3000), (1024, 4096, 2, 700)])
def test_weight_gradient_stays_inside_its_scratch(M, N, K, T, algo):
    """Through the raw C ABI with exactly the scratch dd_workspace_bytes asks for and a guard pattern behind it."""
    lib = dd.load_library()
    offsets, values, X, dY = random_case(M, N, K, T, "bf16", seed=T)
    d_off, d_X, d_dY = torch.from_numpy(offsets).cuda(), to_dev(X, "bf16"), to_dev(dY, "bf16")
    dV = torch.empty((K, min(M, N)), dtype=torch.float32, device="cuda")
    l = dd.make_layer(T, M, N, K, torch.bfloat16, ALGOS[algo])
    need = dd.dd_workspace_bytes(dd.DD_OP_BWD_WEIGHT, l)
    assert need > 0
    guard = 1 << 20
    ws = torch.full((need + guard,), 0xCD, dtype=torch.uint8, device="cuda")
    vp = ctypes.c_void_p
    st = lib.dd_bwd_weight(ctypes.byref(l), vp(d_X.data_ptr()), vp(d_dY.data_ptr()), vp(d_off.data_ptr()),
                           vp(dV.data_ptr()), vp(ws.data_ptr()), need, vp(torch.cuda.current_stream().cuda_stream))
    assert st == 0
    torch.cuda.synchronize()
    assert bool((ws[need:] == 0xCD).all()), "dd_bwd_weight wrote past the scratch it asked for"
    rng = np.random.default_rng(3)
    ks, ps = rng.integers(0, K, 96), rng.integers(0, min(M, N), 96)
    assert rel_err(to_host(dV)[ks, ps], orc.bwd_weight_sampled(X, dY, offsets, ks, ps)) <= TOL_DV
    short = lib.dd_bwd_weight(ctypes.byref(l), vp(d_X.data_ptr()), vp(d_dY.data_ptr()), vp(d_off.data_ptr()),
                              vp(dV.data_ptr()), vp(ws.data_ptr()), need - 256, vp(0))
    assert short == 3


def test_misaligned_matrices_take_the_general_kernels():
    """A matrix that starts 2 bytes past a 16-byte boundary cannot use the 16-byte loads of these kernels: DD_ALGO_VECTOR
    and DD_ALGO_AUTO still answer (general vector kernels), same results within tolerance."""
    M, N, K, T = 256, 512, 3, 90
    offsets, values, X, dY = random_case(M, N, K, T, "bf16", seed=9)

    def shifted(a):
        flat = torch.empty(a.size + 8, dtype=torch.bfloat16, device="cuda")
        flat[1:1 + a.size] = to_dev(a, "bf16").reshape(-1)
        v = flat[1:1 + a.size].view(a.shape)
        assert v.data_ptr() % 16 == 2
        return v

    d_off, d_val = torch.from_numpy(offsets).cuda(), to_dev(values, "bf16")
    for algo in (dd.DD_ALGO_VECTOR, dd.DD_ALGO_AUTO):
        Y = dd.dd_fwd(shifted(X), d_off, d_val, N, algo=algo)
        dX = dd.dd_bwd_input(shifted(dY), d_off, d_val, M, algo=algo)
        dV = dd.dd_bwd_weight(shifted(X), shifted(dY), d_off, algo=algo)
        torch.cuda.synchronize()
        assert rel_err(to_host(Y), orc.fwd(X, offsets, values, N)) <= TOL["bf16"]
        assert rel_err(to_host(dX), orc.bwd_input(dY, offsets, values, M)) <= TOL["bf16"]
        assert rel_err(to_host(dV), orc.bwd_weight(X, dY, offsets)) <= TOL_DV
