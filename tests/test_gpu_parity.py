"""GPU parity: every entry point of the C ABI against the CPU oracle, element by element on
small seeded cases (several tiles plus ragged tails, all edge cases), and on sampled outputs
at the full benchmark sizes."""
import numpy as np
import pytest
import torch

import paper_2506_11449_amd as dd
from oracle import dd_oracle as orc
from paper_2506_11449_amd import synth
from tests.parity_util import ALGOS, TOL, TOL_DV, random_case, rel_err, to_dev, to_host

pytestmark = pytest.mark.gpu

# (M, N, K, T): squares, both rectangular orientations, widths that are no multiple of 64,
# token counts that are no multiple of any tile.
SMALL = [
    (64, 64, 8, 16),
    (48, 48, 5, 33),
    (100, 100, 13, 70),
    (768, 768, 77, 300),
    (64, 192, 20, 50),
    (192, 64, 20, 50),
    (100, 260, 31, 129),
    (260, 100, 31, 129),
    (768, 3072, 307, 130),
    (3072, 768, 307, 130),
    (1024, 1024, 51, 257),
    (128, 128, 13, 1),
    (256, 128, 26, 161),
    (128, 384, 40, 415),
    (512, 512, 3, 700),
    (128, 8192, 100, 70),
    (8192, 128, 100, 70),
    (2048, 2048, 20, 100),
    (384, 1152, 60, 333),
    (256, 384, 38, 200),
    (2048, 2048, 1500, 100),
    (256, 256, 256, 90),
    (640, 128, 30, 77),
    (192, 576, 50, 130),
    (33, 7, 4, 19),
    (7, 33, 4, 19),
    (1, 1, 1, 5),
    (300, 300, 300, 65),
]


def matrix_shape_ok(M, N, dtype):
    """Shapes the matrix-core kernels cover: bf16 storage, both feature counts multiples of 128."""
    return dtype == "bf16" and M % 128 == 0 and N % 128 == 0 and max(M, N) <= 8192


def matrix_wgrad_shape_ok(M, N, dtype):
    """The matrix-core weight gradient tiles 192 x 192, 128 x 256 or 128 x 128."""
    both = lambda d: M % d == 0 and N % d == 0
    return dtype == "bf16" and (both(192) or both(128)) and max(M, N) <= 8192


def _call(fn, *args, algo):
    """Run one entry point; a forced kernel family that does not cover the case must say so."""
    try:
        return fn(*args, algo=algo)
    except dd.DynaDiagError as e:
        if algo != dd.DD_ALGO_AUTO and e.status == 2:
            return None
        raise


def run_all(offsets, values, X, dY, dtype, algo):
    T, M = X.shape
    N = dY.shape[1]
    d_off = torch.from_numpy(np.asarray(offsets, dtype=np.int32)).cuda()
    d_val, d_X, d_dY = to_dev(values, dtype), to_dev(X, dtype), to_dev(dY, dtype)
    Y = _call(dd.dd_fwd, d_X, d_off, d_val, N, algo=algo)
    dX = _call(dd.dd_bwd_input, d_dY, d_off, d_val, M, algo=algo)
    dV = _call(dd.dd_bwd_weight, d_X, d_dY, d_off, algo=algo)
    torch.cuda.synchronize()
    if algo == dd.DD_ALGO_MATRIX:
        ok = matrix_shape_ok(M, N, dtype) and T > 0
        assert (Y is not None) == ok and (dX is not None) == ok
        assert (dV is not None) == (matrix_wgrad_shape_ok(M, N, dtype) and T > 0)
    else:
        assert Y is not None and dX is not None and dV is not None
    return tuple(None if r is None else to_host(r) for r in (Y, dX, dV))


def check_against_oracle(offsets, values, X, dY, dtype, algo):
    M, N = X.shape[1], dY.shape[1]
    Y, dX, dV = run_all(offsets, values, X, dY, dtype, algo)
    if Y is not None:
        assert rel_err(Y, orc.fwd(X, offsets, values, N)) <= TOL[dtype]
    if dX is not None:
        assert rel_err(dX, orc.bwd_input(dY, offsets, values, M)) <= TOL[dtype]
    if dV is not None:
        assert rel_err(dV, orc.bwd_weight(X, dY, offsets)) <= TOL_DV


@pytest.mark.parametrize("algo", ["vector", "matrix", "auto"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("M,N,K,T", SMALL)
def test_small_cases_elementwise(M, N, K, T, dtype, algo):
    offsets, values, X, dY = random_case(M, N, K, T, dtype, seed=1000 * M + 10 * N + K)
    check_against_oracle(offsets, values, X, dY, dtype, ALGOS[algo])


PREPARED = [(768, 768, 77, 300), (768, 3072, 307, 130), (3072, 768, 307, 130), (128, 128, 13, 1), (256, 128, 26, 161),
            (128, 384, 40, 415), (1024, 1024, 51, 257), (384, 1152, 60, 333)]


@pytest.mark.parametrize("M,N,K,T", PREPARED)
def test_prepared_products(M, N, K, T):
    """dd_prepare once, then forward and backward-input products that read neither offsets nor values:
    against the oracle, bit-identical to the calls that rebuild the operands themselves, and still right
    after the block has been refilled for other offsets (duplicates and a negative one among them)."""
    offsets, values, X, dY = random_case(M, N, K, T, "bf16", seed=77 * M + N + K)
    d_X, d_dY = to_dev(X, "bf16"), to_dev(dY, "bf16")
    prepared = None
    for round_ in range(2):
        if round_ == 1:
            offsets = offsets.copy()
            offsets[0] = offsets[-1]
            offsets[K // 2] = offsets[-1] - max(M, N)
        d_off = torch.from_numpy(offsets).cuda()
        d_val = to_dev(values, "bf16")
        prepared = dd.dd_prepare(d_off, d_val, M, N, prepared=prepared)
        Y = dd.dd_fwd(d_X, None, None, N, prepared=prepared)
        dX = dd.dd_bwd_input(d_dY, None, None, M, prepared=prepared)
        Y2 = dd.dd_fwd(d_X, d_off, d_val, N, algo=dd.DD_ALGO_MATRIX)
        dX2 = dd.dd_bwd_input(d_dY, d_off, d_val, M, algo=dd.DD_ALGO_MATRIX)
        dV = dd.dd_bwd_weight(d_X, d_dY, d_off, algo=dd.DD_ALGO_PREPARED)  # same kernels as DD_ALGO_MATRIX
        torch.cuda.synchronize()
        assert torch.equal(Y.view(torch.int16), Y2.view(torch.int16))
        assert torch.equal(dX.view(torch.int16), dX2.view(torch.int16))
        assert rel_err(to_host(Y), orc.fwd(X, offsets, values, N)) <= TOL["bf16"]
        assert rel_err(to_host(dX), orc.bwd_input(dY, offsets, values, M)) <= TOL["bf16"]
        assert rel_err(to_host(dV), orc.bwd_weight(X, dY, offsets)) <= TOL_DV


@pytest.mark.parametrize("M,N,K", [(768, 768, 77), (128, 384, 40), (384, 128, 30), (1024, 1024, 51), (128, 128, 128),
                                   (256, 256, 1), (768, 3072, 307), (2048, 512, 60)])
def test_select_and_prepare_in_one_call(M, N, K):
    """dd_select_prepare against the oracle's selection and, bit for bit, against dd_prepare on those offsets; layers
    of up to 1024 candidates take one launch, the last two cases two.  Scores carry ties, a NaN and signed zeros."""
    D, L = max(M, N), min(M, N)
    rng = np.random.default_rng(M * 7 + N + K)
    scores = np.round(rng.standard_normal(D) * 4).astype(np.float32) / 4  # heavily tied
    scores[D // 3] = np.nan
    scores[D // 2], scores[D // 2 + 1] = 0.0, -0.0
    values = synth.round_to_bf16((rng.standard_normal((K, L)) * 0.02).astype(np.float32))
    X = synth.round_to_bf16(rng.standard_normal((150, M)).astype(np.float32))
    d_scores, d_val = torch.from_numpy(scores).cuda(), to_dev(values, "bf16")
    offsets = orc.select(scores, K)[0]
    for round_ in range(2):  # the second time into the blocks of the first
        if round_ == 0:
            d_off, prepared = dd.dd_select_prepare(d_scores, d_val, M, N)
        else:
            d_off.fill_(-1)
            prepared.buf.fill_(0xAB)
            dd.dd_select_prepare(d_scores, d_val, M, N, offsets_out=d_off, prepared=prepared)
        assert np.array_equal(d_off.cpu().numpy(), offsets)
        separate = dd.dd_prepare(torch.from_numpy(offsets).cuda(), d_val, M, N)
        assert torch.equal(prepared.buf, separate.buf)
    Y = dd.dd_fwd(to_dev(X, "bf16"), None, None, N, prepared=prepared)
    assert rel_err(to_host(Y), orc.fwd(X, offsets, values, N)) <= TOL["bf16"]


def test_prepared_refuses_what_the_matrix_cores_do_not_cover():
    off = torch.zeros(4, dtype=torch.int32, device="cuda")
    for M, N, dtype in ((100, 768, torch.bfloat16), (768, 768, torch.float32)):
        val = torch.zeros((4, min(M, N)), dtype=dtype, device="cuda")
        with pytest.raises(dd.DynaDiagError) as e:
            dd.dd_prepare(off, val, M, N)
        assert e.value.status == 2


@pytest.mark.parametrize("M,N,K,T", [(128, 8192, 100, 1300), (8192, 128, 100, 1300), (512, 2048, 60, 5300),
                                     (2048, 512, 60, 5301)])
def test_more_tiles_than_cus(M, N, K, T):
    """Products whose result has more than 256 tiles of 160 x 256: each workgroup walks several tiles with the
    pipeline running through (two k-slices per tile in the widest cases, a ragged last token tile)."""
    offsets, values, X, dY = random_case(M, N, K, T, "bf16", seed=M + N + T)
    check_against_oracle(offsets, values, X, dY, "bf16", ALGOS["matrix"])
    d_off, d_val = torch.from_numpy(offsets).cuda(), to_dev(values, "bf16")
    prepared = dd.dd_prepare(d_off, d_val, M, N)
    Y = dd.dd_fwd(to_dev(X, "bf16"), None, None, N, prepared=prepared)
    dX = dd.dd_bwd_input(to_dev(dY, "bf16"), None, None, M, prepared=prepared)
    assert rel_err(to_host(Y), orc.fwd(X, offsets, values, N)) <= TOL["bf16"]
    assert rel_err(to_host(dX), orc.bwd_input(dY, offsets, values, M)) <= TOL["bf16"]


@pytest.mark.parametrize("algo", ["vector", "matrix", "auto"])
@pytest.mark.parametrize("M,N,K,bands", [(768, 768, 77, 5), (768, 768, 77, 1), (384, 1152, 115, 4), (1152, 384, 60, 7),
                                         (100, 260, 31, 3)])
def test_clustered_offsets(M, N, K, bands, algo):
    """Runs of adjacent diagonals (the structure learned offsets are expected to have), some wrapping past D."""
    offsets = synth.draw_offsets_clustered(max(M, N), K, bands, seed=M + N + bands)
    for dtype in ("f32", "bf16"):
        _, values, X, dY = random_case(M, N, K, 150, dtype, seed=K, offsets=offsets)
        check_against_oracle(offsets, values, X, dY, dtype, ALGOS[algo])


@pytest.mark.parametrize("algo", ["vector", "matrix", "auto"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_tiny_config(dtype, algo):
    layer = synth.WORKLOADS["tiny"][0]
    offsets, values, X, dY = synth.layer_inputs(layer, seed=2506)
    if dtype == "bf16":
        values, X, dY = map(synth.round_to_bf16, (values, X, dY))
    check_against_oracle(offsets, values, X, dY, dtype, ALGOS[algo])


@pytest.mark.parametrize("algo", ["vector", "matrix", "auto"])
@pytest.mark.parametrize("M,N", [(96, 96), (40, 136), (136, 40)])
def test_offset_edge_cases(M, N, algo):
    D = max(M, N)
    cases = {
        "single_main": [0],
        "single_last": [D - 1],
        "negative": [-1, -D, -D - 3, 2 * D + 5],
        "duplicates": [3, 3, 3, 17],
        "unsorted": [50, 2, 31, 7, 90 % D],
        "adjacent_run": list(range(10, 26)),
    }
    for name, offs in cases.items():
        for dtype in ("f32", "bf16"):
            offsets, values, X, dY = random_case(M, N, len(offs), 37, dtype, seed=len(name) + M, offsets=offs)
            check_against_oracle(offsets, values, X, dY, dtype, ALGOS[algo])


@pytest.mark.parametrize("algo", ["vector", "matrix", "auto"])
def test_all_diagonals_is_dense(algo):
    for M, N in ((64, 64), (32, 80), (80, 32)):
        D = max(M, N)
        offsets, values, X, dY = random_case(M, N, D, 21, "f32", seed=D, offsets=np.arange(D))
        check_against_oracle(offsets, values, X, dY, "f32", ALGOS[algo])


@pytest.mark.parametrize("algo", ["vector", "matrix", "auto"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_identity_and_shift(dtype, algo):
    """Offset o with all-ones values moves column i to column (i + o) mod n, exactly."""
    X = np.random.default_rng(1).standard_normal((9, 128)).astype(np.float32)
    if dtype == "bf16":
        X = synth.round_to_bf16(X)
    ones = to_dev(np.ones((1, 128), np.float32), dtype)
    for o in (0, 1, 127, -5):
        off = torch.tensor([o], dtype=torch.int32, device="cuda")
        Y = _call(dd.dd_fwd, to_dev(X, dtype), off, ones, 128, algo=ALGOS[algo])
        if Y is None:
            assert algo == "matrix" and dtype == "f32"
            continue
        np.testing.assert_array_equal(to_host(Y), np.roll(X, o, axis=1).astype(np.float64))


@pytest.mark.parametrize("algo", ["vector", "matrix", "auto"])
def test_zero_tokens(algo):
    off = torch.tensor([1, 5], dtype=torch.int32, device="cuda")
    val = torch.ones((2, 16), device="cuda")
    X = torch.empty((0, 16), device="cuda")
    assert dd.dd_fwd(X, off, val, 16, algo=ALGOS[algo]).shape == (0, 16)
    assert dd.dd_bwd_input(X, off, val, 16, algo=ALGOS[algo]).shape == (0, 16)
    dV = _call(dd.dd_bwd_weight, X, X, off, algo=ALGOS[algo])
    if dV is not None:
        assert torch.count_nonzero(dV).item() == 0


@pytest.mark.parametrize("algo", ["vector", "matrix", "auto"])
def test_weight_gradient_is_deterministic(algo):
    offsets, values, X, dY = random_case(256, 256, 26, 5000, "bf16", seed=77)
    d_off = torch.from_numpy(offsets).cuda()
    d_X, d_dY = to_dev(X, "bf16"), to_dev(dY, "bf16")
    a = _call(dd.dd_bwd_weight, d_X, d_dY, d_off, algo=ALGOS[algo])
    if a is None:
        pytest.skip("this kernel family has no weight-gradient kernel for the shape")
    a = a.clone()
    b = dd.dd_bwd_weight(d_X, d_dY, d_off, algo=ALGOS[algo])
    assert torch.equal(a, b)


# ---- full benchmark sizes, in the launch configuration bench.py times ----

@pytest.mark.parametrize("algo", ["vector", "matrix", "auto"])
def test_vitb_attention_projection_full(algo):
    """ViT-Base attention projection, 768x768, 90 % sparse, 12608 tokens, bf16: every element."""
    layer = synth.WORKLOADS["vitb_attn_proj"][0]
    offsets, values, X, dY = synth.layer_inputs(layer, seed=2506)
    check_against_oracle(offsets, values, X, dY, "bf16", ALGOS[algo])


def test_vitb_attention_projection_full_as_benchmarked():
    """The launch configuration bench.py times: offsets from the selection kernel, operands prepared once, both
    products on them, the weight gradient by itself; 12608 tokens, every element."""
    layer = synth.WORKLOADS["vitb_attn_proj"][0]
    _, values, X, dY = synth.layer_inputs(layer, seed=2506)
    scores = synth.draw_scores(1, layer.D, seed=2506)
    M, N, K = layer.in_features, layer.out_features, layer.K
    d_off = dd.dd_select_diagonals(torch.from_numpy(scores).cuda(), K)
    offsets = orc.select(scores, K)[0]
    assert np.array_equal(d_off[0].cpu().numpy(), offsets)
    d_val, d_X, d_dY = to_dev(values, "bf16"), to_dev(X, "bf16"), to_dev(dY, "bf16")
    prepared = dd.dd_prepare(d_off[0], d_val, M, N)
    Y = dd.dd_fwd(d_X, None, None, N, prepared=prepared)
    dX = dd.dd_bwd_input(d_dY, None, None, M, prepared=prepared)
    dV = dd.dd_bwd_weight(d_X, d_dY, d_off[0])
    assert rel_err(to_host(Y), orc.fwd(X, offsets, values, N)) <= TOL["bf16"]
    assert rel_err(to_host(dX), orc.bwd_input(dY, offsets, values, M)) <= TOL["bf16"]
    assert rel_err(to_host(dV), orc.bwd_weight(X, dY, offsets)) <= TOL_DV


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("M,N", [(65535, 8), (8, 65535)])
def test_widest_layer(M, N, dtype):
    """The largest feature count the products take (65535 candidate diagonals), in both orientations."""
    offsets, values, X, dY = random_case(M, N, 3, 3, dtype, seed=M + 2 * N, offsets=[65534, 0, -40000])
    check_against_oracle(offsets, values, X, dY, dtype, ALGOS["auto"])


@pytest.mark.parametrize("algo", ["vector", "matrix"])
def test_many_tokens_sampled(algo):
    """300001 tokens through a narrow layer: thousands of tiles per product, token counts far past any 16-bit grid
    limit, a ragged last tile; sampled token rows and sampled gradient entries against the oracle."""
    layer = synth.Layer("narrow", 300001, 128, 256, 26, "bf16")
    _sampled_check(layer, 7, ALGOS[algo], n_rows=64, n_entries=128)


def _sampled_check(layer, seed, algo, n_rows=48, n_entries=256):
    offsets, values, X, dY = synth.layer_inputs(layer, seed)
    M, N = layer.in_features, layer.out_features
    Y, dX, dV = run_all(offsets, values, X, dY, layer.dtype, algo)
    assert Y is not None and dX is not None
    rng = np.random.default_rng(seed)
    rows = np.unique(np.concatenate([[0, layer.tokens - 1], rng.integers(0, layer.tokens, n_rows)]))
    # token rows are independent: the oracle on a subset of rows gives those rows of the full result
    assert rel_err(Y[rows], orc.fwd(X[rows], offsets, values, N)) <= TOL[layer.dtype]
    assert rel_err(dX[rows], orc.bwd_input(dY[rows], offsets, values, M)) <= TOL[layer.dtype]
    ks = rng.integers(0, layer.K, n_entries)
    ps = rng.integers(0, layer.L, n_entries)
    ks[:2], ps[:2] = [0, layer.K - 1], [0, layer.L - 1]
    assert np.all(np.isfinite(Y)) and np.all(np.isfinite(dX))
    if dV is not None:
        ref = orc.bwd_weight_sampled(X, dY, offsets, ks, ps)
        assert rel_err(dV[ks, ps], ref) <= TOL_DV
        assert np.all(np.isfinite(dV))


@pytest.mark.parametrize("algo", ["vector", "matrix", "auto"])
@pytest.mark.parametrize("which", [0, 1])
def test_vitb_mlp_sampled(which, algo):
    _sampled_check(synth.WORKLOADS["vitb_mlp"][which], 2506 + which, ALGOS[algo])


@pytest.mark.parametrize("algo", ["vector", "matrix", "auto"])
@pytest.mark.parametrize("name", [l.name for l in synth.WORKLOADS["vitl"]])
def test_vitl_sampled(name, algo):
    """All nine layer x sparsity cases of the ViT-Large configuration (1024^2, 1024 -> 4096, 4096 -> 1024 at
    80 / 90 / 95 %), 25216 tokens."""
    layer = next(l for l in synth.WORKLOADS["vitl"] if l.name == name)
    _sampled_check(layer, 4096, ALGOS[algo], n_rows=24, n_entries=128)


@pytest.mark.parametrize("algo", ["matrix", "auto"])
@pytest.mark.parametrize("which", [0, 4, 5])
def test_vitb_stack_sampled(which, algo):
    """One block of the ViT-Base-depth stack at 256 x 197 tokens: attention projection, fc1, fc2."""
    _sampled_check(synth.WORKLOADS["vitb_stack"][which], 7000 + which, ALGOS[algo], n_rows=16, n_entries=96)


def test_stack_selection_batched():
    """The per-step re-selection of the stack: 48 score vectors of 768 and 24 of 3072 in two launches."""
    for B, D, K in ((48, 768, 77), (24, 3072, 307)):
        _select_check(synth.draw_scores(B, D, seed=B + D), K)


# ---- selection: bit-exact ----

def _select_check(scores, K):
    got = dd.dd_select_diagonals(torch.from_numpy(scores).cuda(), K).cpu().numpy()
    np.testing.assert_array_equal(got, orc.select(scores, K))


def test_select_matches_oracle_bit_exactly():
    for D, K, B in ((64, 8, 1), (768, 77, 48), (3072, 307, 24), (1024, 51, 3), (4096, 819, 3), (1000, 1, 2),
                    (100, 100, 2), (65536, 6000, 1), (5, 3, 7)):
        _select_check(synth.draw_scores(B, D, seed=D + K), K)


def test_select_ties_nan_and_signed_zero():
    rng = np.random.default_rng(5)
    q = (np.round(rng.standard_normal((6, 777)) * 2) / 2).astype(np.float32)  # tie-heavy
    q[q == 0] = np.where(rng.random(np.count_nonzero(q == 0)) < 0.5, -0.0, 0.0)
    for K in (1, 50, 400, 777):
        _select_check(q, K)
    s = rng.standard_normal((4, 300)).astype(np.float32)
    s[:, ::7] = np.nan
    s[1, :] = np.nan
    s[2, 5] = np.inf
    s[2, 6] = -np.inf
    for K in (1, 40, 280, 300):
        _select_check(s, K)
    _select_check(np.zeros((2, 130), np.float32), 17)


def test_select_feeds_forward_without_leaving_the_device():
    layer = synth.WORKLOADS["tiny"][0]
    _, values, X, _ = synth.layer_inputs(layer, seed=9)
    scores = synth.draw_scores(1, layer.D, seed=9)
    d_off = dd.dd_select_diagonals(torch.from_numpy(scores).cuda(), layer.K)
    Y = dd.dd_fwd(to_dev(X, "f32"), d_off[0], to_dev(values, "f32"), layer.out_features)
    ref = orc.fwd(X, orc.select(scores, layer.K)[0], values, layer.out_features)
    assert rel_err(to_host(Y), ref) <= TOL["f32"]


@pytest.mark.parametrize("M,N,K,T", [(768, 3072, 307, 25216), (768, 768, 77, 50432)])
def test_weight_gradient_misaligned_inputs_stay_inside_the_workspace(M, N, K, T):
    """X and dY that start one bf16 element past a 16-byte boundary: DD_ALGO_AUTO then runs the vector kernels, which
    cut the tokens into more chunks than the matrix-core ones.  Called through the raw C ABI with exactly the scratch
    dd_workspace_bytes asks for and a guard pattern behind it; sampled gradient entries against the oracle.  The
    forced matrix-core family refuses such inputs."""
    import ctypes
    lib = dd.load_library()
    layer = synth.Layer("misaligned", T, M, N, K, "bf16")
    offsets, values, X, dY = synth.layer_inputs(layer, seed=31)
    d_off = torch.from_numpy(offsets).cuda()

    def shifted(a):  # a contiguous [rows x cols] bf16 view that starts 2 bytes past a 16-byte boundary
        flat = torch.empty(a.size + 8, dtype=torch.bfloat16, device="cuda")
        flat[1:1 + a.size] = to_dev(a, "bf16").reshape(-1)
        v = flat[1:1 + a.size].view(a.shape)
        assert v.data_ptr() % 16 == 2 and v.is_contiguous()
        return v

    d_X, d_dY = shifted(X), shifted(dY)
    dV = torch.empty((K, min(M, N)), dtype=torch.float32, device="cuda")
    l = dd.make_layer(T, M, N, K, torch.bfloat16, dd.DD_ALGO_AUTO)
    need = dd.dd_workspace_bytes(dd.DD_OP_BWD_WEIGHT, l)
    guard = 1 << 20
    ws = torch.full((need + guard,), 0xCD, dtype=torch.uint8, device="cuda")
    assert ws.data_ptr() % 256 == 0
    vp = ctypes.c_void_p
    stream = vp(torch.cuda.current_stream().cuda_stream)
    st = lib.dd_bwd_weight(ctypes.byref(l), vp(d_X.data_ptr()), vp(d_dY.data_ptr()), vp(d_off.data_ptr()),
                           vp(dV.data_ptr()), vp(ws.data_ptr()), need, stream)
    assert st == 0
    torch.cuda.synchronize()
    assert bool((ws[need:] == 0xCD).all()), "dd_bwd_weight wrote past the scratch it asked for"
    rng = np.random.default_rng(3)
    ks, ps = rng.integers(0, K, 96), rng.integers(0, min(M, N), 96)
    assert rel_err(to_host(dV)[ks, ps], orc.bwd_weight_sampled(X, dY, offsets, ks, ps)) <= TOL_DV
    for algo in (dd.DD_ALGO_MATRIX, dd.DD_ALGO_PREPARED):
        lm = dd.make_layer(T, M, N, K, torch.bfloat16, algo)
        st = lib.dd_bwd_weight(ctypes.byref(lm), vp(d_X.data_ptr()), vp(d_dY.data_ptr()), vp(d_off.data_ptr()),
                               vp(dV.data_ptr()), vp(ws.data_ptr()), need + guard, stream)
        assert st == 2


BLOCKS = [(768, 768, 77, 2, 300), (768, 768, 77, 5, 1290), (768, 768, 77, 0, 517), (384, 1152, 115, 4, 333),
          (1152, 384, 60, 7, 333), (768, 3072, 307, 3, 700), (3072, 768, 307, 3, 257), (128, 128, 13, 1, 1),
          (1024, 1024, 51, 0, 600), (256, 8192, 100, 2, 70), (8192, 256, 100, 2, 70), (512, 512, 512, 0, 90)]


@pytest.mark.parametrize("M,N,K,bands,T", BLOCKS)
def test_block_skipping_products(M, N, K, bands, T):
    """DD_ALGO_BLOCKS: the products on prepared operands that skip every 32 x 16 operand block no diagonal crosses.
    Clustered offsets (runs of adjacent diagonals, some wrapping), uniform ones (nothing to skip) and the dense case;
    both orientations, ragged token counts; against the oracle, and against the kernel that skips nothing."""
    D = max(M, N)
    offsets = (synth.draw_offsets_clustered(D, K, bands, seed=M + N + bands) if bands
               else synth.draw_offsets(D, K, seed=M + N))
    _, values, X, dY = random_case(M, N, K, T, "bf16", seed=K + T, offsets=offsets)
    d_off, d_val = torch.from_numpy(offsets).cuda(), to_dev(values, "bf16")
    d_X, d_dY = to_dev(X, "bf16"), to_dev(dY, "bf16")
    prepared = dd.dd_prepare(d_off, d_val, M, N)
    Y = dd.dd_fwd(d_X, d_off, None, N, prepared=prepared, algo=dd.DD_ALGO_BLOCKS)
    dX = dd.dd_bwd_input(d_dY, d_off, None, M, prepared=prepared, algo=dd.DD_ALGO_BLOCKS)
    Y2 = dd.dd_fwd(d_X, None, None, N, prepared=prepared)
    dX2 = dd.dd_bwd_input(d_dY, None, None, M, prepared=prepared)
    torch.cuda.synchronize()
    assert rel_err(to_host(Y), orc.fwd(X, offsets, values, N)) <= TOL["bf16"]
    assert rel_err(to_host(dX), orc.bwd_input(dY, offsets, values, M)) <= TOL["bf16"]
    # a skipped block holds zeros only, so both kernels add the same products; they may round the fp32 sums differently
    assert rel_err(to_host(Y), to_host(Y2)) <= 2.0 ** -8
    assert rel_err(to_host(dX), to_host(dX2)) <= 2.0 ** -8


def test_block_skipping_needs_offsets_and_a_prepared_block():
    import ctypes
    lib = dd.load_library()
    l = dd.make_layer(64, 768, 768, 77, torch.bfloat16, dd.DD_ALGO_BLOCKS)
    one = ctypes.c_void_p(256)  # never dereferenced: refused on the host
    need = dd.dd_workspace_bytes(dd.DD_OP_FWD, l)
    assert need == 2 * 768 * 768 * 2
    assert lib.dd_fwd(ctypes.byref(l), one, None, None, one, one, need, None) == 1      # no offsets
    assert lib.dd_fwd(ctypes.byref(l), one, one, None, one, one, need - 1, None) == 3   # block too small
    l32 = dd.make_layer(64, 768, 768, 77, torch.float32, dd.DD_ALGO_BLOCKS)
    assert lib.dd_fwd(ctypes.byref(l32), one, one, None, one, one, need, None) == 2     # fp32 storage


@pytest.mark.parametrize("M,N,K", [(3072, 768, 307), (768, 3072, 307), (3072, 768, 4), (768, 3072, 4)])
def test_more_than_2_31_elements(M, N, K):
    """700001 tokens through a 3072-wide side: the wide matrix has 2.15e9 elements (4.3 GB), so the rows past token 699050
    start beyond 2^31 elements.  Inputs are drawn on the device; the token rows checked against the oracle include the
    first ones past that limit and the last; the weight gradient is checked through a property that holds at any size --
    it is additive over token ranges (each half has fewer than 2^31 elements and such sizes are checked against the
    oracle elsewhere) -- and on sampled entries against the oracle over a window of tokens with all others zeroed."""
    T, D, L = 700001, max(M, N), min(M, N)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(M + K)
    X = torch.randn((T, M), device="cuda", generator=gen, dtype=torch.float32).to(torch.bfloat16)
    dY = torch.randn((T, N), device="cuda", generator=gen, dtype=torch.float32).to(torch.bfloat16)
    offsets = synth.draw_offsets(D, K, seed=5)
    values = synth.round_to_bf16(synth.draw_normal((K, L), 0.02, 5, 10))
    d_off, d_val = torch.from_numpy(offsets).cuda(), to_dev(values, "bf16")
    Y = dd.dd_fwd(X, d_off, d_val, N)
    dX = dd.dd_bwd_input(dY, d_off, d_val, M)
    limit = (1 << 31) // D  # first token row that starts past 2^31 elements of the wide matrix
    rng = np.random.default_rng(1)
    rows = np.unique(np.concatenate([[0, limit - 1, limit, limit + 1, T - 2, T - 1], rng.integers(0, T, 24),
                                     rng.integers(limit, T, 24)]))
    idx = torch.from_numpy(rows).cuda()
    assert rel_err(to_host(Y[idx]), orc.fwd(to_host(X[idx]), offsets, values, N)) <= TOL["bf16"]
    assert rel_err(to_host(dX[idx]), orc.bwd_input(to_host(dY[idx]), offsets, values, M)) <= TOL["bf16"]
    del Y, dX
    dV = dd.dd_bwd_weight(X, dY, d_off)
    half = 350000
    dV_a = dd.dd_bwd_weight(X[:half], dY[:half], d_off)
    dV_b = dd.dd_bwd_weight(X[half:], dY[half:], d_off)
    assert rel_err(to_host(dV), to_host(dV_a) + to_host(dV_b)) <= TOL_DV
    # a window of 64 tokens around the limit and the last 64 kept, everything else zero: the full-size call then
    # has to find exactly those rows, and the oracle needs only them
    keep = np.concatenate([np.arange(limit - 32, limit + 32), np.arange(T - 64, T)])
    kidx = torch.from_numpy(keep).cuda()
    Xk, dYk = X[kidx].clone(), dY[kidx].clone()
    X.zero_()
    dY.zero_()
    X[kidx], dY[kidx] = Xk, dYk
    dV_w = dd.dd_bwd_weight(X, dY, d_off)
    assert rel_err(to_host(dV_w), orc.bwd_weight(to_host(Xk), to_host(dYk), offsets)) <= TOL_DV
