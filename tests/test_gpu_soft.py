"""GPU parity of the soft TopK weights, their derivative and the scaling of the diagonals (Sec. 3.2,
Eq. 4 and Eq. 5) against the CPU oracle, plus the full differentiable chain through the layer."""
import numpy as np
import pytest
import torch

import paper_2506_11449_amd as dd
from oracle import dd_oracle as orc
from paper_2506_11449_amd import synth
from tests.parity_util import TOL, TOL_DV, rel_err, to_dev, to_host

pytestmark = pytest.mark.gpu

TOL_SOFT = 1e-5  # fp32 exp and sums against the fp64 oracle, as max|gpu - ref| / max|ref|


@pytest.mark.parametrize("B,D,K", [(1, 64, 8), (3, 768, 77), (2, 3072, 307), (1, 1000, 1), (2, 100, 100), (1, 5, 2)])
@pytest.mark.parametrize("temperature", [0.05, 1.0, 30.0])
def test_soft_topk_forward_and_backward(B, D, K, temperature):
    scores = synth.draw_scores(B, D, seed=D + K)
    d_scores_in = torch.from_numpy(scores).cuda()
    at = dd.dd_soft_topk(d_scores_in, K, temperature)
    ref = orc.soft_topk(scores, K, temperature)
    assert rel_err(to_host(at), ref) <= TOL_SOFT
    assert float(at.max()) <= 1.0
    g = synth.draw_normal((B, D), 1.0, seed=9, stream=D)
    got = to_host(dd.dd_soft_topk_bwd(d_scores_in, K, temperature, torch.from_numpy(g).cuda()))
    ref_b = orc.soft_topk_bwd(scores, K, temperature, g)
    # An entry whose weight sits on the clamp within fp32 resolution may fall on either side of the min, and then
    # its own derivative is either the formula's or zero: those entries are left out of the comparison, every
    # other entry is still checked (the clamp decision of entry i only enters entry i of the result).
    s = np.exp((scores.astype(np.float64) - scores.max(axis=1, keepdims=True)) / temperature)
    s /= s.sum(axis=1, keepdims=True)
    decided = np.abs(K * s - 1.0) > 1e-4
    assert decided.sum() >= decided.size - 2 * B  # the mask may drop a stray entry, never the test
    # the derivative is (K / T) s_i (g_i - sum_j g_j s_j): when one weight takes nearly everything the
    # bracket cancels to g_i (1 - s_i), so the fp32 rounding of s_i (2^-24) leaves an absolute error of
    # about (K / T) |g| 2^-24 whatever the size of the result; a few of those are allowed on top
    bound = 5 * TOL_SOFT * np.max(np.abs(ref_b)) + 4 * 2.0 ** -24 * (K / temperature) * np.max(np.abs(g))
    assert np.max(np.abs(got - ref_b)[decided]) <= bound


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("D,L,K", [(64, 64, 8), (768, 768, 77), (3072, 768, 307), (100, 52, 7)])
def test_scale_values_and_adjoint(D, L, K, dtype):
    rng = np.random.default_rng(D + L + K)
    offsets = np.sort(rng.permutation(D)[:K]).astype(np.int32)
    if K > 3:
        offsets[1] = offsets[0]          # a repeated offset
        offsets[2] -= D                  # a negative one
    alpha = rng.uniform(0.0, 1.0, D).astype(np.float32)
    V = (rng.standard_normal((K, L)) * 0.02).astype(np.float32)
    if dtype == "bf16":
        V = synth.round_to_bf16(V)
    dValues = rng.standard_normal((K, L)).astype(np.float32)
    d_off, d_alpha, d_V = torch.from_numpy(offsets).cuda(), torch.from_numpy(alpha).cuda(), to_dev(V, dtype)
    eff = dd.dd_scale_values(d_off, d_alpha, d_V)
    assert rel_err(to_host(eff), orc.scale_values(offsets, alpha, V)) <= TOL[dtype]
    dV, dalpha = dd.dd_scale_values_bwd(d_off, d_alpha, d_V, torch.from_numpy(dValues).cuda())
    ref_dV, ref_dalpha = orc.scale_values_bwd(offsets, alpha, V, dValues)
    assert rel_err(to_host(dV), ref_dV) <= TOL_DV
    assert rel_err(to_host(dalpha), ref_dalpha) <= TOL_DV
    untouched = np.setdiff1d(np.arange(D), offsets % D)
    assert np.count_nonzero(to_host(dalpha)[untouched]) == 0


def test_differentiable_chain_scores_to_loss():
    """scores -> soft TopK -> select -> scale -> fwd -> <dY, Y>, and back to d scores: the chain the
    training method differentiates (Sec. 3.2), every link on the GPU, against the oracle's chain."""
    layer = synth.WORKLOADS["tiny"][0]
    D, L, K, N = layer.D, layer.L, layer.K, layer.out_features
    temperature = 0.7
    _, V, X, dY = synth.layer_inputs(layer, seed=11)
    scores = synth.draw_scores(1, D, seed=11)
    d_scores = torch.from_numpy(scores).cuda()
    d_V, d_X, d_dY = to_dev(V, "f32"), to_dev(X, "f32"), to_dev(dY, "f32")
    off = dd.dd_select_diagonals(d_scores, K)[0]
    at = dd.dd_soft_topk(d_scores, K, temperature)[0]
    eff = dd.dd_scale_values(off, at, d_V)
    Y = dd.dd_fwd(d_X, off, eff, N)
    dValues = dd.dd_bwd_weight(d_X, d_dY, off)
    dV, dat = dd.dd_scale_values_bwd(off, at, d_V, dValues)
    dsc = dd.dd_soft_topk_bwd(d_scores, K, temperature, dat[None, :])
    # the same chain on the oracle
    o_off = orc.select(scores, K)[0]
    o_at = orc.soft_topk(scores, K, temperature)[0]
    o_eff = orc.scale_values(o_off, o_at, V)
    o_Y = orc.fwd(X, o_off, o_eff, N)
    o_dValues = orc.bwd_weight(X, dY, o_off)
    o_dV, o_dat = orc.scale_values_bwd(o_off, o_at, V, o_dValues)
    o_dsc = orc.soft_topk_bwd(scores, K, temperature, o_dat)
    np.testing.assert_array_equal(off.cpu().numpy(), o_off)
    assert rel_err(to_host(Y), o_Y) <= 2e-5
    assert rel_err(to_host(dV), o_dV) <= 2e-5
    assert rel_err(to_host(dsc)[0], o_dsc[0]) <= 1e-4


# ---- the same steps folded into the launches of the layer's own path ----

@pytest.mark.parametrize("B,D,K", [(1, 64, 8), (48, 768, 77), (24, 3072, 307), (2, 1000, 1), (2, 100, 100), (1, 65536, 500)])
def test_select_soft_is_the_two_calls_in_one_launch(B, D, K):
    scores = synth.draw_scores(B, D, seed=3 * D + K)
    scores[0, D // 3] = np.nan
    scores[0, 1], scores[0, 2] = 0.0, -0.0
    d_scores = torch.from_numpy(scores).cuda()
    for temperature in (0.3, 5.0):
        off, at = dd.dd_select_soft(d_scores, K, temperature)
        assert torch.equal(off, dd.dd_select_diagonals(d_scores, K))
        assert torch.equal(at.view(torch.int32), dd.dd_soft_topk(d_scores, K, temperature).view(torch.int32))
        np.testing.assert_array_equal(off.cpu().numpy(), orc.select(scores, K))
    clean = synth.draw_scores(B, D, seed=D)
    off, at = dd.dd_select_soft(torch.from_numpy(clean).cuda(), K, 0.7)
    assert rel_err(to_host(at), orc.soft_topk(clean, K, 0.7)) <= TOL_SOFT


@pytest.mark.parametrize("M,N,K", [(768, 768, 77), (128, 384, 40), (384, 128, 30), (768, 3072, 307)])
def test_prepare_scaled_builds_what_scaling_then_preparing_builds(M, N, K):
    D, L = max(M, N), min(M, N)
    rng = np.random.default_rng(M + 3 * N + K)
    offsets = np.sort(rng.permutation(D)[:K]).astype(np.int32)
    offsets[1] = offsets[0]      # a repeated offset
    offsets[2] -= D              # a negative one
    alpha = rng.uniform(0.0, 1.0, D).astype(np.float32)
    V = synth.round_to_bf16((rng.standard_normal((K, L)) * 0.02).astype(np.float32))
    X = synth.round_to_bf16(rng.standard_normal((200, M)).astype(np.float32))
    d_off, d_alpha, d_V = torch.from_numpy(offsets).cuda(), torch.from_numpy(alpha).cuda(), to_dev(V, "bf16")
    fused = dd.dd_prepare_scaled(d_off, d_alpha, d_V, M, N)
    two_steps = dd.dd_prepare(d_off, dd.dd_scale_values(d_off, d_alpha, d_V), M, N)
    assert torch.equal(fused.buf, two_steps.buf)
    Y = dd.dd_fwd(to_dev(X, "bf16"), None, None, N, prepared=fused)
    assert rel_err(to_host(Y), orc.fwd(X, offsets, orc.scale_values(offsets, alpha, V), N)) <= TOL["bf16"]


@pytest.mark.parametrize("M,N,K,T", [(768, 768, 77, 4133), (128, 384, 40, 415), (384, 128, 30, 700), (768, 3072, 307, 1300),
                                     (1024, 1024, 51, 257)])
def test_bwd_weight_scaled_is_the_weight_gradient_and_the_adjoint_of_the_scaling(M, N, K, T):
    D, L = max(M, N), min(M, N)
    rng = np.random.default_rng(M + N + K + T)
    offsets = np.sort(rng.permutation(D)[:K]).astype(np.int32)
    offsets[1] = offsets[0]      # a repeated offset: both copies get the same gradient, their dots add up
    offsets[2] -= D
    alpha = rng.uniform(0.0, 1.0, D).astype(np.float32)
    V = synth.round_to_bf16((rng.standard_normal((K, L)) * 0.02).astype(np.float32))
    d_off, d_alpha, d_V = torch.from_numpy(offsets).cuda(), torch.from_numpy(alpha).cuda(), to_dev(V, "bf16")
    dV = dalpha = None
    for round_ in range(2):  # the second call finds the first one's ticket and dots in the scratch
        X = synth.round_to_bf16(rng.standard_normal((T, M)).astype(np.float32))
        dY = synth.round_to_bf16(rng.standard_normal((T, N)).astype(np.float32))
        d_X, d_dY = to_dev(X, "bf16"), to_dev(dY, "bf16")
        dV, dalpha = dd.dd_bwd_weight_scaled(d_X, d_dY, d_off, d_alpha, d_V, dV=dV, d_alpha_tilde=dalpha)
        ref_dV, ref_dalpha = orc.scale_values_bwd(offsets, alpha, V, orc.bwd_weight(X, dY, offsets))
        assert rel_err(to_host(dV), ref_dV) <= TOL_DV
        assert rel_err(to_host(dalpha), ref_dalpha) <= TOL_DV
        untouched = np.setdiff1d(np.arange(D), offsets % D)
        assert np.count_nonzero(to_host(dalpha)[untouched]) == 0
        dV2, dalpha2 = dd.dd_scale_values_bwd(d_off, d_alpha, d_V, dd.dd_bwd_weight(d_X, d_dY, d_off))
        assert torch.equal(dV, dV2)
        assert rel_err(to_host(dalpha), to_host(dalpha2)) <= TOL_DV


def test_bwd_weight_scaled_refuses_what_its_kernels_do_not_cover():
    off = torch.zeros(4, dtype=torch.int32, device="cuda")
    for M, N, dtype in ((100, 768, torch.bfloat16), (768, 768, torch.float32)):
        X = torch.zeros((8, M), dtype=dtype, device="cuda")
        dY = torch.zeros((8, N), dtype=dtype, device="cuda")
        V = torch.zeros((4, min(M, N)), dtype=dtype, device="cuda")
        alpha = torch.zeros(max(M, N), device="cuda")
        with pytest.raises(dd.DynaDiagError) as e:
            dd.dd_bwd_weight_scaled(X, dY, off, alpha, V)
        assert e.value.status == 2


def test_differentiable_chain_through_the_fused_calls():
    """The chain of the test above on a layer the matrix cores cover (768 -> 768, bf16), with the fused calls:
    scores -> dd_select_soft -> dd_prepare_scaled -> dd_fwd; back: dd_bwd_weight_scaled -> dd_soft_topk_bwd."""
    M = N = D = L = 768
    K, T, temperature = 77, 1000, 0.7
    rng = np.random.default_rng(21)
    V = synth.round_to_bf16((rng.standard_normal((K, L)) * 0.02).astype(np.float32))
    X = synth.round_to_bf16(rng.standard_normal((T, M)).astype(np.float32))
    dY = synth.round_to_bf16(rng.standard_normal((T, N)).astype(np.float32))
    scores = synth.draw_scores(1, D, seed=21)
    d_scores, d_V, d_X, d_dY = torch.from_numpy(scores).cuda(), to_dev(V, "bf16"), to_dev(X, "bf16"), to_dev(dY, "bf16")
    off, at = dd.dd_select_soft(d_scores, K, temperature)
    prepared = dd.dd_prepare_scaled(off[0], at[0], d_V, M, N)
    Y = dd.dd_fwd(d_X, None, None, N, prepared=prepared)
    dV, dat = dd.dd_bwd_weight_scaled(d_X, d_dY, off[0], at[0], d_V)
    dsc = dd.dd_soft_topk_bwd(d_scores, K, temperature, dat[None, :])
    o_off = orc.select(scores, K)[0]
    o_at = orc.soft_topk(scores, K, temperature)[0]
    o_Y = orc.fwd(X, o_off, orc.scale_values(o_off, o_at, V), N)
    o_dV, o_dat = orc.scale_values_bwd(o_off, o_at, V, orc.bwd_weight(X, dY, o_off))
    o_dsc = orc.soft_topk_bwd(scores, K, temperature, o_dat)
    np.testing.assert_array_equal(off[0].cpu().numpy(), o_off)
    assert rel_err(to_host(Y), o_Y) <= TOL["bf16"]
    assert rel_err(to_host(dV), o_dV) <= 2e-5      # two fp32 links (gradient, scaling), 1e-5 each
    assert rel_err(to_host(dsc)[0], o_dsc[0]) <= 1e-4  # four links, the last one amplifies by K/T (as in the test above)
