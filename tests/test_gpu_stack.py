"""The training step over the ViT-Base-depth stack (re-selection of every layer's diagonals, operand build, forward,
backward-input and weight-gradient products of every layer) end to end against the CPU oracle: one block at the full
256 x 197 tokens on sampled outputs, and two blocks at a few hundred tokens element by element."""
import numpy as np
import pytest
import torch

import paper_2506_11449_amd as dd
from oracle import dd_oracle as orc
from paper_2506_11449_amd.stack import StackStep
from tests.parity_util import TOL, TOL_DV, rel_err, to_host

pytestmark = pytest.mark.gpu


def _expected_offsets(st, r):
    """The oracle's selection for score set r, per group: [n_layers x K]."""
    sel = {name: orc.select(st.host_scores[name][r % st.score_sets], st.select_K[name]) for name in st.select_out}
    return {g.name: sel[g.select][g.select_row0:g.select_row0 + g.n_layers] for g in st.groups.values()}


def _check_selection_and_operands(st, r):
    want = _expected_offsets(st, r)
    for g in st.groups.values():
        np.testing.assert_array_equal(g.offsets.cpu().numpy(), want[g.name])
        for j in range(g.n_layers):  # the batched build equals the per-layer one, bit for bit
            single = dd.dd_prepare(g.offsets[j].clone(), g.values[j].clone(), g.M, g.N)
            assert torch.equal(single.buf, g.prepared[j].buf)
    return want


def test_two_blocks_every_element():
    """24-fold smaller in tokens, two blocks: buffer sets are shared between layers (rotation), so the products are
    checked for the layer that used each set last in its pass, the weight gradients for every layer."""
    st = StackStep(blocks=2, tokens=333, sets_attn=3, sets_mlp=1, score_sets=2, seed=11, distinct_sets=True)
    for r in range(2):  # the second step re-selects from other scores into the same buffers
        st.step()
        torch.cuda.synchronize()
        want = _check_selection_and_operands(st, r)
        last_fwd, last_bwd = {}, {}
        for name, j in st.layers:
            last_fwd[(name, j % st.groups[name].sets)] = j
        for name, j in reversed(st.layers):
            last_bwd[(name, j % st.groups[name].sets)] = j
        for g in st.groups.values():
            values = st.host_inputs[g.name + "_values"]
            for s in range(g.sets):
                X, dY = st.host_inputs[g.name][s]
                j = last_fwd[(g.name, s)]
                assert rel_err(to_host(g.Y[s]), orc.fwd(X, want[g.name][j], values[j], g.N)) <= TOL["bf16"]
                j = last_bwd[(g.name, s)]
                assert rel_err(to_host(g.dX[s]), orc.bwd_input(dY, want[g.name][j], values[j], g.M)) <= TOL["bf16"]
            for j in range(g.n_layers):
                X, dY = st.host_inputs[g.name][j % g.sets]
                assert rel_err(to_host(g.dValues[j]), orc.bwd_weight(X, dY, want[g.name][j])) <= TOL_DV


def test_one_block_at_full_size_sampled():
    """One block (four attention projections, fc1, fc2) at 50432 tokens, every layer with buffers of its own, in the
    launch configuration bench.py times: selection bit-exact, sampled token rows of every Y and dX, sampled entries
    of every weight gradient."""
    st = StackStep(blocks=1, tokens=256 * 197, sets_attn=4, sets_mlp=1, score_sets=2, seed=2506, distinct_sets=True)
    st.step()
    st.step()
    torch.cuda.synchronize()
    want = _check_selection_and_operands(st, 1)
    rng = np.random.default_rng(5)
    rows = np.unique(np.concatenate([[0, st.tokens - 1], rng.integers(0, st.tokens, 14)]))
    for g in st.groups.values():
        values = st.host_inputs[g.name + "_values"]
        for j in range(g.n_layers):
            s = j % g.sets
            X, dY = st.host_inputs[g.name][s]
            off = want[g.name][j]
            Y, dX = to_host(g.Y[s][rows]), to_host(g.dX[s][rows])
            assert rel_err(Y, orc.fwd(X[rows], off, values[j], g.N)) <= TOL["bf16"]
            assert rel_err(dX, orc.bwd_input(dY[rows], off, values[j], g.M)) <= TOL["bf16"]
            ks, ps = rng.integers(0, g.K, 64), rng.integers(0, g.L, 64)
            ks[:2], ps[:2] = [0, g.K - 1], [0, g.L - 1]
            dV = to_host(g.dValues[j])
            assert np.all(np.isfinite(dV))
            assert rel_err(dV[ks, ps], orc.bwd_weight_sampled(X, dY, off, ks, ps)) <= TOL_DV
