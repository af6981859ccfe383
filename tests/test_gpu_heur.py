"""GPU parity of the DiagHeur entry points (appendix on the heuristics-based method) against the CPU oracle:
the magnitude of each diagonal within fp32 summation error, the update of the active set bit-exactly."""
import numpy as np
import pytest
import torch

import paper_2506_11449_amd as dd
from oracle import dd_oracle as orc
from paper_2506_11449_amd import synth
from tests.parity_util import to_dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("K,L", [(1, 1), (8, 64), (77, 768), (307, 768), (5, 1000), (3, 4097)])
def test_diag_magnitude(K, L, dtype):
    rng = np.random.default_rng(K * 7919 + L)
    V = (rng.standard_normal((K, L)) * 0.02).astype(np.float32)
    if dtype == "bf16":
        V = synth.round_to_bf16(V)
    V[0, 0] = 0.0
    got = dd.dd_diag_magnitude(to_dev(V, dtype)).cpu().numpy().astype(np.float64)
    ref = orc.diag_magnitude(V)
    # fp32 sum of L non-negative terms in a tree: relative error below L * 2^-24 by a wide margin
    assert np.max(np.abs(got - ref)) <= 1e-5 * np.max(ref)


def _check_update(D, offsets, mags, rnd, n_drop):
    new, src = dd.dd_diagheur_update(D, torch.from_numpy(offsets).cuda(), torch.from_numpy(mags).cuda(),
                                     torch.from_numpy(rnd).cuda(), n_drop)
    torch.cuda.synchronize()
    ref_new, ref_src = orc.diagheur_update(D, offsets, mags, rnd, n_drop)
    assert new.cpu().numpy().tolist() == ref_new.tolist()
    assert src.cpu().numpy().tolist() == ref_src.tolist()


@pytest.mark.parametrize("D,K,n_drop,seed", [(64, 8, 3, 0), (64, 8, 0, 1), (64, 8, 8, 2), (64, 32, 32, 3), (768, 77, 23, 4),
                                             (3072, 307, 92, 5), (4096, 819, 245, 6), (1, 1, 0, 7), (33, 32, 1, 8),
                                             (20000, 2000, 600, 9), (65536, 300, 90, 10)])
def test_diagheur_update_random(D, K, n_drop, seed):
    rng = np.random.default_rng(seed)
    offsets = rng.permutation(D)[:K].astype(np.int32)      # unsorted, as a caller may hold them
    mags = np.abs(rng.standard_normal(K)).astype(np.float32)
    rnd = rng.random(D).astype(np.float32)
    _check_update(D, offsets, mags, rnd, n_drop)


@pytest.mark.parametrize("D,K,n_drop", [(64, 16, 5), (768, 77, 23), (300, 150, 150)])
def test_diagheur_update_ties_nan_and_offsets_outside_the_range(D, K, n_drop):
    rng = np.random.default_rng(D + K)
    offsets = rng.permutation(D)[:K].astype(np.int32)
    offsets[0] -= D            # a negative offset and one beyond D name the same diagonals modulo D
    offsets[1] += 2 * D
    mags = rng.integers(0, 3, K).astype(np.float32)        # heavy ties: broken by lower offset
    mags[2] = np.nan                                        # ranks below every number
    mags[3] = np.inf
    rnd = (rng.integers(0, 4, D) / 4).astype(np.float32)
    rnd[rng.integers(0, D, 5)] = np.nan
    rnd[7] = -0.0
    _check_update(D, offsets, mags, rnd, n_drop)


def test_diagheur_chain_on_the_device():
    """Magnitudes from the values, update, and the forward product with the new set: nothing leaves the device
    between the steps; the new offsets drive dd_fwd as they are."""
    layer = synth.WORKLOADS["vitb_attn_proj"][0]
    D, K, L = layer.D, layer.K, layer.L
    offsets, values, X, _ = synth.layer_inputs(layer, seed=11)
    X = X[:256]
    rng = np.random.default_rng(12)
    rnd = rng.random(D).astype(np.float32)
    d_val = to_dev(values, "bf16")
    d_off = torch.from_numpy(offsets).cuda()
    mag = dd.dd_diag_magnitude(d_val)
    new, src = dd.dd_diagheur_update(D, d_off, mag, torch.from_numpy(rnd).cuda(), 23)
    # the caller's move: kept diagonals carry their values over, grown ones start at zero
    keep = src >= 0
    new_val = torch.zeros_like(d_val)
    new_val[keep] = d_val[src[keep].long()]
    Y = dd.dd_fwd(to_dev(X, "bf16"), new, new_val, layer.out_features)
    torch.cuda.synchronize()
    ref_new, ref_src = orc.diagheur_update(D, offsets, mag.cpu().numpy(), rnd, 23)
    assert new.cpu().numpy().tolist() == ref_new.tolist() and src.cpu().numpy().tolist() == ref_src.tolist()
    ref_val = np.zeros_like(values)
    ref_val[ref_src >= 0] = values[ref_src[ref_src >= 0]]
    ref = orc.fwd(X, ref_new, ref_val, layer.out_features)
    got = Y.to(torch.float64).cpu().numpy()
    assert np.max(np.abs(got - ref)) <= 2e-2 * np.max(np.abs(ref))
