"""Helpers shared by the GPU parity tests: move seeded numpy inputs to the device, call the
C ABI through the binding, bring results back as float64."""
import numpy as np
import torch

import paper_2506_11449_amd as dd
from paper_2506_11449_amd import synth

# Tolerances, as max|gpu - oracle| / max|oracle| over a tensor.
#  fp32 storage: products and sums in fp32; K (or T/splits) terms of random sign -> a few ulp.
#  bf16 storage: inputs are exact, the fp32 sum is rounded once to bf16 (2^-9 relative).
TOL = {"f32": 1e-5, "bf16": 2e-2}
# dValues is always stored in fp32, whatever the inputs.
TOL_DV = 1e-5

ALGOS = {"auto": dd.DD_ALGO_AUTO, "vector": dd.DD_ALGO_VECTOR, "matrix": dd.DD_ALGO_MATRIX}


def to_dev(a, dtype):
    """fp32 numpy array (already representable in `dtype`) -> GPU tensor of that storage type."""
    if dtype == "bf16":
        bits = synth.bf16_bits(a)
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def to_host(t):
    """GPU tensor -> float64 numpy (exact)."""
    return t.detach().to(torch.float64).cpu().numpy()


def rel_err(got, ref):
    scale = np.max(np.abs(ref))
    if scale == 0:
        return float(np.max(np.abs(got)))
    return float(np.max(np.abs(got - ref)) / scale)


def random_case(M, N, K, T, dtype, seed, offsets=None):
    rng = np.random.default_rng(seed)
    D, L = max(M, N), min(M, N)
    if offsets is None:
        offsets = np.sort(rng.permutation(D)[:K]).astype(np.int32)
    offsets = np.asarray(offsets, dtype=np.int32)
    values = (rng.standard_normal((len(offsets), L)) * 0.02).astype(np.float32)
    X = rng.standard_normal((T, M)).astype(np.float32)
    dY = rng.standard_normal((T, N)).astype(np.float32)
    if dtype == "bf16":
        values, X, dY = synth.round_to_bf16(values), synth.round_to_bf16(X), synth.round_to_bf16(dY)
    return offsets, values, X, dY
