"""Seeded synthetic inputs for the diagonally-sparse linear layer.

This module holds no arithmetic of the method: it only draws random numbers, rounds them to
the storage type and names the workload shapes.  Both the HIP path and the CPU oracle are
fed from here (the tests and the benchmark call it and hand the same arrays to both sides).

Workload shapes follow the ViT configurations the paper trains (Sec. 4.1: 224x224 images in
16x16 patches give 196 + 1 = 197 tokens per image; ViT-Base width 768, MLP width 3072;
ViT-Large 1024 / 4096).  The dataset itself is not needed: a layer's cost depends only on
its shape, its number of diagonals and where they sit.
"""
from dataclasses import dataclass

import numpy as np


def num_diagonals(D, sparsity_percent):
    """K = round((1 - S) * D), in integer arithmetic (Sec. 3.1, footnote on K)."""
    return ((100 - sparsity_percent) * D + 50) // 100


def _rng(seed, *stream):
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(seed), *map(int, stream)])))


def draw_offsets(D, K, seed, stream=0):
    """K distinct offsets uniform in [0, D), ascending (int32)."""
    perm = _rng(seed, 1, stream).permutation(D)[:K]
    return np.sort(perm).astype(np.int32)


def draw_offsets_clustered(D, K, bands, seed, stream=0):
    """K distinct offsets in `bands` runs of adjacent diagonals (run starts uniform, runs may wrap past D and
    never overlap), ascending (int32): a stand-in for learned offsets that cluster, of which none exist here."""
    rng = _rng(seed, 3, stream)
    widths = np.full(bands, K // bands)
    widths[:K % bands] += 1
    gap_total = D - K
    # distribute the free candidates over the gaps between consecutive runs (cyclically), then rotate
    cuts = np.sort(rng.integers(0, gap_total + 1, bands - 1)) if bands > 1 else np.array([], dtype=np.int64)
    gaps = np.diff(np.concatenate([[0], cuts, [gap_total]]))
    start = int(rng.integers(0, D))
    out = []
    for w, g in zip(widths, gaps):
        out.extend((start + i) % D for i in range(int(w)))
        start += int(w) + int(g)
    return np.sort(np.array(out, dtype=np.int64)).astype(np.int32)


def draw_normal(shape, std, seed, stream):
    """fp32 N(0, std^2) samples."""
    return (_rng(seed, 2, stream).standard_normal(shape, dtype=np.float32) * np.float32(std)).astype(np.float32)


def bf16_bits(a):
    """fp32 array -> uint16 array of bfloat16 bit patterns, round-to-nearest-even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    bits = (rounded >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(a)
    if nan.any():
        bits = np.where(nan, np.uint16(0x7FC0), bits)
    return bits


def bf16_to_f32(bits):
    """uint16 bfloat16 bit patterns -> the fp32 values they stand for (exact)."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(a):
    """fp32 array rounded to the nearest bfloat16, returned as fp32."""
    return bf16_to_f32(bf16_bits(a))


@dataclass(frozen=True)
class Layer:
    name: str
    tokens: int
    in_features: int
    out_features: int
    K: int
    dtype: str  # "f32" or "bf16"

    @property
    def D(self):
        return max(self.in_features, self.out_features)

    @property
    def L(self):
        return min(self.in_features, self.out_features)


def layer_inputs(layer, seed):
    """offsets, values, X, dY (fp32 arrays; already rounded to bf16 values if layer.dtype says so)."""
    offsets = draw_offsets(layer.D, layer.K, seed)
    values = draw_normal((layer.K, layer.L), 0.02, seed, 10)
    X = draw_normal((layer.tokens, layer.in_features), 1.0, seed, 11)
    dY = draw_normal((layer.tokens, layer.out_features), 1.0, seed, 12)
    if layer.dtype == "bf16":
        values, X, dY = round_to_bf16(values), round_to_bf16(X), round_to_bf16(dY)
    return offsets, values, X, dY


def draw_scores(batch, D, seed, stream=0):
    """Importance scores alpha, one row per layer: fp32 N(0, 1)."""
    return draw_normal((batch, D), 1.0, seed, 100 + stream)


def _sparse(name, tokens, m, n, s, dtype="bf16"):
    return Layer(name, tokens, m, n, num_diagonals(max(m, n), s), dtype)


# The benchmark configurations, by name.
WORKLOADS = {
    "tiny": [Layer("tiny_64", 16, 64, 64, 8, "f32")],
    "vitb_attn_proj": [_sparse("vitb_attn_proj", 64 * 197, 768, 768, 90)],
    "vitb_mlp": [_sparse("vitb_fc1", 128 * 197, 768, 3072, 90),
                 _sparse("vitb_fc2", 128 * 197, 3072, 768, 90)],
    "vitl": [_sparse(f"vitl_{m}x{n}_s{s}", 128 * 197, m, n, s)
             for (m, n) in ((1024, 1024), (1024, 4096), (4096, 1024)) for s in (80, 90, 95)],
    "vitb_stack": ([_sparse("stack_attn", 256 * 197, 768, 768, 90)] * 4
                   + [_sparse("stack_fc1", 256 * 197, 768, 3072, 90),
                      _sparse("stack_fc2", 256 * 197, 3072, 768, 90)]),  # one block; x12 in depth
}
