"""One training step over a stack of diagonally-sparse layers, as a sequence of calls of the C ABI.

The stack is the ViT-Base-depth configuration: `blocks` transformer blocks, each with four 768 -> 768 attention
projections, one 768 -> 3072 and one 3072 -> 768 MLP layer, all 90 % sparse.  A step re-selects every layer's
diagonals from fresh importance scores (Sec. 3.2 Eq. 4: one batched dd_select_diagonals per number of candidates),
rebuilds the dense operands of the products from them (one dd_prepare_batched per layer shape), and runs dd_fwd for
every layer in order, then dd_bwd_input and dd_bwd_weight for every layer in reverse order.

This module only sequences calls and owns the device buffers they work on; every arithmetic step runs in the
library's kernels.  The layers are not chained (weights drawn at N(0, 0.02^2) shrink activations layer by layer until
they underflow): each layer reads seeded N(0, 1) inputs of its own shape, from buffer sets that rotate so that a
product does not find its operands in the Infinity Cache left there by its predecessor.
"""
from dataclasses import dataclass, field

import numpy as np
import torch

from . import binding as dd
from . import synth


@dataclass
class Group:
    """All layers of the stack that share one shape."""
    name: str
    M: int
    N: int
    K: int
    n_layers: int
    sets: int
    select: str = ""         # name of the batched selection this group's offsets come from
    select_row0: int = 0     # first row of that batch
    X: list = field(default_factory=list)      # [sets] of [T x M]
    dY: list = field(default_factory=list)     # [sets] of [T x N]
    Y: list = field(default_factory=list)
    dX: list = field(default_factory=list)
    values: torch.Tensor = None                # [n_layers x K x L]
    dValues: torch.Tensor = None               # [n_layers x K x L] fp32
    prepared: list = None                      # [n_layers] blocks of one buffer
    offsets: torch.Tensor = None               # [n_layers x K] view into the selection's output

    @property
    def D(self):
        return max(self.M, self.N)

    @property
    def L(self):
        return min(self.M, self.N)


def _to_dev_bf16(a, device):
    return torch.from_numpy(synth.bf16_bits(a).view(np.int16)).to(device).view(torch.bfloat16)


class StackStep:
    def __init__(self, blocks=12, tokens=256 * 197, sets_attn=4, sets_mlp=2, score_sets=4, seed=2506,
                 distinct_sets=False, device_inputs=False, sparsity_percent=90, device="cuda:0"):
        """distinct_sets: every buffer set of a shape holds values of its own (else set 0's values at other
        addresses).  device_inputs: X and dY are drawn on the device (seeded torch generator) instead of on the host --
        quicker for the benchmark; the parity tests draw on the host, where the oracle reads the same arrays."""
        self.blocks, self.tokens, self.seed, self.device = blocks, tokens, seed, torch.device(device)
        self.score_sets = score_sets
        K_attn = synth.num_diagonals(768, sparsity_percent)
        K_mlp = synth.num_diagonals(3072, sparsity_percent)
        self.groups = {
            "attn": Group("attn", 768, 768, K_attn, 4 * blocks, sets_attn, "d768", 0),
            "fc1": Group("fc1", 768, 3072, K_mlp, blocks, sets_mlp, "d3072", 0),
            "fc2": Group("fc2", 3072, 768, K_mlp, blocks, sets_mlp, "d3072", blocks),
        }
        # layer order of the stack: (group, index inside the group)
        self.layers = []
        for b in range(blocks):
            self.layers += [("attn", 4 * b + i) for i in range(4)] + [("fc1", b), ("fc2", b)]
        # importance scores: `score_sets` seeded draws per batched selection, used in rotation step by step
        self.host_scores = {"d768": [synth.draw_scores(4 * blocks, 768, seed, stream=r) for r in range(score_sets)],
                            "d3072": [synth.draw_scores(2 * blocks, 3072, seed, stream=100 + r)
                                      for r in range(score_sets)]}
        self.scores = {k: [torch.from_numpy(a).to(self.device) for a in v] for k, v in self.host_scores.items()}
        self.select_K = {"d768": K_attn, "d3072": K_mlp}
        self.select_out = {"d768": torch.empty((4 * blocks, K_attn), dtype=torch.int32, device=self.device),
                           "d3072": torch.empty((2 * blocks, K_mlp), dtype=torch.int32, device=self.device)}
        self.host_inputs = {}
        for gi, g in enumerate(self.groups.values()):
            host = []
            if device_inputs:
                gen = torch.Generator(device=self.device)
                gen.manual_seed(seed + gi)
                for s in range(g.sets if distinct_sets else 1):
                    g.X.append(torch.randn((tokens, g.M), device=self.device, generator=gen).to(torch.bfloat16))
                    g.dY.append(torch.randn((tokens, g.N), device=self.device, generator=gen).to(torch.bfloat16))
            for s in range(0 if device_inputs else (g.sets if distinct_sets else 1)):
                X = synth.round_to_bf16(synth.draw_normal((tokens, g.M), 1.0, seed, 1000 * gi + 10 * s + 1))
                dY = synth.round_to_bf16(synth.draw_normal((tokens, g.N), 1.0, seed, 1000 * gi + 10 * s + 2))
                host.append((X, dY))
                g.X.append(_to_dev_bf16(X, self.device))
                g.dY.append(_to_dev_bf16(dY, self.device))
            for s in range(len(g.X), g.sets):  # same values at other addresses
                g.X.append(g.X[0].clone())
                g.dY.append(g.dY[0].clone())
            self.host_inputs[g.name] = host
            g.Y = [torch.empty((tokens, g.N), dtype=torch.bfloat16, device=self.device) for _ in range(g.sets)]
            g.dX = [torch.empty((tokens, g.M), dtype=torch.bfloat16, device=self.device) for _ in range(g.sets)]
            values = synth.round_to_bf16(synth.draw_normal((g.n_layers, g.K, g.L), 0.02, seed, 1000 * gi + 3))
            self.host_inputs[g.name + "_values"] = values
            g.values = _to_dev_bf16(values, self.device)
            g.dValues = torch.empty((g.n_layers, g.K, g.L), dtype=torch.float32, device=self.device)
            g.offsets = self.select_out[g.select][g.select_row0:g.select_row0 + g.n_layers]
        self.ws = dd.Workspace()
        self.steps_done = 0

    # ---- the parts of a step, each a plain sequence of C-ABI calls on the current stream ----

    def select(self, r):
        for name, out in self.select_out.items():
            dd.dd_select_diagonals(self.scores[name][r % self.score_sets], self.select_K[name], offsets_out=out,
                                   ws=self.ws)

    def prepare(self):
        for g in self.groups.values():
            g.prepared = dd.dd_prepare_batched(g.offsets, g.values, g.M, g.N, prepared=g.prepared)

    def forward(self):
        for name, j in self.layers:
            g = self.groups[name]
            s = j % g.sets
            dd.dd_fwd(g.X[s], None, None, g.N, Y=g.Y[s], prepared=g.prepared[j])

    def backward_input(self):
        for name, j in reversed(self.layers):
            g = self.groups[name]
            s = j % g.sets
            dd.dd_bwd_input(g.dY[s], None, None, g.M, dX=g.dX[s], prepared=g.prepared[j])

    def backward_weight(self):
        for name, j in reversed(self.layers):
            g = self.groups[name]
            s = j % g.sets
            dd.dd_bwd_weight(g.X[s], g.dY[s], g.offsets[j], dValues=g.dValues[j], ws=self.ws)

    def backward(self):
        """Layer by layer in reverse order, input gradient then weight gradient, as backpropagation issues them."""
        for name, j in reversed(self.layers):
            g = self.groups[name]
            s = j % g.sets
            dd.dd_bwd_input(g.dY[s], None, None, g.M, dX=g.dX[s], prepared=g.prepared[j])
            dd.dd_bwd_weight(g.X[s], g.dY[s], g.offsets[j], dValues=g.dValues[j], ws=self.ws)

    def step(self):
        self.select(self.steps_done)
        self.prepare()
        self.forward()
        self.backward()
        self.steps_done += 1

    # ---- bookkeeping for the benchmark ----

    def flops_per_product(self):
        """Algorithmic flops 2 T K L of one product, summed over the layers of the stack."""
        return sum(2.0 * self.tokens * g.K * g.L * g.n_layers for g in self.groups.values())

    def dense_flops_per_product(self):
        return sum(2.0 * self.tokens * g.M * g.N * g.n_layers for g in self.groups.values())

    def bytes_per_product(self):
        """Algorithmic bytes of one forward / backward-input product, summed over the layers."""
        return sum((2 * self.tokens * (g.M + g.N) + 2 * g.K * g.L + 4 * g.K) * g.n_layers for g in self.groups.values())

    def bytes_per_weight_gradient(self):
        return sum((2 * self.tokens * (g.M + g.N) + 4 * g.K * g.L + 4 * g.K) * g.n_layers for g in self.groups.values())
