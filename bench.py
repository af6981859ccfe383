#!/usr/bin/env python3
"""Benchmark of the diagonally-sparse layer's hot path on one MI355X.

Default workload: one training step over the ViT-Base-depth stack -- 12 blocks x (four 768 -> 768 attention
projections + 768 -> 3072 + 3072 -> 768), all 90 % sparse, 256 x 197 = 50432 tokens, bf16 storage with fp32
accumulation.  A step is one pass of the whole path: the diagonals of all 72 layers re-selected from fresh seeded
importance scores (one batched dd_select_diagonals per candidate count), the dense operands rebuilt from them
(one dd_prepare_batched per layer shape), then dd_fwd for every layer and dd_bwd_input + dd_bwd_weight for every
layer in reverse order.  Inputs are resident in HBM; buffer sets rotate so that no product finds its operands in
the 256 MB Infinity Cache.  The metric is the effective (sparse) rate, sum over layers of 3 * 2 T K L / t_step.

Prints ONE JSON line.  Besides the contract fields it carries
  roofline      the kernel with the largest summed time against the ceiling that bounds the method's arithmetic,
  cpu_baseline  the CPU oracle timed on this host's cores on a slice of the workload (a baseline, not a target),
  breakdown     per-entry-point and per-shape times of the step, the dense bf16 GEMMs of the same shapes (hipBLASLt /
                rocBLAS through torch, with the fastest solution per GEMM where a tuning file is present), speedups,
                and one sub-line per layer of the smaller configurations (ViT-B attention projection, ViT-B MLP pair,
                the nine ViT-L layer x sparsity cases, Tiny).

Other modes:  --workload NAME times a step over that workload's layers instead (select + prepare + three products
per layer); --tune-dense writes the tuning file of the dense baseline; --table prints the per-layer table as
markdown; --k-sweep times both kernel families over K (the evidence behind DD_ALGO_AUTO's switch).
"""
import argparse
import json
import os
import sys
import tempfile
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
VALU_FP32_PEAK_TFLOPS = 157.3  # MI355X fp32 vector, published (256 CU x 128 lanes-flop x 2 x 2.4 GHz)
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix, published
DENSE_TUNING_FILE = os.path.join(ROOT, "bench_dense_gemm_tuned.csv")
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")
PAPER_CONTEXT = ("paper reports 3.13x inference / 1.59x training speedup at 90 % sparsity, ViT-Base end to end, "
                 "on an A100 (abstract, Sec. 4.2.3): another machine, context only")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="vitb_stack",
                    choices=["vitb_stack", "vitb_attn_proj", "vitb_mlp", "vitl", "tiny"])
    ap.add_argument("--sets", type=int, default=0, help="rotating buffer sets per shape (0: enough to exceed the "
                                                        "Infinity Cache)")
    ap.add_argument("--algo", default="auto", choices=["auto", "vector", "matrix"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="leave out the sub-lines of the smaller configurations")
    ap.add_argument("--offset-bands", type=int, default=0,
                    help="0: seeded uniform offsets (the benchmark); n > 0: the K diagonals in n runs of adjacent ones")
    ap.add_argument("--per-layer", action="store_true",
                    help="with --workload vitb_stack: time the distinct layers of one block one by one (select + prepare + "
                         "three products each) instead of the whole stack step")
    ap.add_argument("--tune-dense", action="store_true",
                    help="search hipBLASLt / rocBLAS for the fastest solution of every dense GEMM the benchmark "
                         "compares with and write them to bench_dense_gemm_tuned.csv (minutes)")
    ap.add_argument("--table", action="store_true", help="print the per-layer table as markdown instead of JSON")
    ap.add_argument("--k-sweep", action="store_true", help="vector family, matrix family and DD_ALGO_AUTO over K on four shapes")
    ap.add_argument("--saturation", action="store_true",
                    help="where the products stop scaling: prepared dd_fwd (and the dense GEMM) with 3 ... 255 result tiles "
                         "in flight, one per CU, and on random against all-zero operands at the stack's shapes")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy a few times (a known-size reference for the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    return ap.parse_args()


def time_loop(torch, fn, n, warmup=5):
    """Average milliseconds per call of fn(i), timed with events on the launch stream."""
    for i in range(warmup):
        fn(i)
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for i in range(n):
        fn(i)
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) / n


# ---------------------------------------------------------------------------------------------------------------
# dense baseline: torch.matmul = hipBLASLt / rocBLAS; with a tuning file, the fastest solution of either per GEMM
# ---------------------------------------------------------------------------------------------------------------

class DenseBaseline:
    def __init__(self, torch, tune=False):
        self.torch, self.tuned, self.solutions = torch, False, {}
        self.tunable = None
        try:
            import torch.cuda.tunable as tunable
        except Exception:
            return
        if tune:
            tunable.enable(True)
            tunable.tuning_enable(True)
            tunable.set_max_tuning_duration(15)
            tunable.set_max_tuning_iterations(10)
            tunable.set_filename(DENSE_TUNING_FILE)
            self.tunable, self.tuned = tunable, True
        elif os.path.exists(DENSE_TUNING_FILE):
            try:
                tunable.enable(True)
                tunable.tuning_enable(False)
                tunable.set_filename(DENSE_TUNING_FILE)
                if tunable.read_file(DENSE_TUNING_FILE):
                    self.tunable, self.tuned = tunable, True
                else:
                    tunable.enable(False)
            except Exception:
                self.tuned = False

    def off(self):
        if self.tunable is not None:
            self.tunable.enable(False)

    def on(self):
        if self.tunable is not None:
            self.tunable.enable(True)

    def chosen(self):
        """GEMM signature -> solution name, as the tuning results hold them."""
        if self.tunable is None:
            return {}
        try:
            return {f"{r[0]} {r[1]}": r[2] for r in self.tunable.get_results()}
        except Exception:
            return {}

    def time_gemms(self, X, dY, Y, dX, n):
        """us of the three dense GEMMs of a layer over the rotating sets X[s] [T x M], dY[s] [T x N]."""
        torch = self.torch
        M, N = X[0].shape[1], dY[0].shape[1]
        S = len(X)
        W = torch.randn((M, N), device=X[0].device, dtype=X[0].dtype) * 0.02
        dW = torch.empty((M, N), device=X[0].device, dtype=X[0].dtype)
        self.on()
        out = {"fwd": time_loop(torch, lambda i: torch.matmul(X[i % S], W, out=Y[i % S]), n) * 1e3,
               "dgrad": time_loop(torch, lambda i: torch.matmul(dY[i % S], W.t(), out=dX[i % S]), n) * 1e3,
               "wgrad": time_loop(torch, lambda i: torch.matmul(X[i % S].t(), dY[i % S], out=dW), n) * 1e3}
        self.off()
        return out


# ---------------------------------------------------------------------------------------------------------------
# one layer: every entry point by itself, rotating buffer sets
# ---------------------------------------------------------------------------------------------------------------

class LayerBench:
    def __init__(self, torch, dd, synth, layer, algo, sets=0, offset_bands=0, seed=2506):
        self.torch, self.dd, self.layer = torch, dd, layer
        T, M, N, K = layer.tokens, layer.in_features, layer.out_features, layer.K
        self.T, self.M, self.N, self.K, self.L, self.D = T, M, N, K, layer.L, layer.D
        self.tdtype = torch.bfloat16 if layer.dtype == "bf16" else torch.float32
        e = 2 if layer.dtype == "bf16" else 4
        if sets <= 0:  # the operands of one product, times the sets, exceed the Infinity Cache twice over
            sets = max(2, min(8, -(-(512 << 20) // max(1, e * T * (M + N)))))
        self.S = S = sets
        self.algo = {"auto": dd.DD_ALGO_AUTO, "vector": dd.DD_ALGO_VECTOR, "matrix": dd.DD_ALGO_MATRIX}[algo]
        gen = torch.Generator(device="cuda")
        gen.manual_seed(seed)
        self.X = [torch.randn((T, M), device="cuda", generator=gen).to(self.tdtype) for _ in range(S)]
        self.dY = [torch.randn((T, N), device="cuda", generator=gen).to(self.tdtype) for _ in range(S)]
        self.Y = [torch.empty((T, N), dtype=self.tdtype, device="cuda") for _ in range(S)]
        self.dX = [torch.empty((T, M), dtype=self.tdtype, device="cuda") for _ in range(S)]
        values = synth.draw_normal((K, self.L), 0.02, seed, 10)
        scores = synth.draw_scores(1, self.D, seed)
        if offset_bands > 0:  # the selection then returns exactly the clustered set
            scores[0, synth.draw_offsets_clustered(self.D, K, offset_bands, seed)] += 100.0
        self.host = (values, scores)
        if layer.dtype == "bf16":
            self.values = torch.from_numpy(synth.bf16_bits(values).view(np.int16)).cuda().view(torch.bfloat16)
        else:
            self.values = torch.from_numpy(values).cuda()
        self.scores = torch.from_numpy(scores).cuda()
        self.off = torch.empty((1, K), dtype=torch.int32, device="cuda")
        self.dV = torch.empty((K, self.L), dtype=torch.float32, device="cuda")
        self.ws = dd.Workspace()
        self.prepared = None
        probe = dd.make_layer(T, M, N, K, self.tdtype, dd.DD_ALGO_PREPARED)
        self.use_prepare = (algo != "vector" and dd.dd_workspace_bytes(dd.DD_OP_PREPARE, probe) > 0 and
                            (algo == "matrix" or dd.dd_workspace_bytes(
                                dd.DD_OP_FWD, dd.make_layer(T, M, N, K, self.tdtype, dd.DD_ALGO_AUTO)) > 0))
        self.select(0)
        if self.use_prepare:
            self.prepare(0)
        torch.cuda.synchronize()

    # entry points
    def select(self, i):
        self.dd.dd_select_diagonals(self.scores, self.K, offsets_out=self.off, ws=self.ws)

    def prepare(self, i):
        self.prepared = self.dd.dd_prepare(self.off[0], self.values, self.M, self.N, prepared=self.prepared)

    def select_prepare(self, i):
        self.prepared = self.dd.dd_select_prepare(self.scores[0], self.values, self.M, self.N, offsets_out=self.off[0],
                                                  prepared=self.prepared)[1]

    def fwd_alone(self, i):
        s = i % self.S
        self.dd.dd_fwd(self.X[s], self.off[0], self.values, self.N, Y=self.Y[s], algo=self.algo, ws=self.ws)

    def bwd_input_alone(self, i):
        s = i % self.S
        self.dd.dd_bwd_input(self.dY[s], self.off[0], self.values, self.M, dX=self.dX[s], algo=self.algo, ws=self.ws)

    def fwd(self, i):
        if not self.use_prepare:
            return self.fwd_alone(i)
        s = i % self.S
        self.dd.dd_fwd(self.X[s], None, None, self.N, Y=self.Y[s], prepared=self.prepared)

    def bwd_input(self, i):
        if not self.use_prepare:
            return self.bwd_input_alone(i)
        s = i % self.S
        self.dd.dd_bwd_input(self.dY[s], None, None, self.M, dX=self.dX[s], prepared=self.prepared)

    def fwd_blocks(self, i):  # prepared operands, empty 32 x 16 operand blocks skipped
        s = i % self.S
        self.dd.dd_fwd(self.X[s], self.off[0], None, self.N, Y=self.Y[s], prepared=self.prepared,
                       algo=self.dd.DD_ALGO_BLOCKS)

    def bwd_input_blocks(self, i):
        s = i % self.S
        self.dd.dd_bwd_input(self.dY[s], self.off[0], None, self.M, dX=self.dX[s], prepared=self.prepared,
                             algo=self.dd.DD_ALGO_BLOCKS)

    def bwd_weight(self, i):
        s = i % self.S
        self.dd.dd_bwd_weight(self.X[s], self.dY[s], self.off[0], dValues=self.dV, algo=self.algo, ws=self.ws)

    def step(self, i):
        if self.use_prepare:
            self.select_prepare(i)
        else:
            self.select(i)
        self.fwd(i)
        self.bwd_input(i)
        self.bwd_weight(i)

    def flops(self):
        return 2.0 * self.T * self.K * self.L

    def dense_flops(self):
        return 2.0 * self.T * self.M * self.N

    def measure(self, n, dense=None):
        """One sub-line: us per entry point, rates, and the comparison with the dense GEMMs."""
        torch = self.torch
        for i in range(30):  # fresh buffers and an idle chip: the first dozen milliseconds run slow
            self.step(i)
        us = {"dd_select_diagonals": time_loop(torch, self.select, n) * 1e3,
              "dd_fwd": time_loop(torch, self.fwd, n) * 1e3,
              "dd_bwd_input": time_loop(torch, self.bwd_input, n) * 1e3,
              "dd_bwd_weight": time_loop(torch, self.bwd_weight, n) * 1e3}
        if self.use_prepare:
            us["dd_prepare"] = time_loop(torch, self.prepare, n) * 1e3
            us["dd_select_prepare"] = time_loop(torch, self.select_prepare, n) * 1e3
            us["dd_fwd_self_contained"] = time_loop(torch, self.fwd_alone, n) * 1e3
            us["dd_bwd_input_self_contained"] = time_loop(torch, self.bwd_input_alone, n) * 1e3
            self.prepare(0)
            if self.D <= 8192:
                us["dd_fwd_blocks"] = time_loop(torch, self.fwd_blocks, n) * 1e3
                us["dd_bwd_input_blocks"] = time_loop(torch, self.bwd_input_blocks, n) * 1e3
        # What reading dY once for both backward products could save at most: the same calls on ONE buffer set, so that
        # whatever the caches can hold of X and dY is served from them (at 12608 tokens everything fits the 256 MB
        # memory-side cache), and the two products of one layer back to back on the same dY, as a training step
        # issues them (the second then finds dY where the first left it).
        us["cache_hot"] = {"dd_bwd_input": time_loop(torch, lambda i: self.bwd_input(0), n) * 1e3,
                           "dd_bwd_weight": time_loop(torch, lambda i: self.bwd_weight(0), n) * 1e3}

        def pair(i):
            self.bwd_input(i)
            self.bwd_weight(i)
        us["dd_bwd_input+dd_bwd_weight_same_dY"] = time_loop(torch, pair, n) * 1e3
        if self.use_prepare:  # the backward pass as one call: runs of tokens that keep dY in the memory-side cache
            dX2 = [torch.empty_like(x) for x in self.dX]

            def fused(i):
                s = i % self.S
                self.dd.dd_bwd(self.X[s], self.dY[s], self.off[0], None, dX=dX2[s], dValues=self.dV, prepared=self.prepared,
                               ws=self.ws)
            us["dd_bwd"] = time_loop(torch, fused, n) * 1e3
            del dX2
        line = {"layer": f"{self.M}->{self.N}", "tokens": self.T, "K": self.K, "dtype": self.layer.dtype,
                "buffer_sets": self.S, "us": us,
                "sparse_tflops": {k: self.flops() / us[k] / 1e6 for k in ("dd_fwd", "dd_bwd_input", "dd_bwd_weight")},
                "frac_of_fp32_vector_peak": {k: self.flops() / us[k] / 1e6 / VALU_FP32_PEAK_TFLOPS
                                             for k in ("dd_fwd", "dd_bwd_input", "dd_bwd_weight")},
                "dense_equivalent_tflops": {k: self.dense_flops() / us[k] / 1e6
                                            for k in ("dd_fwd", "dd_bwd_input", "dd_bwd_weight")}}
        if dense is not None and self.layer.dtype == "bf16":
            g = dense.time_gemms(self.X, self.dY, self.Y, self.dX, n)
            ours_training = us["dd_fwd"] + us["dd_bwd_input"] + us["dd_bwd_weight"] + us.get("dd_prepare", 0.0)
            line["dense_gemm_us"] = g
            line["speedup_vs_dense"] = {
                "fwd_only_prepared": g["fwd"] / us["dd_fwd"],          # inference: weights fixed, operands built once
                "fwd_only_self_contained": g["fwd"] / us.get("dd_fwd_self_contained", us["dd_fwd"]),
                "fwd_bwd": (g["fwd"] + g["dgrad"] + g["wgrad"]) / ours_training}  # training, operand build charged
        return line


def helper_paths(b, n):
    """The differentiable selection (Sec. 3.2 Eq. 4-5) and the heuristic update of the active set beside one layer's
    step: step by step, and folded into the launches of the layer's own path.  us per call."""
    torch, dd = b.torch, b.dd
    K, D = b.K, b.D
    at = dd.dd_soft_topk(b.scores, K, 1.0)
    V = b.values.clone()
    eff = torch.empty_like(V)
    dsc_in = torch.randn((1, D), device="cuda")
    t = lambda fn: time_loop(torch, fn, n) * 1e3
    steps = {"dd_soft_topk": t(lambda i: dd.dd_soft_topk(b.scores, K, 1.0, alpha_tilde=at)),
             "dd_scale_values": t(lambda i: dd.dd_scale_values(b.off[0], at[0], V, values_eff=eff)),
             "dd_scale_values_bwd": t(lambda i: dd.dd_scale_values_bwd(b.off[0], at[0], V, b.dV, ws=b.ws)),
             "dd_soft_topk_bwd": t(lambda i: dd.dd_soft_topk_bwd(b.scores, K, 1.0, dsc_in))}
    out = {"step_by_step": steps, "step_by_step_sum": sum(steps.values())}
    if b.use_prepare:
        dV2 = torch.empty_like(b.dV)
        dat = torch.empty(D, device="cuda")
        prep = dd.dd_prepare_scaled(b.off[0], at[0], V, b.M, b.N)
        fused = {"dd_select_soft": t(lambda i: dd.dd_select_soft(b.scores, K, 1.0, offsets_out=b.off, alpha_tilde=at)),
                 "dd_select_diagonals": t(b.select),
                 "dd_prepare_scaled": t(lambda i: dd.dd_prepare_scaled(b.off[0], at[0], V, b.M, b.N, prepared=prep)),
                 "dd_prepare": t(b.prepare),
                 "dd_bwd_weight_scaled": t(lambda i: dd.dd_bwd_weight_scaled(b.X[i % b.S], b.dY[i % b.S], b.off[0], at[0],
                                                                             V, dV=dV2, d_alpha_tilde=dat, ws=b.ws)),
                 "dd_bwd_weight": t(b.bwd_weight)}
        out["folded_into_the_path"] = fused
        out["folded_extra_over_the_plain_path"] = (fused["dd_select_soft"] - fused["dd_select_diagonals"] +
                                                   fused["dd_prepare_scaled"] - fused["dd_prepare"] +
                                                   fused["dd_bwd_weight_scaled"] - fused["dd_bwd_weight"] +
                                                   steps["dd_soft_topk_bwd"])
    rnd = torch.rand(D, device="cuda")
    mag = dd.dd_diag_magnitude(b.values)
    n_drop = max(1, (3 * K) // 10)  # RigL's initial drop fraction
    out["diagheur"] = {"dd_diag_magnitude": t(lambda i: dd.dd_diag_magnitude(b.values, magnitudes=mag)),
                       "dd_diagheur_update": t(lambda i: dd.dd_diagheur_update(D, b.off[0], mag, rnd, n_drop, ws=b.ws))}
    b.select(0)
    if b.use_prepare:
        b.prepare(0)
    return out


def cpu_baseline_layers(layers, token_slice, scale, what, synth):
    """The oracle, as it stands, on the host cores over `token_slice` tokens of each layer; scaled to the step."""
    from oracle import dd_oracle as orc
    cases = []
    for i, l in enumerate(layers):
        small = synth.Layer(l.name, token_slice, l.in_features, l.out_features, l.K, l.dtype)
        cases.append((l, synth.layer_inputs(small, seed=2506 + i), synth.draw_scores(1, l.D, seed=2506 + i)))
    reps, t0 = 0, time.perf_counter()
    while True:
        for l, (offsets, values, X, dY), scores in cases:
            orc.select(scores, l.K)
            orc.fwd(X, offsets, values, l.out_features)
            orc.bwd_input(dY, offsets, values, l.in_features)
            orc.bwd_weight(X, dY, offsets)
        reps += 1
        dt = time.perf_counter() - t0
        if dt > 10.0 or reps >= 40:
            break
    flops = sum(3 * 2.0 * token_slice * l.K * l.L for l in layers) * reps
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"{what}; {reps} repetitions in {dt:.1f} s; the rate is per token, so it stands for the whole "
                      f"step (which is {scale:.0f}x this sample); dense fp64 loops, so the oracle performs about "
                      f"{layers[0].D / layers[0].K:.0f}x the sparse flops it is credited with"}


def distinct(layers):
    seen, out = set(), []
    for l in layers:
        key = (l.tokens, l.in_features, l.out_features, l.K, l.dtype)
        if key not in seen:
            seen.add(key)
            out.append(l)
    return out


def stored_traffic(workload, kernel):
    """HBM bytes per launch from the committed rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE), if any."""
    try:
        rec = json.load(open(TRAFFIC_FILE)).get(workload, {}).get(kernel)
    except Exception:
        return None, None
    if rec is None:
        return None, None
    if isinstance(rec, dict):
        return rec.get("bytes_per_launch"), rec.get("source")
    return rec, "profiles/hbm_traffic.json"


def roofline_block(flops, nbytes, seconds, launches, kernel, workload, dense_flops, executed_on, per_entry):
    """`flops`, `nbytes`, `seconds`: sums over `launches` launches of the dominant kernel."""
    alu_bound = flops / (VALU_FP32_PEAK_TFLOPS * 1e12) >= nbytes / (HBM_PEAK_GBS * 1e9)
    traffic, source = stored_traffic(workload, kernel)
    if alu_bound:
        achieved = flops / seconds / 1e12
        r = {"bound": "alu", "achieved": achieved, "peak": VALU_FP32_PEAK_TFLOPS, "unit": "TFLOP/s",
             "frac": achieved / VALU_FP32_PEAK_TFLOPS}
    else:
        achieved = nbytes / seconds / 1e9
        r = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS}
    r.update({"traffic": traffic,
              "traffic_source": (source or "none measured for this workload") +
                                " (a stored figure from rocprofv3 --pmc runs, not measured in this run)",
              "kernel": kernel, "launches_per_step": launches, "avg_launch_us": seconds / launches * 1e6,
              "flops_per_launch": flops / launches, "bytes_per_launch": nbytes / launches,
              "flop_per_byte": flops / nbytes, "achieved_gbs": nbytes / seconds / 1e9,
              "frac_of_hbm_peak": nbytes / seconds / 1e9 / HBM_PEAK_GBS,
              "executed_on": executed_on,
              # what the matrix cores execute is the dense contraction over all D candidate diagonals
              "dense_equivalent_tflops": dense_flops / seconds / 1e12,
              "dense_equivalent_frac_of_mfma_peak": dense_flops / seconds / 1e12 / MFMA_BF16_PEAK_TFLOPS,
              "frac_per_entry_point": per_entry})
    return r


# ---------------------------------------------------------------------------------------------------------------

def run_stack(args, torch, dd, synth, dense):
    from paper_2506_11449_amd.stack import StackStep
    steps = args.steps if args.steps is not None else 20
    warmup = args.warmup if args.warmup is not None else 3
    st = StackStep(blocks=12, tokens=256 * 197, sets_attn=args.sets or 4, sets_mlp=args.sets or 2, score_sets=4,
                   seed=2506, device_inputs=True)
    torch.cuda.synchronize()

    # ---- the timed region of the contract: W warm-up steps, then exactly K steps ----
    for _ in range(warmup):
        st.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        st.step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
    flops = st.flops_per_product()
    value = 3 * flops / (ms_per_step * 1e-3) / 1e12

    # ---- per entry point: all its launches of one step between two events on the launch stream ----
    n = max(3, min(10, steps))
    parts = {"dd_select_diagonals": time_loop(torch, lambda i: st.select(i), n),
             "dd_prepare_batched": time_loop(torch, lambda i: st.prepare(), n),
             "dd_fwd": time_loop(torch, lambda i: st.forward(), n),
             "dd_bwd_input": time_loop(torch, lambda i: st.backward_input(), n),
             "dd_bwd_weight": time_loop(torch, lambda i: st.backward_weight(), n)}
    n_layers = len(st.layers)
    # dd_fwd and dd_bwd_input on prepared operands are one launch of the same kernel each
    # (mm_persistent_kernel<160, 256, 8>: every result here has more tiles than the chip has CUs)
    mm_s = (parts["dd_fwd"] + parts["dd_bwd_input"]) * 1e-3
    wg_s = parts["dd_bwd_weight"] * 1e-3
    per_entry = {k: flops / (parts[k] * 1e-3) / 1e12 / VALU_FP32_PEAK_TFLOPS
                 for k in ("dd_fwd", "dd_bwd_input", "dd_bwd_weight")}
    if mm_s >= wg_s:
        roofline = roofline_block(2 * flops, 2 * st.bytes_per_product(), mm_s, 2 * n_layers, "mm_persistent_kernel",
                                  "vitb_stack", 2 * st.dense_flops_per_product(),
                                  "matrix cores (dense contraction over all D candidate diagonals); the kernel serves "
                                  "dd_fwd and dd_bwd_input", per_entry)
    else:
        roofline = roofline_block(flops, st.bytes_per_weight_gradient(), wg_s, n_layers, "wgrad_mm_kernel",
                                  "vitb_stack", st.dense_flops_per_product(),
                                  "matrix cores (dense contraction over tokens, diagonals kept in the epilogue)",
                                  per_entry)

    breakdown = {"ms_per_step_by_entry_point": parts,
                 "ms_sum_of_entry_points": sum(parts.values()),
                 "sparse_tflops": {k: flops / (parts[k] * 1e-3) / 1e12 for k in ("dd_fwd", "dd_bwd_input", "dd_bwd_weight")},
                 "dense_equivalent_tflops": {k: st.dense_flops_per_product() / (parts[k] * 1e-3) / 1e12
                                             for k in ("dd_fwd", "dd_bwd_input", "dd_bwd_weight")},
                 "paper_context": PAPER_CONTEXT}

    # ---- per shape of the stack, and the dense GEMMs of the same shapes ----
    shapes = {}
    for g in (st.groups.values() if dense is not None else ()):
        S = g.sets
        j0 = 0
        us = {"dd_fwd": time_loop(torch, lambda i: dd.dd_fwd(g.X[i % S], None, None, g.N, Y=g.Y[i % S],
                                                             prepared=g.prepared[j0]), 50, warmup=10) * 1e3,
              "dd_bwd_input": time_loop(torch, lambda i: dd.dd_bwd_input(g.dY[i % S], None, None, g.M, dX=g.dX[i % S],
                                                                         prepared=g.prepared[j0]), 50, warmup=10) * 1e3,
              "dd_bwd_weight": time_loop(torch, lambda i: dd.dd_bwd_weight(g.X[i % S], g.dY[i % S], g.offsets[j0],
                                                                           dValues=g.dValues[j0], ws=st.ws), 50, warmup=10) * 1e3}
        line = {"layers": g.n_layers, "K": g.K, "us": us,
                "frac_of_fp32_vector_peak": {k: 2.0 * st.tokens * g.K * g.L / v / 1e6 / VALU_FP32_PEAK_TFLOPS
                                             for k, v in us.items()},
                "dense_equivalent_tflops": {k: 2.0 * st.tokens * g.M * g.N / v / 1e6 for k, v in us.items()}}
        if dense is not None:
            line["dense_gemm_us"] = dense.time_gemms(g.X, g.dY, g.Y, g.dX, 20)
            line["speedup_vs_dense"] = {"fwd_only_prepared": line["dense_gemm_us"]["fwd"] / us["dd_fwd"],
                                        "fwd_bwd": sum(line["dense_gemm_us"].values()) / sum(us.values())}
        shapes[f"{g.M}->{g.N}"] = line
    if shapes:
        breakdown["stack_shapes"] = shapes
    if dense is not None:
        dense_ms = sum(sum(l["dense_gemm_us"].values()) * l["layers"] for l in shapes.values()) * 1e-3
        dense_fwd_ms = sum(l["dense_gemm_us"]["fwd"] * l["layers"] for l in shapes.values()) * 1e-3
        breakdown["dense_stack_ms"] = {"fwd": dense_fwd_ms, "fwd_dgrad_wgrad": dense_ms,
                                       "tuned": dense.tuned, "solutions": dense.chosen()}
        breakdown["speedup_vs_dense"] = {
            # inference: operands built once, weights fixed; training: the whole step, selection and operand build in
            "fwd_only": dense_fwd_ms / parts["dd_fwd"],
            "training_step": dense_ms / ms_per_step}

    out = {"metric": "diag-sparse linear fwd+bwd effective TFLOP/s, % roofline, speedup vs dense GEMM",
           "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
           "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "bf16", "data": "synthetic",
           "config": {"workload": "ViT-Base-depth stack: 12 blocks x (4 x 768->768 + 768->3072 + 3072->768), 90% sparse "
                                  "(K=77 / 307 diagonals), tokens=256x197=50432, bf16 storage, fp32 accumulate, "
                                  "TopK re-selection of all 72 layers every step",
                      "step": "2 x dd_select_diagonals (48 x 768, 24 x 3072) + 3 x dd_prepare_batched + 72 x dd_fwd + "
                              "72 x (dd_bwd_input + dd_bwd_weight); layers not chained, rotating buffer sets",
                      "offsets": "re-selected every step from seeded N(0,1) scores (uniform)",
                      "layers": n_layers, "tokens": st.tokens,
                      "buffer_sets": {g.name: g.sets for g in st.groups.values()}},
           "roofline": roofline, "breakdown": breakdown}
    if not args.no_cpu_baseline:
        block = synth.WORKLOADS["vitb_stack"]
        out["cpu_baseline"] = cpu_baseline_layers(
            block, st.tokens // 16, 16 * 12,
            f"one block of the stack (4 x 768->768, 768->3072, 3072->768; select + fwd + bwd_input + bwd_weight each) "
            f"on a 1/16 slice of the tokens ({st.tokens // 16} rows)", synth)
    del st
    torch.cuda.empty_cache()
    return out


def run_layers(args, torch, dd, synth, dense, workload):
    """A step = every layer of the workload: selection + operand build, forward, both backward products."""
    layers = synth.WORKLOADS[workload]
    small = workload in ("tiny", "vitb_attn_proj")
    steps = args.steps if args.steps is not None else (200 if small else 20)
    warmup = args.warmup if args.warmup is not None else (20 if small else 3)
    benches = [LayerBench(torch, dd, synth, l, args.algo, args.sets, args.offset_bands, seed=2506 + i)
               for i, l in enumerate(distinct(layers))]
    torch.cuda.synchronize()
    for i in range(warmup):
        for b in benches:
            b.step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        for b in benches:
            b.step(i)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
    flops = sum(b.flops() for b in benches)
    value = 3 * flops / (ms_per_step * 1e-3) / 1e12
    n = max(20, min(steps, 100))
    lines = [b.measure(n, dense) for b in benches]
    if workload == "vitb_attn_proj":
        lines[0]["selection_helpers_us"] = helper_paths(benches[0], n)
    e = 2 if layers[0].dtype == "bf16" else 4
    per = {k: sum(l["us"][k] for l in lines) * 1e-6 for k in ("dd_fwd", "dd_bwd_input", "dd_bwd_weight")}
    dominant = max(per, key=per.get)
    nbytes = sum(e * b.T * (b.M + b.N) + (4 if dominant == "dd_bwd_weight" else e) * b.K * b.L + 4 * b.K for b in benches)
    on_matrix = benches[0].use_prepare
    roofline = roofline_block(flops, nbytes, per[dominant], len(benches), dominant, workload,
                              sum(b.dense_flops() for b in benches),
                              "matrix cores (dense contraction over all D candidate diagonals)" if on_matrix
                              else "vector ALUs",
                              {k: flops / per[k] / 1e12 / VALU_FP32_PEAK_TFLOPS for k in per})
    out = {"metric": "diag-sparse linear fwd+bwd effective TFLOP/s, % roofline, speedup vs dense GEMM",
           "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
           "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": layers[0].dtype, "data": "synthetic",
           "config": {"workload": workload + ": " + ", ".join(f"{b.M}->{b.N} K={b.K} T={b.T}" for b in benches),
                      "step": "per layer: dd_select_prepare (dd_select_diagonals + dd_prepare as one call) + dd_fwd + "
                              "dd_bwd_input + dd_bwd_weight" if on_matrix else
                              "per layer: dd_select_diagonals + dd_fwd + dd_bwd_input + dd_bwd_weight",
                      "offsets": "uniform" if args.offset_bands == 0 else f"{args.offset_bands} runs of adjacent diagonals",
                      "algo": args.algo},
           "roofline": roofline,
           "breakdown": {"layers": lines, "paper_context": PAPER_CONTEXT,
                         "dense_tuned": bool(dense and dense.tuned)}}
    if not args.no_cpu_baseline:
        frac = 1 if small else 16
        out["cpu_baseline"] = cpu_baseline_layers(
            distinct(layers), layers[0].tokens // frac, frac,
            f"every distinct layer of {workload} (select + fwd + bwd_input + bwd_weight) on "
            f"{'all' if frac == 1 else '1/16 of'} the tokens", synth)
    return out, lines


def config_sublines(args, torch, dd, synth, dense):
    """One sub-line per distinct layer of the smaller configurations; each layer's buffers are freed before the next."""
    out = {}
    for name in ("tiny", "vitb_attn_proj", "vitb_mlp", "vitl") + (("vitb_stack",) if args.table else ()):
        lines = []
        for i, l in enumerate(distinct(synth.WORKLOADS[name])):
            b = LayerBench(torch, dd, synth, l, "auto", 0, 0, seed=2506 + i)
            lines.append(b.measure(30, dense))
            if name == "vitb_attn_proj":
                lines[-1]["selection_helpers_us"] = helper_paths(b, 30)
            del b
            torch.cuda.empty_cache()
        out[name] = lines
    return out


def tune_dense(torch, dd, synth, dense):
    """Every dense GEMM the benchmark compares with, once, with the search switched on."""
    seen = set()
    for name in ("vitb_stack", "vitb_attn_proj", "vitb_mlp", "vitl"):
        for l in distinct(synth.WORKLOADS[name]):
            key = (l.tokens, l.in_features, l.out_features)
            if key in seen or l.dtype != "bf16":
                continue
            seen.add(key)
            X = [torch.randn((l.tokens, l.in_features), device="cuda").to(torch.bfloat16)]
            dY = [torch.randn((l.tokens, l.out_features), device="cuda").to(torch.bfloat16)]
            Y, dX = [torch.empty_like(dY[0])], [torch.empty_like(X[0])]
            t = dense.time_gemms(X, dY, Y, dX, 5)
            print(f"tuned {key}: {t}", file=sys.stderr, flush=True)
            del X, dY, Y, dX
            torch.cuda.empty_cache()
    # the file in the layout torch reads back: validators first, then one line per GEMM
    with open(DENSE_TUNING_FILE, "w") as f:
        for key, val in dense.tunable.get_validators():
            f.write(f"Validator,{key},{val}\n")
        for r in dense.tunable.get_results():
            f.write(",".join(str(x) for x in r) + "\n")
    dense.tunable.set_filename(os.path.join(tempfile.gettempdir(), "tunableop_scratch.csv"))  # torch's own copy at exit
    print(f"wrote {DENSE_TUNING_FILE}", file=sys.stderr)


def k_sweep(torch, dd, synth):
    """us per self-contained call over K: DD_ALGO_VECTOR (K <= 16: the kernels for a handful of diagonals), DD_ALGO_MATRIX
    (dense operand rebuilt inside the call) and what DD_ALGO_AUTO picks."""
    rows = []
    for (M, N, T) in ((768, 768, 12608), (1024, 1024, 25216), (768, 3072, 25216), (3072, 768, 25216)):
        D = max(M, N)
        for K in (1, 2, 4, 8, 12, 16, 21, 24, 32, 48, 64, D // 8):
            l = synth.Layer(f"sweep_{M}_{N}_{K}", T, M, N, K, "bf16")
            t = {}
            for algo in ("vector", "matrix", "auto"):
                b = LayerBench(torch, dd, synth, l, algo, 0, 0)
                t[algo] = {"fwd": time_loop(torch, b.fwd_alone, 20) * 1e3,
                           "bwd_input": time_loop(torch, b.bwd_input_alone, 20) * 1e3,
                           "bwd_weight": time_loop(torch, b.bwd_weight, 20) * 1e3}
                del b
            rows.append({"M": M, "N": N, "T": T, "K": K, "us": t,
                         "hbm_floor_us": 2 * T * (M + N) / 8e12 * 1e6})
            print(json.dumps(rows[-1]), file=sys.stderr, flush=True)
    return rows


def saturation(torch, dd, synth, dense):
    """Two experiments on the prepared forward product (and torch.matmul on the same shapes):
    occupancy -- T = 160 * blocks tokens give blocks * N/256 result tiles of 160 x 256, one per CU, so the time per call
    is the time of one tile with that many CUs busy; data -- the stack's shapes on random and on all-zero operands
    (zeros switch no multiplier inputs: what is left of the difference is not arithmetic power)."""
    out = {"occupancy": [], "data": []}

    def run(T, M, N, K, zero, n=30):
        off = torch.from_numpy(synth.draw_offsets(max(M, N), K, 2506)).cuda()
        mk = (lambda *sh: torch.zeros(*sh, device="cuda", dtype=torch.bfloat16)) if zero else \
             (lambda *sh: torch.randn(*sh, device="cuda").to(torch.bfloat16))
        val = mk(K, min(M, N)) * 0.02
        sets = 4
        X = [mk(T, M) for _ in range(sets)]
        Y = [torch.empty(T, N, device="cuda", dtype=torch.bfloat16) for _ in range(sets)]
        prep = dd.dd_prepare(off, val.to(torch.bfloat16), M, N)
        W = mk(M, N)
        t_dd = min(time_loop(torch, lambda i: dd.dd_fwd(X[i % sets], None, None, N, Y=Y[i % sets], prepared=prep), n)
                   for _ in range(3)) * 1e3
        t_mm = None
        if dense is not None:
            dense.on()
            t_mm = min(time_loop(torch, lambda i: torch.matmul(X[i % sets], W, out=Y[i % sets]), n) for _ in range(3)) * 1e3
            dense.off()
        return t_dd, t_mm

    for (M, N, K) in ((768, 768, 77), (2048, 768, 205)):
        for blocks in (1, 4, 8, 16, 32, 48, 64, 85):
            T = 160 * blocks
            t_dd, t_mm = run(T, M, N, K, zero=False)
            tiles = blocks * (N // 256)
            out["occupancy"].append({"M": M, "N": N, "tokens": T, "tiles": tiles, "dd_fwd_us": t_dd, "dense_gemm_us": t_mm,
                                     "dd_fwd_dense_equivalent_tflops": 2.0 * T * M * N / t_dd / 1e6,
                                     "dd_fwd_tflops_per_busy_cu": 2.0 * T * M * N / t_dd / 1e6 / tiles})
            print(json.dumps(out["occupancy"][-1]), file=sys.stderr, flush=True)
    for (M, N, K) in ((768, 768, 77), (768, 3072, 307), (3072, 768, 307)):
        row = {"M": M, "N": N, "tokens": 50432}
        for zero in (False, True):
            t_dd, t_mm = run(50432, M, N, K, zero)
            row["zero" if zero else "random"] = {"dd_fwd_us": t_dd, "dense_gemm_us": t_mm}
        out["data"].append(row)
        print(json.dumps(row), file=sys.stderr, flush=True)
    return out


def markdown_table(lines_by_config):
    out = ["| layer | T | K | prepare | fwd | bwd_input | bwd_weight | dense fwd / dgrad / wgrad | frac of 157.3 fwd / bwd_input / bwd_weight | fwd-only speedup (prepared / self-contained) | fwd+bwd speedup |",
           "|---|---|---|---|---|---|---|---|---|---|---|"]
    for name, lines in lines_by_config.items():
        for l in lines:
            us, g, sp = l["us"], l.get("dense_gemm_us"), l.get("speedup_vs_dense")
            fr = l["frac_of_fp32_vector_peak"]
            prep = f"{us['dd_prepare']:.1f}" if "dd_prepare" in us else "-"  # fp32 storage has no dense operand
            out.append(f"| {l['layer']} ({name}) | {l['tokens']} | {l['K']} | {prep} | "
                       f"{us['dd_fwd']:.1f} | {us['dd_bwd_input']:.1f} | {us['dd_bwd_weight']:.1f} | " +
                       (f"{g['fwd']:.1f} / {g['dgrad']:.1f} / {g['wgrad']:.1f}" if g else "") + " | " +
                       f"{fr['dd_fwd']:.2f} / {fr['dd_bwd_input']:.2f} / {fr['dd_bwd_weight']:.2f} | " +
                       (f"{sp['fwd_only_prepared']:.2f}x / {sp['fwd_only_self_contained']:.2f}x | {sp['fwd_bwd']:.2f}x"
                        if sp else " | ") + " |")
    return "\n".join(out)


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus must be 1 (no multi-GPU path exists).",
              file=sys.stderr)
        return 2
    import torch
    import paper_2506_11449_amd as dd
    from paper_2506_11449_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    dd.load_library()
    dense = None if args.no_dense else DenseBaseline(torch, tune=args.tune_dense)
    if dense is not None:
        dense.off()  # only the baseline's own GEMMs go through the tuned path

    if args.tune_dense:
        tune_dense(torch, dd, synth, dense)
        return 0
    if args.k_sweep:
        print(json.dumps({"k_sweep": k_sweep(torch, dd, synth)}))
        return 0
    if args.saturation:
        print(json.dumps({"saturation": saturation(torch, dd, synth, dense)}))
        return 0
    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.workload == "vitb_stack" and not args.per_layer and args.offset_bands == 0:
        out = run_stack(args, torch, dd, synth, dense)
        if not args.no_configs:
            out["breakdown"]["configs"] = config_sublines(args, torch, dd, synth, dense)
        if args.table:
            print(markdown_table(out["breakdown"].get("configs", {})))
            return 0
    else:
        out, lines = run_layers(args, torch, dd, synth, dense, args.workload)
        if args.table:
            print(markdown_table({args.workload: lines}))
            return 0
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
