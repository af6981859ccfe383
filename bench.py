#!/usr/bin/env python3
"""Benchmark of the diagonally-sparse layer's hot path on one MI355X.

A step is one pass of the whole path over one batch: the selection of the diagonals and the build
of the dense operands from them (dd_select_prepare = dd_select_diagonals + dd_prepare in one call),
dd_fwd, dd_bwd_input and dd_bwd_weight of the ViT-Base attention projection (768 -> 768, 90 % sparse,
K = 77, 12608 tokens, bf16 storage, fp32 accumulation) with inputs already resident in HBM.  The
metric is the effective (sparse) rate 3 * 2*T*K*L / t_step.  Buffers rotate over several sets
so that a step does not find its operands in the 256 MB Infinity Cache.

Prints ONE JSON line.  Besides the contract fields it carries
  roofline      the dominant kernel against the ceiling that bounds it,
  cpu_baseline  the CPU oracle timed on this host's cores (a baseline, not a target),
  breakdown     per-function times, the dense bf16 GEMM (hipBLASLt through torch.matmul) of the
                same shape, and the paper's own speedups for context.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
VALU_FP32_PEAK_TFLOPS = 157.3  # MI355X fp32 vector, published (256 CU x 128 lanes-flop x 2 x 2.4 GHz)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--sets", type=int, default=8, help="rotating buffer sets (working set > Infinity Cache)")
    ap.add_argument("--workload", default="vitb_attn_proj")
    ap.add_argument("--algo", default="auto", choices=["auto", "vector", "matrix"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--offset-bands", type=int, default=0,
                    help="0: seeded uniform offsets (the benchmark); n > 0: the K diagonals in n runs of adjacent ones")
    ap.add_argument("--no-prepare", action="store_true", help="every product rebuilds its dense operand itself")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy a few times (a known-size reference for the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    return ap.parse_args()


def time_loop(torch, fn, sets, steps, warmup):
    """Average milliseconds per call of fn(i % sets), timed with events on the launch stream."""
    for i in range(warmup):
        fn(i % sets)
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for i in range(steps):
        fn(i % sets)
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) / steps


def cpu_baseline(layer, offsets, values, X, dY, scores):
    """The oracle, as it stands, on the host cores: the whole workload, repeated for ~10 s."""
    from oracle import dd_oracle as orc
    reps, t0 = 0, time.perf_counter()
    while True:
        orc.select(scores, layer.K)
        orc.fwd(X, offsets, values, layer.out_features)
        orc.bwd_input(dY, offsets, values, layer.in_features)
        orc.bwd_weight(X, dY, offsets)
        reps += 1
        dt = time.perf_counter() - t0
        if dt > 10.0 or reps >= 40:
            break
    flops = 3 * 2.0 * layer.tokens * layer.K * layer.L * reps
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"whole {layer.name} workload (select + fwd + bwd_input + bwd_weight, all {layer.tokens} "
                      f"tokens), {reps} repetitions, {dt:.1f} s; dense fp64 loops, so it performs "
                      f"{layer.D / layer.K:.1f}x the sparse flops it is credited with"}


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
    algo = {"auto": dd.DD_ALGO_AUTO, "vector": dd.DD_ALGO_VECTOR, "matrix": dd.DD_ALGO_MATRIX}[args.algo]

    layer = synth.WORKLOADS[args.workload][0]
    T, M, N, K, L, D = layer.tokens, layer.in_features, layer.out_features, layer.K, layer.L, layer.D
    tdtype = torch.bfloat16 if layer.dtype == "bf16" else torch.float32

    def dev(a):
        if layer.dtype == "bf16":
            return torch.from_numpy(synth.bf16_bits(a).view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(a).cuda()

    # set 0 holds the seeded inputs; the other sets are device-side copies (same values, other addresses)
    offsets, values, X, dY = synth.layer_inputs(layer, seed=2506)
    scores = synth.draw_scores(1, D, seed=2506)
    if args.offset_bands > 0:  # the selection then returns exactly the clustered set
        scores[0, synth.draw_offsets_clustered(D, K, args.offset_bands, seed=2506)] += 100.0
    S = max(1, args.sets)
    d_val = dev(values)
    d_scores = torch.from_numpy(scores).cuda()
    d_X = [dev(X)] + [None] * (S - 1)
    d_dY = [dev(dY)] + [None] * (S - 1)
    for s in range(1, S):
        d_X[s], d_dY[s] = d_X[0].clone(), d_dY[0].clone()
    d_Y = [torch.empty((T, N), dtype=tdtype, device="cuda") for _ in range(S)]
    d_dX = [torch.empty((T, M), dtype=tdtype, device="cuda") for _ in range(S)]
    d_dV = torch.empty((K, L), dtype=torch.float32, device="cuda")
    d_off = torch.empty((1, K), dtype=torch.int32, device="cuda")
    ws = dd.Workspace()

    def f_select(s):
        dd.dd_select_diagonals(d_scores, K, offsets_out=d_off, ws=ws)

    def f_fwd_alone(s):
        dd.dd_fwd(d_X[s], d_off[0], d_val, N, Y=d_Y[s], algo=algo, ws=ws)

    def f_bwd_input_alone(s):
        dd.dd_bwd_input(d_dY[s], d_off[0], d_val, M, dX=d_dX[s], algo=algo, ws=ws)

    # The dense operands of the matrix-core path are built once per step (dd_prepare) and serve both the forward
    # and the backward-input product, as they would in training; where that path does not apply (vector family,
    # fp32 storage) every product is self-contained.
    use_prepare = (not args.no_prepare and args.algo != "vector" and
                   dd.dd_workspace_bytes(5, dd.make_layer(T, M, N, K, tdtype, dd.DD_ALGO_PREPARED)) > 0 and
                   (args.algo == "matrix" or K * 48 >= D))
    prepared = [None]

    def f_prepare(s):
        prepared[0] = dd.dd_prepare(d_off[0], d_val, M, N, prepared=prepared[0])

    def f_fwd(s):
        dd.dd_fwd(d_X[s], None, None, N, Y=d_Y[s], prepared=prepared[0])

    def f_bwd_input(s):
        dd.dd_bwd_input(d_dY[s], None, None, M, dX=d_dX[s], prepared=prepared[0])

    if not use_prepare:
        f_fwd, f_bwd_input = f_fwd_alone, f_bwd_input_alone

    def f_bwd_weight(s):
        dd.dd_bwd_weight(d_X[s], d_dY[s], d_off[0], dValues=d_dV, algo=algo, ws=ws)

    def f_select_prepare(s):  # selection and operand build as one call
        prepared[0] = dd.dd_select_prepare(d_scores[0], d_val, M, N, offsets_out=d_off[0], prepared=prepared[0])[1]

    def step(s):
        if use_prepare:
            f_select_prepare(s)
        else:
            f_select(s)
        f_fwd(s)
        f_bwd_input(s)
        f_bwd_weight(s)

    f_select(0)
    if use_prepare:
        f_prepare(0)
    torch.cuda.synchronize()

    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- the timed region of the contract: W warm-up steps, then exactly K steps ----
    for i in range(args.warmup):
        step(i % S)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i % S)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    flops_product = 2.0 * T * K * L
    value = 3 * flops_product / (ms_per_step * 1e-3) / 1e12

    # ---- per-function device times (events on the launch stream) ----
    n = max(20, args.steps)
    per = {name: time_loop(torch, fn, S, n, 5) for name, fn in
           (("dd_select_diagonals", f_select), ("dd_fwd", f_fwd), ("dd_bwd_input", f_bwd_input),
            ("dd_bwd_weight", f_bwd_weight))}
    alone = {"dd_fwd": per["dd_fwd"], "dd_bwd_input": per["dd_bwd_input"]}
    if use_prepare:
        per["dd_prepare"] = time_loop(torch, f_prepare, S, n, 5)
        per["dd_select_prepare"] = time_loop(torch, f_select_prepare, S, n, 5)
        alone = {"dd_fwd": time_loop(torch, f_fwd_alone, S, n, 5),
                 "dd_bwd_input": time_loop(torch, f_bwd_input_alone, S, n, 5)}
        f_prepare(0)
    hot = {name: time_loop(torch, fn, 1, n, 5) for name, fn in
           (("dd_fwd", f_fwd), ("dd_bwd_input", f_bwd_input), ("dd_bwd_weight", f_bwd_weight))}

    e = 2 if layer.dtype == "bf16" else 4
    bytes_product = e * (T * M + T * N) + e * K * L + 4 * K
    bytes_wgrad = e * (T * M + T * N) + 4 * K * L + 4 * K
    dominant = max(("dd_fwd", "dd_bwd_input", "dd_bwd_weight"), key=lambda k: per[k])
    dom_s = per[dominant] * 1e-3
    dom_bytes = bytes_wgrad if dominant == "dd_bwd_weight" else bytes_product
    intensity = flops_product / dom_bytes
    # the ceiling that binds: flops / 157.3 TFLOP/s against bytes / 8 TB/s
    alu_bound = flops_product / (VALU_FP32_PEAK_TFLOPS * 1e12) >= dom_bytes / (HBM_PEAK_GBS * 1e9)
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get(args.workload, {}).get(dominant)
        except Exception:
            traffic = None
    if alu_bound:
        achieved = flops_product / dom_s / 1e12
        roofline = {"bound": "alu", "achieved": achieved, "peak": VALU_FP32_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": achieved / VALU_FP32_PEAK_TFLOPS, "traffic": traffic}
    else:
        achieved = dom_bytes / dom_s / 1e9
        roofline = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": achieved / HBM_PEAK_GBS, "traffic": traffic}
    roofline.update({"executed_on": "matrix cores (dense contraction over all D candidate diagonals)"
                     if args.algo != "vector" and layer.dtype == "bf16" else "vector ALUs",
                     "dense_equivalent_tflops": 2.0 * T * M * N / dom_s / 1e12,
                     # the dense contraction the matrix cores execute, against their published bf16 peak
                     "dense_equivalent_frac_of_mfma_peak": 2.0 * T * M * N / dom_s / 1e12 / 2500.0,
                     "kernel": dominant, "avg_launch_us": dom_s * 1e6, "flops_per_launch": flops_product,
                     "bytes_per_launch": dom_bytes, "flop_per_byte": intensity,
                     "achieved_tflops": flops_product / dom_s / 1e12, "achieved_gbs": dom_bytes / dom_s / 1e9,
                     # the same fraction for each of the three products (the dominant one is the slowest)
                     "frac_per_entry_point": {
                         k: (flops_product / (per[k] * 1e-3) / 1e12 / VALU_FP32_PEAK_TFLOPS if alu_bound else
                             (bytes_wgrad if k == "dd_bwd_weight" else bytes_product) / (per[k] * 1e-3) / 1e9
                             / HBM_PEAK_GBS)
                         for k in ("dd_fwd", "dd_bwd_input", "dd_bwd_weight")}})

    breakdown = {"us": {k: v * 1e3 for k, v in per.items()},
                 "us_self_contained": {k: v * 1e3 for k, v in alone.items()},
                 "us_cache_hot": {k: v * 1e3 for k, v in hot.items()},
                 "sparse_tflops": {k: flops_product / (per[k] * 1e-3) / 1e12
                                   for k in ("dd_fwd", "dd_bwd_input", "dd_bwd_weight")},
                 "dense_equivalent_tflops": {k: 2.0 * T * M * N / (per[k] * 1e-3) / 1e12
                                             for k in ("dd_fwd", "dd_bwd_input", "dd_bwd_weight")},
                 "paper_context": "paper reports 3.13x inference / 1.59x training speedup at 90 % sparsity, "
                                  "ViT-Base end to end, on an A100 (abstract, Sec. 4.2.3): another machine"}

    # the same step replayed from a HIP graph (one graph holds one step per buffer set): what is left of the step
    # time once the launches cost the host nothing; reported beside the contract's figure, not as it
    try:
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                for s_ in range(S):
                    step(s_)
        torch.cuda.synchronize()
        reps = max(3, args.steps // S)
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            graph.replay()
        torch.cuda.synchronize()
        breakdown["us_step_replayed_from_graph"] = (time.perf_counter() - t0) * 1e6 / (reps * S)
        del graph
    except Exception as exc:  # reported, never fatal: the contract's figures above do not depend on it
        breakdown["us_step_replayed_from_graph"] = None
        breakdown["graph_error"] = repr(exc)[:200]

    # the differentiable selection path (Sec. 3.2, Eq. 4-5), outside the timed step: launch-bound helpers
    d_V = d_val.clone()
    at = dd.dd_soft_topk(d_scores, K, 1.0)
    soft = {"dd_soft_topk": time_loop(torch, lambda s: dd.dd_soft_topk(d_scores, K, 1.0, alpha_tilde=at), S, n, 5),
            "dd_scale_values": time_loop(torch, lambda s: dd.dd_scale_values(d_off[0], at[0], d_V, values_eff=d_val),
                                         S, n, 5),
            "dd_scale_values_bwd": time_loop(torch, lambda s: dd.dd_scale_values_bwd(d_off[0], at[0], d_V, d_dV, ws=ws),
                                             S, n, 5),
            "dd_soft_topk_bwd": time_loop(torch, lambda s: dd.dd_soft_topk_bwd(d_scores, K, 1.0, at), S, n, 5)}
    breakdown["soft_topk_path_us"] = {k: v * 1e3 for k, v in soft.items()}
    # the heuristic update of the active set (appendix on the heuristics-based method), also outside the step
    d_rand = torch.rand(D, device="cuda")
    mag = dd.dd_diag_magnitude(d_val)
    n_drop = max(1, (3 * K) // 10)  # RigL's initial drop fraction
    heur = {"dd_diag_magnitude": time_loop(torch, lambda s: dd.dd_diag_magnitude(d_val, magnitudes=mag), S, n, 5),
            "dd_diagheur_update": time_loop(torch, lambda s: dd.dd_diagheur_update(D, d_off[0], mag, d_rand, n_drop,
                                                                                   ws=ws), S, n, 5)}
    breakdown["diagheur_path_us"] = {k: v * 1e3 for k, v in heur.items()}

    # three layers of this shape reading one input (query, key, value of an attention block), outside the step:
    # one call per product against one call per layer
    if use_prepare:
        G = 3
        g_off = torch.stack([torch.from_numpy(synth.draw_offsets(D, K, seed=2506 + g)) for g in range(G)]).cuda()
        g_val = torch.stack([d_val] * G).contiguous()
        g_prep = dd.dd_prepare_shared(g_off, g_val, M, N)
        one_prep = [dd.dd_prepare(g_off[g], g_val[g], M, N) for g in range(G)]
        g_Y = [torch.empty((G, T, N), dtype=tdtype, device="cuda") for _ in range(S)]
        g_dX = [torch.empty((G, T, M), dtype=tdtype, device="cuda") for _ in range(S)]

        def per_layer_fwd(s):
            for g in range(G):
                dd.dd_fwd(d_X[s], None, None, N, Y=g_Y[s][g], prepared=one_prep[g])

        def per_layer_bwd_input(s):  # without the two additions that would still have to follow
            for g in range(G):
                dd.dd_bwd_input(g_Y[s][g], None, None, M, dX=g_dX[s][g], prepared=one_prep[g])

        shared = {"dd_prepare_shared": time_loop(torch, lambda s: dd.dd_prepare_shared(g_off, g_val, M, N, prepared=g_prep),
                                                 S, n, 5),
                  "dd_fwd_shared": time_loop(torch, lambda s: dd.dd_fwd_shared(d_X[s], g_prep, Y=g_Y[s]), S, n, 5),
                  "dd_bwd_input_shared": time_loop(torch, lambda s: dd.dd_bwd_input_shared(g_Y[s], g_prep, dX=d_dX[s]),
                                                   S, n, 5),
                  "3 x dd_fwd": time_loop(torch, per_layer_fwd, S, n, 5),
                  "3 x dd_bwd_input (unsummed)": time_loop(torch, per_layer_bwd_input, S, n, 5)}
        breakdown["shared_input_3_sets_us"] = {k: v * 1e3 for k, v in shared.items()}
        del g_Y, g_dX

    if not args.no_dense:
        # dense bf16 GEMMs of the same shape (hipBLASLt / rocBLAS via torch.matmul), same rotation
        Wd = torch.randn((M, N), device="cuda", dtype=tdtype) * 0.02
        dWd = torch.empty((M, N), device="cuda", dtype=tdtype)
        g_fwd = time_loop(torch, lambda s: torch.matmul(d_X[s], Wd, out=d_Y[s]), S, n, 5)
        g_dgrad = time_loop(torch, lambda s: torch.matmul(d_dY[s], Wd.t(), out=d_dX[s]), S, n, 5)
        g_wgrad = time_loop(torch, lambda s: torch.matmul(d_X[s].t(), d_dY[s], out=dWd), S, n, 5)
        breakdown["dense_gemm_us"] = {"fwd": g_fwd * 1e3, "dgrad": g_dgrad * 1e3, "wgrad": g_wgrad * 1e3}
        # per step of training: the operands are built once (with the selection where it is redone every step; the
        # selection itself has no dense counterpart, so only the build is charged here)
        ours_training = per["dd_fwd"] + per["dd_bwd_input"] + per["dd_bwd_weight"] + per.get("dd_prepare", 0.0)
        breakdown["speedup_vs_dense"] = {
            "fwd": g_fwd / alone["dd_fwd"],                   # one self-contained call
            "fwd_prepared": g_fwd / per["dd_fwd"],            # inference: operands built once, weights fixed
            "training": (g_fwd + g_dgrad + g_wgrad) / ours_training}

    out = {
        "metric": "diag-sparse linear fwd+bwd effective TFLOP/s, % roofline, speedup vs dense GEMM",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": layer.dtype, "data": "synthetic",
        "config": {"workload": f"ViT-Base attention projection: {M}->{N}, 90% sparse (K={K} diagonals), "
                               f"tokens={T}, bf16 storage, fp32 accumulate" if args.workload == "vitb_attn_proj"
                   else layer.name,
                   "step": ("dd_select_prepare (dd_select_diagonals and dd_prepare as one call) + dd_fwd + dd_bwd_input + dd_bwd_weight" if use_prepare
                            else "dd_select_diagonals + dd_fwd + dd_bwd_input + dd_bwd_weight"),
                   "offsets": "uniform" if args.offset_bands == 0 else f"{args.offset_bands} runs of adjacent diagonals",
                   "algo": args.algo, "buffer_sets": S, "tokens": T, "in_features": M, "out_features": N, "K": K},
        "roofline": roofline,
        "breakdown": breakdown,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(layer, offsets, values, X, dY, scores)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
