#!/usr/bin/env python3
"""Benchmark of the MXFP4 weight-only-quantised decode linears on one MI355X.

Workload (the second benchmark configuration): the five Llama-7B-shaped decode linears at
M = 1 -- fused QKV [12288x4096], O [4096x4096], gate+up [22016x4096], down [4096x11008] and
the LM head [32000x4096] with the fused argmax -- on seeded synthetic data (Student-t(4)*0.02
weights direct-cast to MXFP4 on the GPU, N(0,1) activations with 8 outlier channels x50).

One step = one pass over the five linears (6 kernel launches).  To keep the 256 MB Infinity
Cache out of the picture every step uses a different one of `--sets` weight sets (>= 2 GB in
total), so each launch streams its weights from HBM.  The timed region replays HIP graphs
(one per weight set) on one stream; inputs are resident in HBM before it starts.

Prints ONE JSON line: value = algorithmic bytes per step / time per step (GB/s), with the
roofline of the dominant kernel and the CPU oracle timed on this machine's host cores beside it.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

METRIC = "MXFP4 WOQ GEMV effective HBM GB/s (% peak) at M=1; us per 7B-shaped decode step"
HBM_PEAK_GBPS = 8000.0


def algorithmic_bytes(m: int, n: int, k: int) -> float:
    """Packed nibbles + scales, read once; activations in; outputs out (BF16)."""
    return n * k * 0.53125 + 2.0 * m * k + 2.0 * m * n


def build_sets(n_sets: int, m: int, dev, keep_bf16: int = 0):
    import torch
    from paper_2503_13565_amd import binding, synth
    shape = synth.LLAMA_7B
    sets = []
    cast_bytes = 0.0
    cast_ms = 0.0
    for layer in range(n_sets):
        lin = {}
        for li, (name, n, k) in enumerate(shape.linears()):
            seed = synth.tensor_seed(0, layer, li)
            w = synth.weights_student_t(n, k, seed=seed, device=dev)
            x = synth.activations_outlier_channels(m, k, seed=seed + 8, device=dev)
            q = torch.empty((n, k // 2), dtype=torch.uint8, device=dev)      # allocated outside the timed span
            s = torch.empty((n, k // 32), dtype=torch.uint8, device=dev)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            binding.mxfp4_direct_cast(w, q=q, s=s)
            e1.record()
            torch.cuda.synchronize()
            if layer > 0:                              # the first layer's casts pay one-time costs
                cast_ms += e0.elapsed_time(e1)
                cast_bytes += n * k * 2.53125
            lin[name] = dict(n=n, k=k, q=q, s=s, x=x, w=w if layer < keep_bf16 else None,
                             y=torch.empty((m, n), dtype=torch.bfloat16, device=dev))
            del w
        lin["lm_head"]["idx"] = torch.empty((m,), dtype=torch.int32, device=dev)
        lin["lm_head"]["val"] = torch.empty((m,), dtype=torch.float32, device=dev)
        sets.append(lin)
    # Where BF16 weights were kept: the casts of those sets again, back to back between two events
    # (same inputs, same outputs), so that the figure is the kernels' and not one host call's latency.
    kept = [t for lin in sets for t in lin.values() if isinstance(t, dict) and t.get("w") is not None]
    if kept:
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for t in kept:
            binding.mxfp4_direct_cast(t["w"], q=t["q"], s=t["s"])
        e1.record()
        torch.cuda.synchronize()
        return sets, sum(t["n"] * t["k"] for t in kept) * 2.53125 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    return sets, (cast_bytes / (cast_ms * 1e-3) / 1e9 if cast_ms > 0 else None)


def run_step(lin, ws):
    from paper_2503_13565_amd import binding
    for name in ("qkv", "o", "gate_up", "down"):
        t = lin[name]
        binding.mxfp4_woq_gemm(t["x"], t["q"], t["s"], y=t["y"])
    t = lin["lm_head"]
    binding.mxfp4_woq_gemm_argmax(t["x"], t["q"], t["s"], workspace=ws, out=(t["idx"], t["val"]))


def run_step_bf16(lin, ws):
    """The same step on the unquantised BF16 weights (what the MXFP4 step is a speed-up over)."""
    from paper_2503_13565_amd import binding
    for name in ("qkv", "o", "gate_up", "down"):
        t = lin[name]
        binding.mxfp4_bf16_gemm(t["x"], t["w"], y=t["y"])
    t = lin["lm_head"]
    binding.mxfp4_bf16_gemm_argmax(t["x"], t["w"], workspace=ws, out=(t["idx"], t["val"]))


def run_verify5_bf16(lin, ws):
    """The target's verification pass over N + 1 = 5 rows on the unquantised weights (section 3.1)."""
    from paper_2503_13565_amd import binding
    for name in ("qkv", "o", "gate_up", "down"):
        t = lin[name]
        binding.mxfp4_bf16_gemm(t["x5"], t["w"], y=t["y5"])
    t = lin["lm_head"]
    binding.mxfp4_bf16_gemm_argmax(t["x5"], t["w"], workspace=ws, out=(t["idx5"], t["val5"]))


def run_step_e4m3(lin, ws):
    """The same step on an 8-bit draft (E4M3 elements with block scales)."""
    from paper_2503_13565_amd import binding
    for name in ("qkv", "o", "gate_up", "down"):
        t = lin[name]
        binding.mxfp4_e4m3_woq_gemm(t["x"], t["q8"], t["s8"], y=t["y"])
    t = lin["lm_head"]
    binding.mxfp4_e4m3_woq_gemm_argmax(t["x"], t["q8"], t["s8"], workspace=ws, out=(t["idx"], t["val"]))


def run_step_e2m3(lin, ws):
    """The same step on a 6-bit draft (E2M3 elements with block scales)."""
    from paper_2503_13565_amd import binding
    for name in ("qkv", "o", "gate_up", "down"):
        t = lin[name]
        binding.mxfp4_e2m3_woq_gemm(t["x"], t["q6"], t["s6"], y=t["y"])
    t = lin["lm_head"]
    binding.mxfp4_e2m3_woq_gemm_argmax(t["x"], t["q6"], t["s6"], workspace=ws, out=(t["idx"], t["val"]))


def run_layer_plain(lin, ws):
    from paper_2503_13565_amd import binding
    for name in ("qkv", "o", "gate_up", "down"):
        t = lin[name]
        binding.mxfp4_woq_gemm(t["x"], t["q"], t["s"], y=t["y"])


def run_layer_fused(lin, ws):
    """The four linears of a decoder layer with what surrounds them fused: the residual add behind
    the o and the down projection (in place), the gate of the MLP behind gate+up (its weight rows
    read as interleaved gate/up pairs: same bytes, same time)."""
    from paper_2503_13565_amd import binding
    t = lin["qkv"]
    binding.mxfp4_woq_gemm(t["x"], t["q"], t["s"], y=t["y"])
    for name in ("o", "down"):
        t = lin[name]
        binding.mxfp4_woq_gemm_fused(t["x"], t["q"], t["s"], residual=t["y"], y=t["y"])
    t = lin["gate_up"]
    binding.mxfp4_woq_gemm_fused(t["x"], t["q"], t["s"], act=binding.ACT_SWIGLU, y=t["h"])


def run_verify8(lin, ws):
    """A verification pass over eight positions on the canonical tensors."""
    from paper_2503_13565_amd import binding
    for name in ("qkv", "o", "gate_up"):
        t = lin[name]
        binding.mxfp4_woq_gemm(t["x8"], t["q"], t["s"], y=t["y8"])


def run_verify8_tiled(lin, ws):
    """The same pass on the tile-major copy of the weights."""
    from paper_2503_13565_amd import binding
    for name in ("qkv", "o", "gate_up"):
        t = lin[name]
        binding.mxfp4_woq_gemm_tiled(t["x8"], t["tw"], y=t["y8"])


DOMINANT = ("qkv", "o", "gate_up", "lm_head")
DOMINANT_KERNEL = "mxfp4::(anonymous namespace)::gemv_reg_kernel<1, 1, 2, 2, 16, false>"


def run_dominant(lin, ws):
    """The four launches of a step that run the dominant kernel instance (every K = 4096 linear)."""
    from paper_2503_13565_amd import binding
    for name in DOMINANT:                               # lm_head: same instance as the fused-argmax call
        t = lin[name]
        binding.mxfp4_woq_gemm(t["x"], t["q"], t["s"], y=t["y"])


def eq1_projection(s_measured: float, verify_cost: float = 1.0):
    """Expected speed-ups of Eq. 1 (arXiv 2503.13565, section 3.2) and of its two-level composition
    (section 3.3) with the draft speed-up S measured here and the acceptance ratios the paper
    reports for its models (sections 4.2, 4.3) as inputs.  N = 4 draft tokens as in the text.
    Eq. 1 prices the verification pass at one target step; `verify_cost` is what it costs here (the
    target's pass over N + 1 rows over its single-row step), and the last figure of each entry uses
    it: (alpha N + 1) / (verify_cost + N / S)."""
    def one(alpha, n, s):
        return (alpha + 1.0 / n) / (1.0 / n + 1.0 / s)

    def two(a_mid, s_mid, a_last, s_last, n=4.0):
        return one(a_mid, n, s_mid * one(a_last, n, s_last / s_mid))
    n = 4.0
    out = {"N": 4, "S_mxfp4_measured": round(s_measured, 3), "S_mxfp4_by_bytes": 3.765,
           "verify_cost_5_rows_over_1": round(verify_cost, 3)}
    for tag, a_q, a_t, s_t in (("llama2_7b_like", 0.712, 0.417, 100.0), ("qwen2.5_7b_like", 0.91, 0.62, 14.0)):
        out[tag] = {
            "alpha_mxfp4_draft": a_q, "alpha_small_draft": a_t, "S_small_draft_assumed": s_t,
            "one_level_mxfp4_draft": round(one(a_q, n, s_measured), 3),
            "one_level_mxfp4_draft_at_S_by_bytes": round(one(a_q, n, 3.765), 3),
            "one_level_small_draft": round(one(a_t, n, s_t), 3),
            "two_level": round(two(a_q, s_measured, a_t, s_t), 3),
            "one_level_mxfp4_draft_with_measured_verify_cost":
                round((a_q * n + 1.0) / (verify_cost + n / s_measured), 3),
        }
    return out


def capture(fn, sets, ws, stream):
    """One HIP graph holding one step per weight set, in order; None if capture is unavailable."""
    import torch
    try:
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            for lin in sets:
                fn(lin, ws)
    except Exception as exc:                            # plain launches still measure the kernels
        print("bench: graph capture failed (%s); timing plain launches" % exc, file=sys.stderr)
        return None
    return g


def runner(graph, fn, sets, ws):
    """run(n): execute n steps, weight sets in rotation -- whole rotations as graph replays, the
    remainder (and everything, without a graph) as plain launches on the current stream."""
    def run(n):
        done = 0
        if graph is not None:
            while n - done >= len(sets):
                graph.replay()
                done += len(sets)
        while done < n:
            fn(sets[done % len(sets)], ws)
            done += 1
    return run


def timed(run, n, stream):
    """Time run(n) on `stream` with HIP events; returns milliseconds in total."""
    import torch
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    with torch.cuda.stream(stream):
        e0.record(stream)
        run(n)
        e1.record(stream)
    torch.cuda.synchronize()
    return e0.elapsed_time(e1)


def cpu_baseline(m: int):
    """The CPU oracle, as it stands, on the same five linears (weight set 0), all host threads."""
    import numpy as np
    import oracle
    from paper_2503_13565_amd import synth
    shape = synth.LLAMA_7B
    threads = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else os.cpu_count()
    threads = max(1, min(threads, oracle.max_threads()))
    t_cast = 0.0
    nbytes = 0.0
    lins = []
    for li, (name, n, k) in enumerate(shape.linears()):
        seed = synth.tensor_seed(0, 0, li)
        w = synth.weights_student_t(n, k, seed=seed)
        x = synth.activations_outlier_channels(m, k, seed=seed + 8)
        wb, xb = synth.to_bits(w), synth.to_bits(x)
        t0 = time.perf_counter()
        q, s = oracle.direct_cast(wb, threads=threads)
        t_cast += time.perf_counter() - t0
        lins.append((name, xb, q, s))
        nbytes += algorithmic_bytes(m, n, k)
    # the whole step, repeated until about ten seconds of it are on the clock (40 times at most)
    t_gemm, reps = 0.0, 0
    while reps < 40 and (t_gemm < 10.0 or reps < 2):
        t1 = time.perf_counter()
        for name, xb, q, s in lins:
            y, _ = oracle.woq_gemm(xb, q, s, threads=threads)
            if name == "lm_head":
                oracle.argmax(y)
        t_gemm += time.perf_counter() - t1
        reps += 1
    per_step = t_gemm / reps
    return {
        "value": nbytes / per_step / 1e9, "unit": "GB/s", "cores": threads, "kind": "oracle",
        "sample": "the full step (the five 7B decode linears at M=%d, FP64 product + argmax) %d times, "
                  "%.1f s in all; the oracle's direct cast of the same weights took %.2f s once "
                  "(not in value)" % (m, reps, t_gemm, t_cast),
        "seconds_per_step": per_step,
    }


def run_stack_bf16(args) -> int:
    """The same stack with unquantised BF16 weights (the target model's step and verification pass;
    arXiv 2503.13565, section 3.2): what the MXFP4 stack's times are compared with."""
    import torch
    from paper_2503_13565_amd import binding, synth
    shape = synth.LLAMA_7B if args.workload == "stack7b" else synth.LLAMA_70B
    layers = args.layers or shape.layers
    m = args.m
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    binding.load()
    ops = []
    for layer in range(layers + 1):
        for li, (name, n, k) in enumerate(shape.linears()):
            if (layer < layers) == (name == "lm_head"):
                continue
            seed = synth.tensor_seed(0, layer, li)
            ops.append(dict(name=name, n=n, k=k, w=synth.weights_student_t(n, k, seed=seed, device=dev),
                            x=synth.activations_outlier_channels(m, k, seed=seed + 8, device=dev),
                            y=torch.empty((m, n), dtype=torch.bfloat16, device=dev)))
    head = ops[-1]
    head["idx"] = torch.empty((m,), dtype=torch.int32, device=dev)
    head["val"] = torch.empty((m,), dtype=torch.float32, device=dev)
    ws = torch.empty((binding.mxfp4_bf16_gemm_argmax_workspace_bytes(m, head["n"], head["k"]),),
                     dtype=torch.uint8, device=dev)

    def step(_lin=None, _ws=None):
        for t in ops[:-1]:
            binding.mxfp4_bf16_gemm(t["x"], t["w"], y=t["y"])
        binding.mxfp4_bf16_gemm_argmax(head["x"], head["w"], workspace=ws, out=(head["idx"], head["val"]))

    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        step()
    torch.cuda.synchronize()
    graph = None if args.no_graph else capture(step, [None], ws, stream)
    run = runner(graph, step, [None], ws)
    steps = max(1, args.steps // 24)
    timed(run, max(1, args.warmup // 12), stream)
    ms_per_step = timed(run, steps, stream) / steps
    step_bytes = sum(2.0 * t["n"] * t["k"] + 2.0 * m * t["k"] + 2.0 * m * t["n"] for t in ops)
    value = step_bytes / (ms_per_step * 1e-3) / 1e9
    print(json.dumps({
        "metric": "BF16-weight linear stack, effective HBM GB/s (the unquantised reference of the MXFP4 stack)",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": steps, "warmup": max(1, args.warmup // 12),
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s with BF16 weights: %d layers x (qkv, o, gate_up, down) + lm_head with argmax, "
                               "M=%d, %.2f GB resident" % (shape.name, layers, m,
                                                           sum(2.0 * t["n"] * t["k"] for t in ops) / 1e9),
                   "M": m, "launch": "hip graph replay" if graph is not None else "stream launches"},
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBPS, 2), "us_per_step": round(ms_per_step * 1e3, 2),
        "bytes_per_step": step_bytes, "roofline": None, "cpu_baseline": None}))
    return 0


def run_stack(args) -> int:
    """Optional workloads: the whole linear-only decode step of a model-shaped weight stack that
    is resident in HBM (the fourth and fifth benchmark configurations).  One step = 4 linears per
    layer + the LM head with argmax, every layer with its own weights (cold by construction)."""
    import torch
    from paper_2503_13565_amd import binding, synth
    shape = synth.LLAMA_7B if args.workload == "stack7b" else synth.LLAMA_70B
    layers = args.layers or shape.layers
    m = args.m
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    binding.load()
    ops = []
    cast_ms = cast_bytes = 0.0
    for layer in range(layers + 1):
        for li, (name, n, k) in enumerate(shape.linears()):
            if (layer < layers) == (name == "lm_head"):
                continue                                 # layers hold 4 linears; the head comes last
            seed = synth.tensor_seed(0, layer, li)
            w = synth.weights_student_t(n, k, seed=seed, device=dev)
            q = torch.empty((n, k // 2), dtype=torch.uint8, device=dev)
            s = torch.empty((n, k // 32), dtype=torch.uint8, device=dev)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            binding.mxfp4_direct_cast(w, q=q, s=s)
            e1.record()
            torch.cuda.synchronize()
            if layer > 0:
                cast_ms += e0.elapsed_time(e1)
                cast_bytes += n * k * 2.53125
            del w
            ops.append(dict(name=name, n=n, k=k, q=q, s=s,
                            x=synth.activations_outlier_channels(m, k, seed=seed + 8, device=dev),
                            y=torch.empty((m, n), dtype=torch.bfloat16, device=dev)))
    # one split-K scratch buffer serves every linear: the calls of a step run one after the other
    sk_bytes = max(binding.mxfp4_woq_gemm_workspace_bytes(m, t["n"], t["k"]) for t in ops[:-1])
    sk = torch.empty((sk_bytes,), dtype=torch.uint8, device=dev) if sk_bytes else None
    n_tiled = 0
    if args.tiled:
        # a pure verifier keeps only the tile-major copy of a linear
        for t in ops[:-1]:
            tw = binding.mxfp4_tile_repack(t["q"], t["s"])
            try:
                binding.mxfp4_woq_gemm_tiled(t["x"], tw, y=t["y"], workspace=sk)
            except binding.Mxfp4Error:
                continue
            t["tw"], t["q"], t["s"] = tw, None, None
            n_tiled += 1
        torch.cuda.synchronize()
    head = ops[-1]
    head["idx"] = torch.empty((m,), dtype=torch.int32, device=dev)
    head["val"] = torch.empty((m,), dtype=torch.float32, device=dev)
    ws = torch.empty((binding.mxfp4_woq_gemm_argmax_workspace_bytes(m, head["n"], head["k"]),),
                     dtype=torch.uint8, device=dev)
    if args.tiled:
        tw = binding.mxfp4_tile_repack(head["q"], head["s"])
        try:
            binding.mxfp4_woq_gemm_tiled_argmax(head["x"], tw, workspace=ws, out=(head["idx"], head["val"]))
            head["tw"], head["q"], head["s"] = tw, None, None
            n_tiled += 1
        except binding.Mxfp4Error:
            pass
        torch.cuda.synchronize()

    def step(_lin=None, _ws=None):
        for t in ops[:-1]:
            if "tw" in t:
                binding.mxfp4_woq_gemm_tiled(t["x"], t["tw"], y=t["y"], workspace=sk)
            else:
                binding.mxfp4_woq_gemm(t["x"], t["q"], t["s"], y=t["y"], workspace=sk)
        if "tw" in head:
            binding.mxfp4_woq_gemm_tiled_argmax(head["x"], head["tw"], workspace=ws, out=(head["idx"], head["val"]))
        else:
            binding.mxfp4_woq_gemm_argmax(head["x"], head["q"], head["s"], workspace=ws, out=(head["idx"], head["val"]))

    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        step()
    torch.cuda.synchronize()
    graph = None if args.no_graph else capture(step, [None], ws, stream)
    run = runner(graph, step, [None], ws)
    steps = max(1, args.steps // 24)
    timed(run, max(1, args.warmup // 12), stream)
    graph_ms_per_step = timed(run, steps, stream) / steps
    plain_ms = timed(runner(None, step, [None], ws), max(1, steps // 2), stream) / max(1, steps // 2)
    # the same launches issued by one library call per step (the host loop is the library's)
    def weights_of(t):
        return dict(w=t["tw"]) if "tw" in t else dict(q=t["q"], s=t["s"])

    group = binding.GemmGroup([dict(x=t["x"], y=t["y"], **weights_of(t)) for t in ops[:-1]] +
                              [dict(x=head["x"], argmax=True, out=(head["idx"], head["val"]), **weights_of(head))])

    def step_grouped(_lin=None, _ws=None):
        group.run()

    timed(runner(None, step_grouped, [None], ws), 1, stream)
    grouped_ms = timed(runner(None, step_grouped, [None], ws), steps, stream) / steps
    # the headline is the faster of the two ways to issue the same kernels, named in config.launch
    launch = "hip graph replay" if graph is not None else "stream launches"
    ms_per_step = graph_ms_per_step
    if grouped_ms < graph_ms_per_step:
        launch, ms_per_step = "stream launches from one grouped library call per step", grouped_ms
    step_bytes = sum(algorithmic_bytes(m, t["n"], t["k"]) for t in ops)
    step_weight_bytes = sum(t["n"] * t["k"] * 0.53125 for t in ops)
    value = step_bytes / (ms_per_step * 1e-3) / 1e9
    out = {
        "metric": METRIC, "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": steps,
        "warmup": max(1, args.warmup // 12), "ms_per_step": round(ms_per_step, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: %d layers x (qkv, o, gate_up, down) + lm_head with argmax, M=%d, "
                               "%.2f GB of MXFP4 resident, %d launches per step"
                               % (shape.name, layers, m, step_weight_bytes / 1e9, len(ops) + 1),
                   "M": m, "launch": launch, "linears_on_tile_major_weights": n_tiled},
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "us_per_step": round(ms_per_step * 1e3, 2), "us_per_step_graph_replay": round(graph_ms_per_step * 1e3, 2),
        "us_per_step_plain_launches": round(plain_ms * 1e3, 2),
        "us_per_step_grouped_call": round(grouped_ms * 1e3, 2),
        "bytes_per_step": step_bytes,
        "tflops": round(2.0 * m * sum(t["n"] * t["k"] for t in ops) / (ms_per_step * 1e-3) / 1e12, 3),
        "direct_cast_GBps": round(cast_bytes / (cast_ms * 1e-3) / 1e9, 1) if cast_ms > 0 else None,
        "roofline": {"bound": "hbm", "achieved": round(value, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(value / HBM_PEAK_GBPS, 4), "traffic": None,
                     "kernel": "whole step (all launches, gaps included)"},
        "cpu_baseline": None,
    }
    print(json.dumps(out))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=240)
    ap.add_argument("--warmup", type=int, default=24)
    ap.add_argument("--sets", type=int, default=12, help="distinct weight sets rotated over (12 = 2.1 GB)")
    ap.add_argument("--m", type=int, default=1, help="activation rows (1 = decode)")
    ap.add_argument("--no-graph", action="store_true", help="time plain stream launches instead of graph replays")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--no-bf16", action="store_true", help="skip the BF16-weight comparison step")
    ap.add_argument("--workload", default="decode7b", choices=["decode7b", "stack7b", "stack70b"],
                    help="decode7b (default): the five 7B decode linears over rotating weight sets; "
                         "stack7b / stack70b: the whole linear-only decode step of a resident weight stack")
    ap.add_argument("--layers", type=int, default=0, help="stack workloads: layers to build (0 = the model's)")
    ap.add_argument("--weights", default="mxfp4", choices=["mxfp4", "bf16"],
                    help="stack workloads: bf16 runs the unquantised reference stack")
    ap.add_argument("--tiled", action="store_true",
                    help="stack workloads: verification passes on the tile-major copy of the weights where it can run")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one MI355X: this build has no multi-GPU path (the linears shard by "
              "output rows without collectives). Run with --gpus 1.", file=sys.stderr)
        return 2

    import torch
    from paper_2503_13565_amd import binding, synth
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    binding.load()
    if args.workload != "decode7b":
        return run_stack_bf16(args) if args.weights == "bf16" else run_stack(args)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    m = args.m
    n_bf16 = 0 if args.no_bf16 else min(args.sets, 4)    # 4 x 0.67 GB of BF16 weights: cold too
    sets, cast_gbps = build_sets(args.sets, m, dev, keep_bf16=n_bf16)
    ws = torch.empty((binding.mxfp4_woq_gemm_argmax_workspace_bytes(m, 32000, 4096),), dtype=torch.uint8, device=dev)
    stream = torch.cuda.Stream()
    shape = synth.LLAMA_7B
    step_bytes = sum(algorithmic_bytes(m, n, k) for _, n, k in shape.linears())
    weight_bytes = sum(n * k * 0.53125 for _, n, k in shape.linears())

    # warm every kernel instance outside any capture (first launches set function attributes)
    with torch.cuda.stream(stream):
        for lin in sets:
            run_step(lin, ws)
    torch.cuda.synchronize()

    graph = None if args.no_graph else capture(run_step, sets, ws, stream)
    run_steps = runner(graph, run_step, sets, ws)
    timed(run_steps, args.warmup, stream)
    ms = timed(run_steps, args.steps, stream)
    graph_ms_per_step = ms / args.steps

    # the same steps as plain stream launches (host launch cost included), for the record
    n_plain = max(len(sets), args.steps // 4)
    plain_ms = timed(runner(None, run_step, sets, ws), n_plain, stream) / n_plain
    # and issued by one library call per step (mxfp4_woq_gemm_grouped: the host loop is the library's)
    for lin in sets:
        head = lin["lm_head"]
        lin["group"] = binding.GemmGroup(
            [dict(x=lin[name]["x"], q=lin[name]["q"], s=lin[name]["s"], y=lin[name]["y"])
             for name in ("qkv", "o", "gate_up", "down")] +
            [dict(x=head["x"], q=head["q"], s=head["s"], argmax=True, out=(head["idx"], head["val"]))])
    run_grouped = runner(None, lambda lin, _ws: lin["group"].run(), sets, ws)
    timed(run_grouped, args.warmup, stream)
    grouped_ms = timed(run_grouped, args.steps, stream) / args.steps
    for lin in sets:
        del lin["group"]
    # For the record, not the headline: the same five products declared independent of each other
    # (MXFP4_DESC_INDEPENDENT; the synthetic inputs are, a model's chain of layers is not).  All
    # five then share one launch and the pick's second stage follows: two launches per step
    # instead of six.
    for lin in sets:
        head = lin["lm_head"]
        lin["group"] = binding.GemmGroup(
            [dict(x=lin[name]["x"], q=lin[name]["q"], s=lin[name]["s"], y=lin[name]["y"], independent=True)
             for name in ("down", "qkv", "o", "gate_up")] +
            [dict(x=head["x"], q=head["q"], s=head["s"], argmax=True, out=(head["idx"], head["val"]),
                  independent=True)])
    run_indep = runner(None, lambda lin, _ws: lin["group"].run(), sets, ws)
    timed(run_indep, args.warmup, stream)
    indep_ms = timed(run_indep, args.steps, stream) / args.steps
    for lin in sets:
        del lin["group"]
    # Two ways to issue the same kernels, each timed over exactly `steps` steps: a replayed HIP
    # graph and the library's grouped call on the stream.  The headline is the faster one (named in
    # config.launch); both stay in the record.
    launch = "hip graph replay" if graph is not None else "stream launches"
    ms_per_step = graph_ms_per_step
    run_best = run_steps
    if grouped_ms < graph_ms_per_step:
        launch, ms_per_step = "stream launches from one grouped library call per step", grouped_ms
        for lin in sets:
            head = lin["lm_head"]
            lin["group"] = binding.GemmGroup(
                [dict(x=lin[name]["x"], q=lin[name]["q"], s=lin[name]["s"], y=lin[name]["y"])
                 for name in ("qkv", "o", "gate_up", "down")] +
                [dict(x=head["x"], q=head["q"], s=head["s"], argmax=True, out=(head["idx"], head["val"]))])
        run_best = runner(None, lambda lin, _ws: lin["group"].run(), sets, ws)
    value = step_bytes / (ms_per_step * 1e-3) / 1e9
    # spread of the headline discipline: the same steps again in ten chunks of one rotation each or more
    chunk = max(len(sets), args.steps // 10 // len(sets) * len(sets))
    chunk_us = sorted(timed(run_best, chunk, stream) / chunk * 1e3 for _ in range(10))
    for lin in sets:
        lin.pop("group", None)

    # dominant kernel: the instance that runs qkv, o, gate+up and the LM head (4 of the 6 launches,
    # 86 % of the bytes); average launch duration from events around graph replays of these four
    # launches only, rotating over the weight sets
    dgraph = None if args.no_graph else capture(run_dominant, sets, ws, stream)
    run_dom = runner(dgraph, run_dominant, sets, ws)
    timed(run_dom, len(sets), stream)
    reps = len(sets) * max(2, args.steps // (2 * len(sets)))
    dom_ms = timed(run_dom, reps, stream) / reps
    # the same four launches from one grouped call per set; the shorter average counts (both bound
    # the kernel's duration from above: the events also see the gaps between launches)
    for lin in sets:
        lin["group"] = binding.GemmGroup([dict(x=lin[name]["x"], q=lin[name]["q"], s=lin[name]["s"], y=lin[name]["y"])
                                          for name in DOMINANT])
    run_dom_grouped = runner(None, lambda lin, _ws: lin["group"].run(), sets, ws)
    timed(run_dom_grouped, len(sets), stream)
    dom_ms = min(dom_ms, timed(run_dom_grouped, reps, stream) / reps)
    for lin in sets:
        del lin["group"]
    dom_launch_us = dom_ms * 1e3 / len(DOMINANT)
    dom_bytes = sum(algorithmic_bytes(m, n, k) for name, n, k in shape.linears() if name in DOMINANT) / len(DOMINANT)
    achieved = dom_bytes / (dom_launch_us * 1e-6) / 1e9

    # the unquantised step: same linears, BF16 weights (2 bytes per weight), same launch discipline
    bf16_us = None
    if n_bf16:
        bsets = sets[:n_bf16]
        with torch.cuda.stream(stream):
            for lin in bsets:
                run_step_bf16(lin, ws)
        torch.cuda.synchronize()
        bgraph = None if args.no_graph else capture(run_step_bf16, bsets, ws, stream)
        run_b = runner(bgraph, run_step_bf16, bsets, ws)
        timed(run_b, n_bf16, stream)
        nb = n_bf16 * max(2, args.steps // (4 * n_bf16))
        bf16_us = timed(run_b, nb, stream) / nb * 1e3
        # the target's verification pass over N + 1 = 5 rows on the same BF16 weights
        for lin in bsets:
            for t in lin.values():
                t["x5"] = synth.activations_outlier_channels(5, t["k"], seed=t["n"] + 5, device=dev)
                t["y5"] = torch.empty((5, t["n"]), dtype=torch.bfloat16, device=dev)
            lin["lm_head"]["idx5"] = torch.empty((5,), dtype=torch.int32, device=dev)
            lin["lm_head"]["val5"] = torch.empty((5,), dtype=torch.float32, device=dev)
        ws5 = torch.empty((binding.mxfp4_bf16_gemm_argmax_workspace_bytes(5, 32000, 4096),), dtype=torch.uint8,
                          device=dev)
        with torch.cuda.stream(stream):
            for lin in bsets:
                run_verify5_bf16(lin, ws5)
        torch.cuda.synchronize()
        vgraph = None if args.no_graph else capture(run_verify5_bf16, bsets, ws5, stream)
        run_v = runner(vgraph, run_verify5_bf16, bsets, ws5)
        timed(run_v, n_bf16, stream)
        bf16_verify5_us = timed(run_v, nb, stream) / nb * 1e3
        # further variants on the same four weight sets, each timed like the step above: an 8-bit
        # draft, the decoder layer with fused epilogues, and an 8-row verification pass on the
        # canonical and on the tile-major weights
        def leg(fn):
            with torch.cuda.stream(stream):
                for lin in bsets:
                    fn(lin, ws)
            torch.cuda.synchronize()
            g = None if args.no_graph else capture(fn, bsets, ws, stream)
            r = runner(g, fn, bsets, ws)
            timed(r, n_bf16, stream)
            return timed(r, nb, stream) / nb * 1e3
        for lin in bsets:
            for name, t in lin.items():
                t["q8"], t["s8"] = binding.mxfp4_e4m3_direct_cast(t["w"])
                t["q6"], t["s6"] = binding.mxfp4_e2m3_direct_cast(t["w"])
                t["w"] = None
                if name in ("qkv", "o", "gate_up"):
                    t["x8"] = synth.activations_outlier_channels(8, t["k"], seed=t["n"], device=dev)
                    t["y8"] = torch.empty((8, t["n"]), dtype=torch.bfloat16, device=dev)
                    t["tw"] = binding.mxfp4_tile_repack(t["q"], t["s"])
            lin["gate_up"]["h"] = torch.empty((m, lin["gate_up"]["n"] // 2), dtype=torch.bfloat16, device=dev)
        variants = {
            "e4m3_weights_us_per_step": round(leg(run_step_e4m3), 2),
            "e2m3_weights_us_per_step": round(leg(run_step_e2m3), 2),
            "layer_4_linears_us": round(leg(run_layer_plain), 2),
            "layer_4_linears_fused_epilogues_us": round(leg(run_layer_fused), 2),
            "verify_m8_qkv_o_gateup_us": round(leg(run_verify8), 2),
            "verify_m8_qkv_o_gateup_tile_major_us": round(leg(run_verify8_tiled), 2),
        }
        for lin in bsets:
            for t in lin.values():
                for key in ("q8", "s8", "q6", "s6", "x8", "y8", "x5", "y5", "tw", "h"):
                    t.pop(key, None)

    # what a plain 128-bit read stream gets on this device, over 4 GiB (context for frac)
    buf = torch.empty(4 << 30, dtype=torch.uint8, device=dev)
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    def run_read(n):
        for _ in range(n):
            binding.mxfp4_diag_stream_read(buf, sink)
    timed(run_read, 1, stream)
    read_ms = timed(run_read, 5, stream) / 5
    stream_read_gbps = buf.numel() / (read_ms * 1e-3) / 1e9
    # one plain copy of known size (1 GiB read + 1 GiB written): the reference against which
    # the profiler's FETCH_SIZE / WRITE_SIZE counters are scaled
    half = buf.numel() // 4
    with torch.cuda.stream(stream):
        binding.mxfp4_diag_stream_copy(buf[:half], buf[2 * half:3 * half])
    torch.cuda.synchronize()
    del buf

    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.txt")
    if os.path.exists(tpath):
        for line in open(tpath):
            if line.startswith("gemv_m1_dominant_bytes_per_launch"):
                try:
                    traffic = int(line.split("=")[1])
                except ValueError:
                    traffic = None

    out = {
        "metric": METRIC, "value": round(value, 1), "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "configs[1]: Llama-7B-shaped decode linears at M=%d "
                               "(qkv 12288x4096, o 4096x4096, gate_up 22016x4096, down 4096x11008, "
                               "lm_head 32000x4096 + argmax), %d weight sets rotated (%.2f GB)"
                               % (m, len(sets), len(sets) * weight_bytes / 1e9),
                   "M": m, "launch": launch},
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "us_per_step": round(ms_per_step * 1e3, 2),
        "us_per_step_graph_replay": round(graph_ms_per_step * 1e3, 2),
        "us_per_step_min_median_max_of_10_chunks": [round(chunk_us[0], 2), round((chunk_us[4] + chunk_us[5]) / 2, 2),
                                                    round(chunk_us[-1], 2)],
        "us_per_step_plain_launches": round(plain_ms * 1e3, 2),
        "us_per_step_grouped_call": round(grouped_ms * 1e3, 2),
        "independent_products_merged_launch": {
            "us_per_step": round(indep_ms * 1e3, 2),
            "GBps": round(step_bytes / (indep_ms * 1e-3) / 1e9, 1),
            "frac_of_8TBps": round(step_bytes / (indep_ms * 1e-3) / 1e9 / 8000.0, 4),
            "launches_per_step": 2,
            "note": "not the headline: valid only because the benchmark's five inputs do not depend on each other",
        },
        "bytes_per_step": step_bytes,
        "tflops": round(2.0 * m * sum(n * k for _, n, k in shape.linears()) / (ms_per_step * 1e-3) / 1e12, 3),
        "bf16_weights_us_per_step": None if bf16_us is None else round(bf16_us, 2),
        "speedup_over_bf16_weights": None if bf16_us is None else round(bf16_us / (graph_ms_per_step * 1e3), 3),
        "stream_read_GBps": round(stream_read_gbps, 1),
        "direct_cast_GBps": None if cast_gbps is None else round(cast_gbps, 1),
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                     "kernel": DOMINANT_KERNEL + " (qkv, o, gate_up and lm_head launches)",
                     "bytes_per_launch": dom_bytes, "us_per_launch": round(dom_launch_us, 3)},
    }
    if bf16_us is not None:
        out["eq1_projection"] = eq1_projection(bf16_us / (graph_ms_per_step * 1e3), bf16_verify5_us / bf16_us)
        out["bf16_weights_verify_5_rows_us"] = round(bf16_verify5_us, 2)
        out["variants"] = variants
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(m)
        for key in ("value", "seconds_per_step"):
            out["cpu_baseline"][key] = round(out["cpu_baseline"][key], 4)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
