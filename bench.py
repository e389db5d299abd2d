#!/usr/bin/env python3
"""Benchmark of the MXFP4 weight-only-quantised linear layer on one MI355X.

Headline workload (the second benchmark configuration): the five Llama-7B-shaped decode linears at
M = 1 -- fused QKV [12288x4096], O [4096x4096], gate+up [22016x4096], down [4096x11008] and the LM
head [32000x4096] with the fused argmax -- on seeded synthetic data (Student-t(4)*0.02 weights
direct-cast to MXFP4 on the GPU, N(0,1) activations with 8 outlier channels x50).  One step = one
pass over the five.  Every step uses a different one of `--sets` weight sets (2.1 GB in all), so
nothing is served from the 256 MB Infinity Cache; inputs are resident in HBM before the timed
region.  The same K steps are timed under each launch discipline, each one alone and for exactly K
steps: replays of a HIP graph that holds one rotation of the weight sets, one grouped library call
per step, one chained (persistent) launch per step.  The fastest is the headline; all stay in the line.

Beside it, in the same JSON line: `roofline` (the dominant kernel instance) and `roofline_per_linear`
(every launch of the step), `configs` (the other four benchmark configurations, each as microseconds,
GB/s of algorithmic bytes and % of 8 TB/s), `cpu_baseline` (the CPU oracle on this machine's host cores).
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
DTYPE = "bf16 x mxfp4 (e2m1 + e8m0 per 32) -> f32 accumulate, bf16 out"
STEP_LINEARS = ("qkv", "o", "gate_up", "down")
DOMINANT = ("qkv", "gate_up", "lm_head")      # two workgroups of 8 waves per unit; the o projection (16 rows per unit) runs the 12-wave instance
DOMINANT_KERNEL = "mxfp4::(anonymous namespace)::gemv_reg_kernel<1, 1, 2, 2, 8, false>"


def algorithmic_bytes(m: int, n: int, k: int) -> float:
    """Packed nibbles + scales, read once; activations in; outputs out (BF16)."""
    return n * k * 0.53125 + 2.0 * m * k + 2.0 * m * n


def rate(nbytes: float, us: float) -> dict:
    gbps = nbytes / (us * 1e-6) / 1e9
    return {"us": round(us, 2), "GBps": round(gbps, 1), "pct_of_8TBps": round(100.0 * gbps / HBM_PEAK_GBPS, 2)}


# ---- timing ---------------------------------------------------------------------------------------

class Clock:
    """HIP events on the stream that the work is launched on."""

    def __init__(self, stream):
        self.stream = stream

    def ms(self, fn):
        import torch
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        with torch.cuda.stream(self.stream):
            e0.record(self.stream)
            fn()
            e1.record(self.stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1)

    def capture(self, fn):
        """One HIP graph of fn() (which has run once on this stream already)."""
        import torch
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=self.stream):
            fn()
        return g

    def us_per_call(self, calls, n, warmup):
        """calls: list of zero-argument callables taken in rotation; n timed calls after `warmup`
        untimed ones of the same kind, all in one timed region."""
        def run(count):
            for i in range(count):
                calls[i % len(calls)]()
        if warmup:
            self.ms(lambda: run(warmup))
        return self.ms(lambda: run(n)) * 1e3 / n

    def us_per_call_graphs(self, fns, n, warmup):
        """The same as HIP graph replays, exactly n calls: one graph holds the whole rotation (all
        callables in order), replayed n // len(fns) times, and a second graph the n % len(fns)
        calls that remain.  (A graph per callable would be bound by the host's cost per replay,
        about 15 us, which is more than most of these kernels take.)"""
        import torch
        with torch.cuda.stream(self.stream):
            for f in fns:
                f()
        torch.cuda.synchronize()

        def many(count):
            def run():
                for f in fns[:count]:
                    f()
            return run
        full = self.capture(many(len(fns)))
        rem = self.capture(many(n % len(fns))) if n % len(fns) else None

        def run_n():
            for _ in range(n // len(fns)):
                full.replay()
            if rem is not None:
                rem.replay()
        for _ in range((warmup + len(fns) - 1) // len(fns)):
            self.ms(full.replay)
        return self.ms(run_n) * 1e3 / n, (full, rem)


# ---- tensors --------------------------------------------------------------------------------------

_CAST_BLOCKER = None


def cast_linears(specs, dev, cast_acc, keep_w=False):
    """Student-t weights of some linears [(n, k, seed)], generated on the device, then direct-cast
    back to back between two events (outputs allocated outside the timed span)."""
    import torch
    from paper_2503_13565_amd import binding, synth
    ws = [synth.weights_student_t(n, k, seed=seed, device=dev) for n, k, seed in specs]
    outs = [(torch.empty((n, k // 2), dtype=torch.uint8, device=dev), torch.empty((n, k // 32), dtype=torch.uint8, device=dev))
            for n, k, _ in specs]
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    # a fill kernel ahead of the first event: the host enqueues the event and the casts while it runs, so
    # the span holds the casts back to back and not the host's launch latency after the synchronize
    global _CAST_BLOCKER
    if _CAST_BLOCKER is None or _CAST_BLOCKER.device != torch.device(dev):
        _CAST_BLOCKER = torch.empty((64 << 20,), dtype=torch.uint8, device=dev)
    _CAST_BLOCKER.fill_(0)
    e0.record()
    for w, (q, s) in zip(ws, outs):
        binding.mxfp4_direct_cast(w, q=q, s=s)
    e1.record()
    torch.cuda.synchronize()
    if cast_acc is not None:
        cast_acc["ms"] += e0.elapsed_time(e1)
        cast_acc["bytes"] += sum(n * k for n, k, _ in specs) * 2.53125
        cast_acc["weights"] += sum(n * k for n, k, _ in specs)
        cast_acc["calls"] += len(specs)
        cast_acc["spans"] += 1
    return [dict(n=n, k=k, q=q, s=s, w=w if keep_w else None) for (n, k, _), w, (q, s) in zip(specs, ws, outs)]


def build_sets(n_sets, m, dev, keep_bf16):
    import torch
    from paper_2503_13565_amd import synth
    shape = synth.LLAMA_7B
    sets = []
    for layer in range(n_sets):
        lin = {}
        specs = [(n, k, synth.tensor_seed(0, layer, li)) for li, (name, n, k) in enumerate(shape.linears())]
        cast = cast_linears(specs, dev, None, keep_w=layer < keep_bf16)
        for (name, n, k), (_, _, seed), t in zip(shape.linears(), specs, cast):
            t["x"] = synth.activations_outlier_channels(m, k, seed=seed + 8, device=dev)
            t["y"] = torch.empty((m, n), dtype=torch.bfloat16, device=dev)
            lin[name] = t
        lin["lm_head"]["idx"] = torch.empty((m,), dtype=torch.int32, device=dev)
        lin["lm_head"]["val"] = torch.empty((m,), dtype=torch.float32, device=dev)
        sets.append(lin)
    return sets


def build_stack(shape, m_list, dev, layers=0):
    """The resident weight stack of a model shape: layers x (qkv, o, gate_up, down) + lm_head, every
    layer with weights of its own, generated and cast layer by layer (the BF16 originals are never
    held together); activations and outputs for every M of m_list."""
    import torch
    from paper_2503_13565_amd import synth
    layers = layers or shape.layers
    cast_acc = {"ms": 0.0, "bytes": 0.0, "weights": 0, "calls": 0, "spans": 0}
    ops = []
    for layer in range(layers + 1):
        # layers hold 4 linears; the head comes last
        named = [(li, name, n, k) for li, (name, n, k) in enumerate(shape.linears())
                 if (layer < layers) != (name == "lm_head")]
        cast = cast_linears([(n, k, synth.tensor_seed(0, layer, li)) for li, _, n, k in named], dev, cast_acc)
        for (_, name, _, _), t in zip(named, cast):
            t["name"] = name
            ops.append(t)
    # activations: one row set per linear shape and M (values do not matter for the time; shapes do)
    xs = {}
    for m in m_list:
        for li, (name, n, k) in enumerate(shape.linears()):
            xs[(m, name)] = (synth.activations_outlier_channels(m, k, seed=9000 + 16 * m + li, device=dev),
                             torch.empty((m, n), dtype=torch.bfloat16, device=dev))
    return ops, xs, cast_acc


# ---- the headline step under its launch disciplines ------------------------------------------------

def step_calls(lin, ws):
    from paper_2503_13565_amd import binding
    for name in STEP_LINEARS:
        t = lin[name]
        binding.mxfp4_woq_gemm(t["x"], t["q"], t["s"], y=t["y"])
    t = lin["lm_head"]
    binding.mxfp4_woq_gemm_argmax(t["x"], t["q"], t["s"], workspace=ws, out=(t["idx"], t["val"]))


def step_items(lin, **flags):
    head = lin["lm_head"]
    return ([dict(x=lin[name]["x"], q=lin[name]["q"], s=lin[name]["s"], y=lin[name]["y"], **flags)
             for name in STEP_LINEARS] +
            [dict(x=head["x"], q=head["q"], s=head["s"], argmax=True, out=(head["idx"], head["val"]), **flags)])


def step_calls_bf16(lin, ws):
    """The same step on the unquantised BF16 weights (what the MXFP4 step is a speed-up over)."""
    from paper_2503_13565_amd import binding
    for name in STEP_LINEARS:
        t = lin[name]
        binding.mxfp4_bf16_gemm(t["x"], t["w"], y=t["y"])
    t = lin["lm_head"]
    binding.mxfp4_bf16_gemm_argmax(t["x"], t["w"], workspace=ws, out=(t["idx"], t["val"]))


def verify5_calls_bf16(lin, ws):
    """The target's verification pass over N + 1 = 5 rows on the unquantised weights (section 3.1)."""
    from paper_2503_13565_amd import binding
    for name in STEP_LINEARS:
        t = lin[name]
        binding.mxfp4_bf16_gemm(t["x5"], t["w"], y=t["y5"])
    t = lin["lm_head"]
    binding.mxfp4_bf16_gemm_argmax(t["x5"], t["w"], workspace=ws, out=(t["idx5"], t["val5"]))


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


def cpu_baseline(m: int):
    """The CPU oracle, as it stands, on the same five linears (weight set 0), all host threads."""
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
        "value": round(nbytes / per_step / 1e9, 4), "unit": "GB/s", "cores": threads, "kind": "oracle",
        "sample": "the full step (the five 7B decode linears at M=%d, FP64 product + argmax) %d times, "
                  "%.1f s in all; the oracle's direct cast of the same weights took %.2f s once "
                  "(not in value)" % (m, reps, t_gemm, t_cast),
        "seconds_per_step": round(per_step, 4),
    }


# ---- the other configurations ----------------------------------------------------------------------

def config_single_linear(clock, dev, reps):
    """First configuration: W [4096, 4096] Gaussian with x20 outliers, x [1, 4096]; third configuration,
    first half: the same weights under M = 2 .. 32 rows.  128 copies of the packed weights (1.1 GB) are
    rotated so that every launch streams from HBM."""
    import torch
    from paper_2503_13565_amd import binding, synth
    c0 = synth.config0(device=dev)
    q0, s0 = binding.mxfp4_direct_cast(c0["w"])
    copies = [(q0.clone(), s0.clone()) for _ in range(128)]
    n, k = 4096, 4096
    out = {}
    for m in (1, 2, 4, 8, 16, 32):
        x = c0["x"] if m == 1 else synth.activations_gaussian(m, k, seed=300 + m, device=dev)
        y = torch.empty((m, n), dtype=torch.bfloat16, device=dev)
        fns = [(lambda q=q, s=s: binding.mxfp4_woq_gemm(x, q, s, y=y)) for q, s in copies]
        us, graphs = clock.us_per_call_graphs(fns, reps, len(fns))
        out["M=%d" % m] = rate(algorithmic_bytes(m, n, k), us)
        del graphs
    return out


def config_verify_sweep_lm_head(clock, sets, dev, reps):
    """Third configuration, second half: the LM head [32000 x 4096] with the fused argmax under
    M = k + 1 rows for k = 1, 3, 7, 15, 31 draft tokens, the weight sets of the headline in rotation."""
    import torch
    from paper_2503_13565_amd import binding, synth
    n, k = 32000, 4096
    out = {}
    for m in (2, 4, 8, 16, 32):
        x = synth.activations_outlier_channels(m, k, seed=400 + m, device=dev)
        idx = torch.empty((m,), dtype=torch.int32, device=dev)
        val = torch.empty((m,), dtype=torch.float32, device=dev)
        ws = torch.empty((binding.mxfp4_woq_gemm_argmax_workspace_bytes(m, n, k),), dtype=torch.uint8, device=dev)
        fns = [(lambda t=lin["lm_head"]: binding.mxfp4_woq_gemm_argmax(x, t["q"], t["s"], workspace=ws, out=(idx, val)))
               for lin in sets]
        us, graphs = clock.us_per_call_graphs(fns, reps, len(fns))
        out["M=%d" % m] = rate(algorithmic_bytes(m, n, k), us)
        del graphs
    return out


def stack_step_times(clock, ops, xs, m, reps, with_chain, tiled=False):
    """One linear-only decode step over a resident stack at M rows: a graph replay of all launches,
    one grouped library call, and (M = 1) chained persistent launches.  tiled: every product on the
    tile-major copy of its weights (ops then carry `tw`)."""
    import torch
    from paper_2503_13565_amd import binding
    dev = xs[(m, "lm_head")][0].device
    head = ops[-1]
    idx = torch.empty((m,), dtype=torch.int32, device=dev)
    val = torch.empty((m,), dtype=torch.float32, device=dev)
    sk_bytes = max(binding.mxfp4_woq_gemm_workspace_bytes(m, t["n"], t["k"]) for t in ops[:-1])
    sk = torch.empty((sk_bytes,), dtype=torch.uint8, device=dev) if sk_bytes else None
    ws = torch.empty((binding.mxfp4_woq_gemm_argmax_workspace_bytes(m, head["n"], head["k"]),),
                     dtype=torch.uint8, device=dev)

    def step():
        for t in ops[:-1]:
            x, y = xs[(m, t["name"])]
            if tiled:
                binding.mxfp4_woq_gemm_tiled(x, t["tw"], y=y, workspace=sk)
            else:
                binding.mxfp4_woq_gemm(x, t["q"], t["s"], y=y, workspace=sk)
        if tiled:
            binding.mxfp4_woq_gemm_tiled_argmax(xs[(m, "lm_head")][0], head["tw"], workspace=ws, out=(idx, val))
        else:
            binding.mxfp4_woq_gemm_argmax(xs[(m, "lm_head")][0], head["q"], head["s"], workspace=ws, out=(idx, val))

    def weights_of(t):
        return dict(w=t["tw"]) if tiled else dict(q=t["q"], s=t["s"])
    items = [dict(x=xs[(m, t["name"])][0], y=xs[(m, t["name"])][1], **weights_of(t)) for t in ops[:-1]]
    items.append(dict(x=xs[(m, "lm_head")][0], argmax=True, out=(idx, val), **weights_of(head)))
    nbytes = sum(algorithmic_bytes(m, t["n"], t["k"]) for t in ops)
    res = {}
    us, graphs = clock.us_per_call_graphs([step], reps, 1)
    res["graph_replay"] = rate(nbytes, us)
    del graphs
    group = binding.GemmGroup(items)
    res["grouped_call"] = rate(nbytes, clock.us_per_call([group.run], reps, 1))
    if with_chain and m == 1 and not tiled:
        chain = binding.GemmGroup(items, chained=True, mode=binding.CHAIN_PERSISTENT)
        res["chained_persistent_launches"] = rate(nbytes, clock.us_per_call([chain.run], reps, 1))
        if chain.chain_status() != 0:
            res["chained_persistent_launches"] = {"error": "a barrier wait was given up (status %#x)" % chain.chain_status()}
    best = min((v for v in res.values() if "us" in v), key=lambda v: v["us"])
    res["best"] = dict(best, launches_per_step=len(ops) + 1, bytes_per_step=nbytes,
                       tflops=round(2.0 * m * sum(t["n"] * t["k"] for t in ops) / (best["us"] * 1e-6) / 1e12, 2))
    return res


def config_stack(clock, shape, m_list, reps, dev, with_chain=True, layers=0, tiled=False, tiled_m=()):
    """tiled: the stack only as tile-major copies (a pure verifier); tiled_m: rows for which the step
    is timed on the tile-major copy too, beside the canonical tensors (both copies resident)."""
    from paper_2503_13565_amd import binding
    ops, xs, cast_acc = build_stack(shape, m_list, dev, layers)
    out = {"weights_GB": round(sum(t["n"] * t["k"] * 0.53125 for t in ops) / 1e9, 3),
           "layers": (len(ops) - 1) // 4}
    if tiled or tiled_m:
        for t in ops:
            t["tw"] = binding.mxfp4_tile_repack(t["q"], t["s"])
            if tiled:
                t["q"] = t["s"] = None
    for m in m_list:
        if not tiled:
            out["M=%d" % m] = stack_step_times(clock, ops, xs, m, reps, with_chain)
        if tiled or m in tiled_m:
            out["M=%d on the tile-major copy" % m] = stack_step_times(clock, ops, xs, m, reps, False, tiled=True)
    gbps = cast_acc["bytes"] / (cast_acc["ms"] * 1e-3) / 1e9
    out["direct_cast_all_weights"] = {
        "weights": cast_acc["weights"], "ms": round(cast_acc["ms"], 3), "GBps_moved": round(gbps, 1),
        "pct_of_8TBps": round(100.0 * gbps / HBM_PEAK_GBPS, 2), "calls": cast_acc["calls"],
        "note": "%d cast launches in %d timed spans (a layer's four casts back to back between two events, a fill kernel ahead of the first so that the queue is fed); "
                "2.53125 bytes moved per weight" % (cast_acc["calls"], cast_acc["spans"])}
    return out


# ---- stand-alone stack workloads -------------------------------------------------------------------

def run_stack_only(args) -> int:
    import torch
    from paper_2503_13565_amd import binding, synth
    shape = synth.LLAMA_7B if args.workload == "stack7b" else synth.LLAMA_70B
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    binding.load()
    clock = Clock(torch.cuda.Stream())
    reps = max(2, args.steps // 24)
    if args.weights == "bf16":
        return run_stack_bf16(args, clock, shape, dev, reps)
    res = config_stack(clock, shape, [args.m], reps, dev, layers=args.layers, tiled=args.tiled)
    best = res["M=%d on the tile-major copy" % args.m if args.tiled else "M=%d" % args.m]["best"]
    print(json.dumps({
        "metric": METRIC, "value": best["GBps"], "unit": "GB/s", "n_gpus": 1, "steps": reps, "warmup": 1,
        "ms_per_step": round(best["us"] * 1e-3, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": DTYPE, "data": "synthetic",
        "config": {"workload": "%s: %d layers x (qkv, o, gate_up, down) + lm_head with argmax, M=%d, %.2f GB of "
                               "MXFP4 resident" % (shape.name, res["layers"], args.m, res["weights_GB"]), "M": args.m},
        "stack": res, "roofline": None, "cpu_baseline": None}))
    return 0


def run_stack_bf16(args, clock, shape, dev, reps) -> int:
    """The same stack with unquantised BF16 weights (the target model's step and verification pass;
    arXiv 2503.13565, section 3.2): what the MXFP4 stack's times are compared with."""
    import torch
    from paper_2503_13565_amd import binding, synth
    layers = args.layers or shape.layers
    m = args.m
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

    def step():
        for t in ops[:-1]:
            binding.mxfp4_bf16_gemm(t["x"], t["w"], y=t["y"])
        binding.mxfp4_bf16_gemm_argmax(head["x"], head["w"], workspace=ws, out=(head["idx"], head["val"]))

    us, _ = clock.us_per_call_graphs([step], reps, 1)
    step_bytes = sum(2.0 * t["n"] * t["k"] + 2.0 * m * t["k"] + 2.0 * m * t["n"] for t in ops)
    r = rate(step_bytes, us)
    print(json.dumps({
        "metric": "BF16-weight linear stack, effective HBM GB/s (the unquantised reference of the MXFP4 stack)",
        "value": r["GBps"], "unit": "GB/s", "n_gpus": 1, "steps": reps, "warmup": 1,
        "ms_per_step": round(us * 1e-3, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 x bf16 -> f32 accumulate", "data": "synthetic",
        "config": {"workload": "%s with BF16 weights: %d layers x (qkv, o, gate_up, down) + lm_head with argmax, "
                               "M=%d, %.2f GB resident" % (shape.name, layers, m,
                                                           sum(2.0 * t["n"] * t["k"] for t in ops) / 1e9),
                   "M": m, "launch": "hip graph replay"},
        "pct_of_hbm_peak": r["pct_of_8TBps"], "us_per_step": r["us"], "bytes_per_step": step_bytes,
        "roofline": None, "cpu_baseline": None}))
    return 0


# ---- main -------------------------------------------------------------------------------------------

def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=240)
    ap.add_argument("--warmup", type=int, default=24)
    ap.add_argument("--sets", type=int, default=12, help="distinct weight sets rotated over (12 = 2.1 GB)")
    ap.add_argument("--m", type=int, default=1, help="activation rows (1 = decode)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--no-bf16", action="store_true", help="skip the BF16-weight comparison step and the variants")
    ap.add_argument("--no-configs", action="store_true", help="skip the block of the other four configurations")
    ap.add_argument("--no-70b", action="store_true", help="skip the fifth configuration (36.9 GB stack)")
    ap.add_argument("--workload", default="decode7b", choices=["decode7b", "stack7b", "stack70b"],
                    help="decode7b (default): the five 7B decode linears over rotating weight sets, with the "
                         "other configurations beside them; stack7b / stack70b: only that stack at --m rows")
    ap.add_argument("--layers", type=int, default=0, help="stack workloads: layers to build (0 = the model's)")
    ap.add_argument("--tiled", action="store_true",
                    help="stack workloads: every product on the tile-major copy of its weights")
    ap.add_argument("--weights", default="mxfp4", choices=["mxfp4", "bf16"],
                    help="stack workloads: bf16 runs the unquantised reference stack")
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
        return run_stack_only(args)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    m = args.m
    steps, warmup = max(1, args.steps), max(0, args.warmup)
    n_bf16 = 0 if args.no_bf16 else min(args.sets, 4)    # 4 x 0.67 GB of BF16 weights: cold too
    sets = build_sets(args.sets, m, dev, keep_bf16=n_bf16)
    ws = torch.empty((binding.mxfp4_woq_gemm_argmax_workspace_bytes(m, 32000, 4096),), dtype=torch.uint8, device=dev)
    clock = Clock(torch.cuda.Stream())
    shape = synth.LLAMA_7B
    step_bytes = sum(algorithmic_bytes(m, n, k) for _, n, k in shape.linears())
    weight_bytes = sum(n * k * 0.53125 for _, n, k in shape.linears())

    # --- the step under each launch discipline: exactly `steps` steps after `warmup` of the same kind
    disciplines = {}
    us, step_graphs = clock.us_per_call_graphs([(lambda lin=lin: step_calls(lin, ws)) for lin in sets], steps, warmup)
    disciplines["hip graph replay (one graph per rotation of the weight sets)"] = us
    groups = [binding.GemmGroup(step_items(lin)) for lin in sets]
    disciplines["stream launches from one grouped library call per step"] = clock.us_per_call(
        [g.run for g in groups], steps, warmup)
    chain_note = None
    if m == 1:
        label = "one chained call per step: all five products in one persistent launch"
        chains = [binding.GemmGroup(step_items(lin), chained=True, mode=binding.CHAIN_PERSISTENT) for lin in sets]
        us_chain = clock.us_per_call([c.run for c in chains], steps, warmup)
        if all(c.chain_status() == 0 for c in chains):
            disciplines[label] = us_chain
        else:
            chain_note = "a barrier wait was given up"
        del chains
    plain_us = clock.us_per_call([(lambda lin=lin: step_calls(lin, ws)) for lin in sets], max(len(sets), steps // 4), 0)
    launch = min(disciplines, key=disciplines.get)
    us_per_step = disciplines[launch]
    value = step_bytes / (us_per_step * 1e-6) / 1e9
    # spread of the headline discipline: ten further chunks of one rotation or more
    chunk_us = None
    chunk = max(len(sets), steps // 10 // len(sets) * len(sets))
    if launch.startswith("hip graph"):
        chunk_us = sorted(clock.ms(lambda: [step_graphs[0].replay() for _ in range(chunk // len(sets))]) * 1e3 / chunk
                          for _ in range(10))
    elif launch.startswith("stream launches"):
        chunk_us = sorted(clock.us_per_call([g.run for g in groups], chunk, 0) for _ in range(10))
    # for the record, not the headline: the five products declared independent of each other
    # (MXFP4_DESC_INDEPENDENT; the synthetic inputs are, a model's chain of layers is not)
    indep = [binding.GemmGroup([dict(it, independent=True) for it in
                                (step_items(lin)[3:4] + step_items(lin)[0:3] + step_items(lin)[4:])]) for lin in sets]
    indep_us = clock.us_per_call([g.run for g in indep], steps, warmup)
    del indep

    # --- every launch of the step alone: graph replays of that one launch over the weight sets
    # (twenty rotations whatever `steps` is: these are averages per launch, not the timed step)
    lin_reps = 20 * len(sets)
    per_linear = []
    for name, n, k in shape.linears():
        if name == "lm_head":
            continue
        fns = [(lambda t=lin[name]: binding.mxfp4_woq_gemm(t["x"], t["q"], t["s"], y=t["y"])) for lin in sets]
        us, g = clock.us_per_call_graphs(fns, lin_reps, len(fns))
        per_linear.append(dict(linear=name, N=n, K=k, launches=1, bytes=algorithmic_bytes(m, n, k),
                               **rate(algorithmic_bytes(m, n, k), us)))
        del g
    fns = [(lambda t=lin["lm_head"]: binding.mxfp4_woq_gemm(t["x"], t["q"], t["s"], y=t["y"])) for lin in sets]
    head_us, g = clock.us_per_call_graphs(fns, lin_reps, len(fns))
    del g
    fns = [(lambda t=lin["lm_head"]: binding.mxfp4_woq_gemm_argmax(t["x"], t["q"], t["s"], workspace=ws,
                                                                   out=(t["idx"], t["val"]))) for lin in sets]
    head_pick_us, g = clock.us_per_call_graphs(fns, lin_reps, len(fns))
    del g
    hb = algorithmic_bytes(m, 32000, 4096)
    per_linear.append(dict(linear="lm_head (product only, y written)", N=32000, K=4096, launches=1, bytes=hb,
                           **rate(hb, head_us)))
    per_linear.append(dict(linear="lm_head with fused argmax (product + second stage of the pick)", N=32000, K=4096,
                           launches=2, bytes=hb, **rate(hb, head_pick_us)))
    per_linear.append(dict(linear="argmax second stage (difference of the two lines above)", launches=1,
                           us=round(head_pick_us - head_us, 2)))
    # dominant kernel instance: the K = 4096 launches with more than 40 rows per compute unit (qkv, gate_up,
    # lm_head: 81 % of the bytes)
    dom_names = [p for p in per_linear[:3] if p["linear"] in DOMINANT] + [per_linear[4]]
    dom_us = sum(p["us"] for p in dom_names) / len(dom_names)
    dom_bytes = sum(p["bytes"] for p in dom_names) / len(dom_names)
    achieved = dom_bytes / (dom_us * 1e-6) / 1e9

    # --- the unquantised step and further variants on the first four weight sets
    extra = {}
    if n_bf16:
        bsets = sets[:n_bf16]
        nb = n_bf16 * max(2, steps // (4 * n_bf16))
        bf16_us, g = clock.us_per_call_graphs([(lambda lin=lin: step_calls_bf16(lin, ws)) for lin in bsets], nb, n_bf16)
        del g
        for lin in bsets:
            for t in lin.values():
                t["x5"] = synth.activations_outlier_channels(5, t["k"], seed=t["n"] + 5, device=dev)
                t["y5"] = torch.empty((5, t["n"]), dtype=torch.bfloat16, device=dev)
            lin["lm_head"]["idx5"] = torch.empty((5,), dtype=torch.int32, device=dev)
            lin["lm_head"]["val5"] = torch.empty((5,), dtype=torch.float32, device=dev)
        ws5 = torch.empty((binding.mxfp4_bf16_gemm_argmax_workspace_bytes(5, 32000, 4096),), dtype=torch.uint8,
                          device=dev)
        v5_us, g = clock.us_per_call_graphs([(lambda lin=lin: verify5_calls_bf16(lin, ws5)) for lin in bsets], nb, n_bf16)
        del g
        graph_us = disciplines["hip graph replay (one graph per rotation of the weight sets)"]      # like with like: both as graph replays
        extra["bf16_weights_us_per_step"] = round(bf16_us, 2)
        extra["bf16_weights_verify_5_rows_us"] = round(v5_us, 2)
        extra["speedup_over_bf16_weights"] = round(bf16_us / graph_us, 3)
        extra["eq1_projection"] = eq1_projection(bf16_us / graph_us, v5_us / bf16_us)
        # other element formats as drafts, fused epilogues, a verification pass on both weight layouts
        for lin in bsets:
            for name, t in lin.items():
                t["q8"], t["s8"] = binding.mxfp4_e4m3_direct_cast(t["w"])
                t["q6"], t["s6"] = binding.mxfp4_e2m3_direct_cast(t["w"])
                for fmt in (binding.FMT_E5M2, binding.FMT_E3M2, binding.FMT_T2):
                    t["qf%d" % fmt], t["sf%d" % fmt] = binding.mxfp4_fmt_direct_cast(fmt, t["w"])
                t["w"] = None
                if name in ("qkv", "o", "gate_up"):
                    t["x8"] = synth.activations_outlier_channels(8, t["k"], seed=t["n"], device=dev)
                    t["y8"] = torch.empty((8, t["n"]), dtype=torch.bfloat16, device=dev)
                    t["tw"] = binding.mxfp4_tile_repack(t["q"], t["s"])
            lin["gate_up"]["h"] = torch.empty((m, lin["gate_up"]["n"] // 2), dtype=torch.bfloat16, device=dev)

        def e4m3(lin):
            for name in STEP_LINEARS:
                t = lin[name]
                binding.mxfp4_e4m3_woq_gemm(t["x"], t["q8"], t["s8"], y=t["y"])
            t = lin["lm_head"]
            binding.mxfp4_e4m3_woq_gemm_argmax(t["x"], t["q8"], t["s8"], workspace=ws, out=(t["idx"], t["val"]))

        def e2m3(lin):
            for name in STEP_LINEARS:
                t = lin[name]
                binding.mxfp4_e2m3_woq_gemm(t["x"], t["q6"], t["s6"], y=t["y"])
            t = lin["lm_head"]
            binding.mxfp4_e2m3_woq_gemm_argmax(t["x"], t["q6"], t["s6"], workspace=ws, out=(t["idx"], t["val"]))

        def by_id(fmt):
            def run(lin):
                for name in STEP_LINEARS:
                    t = lin[name]
                    binding.mxfp4_fmt_woq_gemm(fmt, t["x"], t["qf%d" % fmt], t["sf%d" % fmt], y=t["y"])
                t = lin["lm_head"]
                binding.mxfp4_fmt_woq_gemm_argmax(fmt, t["x"], t["qf%d" % fmt], t["sf%d" % fmt], workspace=ws,
                                                  out=(t["idx"], t["val"]))
            return run

        def layer_plain(lin):
            for name in STEP_LINEARS:
                t = lin[name]
                binding.mxfp4_woq_gemm(t["x"], t["q"], t["s"], y=t["y"])

        def layer_fused(lin):
            t = lin["qkv"]
            binding.mxfp4_woq_gemm(t["x"], t["q"], t["s"], y=t["y"])
            for name in ("o", "down"):
                t = lin[name]
                binding.mxfp4_woq_gemm_fused(t["x"], t["q"], t["s"], residual=t["y"], y=t["y"])
            t = lin["gate_up"]
            binding.mxfp4_woq_gemm_fused(t["x"], t["q"], t["s"], act=binding.ACT_SWIGLU, y=t["h"])

        def verify8(lin):
            for name in ("qkv", "o", "gate_up"):
                t = lin[name]
                binding.mxfp4_woq_gemm(t["x8"], t["q"], t["s"], y=t["y8"])

        def verify8_tiled(lin):
            for name in ("qkv", "o", "gate_up"):
                t = lin[name]
                binding.mxfp4_woq_gemm_tiled(t["x8"], t["tw"], y=t["y8"])

        variants = {}
        for key, fn in (("e4m3_weights_us_per_step", e4m3), ("e2m3_weights_us_per_step", e2m3),
                        ("e5m2_weights_us_per_step", by_id(binding.FMT_E5M2)),
                        ("e3m2_weights_us_per_step", by_id(binding.FMT_E3M2)),
                        ("ternary_2bit_weights_us_per_step", by_id(binding.FMT_T2)),
                        ("layer_4_linears_us", layer_plain), ("layer_4_linears_fused_epilogues_us", layer_fused),
                        ("verify_m8_qkv_o_gateup_us", verify8), ("verify_m8_qkv_o_gateup_tile_major_us", verify8_tiled)):
            us, g = clock.us_per_call_graphs([(lambda lin=lin, fn=fn: fn(lin)) for lin in bsets], nb, n_bf16)
            variants[key] = round(us, 2)
            del g
        # attention over a cache held in MXFP4: one head, 4096 tokens of dimension 128, four query rows
        # (64 heads' caches in rotation: 36 MB, more than the L2s hold)
        heads = []
        for h in range(64):
            kq, ks = binding.mxfp4_direct_cast(synth.weights_student_t(4096, 128, seed=900 + h, device=dev))
            vq, vs = binding.mxfp4_direct_cast(synth.weights_student_t(4096, 128, seed=1900 + h, device=dev))
            heads.append(dict(kq=kq, ks=ks, vq=vq, vs=vs))
        qx = synth.activations_outlier_channels(4, 128, seed=77, device=dev)
        px = synth.activations_outlier_channels(4, 4096, seed=78, device=dev)
        sc = torch.empty((4, 4096), dtype=torch.bfloat16, device=dev)
        ov = torch.empty((4, 128), dtype=torch.bfloat16, device=dev)
        wst = torch.empty((binding.mxfp4_woq_gemm_t_workspace_bytes(4, 4096, 128),), dtype=torch.uint8, device=dev)
        us, g = clock.us_per_call_graphs([(lambda h=h: binding.mxfp4_woq_gemm(qx, h["kq"], h["ks"], y=sc)) for h in heads],
                                         4 * len(heads), len(heads))
        variants["cache_head_4096x128_scores_4_rows_us"] = round(us, 2)
        del g
        us, g = clock.us_per_call_graphs([(lambda h=h: binding.mxfp4_woq_gemm_t(px, h["vq"], h["vs"], y=ov, workspace=wst))
                                          for h in heads], 4 * len(heads), len(heads))
        variants["cache_head_4096x128_values_4_rows_us"] = round(us, 2)
        del g, heads
        extra["variants"] = variants
        for lin in bsets:
            for t in lin.values():
                for key in ("q8", "s8", "q6", "s6", "x8", "y8", "x5", "y5", "tw", "h", "qf1", "sf1", "qf2", "sf2", "qf3", "sf3"):
                    t.pop(key, None)

    # --- what a plain 128-bit read stream gets on this device, over 4 GiB (context for frac), and one
    # plain copy of known size: the reference against which the profiler's byte counters are scaled
    buf = torch.empty(4 << 30, dtype=torch.uint8, device=dev)
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    stream_read_gbps = buf.numel() / (clock.us_per_call([lambda: binding.mxfp4_diag_stream_read(buf, sink)], 5, 1) * 1e-6) / 1e9
    half = buf.numel() // 4
    with torch.cuda.stream(clock.stream):
        binding.mxfp4_diag_stream_copy(buf[:half], buf[2 * half:3 * half])
    torch.cuda.synchronize()
    del buf

    # --- the other four configurations
    configs = None
    if not args.no_configs:
        reps = 10 * len(sets)
        single = config_single_linear(clock, dev, reps)
        configs = {
            "config_1_single_linear_4096x4096": single.pop("M=1"),
            "config_3_verification_sweep": {"linear_4096x4096": single,
                                            "lm_head_32000x4096_with_argmax": config_verify_sweep_lm_head(clock, sets, dev, reps)},
        }
        del step_graphs, groups
        sets.clear()
        torch.cuda.empty_cache()
        stack_reps = max(5, steps // 24)
        configs["config_4_llama7b_stack"] = config_stack(clock, synth.LLAMA_7B, [1, 8], stack_reps, dev, tiled_m=(1, 8))
        torch.cuda.empty_cache()
        if not args.no_70b:
            configs["config_5_llama70b_stack"] = config_stack(clock, synth.LLAMA_70B, [1, 4, 16], max(2, stack_reps // 2), dev)
            torch.cuda.empty_cache()

    traffic, traffic_source = None, None
    tpath = os.path.join(ROOT, "profiles", "traffic.txt")
    if os.path.exists(tpath):
        for line in open(tpath):
            if line.startswith("gemv_m1_dominant_bytes_per_launch"):
                try:
                    traffic = int(line.split("=")[1])
                    traffic_source = ("profiles/traffic.txt: rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE passes of this "
                                      "command, scaled by the copy kernel of known size; a stored figure, not "
                                      "counted in this run")
                except ValueError:
                    traffic = None

    out = {
        "metric": METRIC, "value": round(value, 1), "unit": "GB/s", "n_gpus": 1,
        "steps": steps, "warmup": warmup, "ms_per_step": round(us_per_step * 1e-3, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": DTYPE,
        "data": "synthetic",
        "config": {"workload": "configs[1]: Llama-7B-shaped decode linears at M=%d "
                               "(qkv 12288x4096, o 4096x4096, gate_up 22016x4096, down 4096x11008, "
                               "lm_head 32000x4096 + argmax), %d weight sets rotated (%.2f GB)"
                               % (m, args.sets, args.sets * weight_bytes / 1e9),
                   "M": m, "launch": launch},
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "us_per_step": round(us_per_step, 2),
        "us_per_step_by_launch_discipline": {k: round(v, 2) for k, v in disciplines.items()},
        "us_per_step_plain_python_launches": round(plain_us, 2),
        "independent_products_merged_launch": dict(
            rate(step_bytes, indep_us), launches_per_step=2,
            note="not the headline: valid only because the benchmark's five inputs do not depend on each other"),
        "bytes_per_step": step_bytes,
        "tflops": round(2.0 * m * sum(n * k for _, n, k in shape.linears()) / (us_per_step * 1e-6) / 1e12, 3),
        "stream_read_GBps": round(stream_read_gbps, 1),
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic, "traffic_source": traffic_source,
                     "kernel": DOMINANT_KERNEL + " (qkv, gate_up and lm_head launches)",
                     "bytes_per_launch": dom_bytes, "us_per_launch": round(dom_us, 3),
                     "duration_source": "HIP events on the launch stream around %d back-to-back launches of each "
                                        "linear alone, replayed from a graph (weight sets in rotation), averaged over "
                                        "the three linears; the gaps between launches are inside, so the kernel itself "
                                        "is a little shorter (rocprofv3 kernel trace under profiles/)" % lin_reps},
        "roofline_per_linear": per_linear,
    }
    if chunk_us:
        out["us_per_step_min_median_max_of_10_chunks"] = [round(chunk_us[0], 2),
                                                          round((chunk_us[4] + chunk_us[5]) / 2, 2),
                                                          round(chunk_us[-1], 2)]
    if chain_note:
        out["chained_launch_note"] = chain_note
    out.update(extra)
    if configs is not None:
        out["configs"] = configs
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(m)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
