#!/usr/bin/env python3
"""Benchmark of the LazyTensor fused-execution hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input: record the trace
through the C ABI, barrier (cut, hash, cache lookup, lowering on a miss, kernel launches), block
until the device is done.  Inputs are resident in HBM before the timed region starts.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c4|c1|c2|c3|c5]

Without --workload the headline is c4 (the configuration whose fused regions are HBM-bound at a
size that fills the GPU) and the other four configurations run briefly afterwards; their rates
and roofline fractions go under detail.other_configs of the same JSON line.

Prints ONE JSON line: barrier-steps/s for the workload, the roofline of its dominant kernel
(duration measured with HIP events on the library's stream inside the timed steps) and the CPU
oracle timed on the same box.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published


def _profiled_traffic(kernel):
    """HBM bytes per launch of `kernel` as rocprofv3 counted them (FETCH_SIZE and WRITE_SIZE, each
    scaled by what the same counter reads for a 1 GiB device copy): the figure is not measured by
    this process -- counters need the profiler -- but read from the committed summary of the
    profiler runs of this same command, profiles/c4_adam_clip_hbm_traffic.md (line
    "traffic_bytes_per_launch <kernel instance> <bytes>"); None when there is no such line."""
    path = os.path.join(ROOT, "profiles", "c4_adam_clip_hbm_traffic.md")
    try:
        for ln in open(path):
            parts = ln.strip().strip("`").split()
            if len(parts) >= 3 and parts[0] == "traffic_bytes_per_launch" and " ".join(parts[1:-1]) == kernel:
                return int(parts[-1])
    except OSError:
        pass
    return None


MFMA_PEAK_TFLOPS = {"bf16": 2516.6, "f32": 157.3}


_STREAMS = 4   # --streams: streams a barrier may spread independent launches over
_C1_STREAMING_RUN = True   # --no-streaming-run: C1 without its extra run on [16384, 16384] operands


def _gpu_ctx(workspace_bytes):
    from paper_2102_13267_amd import Context
    ctx = Context(device=0, workspace_bytes=workspace_bytes)
    ctx.set_streams(_STREAMS)
    return ctx


def _sync():
    import torch
    torch.cuda.synchronize()


def _time_steps(step_fn, ctx, steps, warmup):
    """Returns (seconds for `steps` steps, per-kernel records of the timed steps, barrier infos)."""
    for _ in range(warmup):
        step_fn()
    _sync()
    ctx.set_profiling(True)
    launches, infos = [], []
    _sync()
    t0 = time.perf_counter()
    for _ in range(steps):
        infos.append(step_fn())
        launches.append(ctx.last_launches())
    _sync()
    dt = time.perf_counter() - t0
    ctx.set_profiling(False)
    # the same steps without event recording, for the headline rate
    _sync()
    t0 = time.perf_counter()
    for _ in range(steps):
        step_fn()
    _sync()
    dt_plain = time.perf_counter() - t0
    return dt_plain, dt, launches, infos


def _time_pipelined(record_fn, ctx, steps):
    """Steps per second when the barrier does not block (section 4's asynchronous execution): the
    host records step i+1 while the device runs step i; one synchronisation at the end.
    `record_fn` records one step and returns what must stay alive until its barrier."""
    _sync()
    t0 = time.perf_counter()
    for _ in range(steps):
        keep = record_fn()
        ctx.barrier(False)
    del keep
    _sync()
    return steps / (time.perf_counter() - t0)


def _dominant(launches):
    """Average duration and algorithmic bytes / flops per launch of the kernel family that takes
    the most device time."""
    agg = {}
    for step in launches:
        for r in step:
            a = agg.setdefault((r["kernel"], r["region"]), {"ms": 0.0, "n": 0, "bytes": r["bytes"], "flops": r["flops"]})
            a["ms"] += r["ms"]
            a["n"] += 1
    (kernel, region), a = max(agg.items(), key=lambda kv: kv[1]["ms"])
    table = [{"kernel": k, "region": rg, "avg_ms": v["ms"] / v["n"], "bytes": v["bytes"], "flops": v["flops"]}
             for (k, rg), v in sorted(agg.items(), key=lambda kv: kv[0][1])]
    return kernel, region, a["ms"] / a["n"], a["bytes"], a["flops"], table


# ---- workloads ---------------------------------------------------------------------------------
def run_c4(steps, warmup, n=268_435_456):
    from workloads import programs
    from workloads.inputs import C4_HYPER, c4_inputs
    ctx = _gpu_ctx(64 << 20)
    inp = c4_inputs(n)
    p, g, m, v = (ctx.tensor(inp[k], donatable=(k != "g")) for k in ("p", "g", "m", "v"))
    state = {"t": 0}

    def step():
        state["t"] += 1
        programs.c4_step(ctx, p, g, m, v, **dict(C4_HYPER, t=state["t"]))
        return ctx.barrier(True)
    dt, dt_prof, launches, infos = _time_steps(step, ctx, steps, warmup)
    kernel, region, avg_ms, kbytes, _, table = _dominant(launches)
    roof = {"bound": "hbm", "kernel": kernel, "achieved": kbytes / (avg_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
            "unit": "GB/s", "traffic": None, "avg_ms": avg_ms, "bytes_per_launch": kbytes}
    roof["frac"] = roof["achieved"] / roof["peak"]
    if n == 268_435_456:
        roof["traffic"] = _profiled_traffic(kernel)
    extra = {"kernels": table, "plan": ctx.dump_plan(), "cache_hits": sum(i.cache_hit for i in infos),
             "bytes_planned_per_step": int(infos[-1].bytes_planned),
             "whole_step_GBps": infos[-1].bytes_planned * steps / dt / 1e9}
    config = {"workload": f"c4: fused Adam + grad-norm clipping over {n} fp32 params, one barrier per step",
              "params": n, "regions": int(infos[-1].n_regions)}

    def cpu(sample=1 << 24):
        from oracle.numeric import Eager
        si = c4_inputs(sample)
        E = Eager()
        ts = [E.tensor(si[k]) for k in ("p", "g", "m", "v")]
        programs.c4_step(E, *ts, **C4_HYPER)           # warm-up
        t0 = time.perf_counter()
        reps = 0
        while time.perf_counter() - t0 < 10.0:
            programs.c4_step(E, *ts, **C4_HYPER)
            reps += 1
        per_param = (time.perf_counter() - t0) / (reps * sample)
        return 1.0 / (per_param * n), f"{reps} oracle steps on {sample} params, scaled linearly to {n}"
    return dt, "f32", config, roof, extra, cpu


def _c1_streaming_rate(n=16384, reps=5):
    """The same trace on [n, n] operands (2 GiB of inputs at n = 16384, not a configuration of the
    benchmark): at the configured size the row kernel's 8 MiB are cache resident and a launch is over
    in microseconds, so this run is what shows the kernel's rate against HBM."""
    import torch
    from workloads import programs
    ctx = _gpu_ctx(64 << 20)
    gen = torch.Generator(device="cuda:0").manual_seed(1001)
    x, y = (torch.rand(n, n, device="cuda:0", generator=gen) * 2 - 1 for _ in range(2))
    b = torch.rand(n, device="cuda:0", generator=gen) * 2 - 1
    tx, ty, tb = ctx.tensor(x), ctx.tensor(y), ctx.tensor(b)
    out = programs.c1_trace(ctx, tx, ty, tb)
    ctx.barrier(True)
    ctx.set_profiling(True)
    ms = []
    for _ in range(reps):
        out = programs.c1_trace(ctx, tx, ty, tb)
        ctx.barrier(True)
        ms.append(min(r["ms"] for r in ctx.last_launches() if r["kernel"].startswith("lt_row_reduce")))
    ctx.set_profiling(False)
    del out
    ctx.close()
    nbytes = 2 * 4 * n * n + 2 * 4 * n
    best = min(ms)
    return {"row_kernel_ms": best, "bytes": nbytes, "GBps": nbytes / (best * 1e-3) / 1e9, "frac_of_hbm_peak": nbytes / (best * 1e-3) / 1e9 / HBM_PEAK_GBS}


def run_c1(steps, warmup, rows=1024, cols=1024):
    from workloads import programs
    from workloads.inputs import c1_inputs
    ctx = _gpu_ctx(64 << 20)
    inp = c1_inputs(rows, cols)
    x, y, b = (ctx.tensor(inp[k]) for k in ("x", "y", "bias"))

    def step():
        out = programs.c1_trace(ctx, x, y, b)
        return ctx.barrier(True)
    dt, dt_prof, launches, infos = _time_steps(step, ctx, steps, warmup)
    kernel, region, avg_ms, kbytes, _, table = _dominant(launches)
    roof = {"bound": "hbm", "kernel": kernel, "achieved": kbytes / (avg_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
            "unit": "GB/s", "traffic": None, "avg_ms": avg_ms, "bytes_per_launch": kbytes}
    roof["frac"] = roof["achieved"] / roof["peak"]
    extra = {"kernels": table, "plan": ctx.dump_plan(), "cache_hits": sum(i.cache_hit for i in infos)}
    config = {"workload": f"c1: 12-op elementwise+reduce trace on fp32 [{rows},{cols}]", "regions": int(infos[-1].n_regions)}
    if rows == 1024 and cols == 1024 and _C1_STREAMING_RUN:
        extra["streaming_run_16384x16384"] = _c1_streaming_rate()

    def cpu():
        from oracle.numeric import Eager
        E = Eager()
        ts = [E.tensor(inp[k]) for k in ("x", "y", "bias")]
        programs.c1_trace(E, *ts)
        t0 = time.perf_counter()
        reps = 0
        while time.perf_counter() - t0 < 10.0:
            programs.c1_trace(E, *ts)
            reps += 1
        return reps / (time.perf_counter() - t0), f"{reps} oracle steps at full size"
    return dt, "f32", config, roof, extra, cpu


def run_c2(steps, warmup):
    from workloads import programs
    from workloads.inputs import c2_inputs
    ctx = _gpu_ctx(256 << 20)
    n_batches = 100
    inp = c2_inputs(steps=n_batches)
    names = ("W1", "b1", "W2", "b2", "W3", "b3")
    params = [ctx.tensor(inp[k], donatable=True) for k in names]
    Xs = [ctx.tensor(inp["X"][i]) for i in range(n_batches)]
    Ls = [ctx.tensor(inp["labels"][i]) for i in range(n_batches)]
    state = {"i": 0}

    def step():
        i = state["i"] % n_batches
        state["i"] += 1
        loss = programs.c2_step(ctx, Xs[i], Ls[i], params, 0.01)
        return ctx.barrier(True)
    dt, dt_prof, launches, infos = _time_steps(step, ctx, steps, warmup)

    def record():
        i = state["i"] % n_batches
        state["i"] += 1
        return programs.c2_step(ctx, Xs[i], Ls[i], params, 0.01)
    pipelined = _time_pipelined(record, ctx, steps)

    # the same steps without tracing (a captured step run again on re-pointed batch tensors), and
    # as HIP graphs (batches copied into fixed tensors so that the addresses come back)
    import torch
    Xt = [torch.from_numpy(inp["X"][i]).cuda() for i in range(n_batches)]
    Lt = [torch.from_numpy(inp["labels"][i]).cuda() for i in range(n_batches)]
    X, L = ctx.tensor(Xt[0].clone()), ctx.tensor(Lt[0].clone())
    loss = programs.c2_step(ctx, X, L, params, 0.01)
    ctx.barrier(True)
    captured = ctx.capture_step()

    def replayed(graphs):
        ctx.set_graphs(graphs)

        def one(i):
            if graphs:
                X._keep.copy_(Xt[i % n_batches])
                L._keep.copy_(Lt[i % n_batches])
            else:
                ctx.rebind(X, Xt[i % n_batches])
                ctx.rebind(L, Lt[i % n_batches])
            captured.replay(blocking=True)
        for i in range(max(warmup, 8)):
            one(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            one(i)
        torch.cuda.synchronize()
        rate = steps / (time.perf_counter() - t0)
        ctx.set_graphs(False)
        return rate
    rate_replay, rate_graph = replayed(False), replayed(True)
    _, _, _, _, _, table = _dominant(launches)
    # the contractions as a family (each is a few microseconds: launch latency, not the matrix cores, bounds them)
    flops = sum(r["flops"] for st in launches for r in st)
    gemm_ms = sum(r["ms"] for st in launches for r in st if r["flops"])
    roof = {"bound": "mfma", "kernel": "lt_gemm_kernel<float, ...> (every contraction of the step)", "achieved": flops / (gemm_ms * 1e-3) / 1e12,
            "peak": MFMA_PEAK_TFLOPS["f32"], "unit": "TFLOP/s", "traffic": None, "gemm_ms_per_step": gemm_ms / len(launches),
            "device_ms_per_step": sum(r["ms"] for st in launches for r in st) / len(launches),
            "launches_per_step": len(launches[-1])}
    roof["frac"] = roof["achieved"] / roof["peak"]
    extra = {"kernels": table, "cache_hits": sum(i.cache_hit for i in infos), "ns_host_per_step": {
        "collect": int(np.mean([i.ns_collect for i in infos])), "hash": int(np.mean([i.ns_hash for i in infos])),
        "launch": int(np.mean([i.ns_launch for i in infos]))}, "steps_per_s_non_blocking_barrier": pipelined,
        "steps_per_s_replayed_without_tracing": rate_replay, "steps_per_s_replayed_as_hip_graphs": rate_graph}
    config = {"workload": "c2: MLP 784-512-512-10 fp32 batch 128, fwd+bwd+SGD, one barrier per step", "regions": int(infos[-1].n_regions)}

    def cpu():
        from oracle.numeric import Eager
        E = Eager()
        ps = [E.tensor(inp[k]) for k in names]
        X, L = E.tensor(inp["X"][0]), E.tensor(inp["labels"][0])
        programs.c2_step(E, X, L, ps, 0.01)
        t0 = time.perf_counter()
        reps = 0
        while time.perf_counter() - t0 < 10.0:
            programs.c2_step(E, X, L, ps, 0.01)
            reps += 1
        return reps / (time.perf_counter() - t0), f"{reps} oracle steps at full size"
    return dt, "f32", config, roof, extra, cpu


def run_c5(steps, warmup):
    """The configured run is `steps` (200) steps from an empty plan cache: that pass gives the hit
    rate, the number of distinct traces and the lowering time per miss (`warmup` is not used: the
    first pass is the warm-up).  The same sequence is then run again, every step a cache hit, for
    the steady-state rate (the headline value: barrier-steps/s are quoted on cache hits), and once
    more with per-launch timing for the roofline entry."""
    from workloads import programs
    from workloads.inputs import c5_batch, c5_inputs
    ctx = _gpu_ctx(1 << 30)
    inp = c5_inputs(steps=steps)
    W = [ctx.tensor(w) for w in inp["W"]]; b = [ctx.tensor(w) for w in inp["b"]]
    Wr = [ctx.tensor(w) for w in inp["Wr"]]; br = [ctx.tensor(w) for w in inp["br"]]
    Xs = [ctx.tensor(c5_batch(i, int(inp["batch"][i]))) for i in range(steps)]
    words = [ctx.tensor(np.array([inp["word"][i]], np.int32)) for i in range(steps)]

    def one_pass():
        infos, keys = [], []
        _sync()
        t0 = time.perf_counter()
        for i in range(steps):
            depth = 1 + int(ctx.fetch(words[i])[0]) % 8      # data-dependent host branch: a trace break
            s, h = programs.c5_forward(ctx, Xs[i], W, b, Wr, br, depth)
            infos.append(ctx.barrier(True))
            keys.append((int(inp["batch"][i]), depth))
        _sync()
        return time.perf_counter() - t0, infos, keys
    dt_first, infos, keys = one_pass()
    misses = [i for i in infos if not i.cache_hit]
    dt, infos2, _ = one_pass()
    assert all(i.cache_hit for i in infos2)
    ctx.set_profiling(True)
    launches = []
    for i in range(steps):
        depth = 1 + int(ctx.fetch(words[i])[0]) % 8
        s, h = programs.c5_forward(ctx, Xs[i], W, b, Wr, br, depth)
        ctx.barrier(True)
        launches.append(ctx.last_launches())
    ctx.set_profiling(False)
    flops = sum(r["flops"] for st in launches for r in st)
    gemm_ms = sum(r["ms"] for st in launches for r in st if r["flops"] or r["kernel"].startswith("lt_split_post"))
    roof = {"bound": "mfma", "kernel": "lt_gemm_kernel<float, ...> (every contraction of the run, with the second launches of split ones)",
            "achieved": flops / (gemm_ms * 1e-3) / 1e12, "peak": MFMA_PEAK_TFLOPS["f32"], "unit": "TFLOP/s", "traffic": None,
            "gemm_ms_total": gemm_ms}
    roof["frac"] = roof["achieved"] / roof["peak"]
    by_batch = {}
    for st, (bsz, _) in zip(launches, keys):
        e = by_batch.setdefault(bsz, [0.0, 0.0])
        e[0] += sum(r["flops"] for r in st)
        e[1] += sum(r["ms"] for r in st if r["flops"] or r["kernel"].startswith("lt_split_post"))
    extra = {"hit_rate_first_pass": 1 - len(misses) / len(infos), "distinct_traces": len(set(keys)), "misses": len(misses),
             "lowering_us_per_miss": float(np.mean([i.ns_lower for i in misses]) / 1e3) if misses else None,
             "steps_per_s_first_pass_with_lowering": steps / dt_first,
             "contraction_TFLOPs_by_batch": {str(k): v[0] / (v[1] * 1e-3) / 1e12 for k, v in sorted(by_batch.items()) if v[1] > 0}}
    config = {"workload": f"c5: 4-layer GELU MLP d=2048 fp32, batch in {{8..1024}}, 1-8 unrolled residual blocks, {steps} steps"}

    def cpu():
        from oracle.numeric import Eager
        E = Eager()
        ow = [[E.tensor(w) for w in inp[k]] for k in ("W", "b", "Wr", "br")]
        t0 = time.perf_counter()
        done = 0
        while done < steps and time.perf_counter() - t0 < 15.0:
            programs.c5_forward(E, E.tensor(c5_batch(done, int(inp["batch"][done]))), *ow, keys[done][1])
            done += 1
        return done / (time.perf_counter() - t0), f"the first {done} steps of the same sequence (batch sizes and depths as drawn)"
    return dt, "f32", config, roof, extra, cpu


def run_c3(steps, warmup, bsz=32, seq=256, d=1024, ffn=4096, heads=16):
    from workloads import programs
    from workloads.inputs import c3_inputs
    import torch
    ctx = _gpu_ctx(8 << 30)
    keys = programs.C3_WEIGHTS + programs.C3_VECTORS

    def setup(B, mk, batch):
        inp = c3_inputs(batch, seq, d, ffn)
        bf = lambda a: torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()   # round to nearest even
        P = {k: mk(bf(inp[k]), "bf16", True) for k in keys}
        M = {k: mk(np.zeros_like(inp[k]), "f32", True) for k in keys}
        V = {k: mk(np.zeros_like(inp[k]), "f32", True) for k in keys}
        return mk(bf(inp["x"]), "bf16", False), mk(bf(inp["dy"]), "bf16", False), P, M, V, heads
    g = setup(ctx, lambda a, dt, don: ctx.tensor(a, dtype=dt, donatable=don), bsz)
    state = {"t": 0}

    def step():
        state["t"] += 1
        y, dx = programs.c3_step(ctx, *g, t=state["t"])     # held until the barrier: the layer output and the input gradient are results
        return ctx.barrier(True)
    dt, dt_prof, launches, infos = _time_steps(step, ctx, steps, warmup)

    def record():
        state["t"] += 1
        return programs.c3_step(ctx, *g, t=state["t"])
    pipelined = _time_pipelined(record, ctx, steps)

    # the same steps without tracing (section 7 of the paper): one more traced step is captured and
    # run again with the two scalars that depend on the step number (Adam's bias corrections) replaced
    def replayed():
        state["t"] += 1
        t0 = state["t"]
        held = programs.c3_step(ctx, *g, t=t0)
        ctx.barrier(True)
        captured = ctx.capture_step()
        base = captured.scalars
        c1, c2 = 1.0 - 0.9 ** t0, 1.0 - 0.999 ** t0

        def one():
            state["t"] += 1
            t = state["t"]
            captured.replay(scalars=[1.0 - 0.9 ** t if v == c1 else 1.0 - 0.999 ** t if v == c2 else v for v in base], blocking=True)
        for _ in range(max(warmup, 2)):
            one()
        torch.cuda.synchronize()
        t_start = time.perf_counter()
        for _ in range(steps):
            one()
        torch.cuda.synchronize()
        rate = steps / (time.perf_counter() - t_start)
        captured.free()
        del held
        return rate
    rate_replay = replayed()
    _, _, _, _, _, table = _dominant(launches)
    n = len(launches)
    gemm = [r for st in launches for r in st if r["flops"]]
    rest = [r for st in launches for r in st if not r["flops"]]
    big = [r for r in gemm if r["flops"] >= 2 * bsz * seq * d * d]           # the projection / FFN GEMMs
    att = [r for r in gemm if r["flops"] < 2 * bsz * seq * d * d]           # per-head score / context GEMMs
    tf = lambda rs: sum(r["flops"] for r in rs) / (sum(r["ms"] for r in rs) * 1e-3) / 1e12 if rs else None
    gb = lambda rs: sum(r["bytes"] for r in rs) / (sum(r["ms"] for r in rs) * 1e-3) / 1e9 if rs else None
    roof = {"bound": "mfma", "kernel": "lt_gemm_bf16_kernel<...> (every contraction of the step)", "achieved": tf(gemm), "peak": MFMA_PEAK_TFLOPS["bf16"],
            "unit": "TFLOP/s", "traffic": None, "gemm_ms_per_step": sum(r["ms"] for r in gemm) / n,
            "flops_per_step": sum(r["flops"] for r in gemm) / n}
    roof["frac"] = roof["achieved"] / roof["peak"]
    extra = {"projection_ffn_gemm_TFLOPs": tf(big), "attention_gemm_TFLOPs": tf(att),
             "non_gemm_ms_per_step": sum(r["ms"] for r in rest) / n, "non_gemm_GBps": gb(rest),
             "non_gemm_bytes_per_step": sum(r["bytes"] for r in rest) / n,
             "device_ms_per_step": sum(r["ms"] for st in launches for r in st) / n,
             "launches_per_step": len(launches[-1]), "kernels": table,
             "cache_hits": sum(i.cache_hit for i in infos), "steps_per_s_non_blocking_barrier": pipelined,
             "steps_per_s_replayed_without_tracing": rate_replay,
             "ns_host_per_step": {"collect": int(np.mean([i.ns_collect for i in infos])),
                                  "hash": int(np.mean([i.ns_hash for i in infos])),
                                  "launch": int(np.mean([i.ns_launch for i in infos]))}}
    config = {"workload": f"c3: transformer encoder layer fwd+bwd+Adam, bf16, batch {bsz} seq {seq} d_model {d} "
                          f"heads {heads} ffn {ffn}, one barrier per step", "regions": int(infos[-1].n_regions)}

    def cpu(sample_batch=2):
        from oracle.numeric import Eager
        E = Eager()
        r = setup(E, lambda a, dt, don: E.tensor(a, dtype=dt), sample_batch)
        t0 = time.perf_counter()
        programs.c3_step(E, *r, t=1)
        el = time.perf_counter() - t0
        return 1.0 / (el * bsz / sample_batch), f"1 oracle step at batch {sample_batch}, scaled linearly to batch {bsz}"
    return dt, "bf16", config, roof, extra, cpu


def run_shapes(steps, warmup):
    """Not a configuration of the benchmark: relu(A x B + bias) in fp32, one barrier per product, at
    the contraction shapes of C2 (forward, backward and weight-gradient layouts) and of C5 (every
    batch size), with HIP events around every launch -- which kernel the lowering picks for a
    shape and what the product costs, for the kernel notes in the design document and a
    rocprofv3 trace per kernel instance.  A "step" is one pass over all shapes."""
    import torch
    ctx = _gpu_ctx(2 << 30)
    shapes = [(128, 512, 784, 0, 0), (128, 512, 512, 0, 0), (128, 10, 512, 0, 0), (128, 512, 512, 0, 1), (128, 512, 10, 0, 1),
              (784, 512, 128, 1, 0), (512, 512, 128, 1, 0), (512, 10, 128, 1, 0)]
    shapes += [(bsz, 2048, 2048, 0, 0) for bsz in (8, 16, 32, 64, 128, 256, 512, 1024)]
    ops = []
    for m, n, k, ta, tb in shapes:
        ops.append((ctx.tensor(torch.randn((k, m) if ta else (m, k), device="cuda")),
                    ctx.tensor(torch.randn((n, k) if tb else (k, n), device="cuda")),
                    ctx.tensor(torch.randn(n, device="cuda")), bool(ta), bool(tb)))

    def one(i):
        a, b, bias, ta, tb = ops[i]
        y = ctx.relu(ctx.add(ctx.matmul(a, b, trans_a=ta, trans_b=tb), bias))
        ctx.barrier(True)
        return y
    for _ in range(max(warmup, 2)):
        for i in range(len(shapes)):
            one(i)
    ctx.set_profiling(True)
    per = [[] for _ in shapes]
    names = [None] * len(shapes)
    for _ in range(steps):
        for i in range(len(shapes)):
            one(i)
            ll = ctx.last_launches()
            per[i].append(sum(r["ms"] for r in ll) * 1e3)
            names[i] = [r["kernel"] for r in ll]
    ctx.set_profiling(False)
    _sync()
    t0 = time.perf_counter()
    for _ in range(steps):
        for i in range(len(shapes)):
            one(i)
    _sync()
    dt = time.perf_counter() - t0
    table = []
    for (m, n, k, ta, tb), us, nm in zip(shapes, per, names):
        med = float(np.median(us))
        table.append({"m": m, "n": n, "k": k, "trans_a": ta, "trans_b": tb, "us_with_events": med,
                      "TFLOPs": 2.0 * m * n * k / med * 1e-6, "launches": nm})
    flops = sum(2.0 * m * n * k for m, n, k, _, _ in shapes)
    total_us = sum(r["us_with_events"] for r in table)
    roof = {"bound": "mfma", "kernel": "every fp32 contraction of the pass", "achieved": flops / total_us * 1e-6, "peak": MFMA_PEAK_TFLOPS["f32"],
            "unit": "TFLOP/s", "traffic": None}
    roof["frac"] = roof["achieved"] / roof["peak"]
    config = {"workload": "shapes: relu(A x B + bias), fp32, the contraction shapes of c2 and c5, one barrier per product"}
    return dt, "f32", config, roof, {"shapes": table}, None


WORKLOADS = {"c1": run_c1, "c2": run_c2, "c3": run_c3, "c4": run_c4, "c5": run_c5, "shapes": run_shapes}


def _build_if_nothing_is_built():
    """liblt.so and the recording extension are loaded as built; only a tree without them is built
    here (in a process of its own, before the package is imported)."""
    pkg = os.path.join(ROOT, "paper_2102_13267_amd")
    have = os.path.exists(os.path.join(pkg, "liblt.so")) and any(f.startswith("_ltrec") and f.endswith(".so") for f in os.listdir(pkg))
    if not have:
        import subprocess
        subprocess.run([sys.executable, "-m", "paper_2102_13267_amd.build"], cwd=ROOT, check=True, stdout=sys.stderr)


def main():
    _build_if_nothing_is_built()
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default=None, choices=sorted(WORKLOADS),
                    help="default: c4 as the headline line, plus a short run of every other config under detail.other_configs")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--streams", type=int, default=4,
                    help="streams a barrier may spread independent launches over (1: all on one stream)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy, so that a rocprofv3 --pmc run of this command "
                         "holds a kernel of known HBM traffic to scale FETCH_SIZE / WRITE_SIZE by")
    ap.add_argument("--no-streaming-run", action="store_true",
                    help="c1: leave out the extra run of the trace on [16384, 16384] operands (a kernel trace of "
                         "the command then holds the configured size only)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU; --gpus must be 1 "
              "(the path would shard by parameter range / batch: every replica records the same trace)", file=sys.stderr)
        sys.exit(2)
    global _STREAMS, _C1_STREAMING_RUN
    _STREAMS = args.streams
    _C1_STREAMING_RUN = not args.no_streaming_run
    defaults = {"c4": (20, 3), "c1": (200, 10), "c2": (200, 10), "c3": (10, 2), "c5": (200, 0), "shapes": (20, 3)}
    headline = args.workload or "c4"
    steps = args.steps if args.steps is not None else defaults[headline][0]
    warmup = args.warmup if args.warmup is not None else defaults[headline][1]
    if args.copy_calibration:
        import torch
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    dt, dtype, config, roof, extra, cpu = WORKLOADS[headline](steps, warmup)
    line = {
        "metric": "barrier-steps/sec", "value": steps / dt, "unit": "steps/s", "n_gpus": 1, "steps": steps,
        "warmup": warmup, "ms_per_step": dt / steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": dtype, "data": "synthetic", "config": config, "roofline": roof,
    }
    if cpu is not None and not args.no_cpu:
        v, sample = cpu()
        line["cpu_baseline"] = {"value": v, "unit": "steps/s", "cores": os.cpu_count(), "kind": "oracle", "sample": sample}
    line["detail"] = extra
    if args.workload is None:
        # the other configurations, each a short run of its own (parity is the tests' business;
        # these are the rates and roofline fractions the design notes quote)
        others = {}
        for w in ("c1", "c2", "c3", "c5"):
            import gc
            gc.collect()
            st, wu = defaults[w]
            odt, odtype, oconfig, oroof, oextra, _ = WORKLOADS[w](st, wu)
            others[w] = {"value": st / odt, "unit": "steps/s", "ms_per_step": odt / st * 1e3, "steps": st, "dtype": odtype,
                         "workload": oconfig["workload"], "roofline": oroof,
                         "detail": {k: v for k, v in oextra.items() if k not in ("kernels", "plan")}}
        line["detail"]["other_configs"] = others
    print(json.dumps(line))


if __name__ == "__main__":
    main()
