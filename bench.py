#!/usr/bin/env python3
"""Benchmark of the CLT-k + low-pass error-feedback step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--select exact|chunk]
                    [--no-per-config] [--no-cpu-baseline]

A "step" is one call of scalecom_step (scalecom_step_layers for the per-layer workload): the
whole path -- accumulate, exact top-k on the cyclic leader, gather, sum over learners,
low-pass memory update -- over one batch of synthetic gradients that already sit in HBM.
Memories are carried from step to step, the leader rotates with the step index.  Memories start
at zero (Alg. 1), and the default of 300 warm-up steps takes the run into the state a training
job spends its time in: error feedback lets the magnitudes pile up just below the selection
threshold (after a few hundred steps a twelve-bit bucket of keys around it holds several per
cent of all elements), which is the hard case for finding the threshold; the first steps of a
run are the easy one.

The headline (`value`, `config`, `roofline`, `cpu_baseline`) is the largest configuration,
large_bf16: 8 learners x 10^9 elements, bfloat16 gradients.  `per_config` holds all five
configurations measured in the same process with the same --steps and --warmup: time per step,
elements per second, the step's and the dominant kernel's fraction of the HBM peak, how many of
the timed steps missed their threshold prediction, and the CPU oracle's rate on a bounded
sample; for the launch-bound tiny configuration also the time per step of a captured HIP graph.

`--select chunk` times the chunk-wise selector of the paper's own implementation (one position
per `rate` consecutive elements) instead of the exact top-k.

Prints ONE JSON line.  `value` is gradient elements per second (n_learners * numel / step
time).  `roofline` is for the dominant kernel (the all-learner pass k_update), timed with HIP
events recorded by the library on its own stream inside the timed region.  `cpu_baseline` is
the single-threaded CPU oracle on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth
HEADLINE = "large_bf16"         # the largest single-GPU configuration
TRAFFIC_FILE = os.path.join("profiles", "k_update_pmc.txt")


def chunk_sizes(w):
    """Chunk-wise selector: the workload's compression rate as the chunk size of every tensor."""
    return [w.rate] * w.n_tensors


def index_set_size(w, select):
    if select == "exact":
        return w.k
    if w.n_tensors == 1:
        return -(-w.numel // w.rate)
    return sum(-(-(b - a) // w.rate) for a, b in zip(w.offsets[:-1], w.offsets[1:]))


def algorithmic_bytes(w, k):
    """Bytes one step must move: read every learner's mem and grad,
    write every mem, one extra look at the leader's (mem, grad) to find the threshold, write
    idx + reduced values."""
    gb = 2 if w.grad_dtype == "bf16" else 4
    n, N = w.n_learners, w.numel
    update = n * N * (4 + gb) + n * N * 4 + k * 8      # the all-learner pass (k_update) and its outputs
    leader = N * (4 + gb)
    return update, update + leader


def recorded_traffic(workload_name):
    """HBM bytes of one all-learner pass (every k_update dispatch of a step together) from the
    committed rocprofv3 --pmc summary (line `traffic_bytes_per_pass[<workload>]: <number>`), or
    None if there is none.  Recorded by an earlier profiler run, not measured by this one."""
    try:
        text = open(os.path.join(ROOT, TRAFFIC_FILE)).read()
    except OSError:
        return None
    m = re.search(r"traffic_bytes_per_pass\[" + re.escape(workload_name) + r"\]:\s*([0-9.eE+]+)", text)
    return float(m.group(1)) if m else None


def _to_host(t):
    import numpy as np
    import torch
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def cpu_oracle_sample(w, select):
    """The oracle as it stands, one thread, on a bounded sample of the workload's first step (zero
    memories; its time per step does not depend on the state).  Whole vectors: the oracle's own
    primitives on the leader (accumulate, selection, gather, memory update) and on ONE other
    learner (accumulate, gather, memory update), scaled to all learners.  Per-tensor workload:
    one whole oracle step."""
    import numpy as np
    import torch

    import oracle
    from paper_2104_11125_amd import workloads

    oracle.build(force=False)
    dev = torch.device("cuda:0")
    n = w.n_learners
    if w.n_tensors > 1:
        grad = [_to_host(g) for g in workloads.gradients(w, 0, dev)]
        mem = [np.zeros(w.numel, np.float32) for _ in range(n)]
        t0 = time.perf_counter()
        if select == "chunk":
            oracle.step_layers_chunked(mem, grad, w.offsets, chunk_sizes(w), w.beta, w.lr, 0)
        else:
            oracle.step_layers(mem, grad, w.offsets, w.ks, w.beta, w.lr, 0)
        per_step = time.perf_counter() - t0
        sample = "one whole oracle step (all learners, all tensors)"
    else:
        shared = workloads.shared_component(w, 0, dev)
        times = []
        idx = None
        vals = []
        for i in (0, 1 % n):                                # the leader of step 0, then one other learner
            g = _to_host(workloads.learner_gradient(w, 0, i, dev, shared=shared))
            m = np.zeros(w.numel, np.float32)
            t0 = time.perf_counter()
            acc = oracle.accumulate(m, g, w.lr)
            if idx is None:
                idx = oracle.chunk_select(acc, w.rate) if select == "chunk" else oracle.topk_select(acc, w.k)
            vals.append(oracle.gather(acc, idx))
            oracle.memory_update(m, acc, idx, w.beta)
            times.append(time.perf_counter() - t0)
            del acc, m, g
            if n == 1:
                break
        t0 = time.perf_counter()
        oracle.reduce(vals)
        t_reduce = (time.perf_counter() - t0) / len(vals)
        del shared
        other = times[1] if len(times) > 1 else 0.0
        per_step = times[0] + (n - 1) * other + n * t_reduce
        sample = (f"the oracle's primitives on the leader ({times[0]:.2f} s with the selection) and on one other learner "
                  f"({other:.2f} s), scaled to {n} learners")
    return {
        "value": n * w.numel / per_step,
        "unit": "elements/s",
        "cores": 1,
        "kind": "oracle",
        "sample": f"first step of the full workload ({n} learners x {w.numel} elements, k={index_set_size(w, select)}, "
                  f"select={select}): {sample}; {per_step * 1e3:.0f} ms/step; host has {os.cpu_count()} logical cores",
        "ms_per_step": per_step * 1e3,
    }


def graph_replay_ms(w, select, pool, dev, replays=50):
    """Time per step of a captured cycle of n_learners steps (one per leader), replayed: what the
    launch-bound small configuration costs without the host's launch overhead in between."""
    import torch

    from paper_2104_11125_amd import binding

    k = index_set_size(w, select)
    side = torch.cuda.Stream(device=dev)
    n = w.n_learners
    with torch.cuda.stream(side):
        ctx = binding.scalecom_init(w.numel, n, torch.float32 if w.grad_dtype != "bf16" else torch.bfloat16, w.n_tensors,
                                    dev, stream=side, k_max=k)
        mem = [torch.zeros(w.numel, device=dev) for _ in range(n)]
        idx = torch.empty(k, dtype=torch.int32, device=dev)
        red = torch.empty(k, dtype=torch.float32, device=dev)

        def cycle(first):
            for j in range(n):
                t = first + j
                if w.n_tensors == 1:
                    ctx.scalecom_step(mem, pool[t % len(pool)], w.k, w.beta, w.lr, t, idx, red)
                else:
                    ctx.scalecom_step_layers(mem, pool[t % len(pool)], w.offsets, w.ks, w.beta, w.lr, t, idx, red)
        for c in range(10):
            cycle(c * n)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        cycle(10 * n)
    for _ in range(5):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(replays):
        graph.replay()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / (replays * n) * 1e3
    ctx.close()
    return ms


def measure(w, args, dev, with_phases):
    """Warm-up, then the timed steps of one workload; everything the JSON line says about it."""
    import torch

    from paper_2104_11125_amd import binding, workloads

    select = args.select
    k = index_set_size(w, select)
    gd = torch.bfloat16 if w.grad_dtype == "bf16" else torch.float32
    ctx = binding.scalecom_init(w.numel, w.n_learners, gd, w.n_tensors, dev, k_max=k)

    # inputs resident in HBM before the timed region: a pool of gradient batches, zero memories
    gbytes = w.n_learners * w.numel * (2 if w.grad_dtype == "bf16" else 4)
    pool_n = max(1, min(args.pool, args.steps + args.warmup, int(150e9 // gbytes)))
    while pool_n > 1 and math.gcd(pool_n, w.n_learners) != 1:
        pool_n -= 1
    pool = [workloads.gradients(w, t, dev) for t in range(pool_n)]
    mem = workloads.zero_memories(w, dev)
    idx = torch.empty(k, dtype=torch.int32, device=dev)
    red = torch.empty(k, dtype=torch.float32, device=dev)

    def one_step(t):
        g = pool[t % pool_n]
        if select == "chunk" and w.n_tensors > 1:
            ctx.scalecom_step_layers_chunked(mem, g, w.offsets, chunk_sizes(w), w.beta, w.lr, t, idx, red)
        elif select == "chunk":
            ctx.scalecom_step_chunked(mem, g, w.rate, w.beta, w.lr, t, idx, red)
        elif w.n_tensors == 1:
            ctx.scalecom_step(mem, g, w.k, w.beta, w.lr, t, idx, red)
        else:
            ctx.scalecom_step_layers(mem, g, w.offsets, w.ks, w.beta, w.lr, t, idx, red)

    for t in range(args.warmup):
        one_step(t)
    warm_stats = ctx.scalecom_selection_stats(reset=True)       # (waits for the stream)
    torch.cuda.synchronize()
    # HIP events around the dominant kernel only, on every 4th step: an event pair costs the
    # stream about 10 us, which the timed region should not carry on every step
    sample_every = 4 if args.steps >= 8 else 1
    ctx.scalecom_timing_begin(args.steps, every=sample_every)
    t0 = time.perf_counter()
    for t in range(args.warmup, args.warmup + args.steps):
        one_step(t)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    timed = ctx.scalecom_timing_read(args.steps)
    stats = ctx.scalecom_selection_stats()
    phases = []
    if with_phases:
        # outside the timed region: a few more steps with an event at every phase boundary
        extra = min(args.steps, 10)
        ctx.scalecom_timing_begin(extra, all_phases=True)
        for t in range(args.warmup + args.steps, args.warmup + args.steps + extra):
            one_step(t)
        phases = ctx.scalecom_timing_read(extra)

    ms_per_step = elapsed / args.steps * 1e3
    fused_bytes, step_bytes = algorithmic_bytes(w, k)
    fused_ms = sum(p[3] for p in timed) / len(timed) if timed else None      # phase 3 = the all-learner pass k_update
    achieved = fused_bytes / (fused_ms * 1e-3) / 1e9 if fused_ms else None
    res = {
        "w": w, "k": k, "pool_n": pool_n, "ms_per_step": ms_per_step, "fused_bytes": fused_bytes,
        "step_bytes": step_bytes, "fused_ms": fused_ms, "achieved": achieved, "launches_timed": len(timed),
        "phases": phases, "stats": stats, "warm_stats": warm_stats,
        "graph_ms": None,
    }
    ctx.close()
    if w.name == "tiny" and select == "exact":
        res["graph_ms"] = graph_replay_ms(w, select, pool, dev)
    del pool, mem, idx, red
    torch.cuda.empty_cache()
    return res


def config_entry(r, n_tensor_steps):
    w = r["w"]
    step_gbps = r["step_bytes"] / (r["ms_per_step"] * 1e-3) / 1e9
    e = {
        "workload": w.name, "n_learners": w.n_learners, "numel": w.numel, "k": r["k"], "grad_dtype": w.grad_dtype,
        "n_tensors": w.n_tensors,
        "ms_per_step": r["ms_per_step"],
        "elements_per_s": w.n_learners * w.numel / (r["ms_per_step"] * 1e-3),
        "algorithmic_bytes_per_step": r["step_bytes"],
        "step_frac_of_hbm_peak": step_gbps / HBM_PEAK_GBPS,
        "k_update_avg_ms": r["fused_ms"],
        "k_update_frac_of_hbm_peak": r["achieved"] / HBM_PEAK_GBPS if r["achieved"] else None,
        "timed_steps": int(r["stats"]["steps"]),
        # of the timed steps' (step, tensor) selections: threshold outside the expected range (two more
        # leader passes), no expectation yet, refinement by full passes, wide range (one more list pass)
        "selections": n_tensor_steps,
        "selection_misses": int(r["stats"]["missed"]),
        "selection_no_prediction": int(r["stats"]["no_prediction"]),
        "selection_full_mode": int(r["stats"]["full_mode"]),
        "selection_wide_range": int(r["stats"]["wide_range"]),
        "warmup_selection_misses": int(r["warm_stats"]["missed"]),
    }
    if r["graph_ms"] is not None:
        e["graph_replay_ms_per_step"] = r["graph_ms"]
    return e


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=300,
                    help="untimed steps from zero memories before the timed ones (see the module docstring)")
    ap.add_argument("--workload", default=HEADLINE, help="the configuration the headline figures are for")
    ap.add_argument("--select", choices=["exact", "chunk"], default="exact")
    ap.add_argument("--no-per-config", action="store_true", help="measure the headline workload only")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--pool", type=int, default=32,
                    help="distinct gradient batches kept in HBM and cycled, standing in for fresh draws every step "
                         "(at most 150 GB of them; lowered until the number has no common factor with the learner "
                         "count, so that no learner leads on the same batch every time)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (all learners are buffers on one MI355X); "
              "--gpus > 1 is not supported", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2104_11125_amd import binding, workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")
    head_w = workloads.by_name(args.workload)
    results = {}
    order = [head_w] + ([] if args.no_per_config else [w for w in workloads.configs() if w.name != head_w.name])
    for w in order:
        print(f"[bench] {w.name}: {w.n_learners} learners x {w.numel} elements, {args.warmup} + {args.steps} steps",
              file=sys.stderr, flush=True)
        results[w.name] = measure(w, args, dev, with_phases=w.name == head_w.name)
    r = results[head_w.name]
    w, k = head_w, r["k"]
    ms_per_step = r["ms_per_step"]
    phases = r["phases"]
    n_ph = len(phases)
    phase_avg = [sum(p[j] for p in phases) / n_ph for j in range(binding.SCALECOM_N_PHASES)] if n_ph else None

    # practical ceiling: the library's plain copy kernel over 1 GiB (read + write)
    ctx = binding.scalecom_init(1024, 1, torch.float32, 1, dev, k_max=1)
    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    for _ in range(2):
        ctx.scalecom_stream_copy(dst, src)
    torch.cuda.synchronize()
    c0 = time.perf_counter()
    for _ in range(10):
        ctx.scalecom_stream_copy(dst, src)
    torch.cuda.synchronize()
    copy_gbps = 10 * 2 * (1 << 30) / (time.perf_counter() - c0) / 1e9
    # what one more dependent launch costs the stream when nothing watches it: the 1 GiB copy followed by 0 or 16
    # copies of 16 bytes (the same kernel with one block), 20 times each way.  A kernel trace of this very command
    # shows the 16-byte copies at about 4.5 us each: the profiler's own share of every dispatch.
    def copies_with_small(n_small):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(20):
            ctx.scalecom_stream_copy(dst, src)
            for _ in range(n_small):
                ctx.scalecom_stream_copy(dst[:16], src[:16])
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / 20
    copies_with_small(16)
    launch_us = (copies_with_small(16) - copies_with_small(0)) / 16 * 1e6
    del src, dst
    ctx.close()
    torch.cuda.empty_cache()

    step_gbps = r["step_bytes"] / (ms_per_step * 1e-3) / 1e9
    traffic = recorded_traffic(w.name) if args.select == "exact" else None
    out = {
        "metric": "clt_k_gradient_elements_per_s",
        "value": w.n_learners * w.numel / (ms_per_step * 1e-3),
        "unit": "elements/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",                     # the path computes in binary32 whatever the gradients are stored as
        "data": "synthetic",
        "config": {
            "workload": w.name, "select": args.select, "n_learners": w.n_learners, "numel": w.numel, "k": k,
            "grad_dtype": w.grad_dtype,
            "n_tensors": w.n_tensors, "beta": w.beta, "lr": w.lr, "gradient_pool": r["pool_n"],
        },
        "timed_steps": int(r["stats"]["steps"]),
        "selection_misses": int(r["stats"]["missed"]),
        "roofline": {
            "bound": "hbm",
            "kernel": "k_update",
            "achieved": r["achieved"],
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": r["achieved"] / HBM_PEAK_GBPS if r["achieved"] else None,
            # HBM bytes of one pass by the profiler's counters, recorded in an earlier run of the same
            # command under rocprofv3 --pmc and read from the file named below; not measured by this run
            "traffic": traffic,
            "traffic_recorded_from": TRAFFIC_FILE if traffic is not None else None,
            "algorithmic_bytes_per_launch": r["fused_bytes"],
            "avg_launch_ms": r["fused_ms"],
            "launches_timed": r["launches_timed"],
            # the pass goes over 8 learners per kernel launch; with more learners the figures above (bytes,
            # duration, traffic) are those of one step's launches together
            "kernel_launches_per_pass": -(-w.n_learners // 8),
        },
        "step_roofline": {
            "algorithmic_bytes_per_step": r["step_bytes"],
            "achieved_GBps": step_gbps,
            "frac_of_peak": step_gbps / HBM_PEAK_GBPS,
            "copy_kernel_GBps": copy_gbps,
            "frac_of_copy_kernel": step_gbps / copy_gbps,
            "dependent_launch_us": launch_us,
            # the extra steps after the timed region, each bracketed by HIP events at every phase boundary
            # (the events themselves add a few microseconds per boundary)
            "event_timed_extra_steps_median_ms": sorted(sum(p) for p in phases)[n_ph // 2] if n_ph else None,
            "phase_ms_untimed_extra_steps": dict(zip(["leader_first_look", "refine", "counts_scan_slots", "update", "reduce"], phase_avg)) if phase_avg else None,
        },
    }
    entries = []
    for cw in workloads.configs():
        if cw.name not in results:
            continue
        e = config_entry(results[cw.name], int(results[cw.name]["stats"]["steps"]) * cw.n_tensors)
        if not args.no_cpu_baseline:
            print(f"[bench] CPU oracle sample of {cw.name}", file=sys.stderr, flush=True)
            base = cpu_oracle_sample(cw, args.select)
            e["cpu_oracle"] = {"elements_per_s": base["value"], "ms_per_step": base["ms_per_step"], "cores": 1,
                               "sample": base["sample"]}
            if cw.name == w.name:
                out["cpu_baseline"] = base
        entries.append(e)
    if not args.no_per_config:
        out["per_config"] = entries
    elif not args.no_cpu_baseline and "cpu_baseline" not in out:
        out["cpu_baseline"] = cpu_oracle_sample(w, args.select)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
