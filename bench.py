#!/usr/bin/env python3
"""Benchmark of the CLT-k + low-pass error-feedback step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--select exact|chunk]
                    [--no-cpu-baseline]

A "step" is one call of scalecom_step (scalecom_step_layers for the per-layer workload): the
whole path -- accumulate, exact top-k on the cyclic leader, gather, sum over learners,
low-pass memory update -- over one batch of synthetic gradients that already sit in HBM.
Memories are carried from step to step, the leader rotates with the step index.  Memories start
at zero (Alg. 1), and the default of 300 warm-up steps takes the run into the state a training
job spends its time in: error feedback lets the magnitudes pile up just below the selection
threshold (after a few hundred steps a twelve-bit bucket of keys around it holds several per
cent of all elements), which is the hard case for finding the threshold; the first steps of a
run are the easy one.

`--select chunk` times the chunk-wise selector of the paper's own implementation (one position
per `rate` consecutive elements: scalecom_step_chunked, or scalecom_step_layers_chunked for the
per-layer workload) instead of the exact top-k.

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
    """HBM bytes per launch of the fused kernel from the committed rocprofv3 --pmc summary
    (line `traffic_bytes_per_launch[<workload>]: <number>`), or None if there is none."""
    path = os.path.join(ROOT, "profiles", "k_update_pmc.txt")
    try:
        text = open(path).read()
    except OSError:
        return None
    m = re.search(r"traffic_bytes_per_launch\[" + re.escape(workload_name) + r"\]:\s*([0-9.eE+]+)", text)
    return float(m.group(1)) if m else None


def cpu_baseline(w, select, budget_s=20.0):
    """The oracle as it stands, single thread, on host copies of the first steps' inputs."""
    import numpy as np
    import torch

    import oracle
    from paper_2104_11125_amd import workloads

    oracle.build(force=False)
    dev = torch.device("cuda:0")
    mem = [np.zeros(w.numel, np.float32) for _ in range(w.n_learners)]
    done, spent = 0, 0.0
    while done < w.steps and (done == 0 or spent + spent / done < budget_s):
        grad = []
        for g in workloads.gradients(w, done, dev):
            grad.append(g.view(torch.int16).cpu().numpy().view(np.uint16) if g.dtype == torch.bfloat16
                        else g.cpu().numpy())
        t0 = time.perf_counter()
        if select == "chunk" and w.n_tensors > 1:
            oracle.step_layers_chunked(mem, grad, w.offsets, chunk_sizes(w), w.beta, w.lr, done)
        elif select == "chunk":
            oracle.step_chunked(mem, grad, w.rate, w.beta, w.lr, done)
        elif w.n_tensors == 1:
            oracle.step(mem, grad, w.k, w.beta, w.lr, done)
        else:
            oracle.step_layers(mem, grad, w.offsets, w.ks, w.beta, w.lr, done)
        spent += time.perf_counter() - t0
        done += 1
    per_step = spent / done
    return {
        "value": w.n_learners * w.numel / per_step,
        "unit": "elements/s",
        "cores": 1,
        "kind": "oracle",
        "sample": f"first {done} step(s) of the full workload ({w.n_learners} learners x {w.numel} elements, "
                  f"k={index_set_size(w, select)}, select={select}), memory carried; {per_step * 1e3:.0f} ms/step; host has {os.cpu_count()} logical cores",
        "ms_per_step": per_step * 1e3,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=300,
                    help="untimed steps from zero memories before the timed ones (see the module docstring)")
    ap.add_argument("--workload", default="resnet50_sized")
    ap.add_argument("--select", choices=["exact", "chunk"], default="exact")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--pool", type=int, default=7,
                    help="distinct gradient batches kept in HBM and cycled (lowered until it has no common "
                         "factor with the learner count, so that no learner leads on the same batch every time)")
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
    w = workloads.by_name(args.workload)
    k = index_set_size(w, args.select)
    gd = torch.bfloat16 if w.grad_dtype == "bf16" else torch.float32
    ctx = binding.scalecom_init(w.numel, w.n_learners, gd, w.n_tensors, dev, k_max=k)

    # inputs resident in HBM before the timed region: a pool of gradient batches, zero memories
    gbytes = w.n_learners * w.numel * (2 if w.grad_dtype == "bf16" else 4)
    pool_n = max(1, min(args.pool, args.steps + args.warmup, int(100e9 // gbytes)))
    while pool_n > 1 and math.gcd(pool_n, w.n_learners) != 1:
        pool_n -= 1
    pool = [workloads.gradients(w, t, dev) for t in range(pool_n)]
    mem = workloads.zero_memories(w, dev)
    idx = torch.empty(k, dtype=torch.int32, device=dev)
    red = torch.empty(k, dtype=torch.float32, device=dev)

    def one_step(t):
        g = pool[t % pool_n]
        if args.select == "chunk" and w.n_tensors > 1:
            ctx.scalecom_step_layers_chunked(mem, g, w.offsets, chunk_sizes(w), w.beta, w.lr, t, idx, red)
        elif args.select == "chunk":
            ctx.scalecom_step_chunked(mem, g, w.rate, w.beta, w.lr, t, idx, red)
        elif w.n_tensors == 1:
            ctx.scalecom_step(mem, g, w.k, w.beta, w.lr, t, idx, red)
        else:
            ctx.scalecom_step_layers(mem, g, w.offsets, w.ks, w.beta, w.lr, t, idx, red)

    for t in range(args.warmup):
        one_step(t)
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
    # outside the timed region: a few more steps with an event at every phase boundary
    extra = min(args.steps, 10)
    ctx.scalecom_timing_begin(extra, all_phases=True)
    for t in range(args.warmup + args.steps, args.warmup + args.steps + extra):
        one_step(t)
    phases = ctx.scalecom_timing_read(extra)

    ms_per_step = elapsed / args.steps * 1e3
    elements = w.n_learners * w.numel
    fused_bytes, step_bytes = algorithmic_bytes(w, k)
    n_ph = len(phases)
    phase_avg = [sum(p[j] for p in phases) / n_ph for j in range(binding.SCALECOM_N_PHASES)] if n_ph else None
    fused_ms = sum(p[3] for p in timed) / len(timed) if timed else None      # phase 3 = the all-learner pass k_update
    achieved = fused_bytes / (fused_ms * 1e-3) / 1e9 if fused_ms else None

    # practical ceiling: the library's plain copy kernel over 1 GiB (read + write)
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
    del src, dst

    out = {
        "metric": "clt_k_gradient_elements_per_s",
        "value": elements / (ms_per_step * 1e-3),
        "unit": "elements/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": w.name, "select": args.select, "n_learners": w.n_learners, "numel": w.numel, "k": k,
            "grad_dtype": w.grad_dtype,
            "n_tensors": w.n_tensors, "beta": w.beta, "lr": w.lr, "gradient_pool": pool_n,
        },
        "roofline": {
            "bound": "hbm",
            "kernel": "k_update",
            "achieved": achieved,
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBPS if achieved else None,
            "traffic": recorded_traffic(w.name) if args.select == "exact" else None,
            "algorithmic_bytes_per_launch": fused_bytes,
            "avg_launch_ms": fused_ms,
            "launches_timed": len(timed),
            # the pass goes over 8 learners per kernel launch; with more learners the figures above are
            # those of one step's launches together
            "kernel_launches_per_pass": -(-w.n_learners // 8),
        },
        "step_roofline": {
            "algorithmic_bytes_per_step": step_bytes,
            "achieved_GBps": step_bytes / (ms_per_step * 1e-3) / 1e9,
            "frac_of_peak": step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS,
            "copy_kernel_GBps": copy_gbps,
            "frac_of_copy_kernel": step_bytes / (ms_per_step * 1e-3) / 1e9 / copy_gbps,
            # the extra steps after the timed region, each bracketed by HIP events at every phase boundary
            # (the events themselves add a few microseconds per boundary)
            "event_timed_extra_steps_ms": [sum(p) for p in phases] if n_ph else None,
            "event_timed_extra_steps_median_ms": sorted(sum(p) for p in phases)[n_ph // 2] if n_ph else None,
            "phase_ms_untimed_extra_steps": dict(zip(["leader_first_look", "refine", "counts_scan_slots", "update", "reduce"], phase_avg)) if phase_avg else None,
        },
    }
    if not args.no_cpu_baseline:
        del pool
        torch.cuda.empty_cache()
        out["cpu_baseline"] = cpu_baseline(w, args.select)
    ctx.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
