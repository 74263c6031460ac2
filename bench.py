#!/usr/bin/env python3
"""Benchmark of the AoT multi-stream DAG executor on one MI355X.

One "step" = one replay of the whole recorded DAG (every task of the workload) on an
input that already sits in the arena, followed by a wait for its completion: the
batch-1 DAG latency. Prints ONE JSON line. Besides the contract fields it reports the
critical-path bound (sum of isolated kernel times along the longest path), the achieved
fraction of it, the overhead per task, the same latency in the other replay modes, a
roofline entry for the kernel that accounts for most GPU time, and the CPU oracle timed
on the host cores of the same box.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
PEAK_FP32_MFMA_TFLOPS = 157.3  # dense fp32 matrix
PEAK_FP32_VALU_TFLOPS = 157.3  # 256 CUs x 128 fp32 FMA lanes x 2 flop x 2.4 GHz

KERNEL_BOUND = {"conv1x1": "mfma", "conv3x3": "alu"}     # everything else streams memory: "hbm"


def percentile(xs, q):
    xs = sorted(xs)
    return xs[min(len(xs) - 1, int(q * len(xs)))]


def time_mode(runner, B, mode, steps, warmup):
    import torch
    B.ng_replay_mode(runner.g, mode)
    for _ in range(warmup):
        B.ng_replay(runner.g)
        B.ng_sync(runner.g)
    torch.cuda.synchronize()
    lat = []
    t_all = time.perf_counter()
    for _ in range(steps):
        t0 = time.perf_counter()
        B.ng_replay(runner.g)
        B.ng_sync(runner.g)
        lat.append((time.perf_counter() - t0) * 1e6)
    torch.cuda.synchronize()
    total = time.perf_counter() - t_all
    return total, lat


def throughput(runner, B, mode, n):
    """Back-to-back replays with one final wait (replays per second)."""
    import torch
    B.ng_replay_mode(runner.g, mode)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(n):
        B.ng_replay(runner.g)
    B.ng_sync(runner.g)
    torch.cuda.synchronize()
    return n / (time.perf_counter() - t0)


def cpu_baseline(workload, budget_s=12.0):
    """The oracle as it stands, timed on this machine's host cores on the same workload."""
    from oracle.forward import forward
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    forward(workload)                      # warm caches
    times, t_end = [], time.perf_counter() + budget_s
    while time.perf_counter() < t_end or len(times) < 2:
        t0 = time.perf_counter()
        forward(workload)
        times.append(time.perf_counter() - t0)
        if len(times) >= 50:
            break
    return {"value": min(times) * 1e6, "unit": "us", "cores": int(cores), "kind": "oracle",
            "sample": f"{len(times)} full forward passes of the same DAG (min wall time)",
            "host_cpus": os.cpu_count()}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--config", default="nasnet_style")
    ap.add_argument("--batch", type=int, default=1, help="only for inception_style")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--per-task", action="store_true", help="also print a per-kernel table to stderr")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the path has no multi-GPU part); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads
    from paper_2012_02732_amd import GraphRunner, binding as B

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    kw = {"batch": args.batch} if args.config == "inception_style" else {}
    w = workloads.make(args.config, **kw)
    runner = GraphRunner(w, "cuda:0")
    sched = runner.prepare()
    n_nodes = len(w.nodes)
    n_tasks = n_nodes - sum(nd.op == "input" for nd in w.nodes)

    # ---- timed region: K replays of the whole DAG, multi-stream graph ----------------
    total, lat = time_mode(runner, B, B.NG_MODE_GRAPH_MULTI, args.steps, args.warmup)
    ms_per_step = total / args.steps * 1e3
    t_e2e = statistics.median(lat)

    # ---- isolated kernel times -> critical path ----------------------------------------
    reps = 30 if n_tasks > 150 else 100
    t_iso = [B.ng_time_task(runner.g, v, reps) for v in range(n_nodes)]
    t_cp, path = B.ng_critical_path(runner.g, t_iso)
    cp_tasks = sum(1 for v in path if t_iso[v] > 0)

    # ---- other replay modes (shorter runs) -----------------------------------------------
    k2 = max(20, args.steps // 5)
    modes = {}
    for name, mode in (("graph_single", B.NG_MODE_GRAPH_SINGLE), ("eager_single", B.NG_MODE_EAGER_SINGLE),
                       ("eager_multi", B.NG_MODE_EAGER_MULTI), ("device_resident", B.NG_MODE_DEVICE_RESIDENT)):
        _, l2 = time_mode(runner, B, mode, k2, 5)
        modes[name] = statistics.median(l2)
    thr = throughput(runner, B, B.NG_MODE_GRAPH_MULTI, max(50, args.steps // 2))
    B.ng_replay_mode(runner.g, B.NG_MODE_GRAPH_MULTI)

    # ---- roofline of the kernel that accounts for most isolated GPU time ------------------
    per_kernel = {}
    for v in range(n_nodes):
        name = B.ng_task_kernel(runner.g, v)
        if not name:
            continue
        nbytes, flops = B.ng_task_work(runner.g, v)
        k = per_kernel.setdefault(name, {"launches": 0, "us": 0.0, "bytes": 0.0, "flops": 0.0})
        k["launches"] += 1
        k["us"] += t_iso[v]
        k["bytes"] += nbytes
        k["flops"] += flops
    dom = max(per_kernel, key=lambda n: per_kernel[n]["us"])
    d = per_kernel[dom]
    bound = next((b for pre, b in KERNEL_BOUND.items() if dom.startswith(pre)), "hbm")
    avg_us = d["us"] / d["launches"]
    if bound == "hbm":
        achieved, peak, unit = d["bytes"] / d["launches"] / avg_us * 1e-3, PEAK_HBM_GBS, "GB/s"
    else:
        achieved = d["flops"] / d["launches"] / avg_us * 1e-6
        peak, unit = (PEAK_FP32_MFMA_TFLOPS if bound == "mfma" else PEAK_FP32_VALU_TFLOPS), "TFLOP/s"
    roofline = {"kernel": dom, "bound": bound, "achieved": achieved, "peak": peak, "unit": unit,
                "frac": achieved / peak, "traffic": None, "launches_per_step": d["launches"],
                "avg_launch_us": avg_us, "share_of_isolated_gpu_time": d["us"] / sum(t_iso)}
    if args.per_task:
        for name, k in sorted(per_kernel.items(), key=lambda kv: -kv[1]["us"]):
            print(f"{name:24s} launches {k['launches']:4d}  total {k['us']:9.1f} us  avg {k['us'] / k['launches']:7.2f} us"
                  f"  {k['bytes'] / k['us'] * 1e-3:8.1f} GB/s  {k['flops'] / k['us'] * 1e-6:8.3f} TFLOP/s", file=sys.stderr)

    out = {
        "metric": "DAG latency at batch 1 (replay + wait, input resident in HBM)",
        "value": ms_per_step * 1e3, "unit": "us",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.config + (f"_b{args.batch}" if args.config == "inception_style" else ""),
                   "input_shape": list(w.input.shape), "tasks": n_tasks, "streams": sched["n_streams"],
                   "sync_edges": sched["n_sync"], "events": sched["n_events"], "replay": "hipGraph multi-stream"},
        "latency_us": {"median": t_e2e, "p10": percentile(lat, 0.10), "p90": percentile(lat, 0.90)},
        "throughput_replays_per_s": thr,
        "critical_path": {"t_cp_us": t_cp, "tasks_on_path": cp_tasks, "sum_isolated_us": sum(t_iso),
                          "fraction_of_bound": t_cp / t_e2e,
                          "overhead_us_per_task": (t_e2e - t_cp) / max(cp_tasks, 1)},
        "other_modes_median_us": modes,
        "multi_vs_single_stream": modes["graph_single"] / t_e2e,
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
    runner.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
