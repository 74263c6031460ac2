#!/usr/bin/env python3
"""Benchmark of the AoT multi-stream DAG executor on one MI355X.

One "step" = one replay of the whole recorded DAG (every task of the workload) on an
input that already sits in the arena, followed by a wait for its completion: the batch-1
DAG latency. The timed region uses the replay mode the library itself found fastest for this DAG in its
trial at capture time (for the NAS-cell workload that is the device-resident mode: one
launch, persistent workgroups walk the recorded schedule); the other modes are timed
afterwards for comparison. Prints ONE JSON line with the
contract fields plus: the critical-path bound (isolated kernel times summed along the
longest path) and the achieved fraction of it, the overhead per task, the other modes, a
roofline entry for the kernel that carries the replay, and the CPU oracle timed on the
host cores of the same box.
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

# HBM bytes of one device-resident replay, from two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE)
# scaled by what the same counters read for a plain 256 MiB copy (2.00 and 1.00): the
# summary with the commands is profiles/resident_kernel_nasnet_style.md.
MEASURED_TRAFFIC_BYTES = {("nasnet_style", "device_resident"): (29251.4 * 2.00 + 43548.7 * 1.00) * 1024}

MODES = {"graph_multi": 0, "graph_single": 1, "eager_single": 2, "eager_multi": 3, "device_resident": 4}
MODE_NAMES = {v: k for k, v in MODES.items()}


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
    ap.add_argument("--mode", default="auto", choices=sorted(MODES) + ["auto"],
                    help="auto = the mode the library's own trial at capture time found fastest")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-modes", action="store_true")
    ap.add_argument("--per-task", action="store_true", help="also print a per-kernel table to stderr")
    ap.add_argument("--timeline", action="store_true",
                    help="device-resident mode: print how many tasks execute at the same time during one traced replay (stderr)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 256 MiB device copy (scale reference for HBM traffic counters)")
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
    auto_mode, auto_trial = B.ng_auto_mode(runner.g)
    if args.mode == "auto":
        args.mode = MODE_NAMES[auto_mode]
    mode = MODES[args.mode]

    if args.copy_probe:
        src = torch.ones(64 << 20, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- timed region: K replays of the whole DAG -----------------------------------------
    total, lat = time_mode(runner, B, mode, args.steps, args.warmup)
    ms_per_step = total / args.steps * 1e3
    t_e2e = statistics.median(lat)
    dev_us = B.ng_time_replay(runner.g, min(args.steps, 200))      # HIP events on the replay's own stream
    thr = throughput(runner, B, mode, max(50, args.steps // 2))

    # ---- isolated kernel times -> critical path ----------------------------------------------
    reps = 20 if n_tasks > 150 else 50
    c_empty = B.ng_time_chain(runner.g, -1, 200)
    c_raw = [B.ng_time_chain(runner.g, v, reps) for v in range(n_nodes)]
    t_iso = [B.ng_time_task(runner.g, v, reps) for v in range(n_nodes)]
    t_cp, path = B.ng_critical_path(runner.g, t_iso)
    t_cp_hi, _ = B.ng_critical_path(runner.g, c_raw)
    t_cp_lo, _ = B.ng_critical_path(runner.g, [max(c - c_empty, 0.0) if c > 0 else 0.0 for c in c_raw])
    cp_tasks = sum(1 for v in path if t_iso[v] > 0)

    # ---- the other replay modes (shorter runs) -----------------------------------------------
    modes = {args.mode: t_e2e}
    if not args.no_other_modes:
        k2 = max(20, args.steps // 5)
        for name, m in MODES.items():
            if name != args.mode:
                modes[name] = statistics.median(time_mode(runner, B, m, k2, 5)[1])
    B.ng_replay_mode(runner.g, mode)

    # ---- roofline of the kernel that carries the replay ----------------------------------------
    per_kernel = {}
    all_bytes = all_flops = 0.0
    for v in range(n_nodes):
        name = B.ng_task_kernel(runner.g, v)
        if not name:
            continue
        nbytes, flops = B.ng_task_work(runner.g, v)
        all_bytes += nbytes
        all_flops += flops
        k = per_kernel.setdefault(name, {"launches": 0, "us": 0.0, "bytes": 0.0, "flops": 0.0})
        k["launches"] += 1
        k["us"] += t_iso[v]
        k["bytes"] += nbytes
        k["flops"] += flops
    if args.mode == "device_resident":
        # one launch of resident_kernel executes every task: algorithmic bytes = sum over the tasks
        achieved = all_bytes / dev_us * 1e-3
        roofline = {"kernel": "resident_kernel", "bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS,
                    "unit": "GB/s", "frac": achieved / PEAK_HBM_GBS,
                    "traffic": MEASURED_TRAFFIC_BYTES.get((args.config, args.mode)),
                    "launches_per_step": 1, "avg_launch_us": dev_us, "algorithmic_bytes_per_launch": all_bytes,
                    "algorithmic_flops_per_launch": all_flops,
                    "note": "latency-bound by construction: the bound that matters is critical_path"}
    else:
        dom = max(per_kernel, key=lambda n: per_kernel[n]["us"])
        d = per_kernel[dom]
        avg_us = d["us"] / d["launches"]
        achieved = d["bytes"] / d["launches"] / avg_us * 1e-3
        roofline = {"kernel": dom, "bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": achieved / PEAK_HBM_GBS, "traffic": None, "launches_per_step": d["launches"],
                    "avg_launch_us": avg_us}
    if args.per_task:
        for name, k in sorted(per_kernel.items(), key=lambda kv: -kv[1]["us"]):
            print(f"{name:24s} launches {k['launches']:4d}  isolated total {k['us']:9.1f} us  avg {k['us'] / k['launches']:7.2f} us"
                  f"  {k['bytes'] / k['us'] * 1e-3:8.1f} GB/s  {k['flops'] / k['us'] * 1e-6:8.3f} TFLOP/s", file=sys.stderr)

    # ---- where the time of one device-resident replay goes (its own trace) -----------------------
    timeline = None
    if args.mode == "device_resident":
        B.ng_resident_trace(runner.g, 1)
        B.ng_replay(runner.g)
        B.ng_sync(runner.g)
        tr = B.ng_resident_trace(runner.g, 0, fetch=True)
        host_of = B.ng_resident_fusion(runner.g)
        ran = [v for v in range(n_nodes) if tr[v] is not None]
        if ran:
            v = max(ran, key=lambda u: tr[u][3])
            span = tr[v][3]
            run_us = wait_us = 0.0
            hops = 0
            while v is not None:                 # walk back along the producer that finished last
                ps = [u for u in w.nodes[v].preds if tr[u] is not None]
                u = max(ps, key=lambda q: tr[q][3]) if ps else None
                run_us += tr[v][3] - tr[v][1]
                wait_us += tr[v][1] - (tr[u][3] if u is not None else 0.0)
                hops += 1
                v = u
            if args.timeline:
                # tasks executing at the same time: a task counts from the moment its last workgroup is past
                # the wait until its last workgroup has stored its tiles
                events = []
                own = [u for u in ran if host_of[u] == -1]        # the others ran inside a producer's tiles / had nothing to do
                for u in own:
                    events.append((tr[u][1], 1))
                    events.append((tr[u][3], -1))
                events.sort()
                hist, level, last_t = {}, 0, 0.0
                for t_ev, d in events:
                    hist[level] = hist.get(level, 0.0) + (t_ev - last_t)
                    level += d
                    last_t = t_ev
                print(f"traced replay: {span:.1f} us, {len(ran)} tasks, {len(own)} of them with workgroups of their own; "
                      f"time with k of those executing:", file=sys.stderr)
                for k in sorted(hist):
                    print(f"  k = {k:2d}: {hist[k]:7.1f} us  {100 * hist[k] / span:5.1f} %", file=sys.stderr)
                busy = sum(tr[u][3] - tr[u][1] for u in own)
                print(f"  sum of task execution intervals {busy:.1f} us = {busy / span:.2f} tasks executing on average; "
                      f"no task executing (hand-overs only) {hist.get(0, 0.0):.1f} us", file=sys.stderr)
            timeline = {"traced_replay_us": span, "tasks_on_realised_chain": hops, "tile_execution_us": run_us,
                        "hand_over_us": wait_us,
                        "note": "one replay with per-entry clock readings (three plain stores per list entry, about 1 % slower): "
                                "tile execution = last workgroup past its wait -> last workgroup stored; hand-over = "
                                "the rest, i.e. a producer's last store -> the consumer past its wait, which includes "
                                "the consumer's input-independent prologue"}

    n_wg, n_entries, xcds, est_us = B.ng_resident_sizes(runner.g)
    fusion = B.ng_resident_fusion(runner.g)
    out = {
        "metric": "DAG latency (µs) at batch 1; % of critical-path bound; µs overhead/task",
        "metric_note": "value = wall time of the K timed steps (each: replay + wait) / K, input resident in HBM; "
                       "the other two parts of the metric are critical_path.fraction_of_bound and .overhead_us_per_task",
        "value": ms_per_step * 1e3, "unit": "us",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.config + (f"_b{args.batch}" if args.config == "inception_style" else ""),
                   "input_shape": list(w.input.shape), "tasks": n_tasks, "streams": sched["n_streams"],
                   "sync_edges": sched["n_sync"], "events": sched["n_events"], "replay": args.mode,
                   "resident_workgroups": n_wg, "resident_xcds": xcds,
                   "resident_tasks_inside_their_producer": sum(h >= 0 for h in fusion),
                   "resident_concats_in_place": sum(h == -2 for h in fusion),
                   "resident_plan_setting_kept": B.ng_resident_plan_kept(runner.g)},
        "latency_us": {"median": t_e2e, "p10": percentile(lat, 0.10), "p90": percentile(lat, 0.90),
                       "device_side": dev_us},
        "throughput_replays_per_s": thr,
        "critical_path": {"t_cp_us": t_cp, "tasks_on_path": cp_tasks, "sum_isolated_us": sum(t_iso),
                          "fraction_of_bound": t_cp / t_e2e, "fraction_of_bound_device_side": t_cp / dev_us,
                          "overhead_us_per_task": (t_e2e - t_cp) / max(cp_tasks, 1),
                          "t_cp_if_chain_time_counts_as_duration_us": t_cp_hi,
                          "t_cp_if_only_time_above_an_empty_kernel_counts_us": t_cp_lo,
                          "empty_kernel_chain_us_per_node": c_empty,
                          "planner_expected_us": est_us,
                          "tasks_on_path_without_workgroups_of_their_own": sum(fusion[v] != -1 for v in path),
                          "note": "t_cp = longest path of the DAG weighted with the isolated time of every task's "
                                  "stand-alone kernel, every task counted; in the device-resident replay some of them "
                                  "run inside their producer's tiles or have nothing to do (counted in the field above)"},
        "resident_timeline": timeline,
        "modes_median_us": modes,
        "auto_mode": {"chosen": MODE_NAMES[auto_mode], "trial_us": {MODE_NAMES[k]: v for k, v in auto_trial.items()}},
        "roofline": roofline,
    }
    if "graph_single" in modes and "graph_multi" in modes:
        out["graph_multi_vs_single_stream"] = modes["graph_single"] / modes["graph_multi"]
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
    runner.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
