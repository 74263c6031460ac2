#!/usr/bin/env python3
"""Benchmark of the AoT multi-stream DAG executor on one MI355X.

One "step" = one replay of the whole recorded DAG (every task of the workload) on an input that
already sits in the arena, followed by a wait for its completion: the DAG latency. The timed
region uses the replay mode the library itself found fastest for the DAG in its trial at capture
time (NG_MODE_AUTO). Prints ONE JSON line: the contract fields for the headline workload
(nasnet_style, batch 1) and, under "configs", the same measurements for all five configurations
and for inception_style at batch 32 (the paper's Table 1 compares multi- and single-stream replay
per network). Per configuration:

  * latency of replay + wait (median, p10, p90), device-side time, throughput;
  * the critical-path time of Section 3 in two forms - `all_tasks`: longest path of the DAG weighted
    with the isolated time of every task's own kernel; `as_executed`: weighted with the isolated time
    of the kernels the chosen replay mode really runs (fused variants timed as themselves, tasks
    without a kernel of their own weigh 0) - and the fraction of the replay latency each one is;
  * isolated time = time the GPU is busy with the kernel when it runs alone, by the device's own
    clock read inside the kernel (ng_time_task_device); the headline workload also gets the two
    estimates from chains of dependent launches as a cross-check;
  * the multi-stream and single-stream HIP graphs and their ratio;
  * a roofline entry for the kernel that dominates the replay.

Other uses:
  bench.py --config C --solo-launches R --sidecar F    launches every task's kernel R times by itself
        (to be run under `rocprofv3 --kernel-trace`), writes what it launched to F;
  bench.py --dispatch-trace kernel_trace.csv --sidecar F   no GPU: critical path from the trace's
        begin-to-end dispatch timestamps.
  bench.py --config C --mode graph_multi --replay-only N   N replays between two markers (under
        `rocprofv3 --kernel-trace`); bench.py --overlap-trace kernel_trace.csv --replay-only N   no GPU:
        how many kernels execute at the same time and the idle gaps between them.
"""
from __future__ import annotations

import argparse
import csv
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
PEAK_MFMA_F32_TFLOPS = 157.3   # MI355X fp32 matrix
RIDGE_FLOP_PER_BYTE = PEAK_MFMA_F32_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9)

# HBM bytes of one launch of the dominant kernel, from two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE; KiB
# per dispatch) scaled by what the same counters read for a plain 256 MiB copy (2.00 and 1.00). Key:
# (workload, kernel). The summaries with the commands are under profiles/.
MEASURED_TRAFFIC_BYTES = {("nasnet_style", "resident_kernel"): (29281.7 * 2.00 + 43689.1 * 1.00) * 1024}   # profiles/resident_kernel_nasnet_style.md

MODES = {"graph_multi": 0, "graph_single": 1, "eager_single": 2, "eager_multi": 3, "device_resident": 4}
MODE_NAMES = {v: k for k, v in MODES.items()}
ALL_CONFIGS = [("tiny_cell", 1), ("chain50", 1), ("random200", 1), ("nasnet_style", 1), ("inception_style", 1), ("inception_style", 32),
               ("nas_cell_cifar_training", 32)]
HEADLINE = ("nasnet_style", 1)


def label(name, batch):
    return name + (f"_b{batch}" if name in ("inception_style", "nas_cell_cifar_training") else "")


def make_workload(name, batch):
    import numpy as np
    import workloads
    if name == "nas_cell_cifar_training":
        # one training iteration (forward, backward, SGD) of the NAS-cell network on CIFAR-sized inputs, the paper's
        # training setting (Section 5); dL/dlogits is a fixed random seed tensor, the step size is tiny so that
        # thousands of timed steps do not drift the weights away
        fwd = workloads.nas_cell_cifar(batch=batch)
        out = fwd.outputs[0]
        seed = (np.random.default_rng(0).standard_normal(fwd.nodes[out].shape) / batch).astype(np.float32)
        return workloads.training_graph(fwd, 1e-6, {out: seed})
    kw = {"batch": batch} if name == "inception_style" else {}
    return workloads.make(name, **kw)


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


def longest_path(preds, weight):
    """Longest path of a DAG whose ids are a topological order: (total, [ids])."""
    n = len(preds)
    best, came = [0.0] * n, [-1] * n
    for v in range(n):
        b = 0.0
        for u in preds[v]:
            if came[v] < 0 or best[u] > b:
                b, came[v] = best[u], u
        best[v] = b + weight[v]
    v = max(range(n), key=lambda i: best[i])
    total, path = best[v], []
    while v >= 0:
        path.append(v)
        v = came[v]
    return total, path[::-1]


def resident_timeline(runner, B, w, n_nodes, verbose):
    """Where the time of one device-resident replay goes, from its own trace."""
    B.ng_resident_trace(runner.g, 1)
    B.ng_replay(runner.g)
    B.ng_sync(runner.g)
    tr = B.ng_resident_trace(runner.g, 0, fetch=True)
    host_of = B.ng_resident_fusion(runner.g)
    ran = [v for v in range(n_nodes) if tr[v] is not None]
    if not ran:
        return None
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
    # tasks executing at the same time: a task counts from the moment its last workgroup is past the wait
    # until its last workgroup has stored its tiles
    own = [u for u in ran if host_of[u] == -1]        # the others ran inside a producer's tiles / had nothing to do
    events = []
    for u in own:
        events.append((tr[u][1], 1))
        events.append((tr[u][3], -1))
    events.sort()
    hist, level, last_t = {}, 0, 0.0
    for t_ev, d in events:
        hist[level] = hist.get(level, 0.0) + (t_ev - last_t)
        level += d
        last_t = t_ev
    busy = sum(tr[u][3] - tr[u][1] for u in own)
    if verbose:
        print(f"traced replay: {span:.1f} us, {len(ran)} tasks, {len(own)} of them with workgroups of their own; "
              f"time with k of those executing:", file=sys.stderr)
        for k in sorted(hist):
            print(f"  k = {k:2d}: {hist[k]:7.1f} us  {100 * hist[k] / span:5.1f} %", file=sys.stderr)
        print(f"  sum of task execution intervals {busy:.1f} us = {busy / span:.2f} tasks executing on average", file=sys.stderr)
    return {"traced_replay_us": span, "tasks_on_realised_chain": hops, "tile_execution_us": run_us, "hand_over_us": wait_us,
            "no_task_executing_us": hist.get(0, 0.0), "tasks_executing_on_average": busy / span,
            "note": "one replay with per-entry clock readings: tile execution = last workgroup past its wait -> last workgroup "
                    "stored; hand-over = the rest (a producer's last store -> the consumer past its wait, the consumer's "
                    "input-independent prologue included)"}


def measure(name, batch, steps, warmup, args, headline):
    """All measurements of one configuration -> dict."""
    import torch
    from paper_2012_02732_amd import GraphRunner, binding as B

    w = make_workload(name, batch)
    t_prep = time.perf_counter()
    runner = GraphRunner(w, "cuda:0")
    sched = runner.prepare()
    t_prep = time.perf_counter() - t_prep
    n_nodes = len(w.nodes)
    n_tasks = n_nodes - sum(nd.op == "input" for nd in w.nodes)
    auto_mode, auto_trial = B.ng_auto_mode(runner.g)
    mode_name = MODE_NAMES[auto_mode] if args.mode == "auto" else args.mode
    mode = MODES[mode_name]
    gm_state, gm_checked = B.ng_graph_multi_check(runner.g)

    # ---- timed region: K replays of the whole DAG ---------------------------------------------
    total, lat = time_mode(runner, B, mode, steps, warmup)
    ms_per_step = total / steps * 1e3
    t_e2e = statistics.median(lat)
    dev_us = B.ng_time_replay(runner.g, min(steps, 200))          # HIP events on the replay's own stream
    thr = throughput(runner, B, mode, max(20, steps // 2))
    floor_us = B.ng_time_launch_floor(runner.g, 200)

    # ---- the other replay modes (shorter runs) --------------------------------------------------
    modes = {mode_name: t_e2e}
    k2 = max(10, steps // 5)
    for other, m in MODES.items():
        if other == mode_name or (not headline and other.startswith("eager")) or args.no_other_modes:
            continue
        if m == 0 and gm_state != 1:
            continue                                               # refused by the library
        modes[other] = statistics.median(time_mode(runner, B, m, k2, 3)[1])
    B.ng_replay_mode(runner.g, mode)

    # ---- isolated kernel times -> critical path ---------------------------------------------------
    reps = args.isolated_reps if batch == 1 else max(5, args.isolated_reps // 3)
    t_iso = [B.ng_time_task_device(runner.g, v, False, reps)[0] for v in range(n_nodes)]
    t_exe = [B.ng_time_task_device(runner.g, v, True, reps)[0] for v in range(n_nodes)]
    exe_name = [B.ng_task_kernel_executed(runner.g, v) for v in range(n_nodes)]
    preds = [list(nd.preds) for nd in w.nodes]
    t_cp, path = longest_path(preds, t_iso)
    t_cp_exe, path_exe = longest_path(preds, t_exe)
    cp_tasks = sum(1 for v in path if t_iso[v] > 0)
    cp_tasks_exe = sum(1 for v in path_exe if t_exe[v] > 0)
    cp = {"definition": "longest path of the DAG weighted with isolated kernel times (Section 3); isolated time = GPU busy time "
                        "of the kernel running alone, device clock read inside the kernel, median of %d launches" % reps,
          "all_tasks": {"t_cp_us": t_cp, "tasks_on_path": cp_tasks, "fraction_of_bound": t_cp / t_e2e,
                        "fraction_of_bound_device_side": t_cp / dev_us, "sum_isolated_us": sum(t_iso),
                        "note": "every task weighted with its own stand-alone kernel, one kernel per task; the replay runs some "
                                "of them inside another task's kernel, so this is not a lower bound for it and can exceed 1"},
          "as_executed": {"t_cp_us": t_cp_exe, "tasks_on_path_with_a_kernel": cp_tasks_exe, "fraction_of_bound": t_cp_exe / t_e2e,
                          "fraction_of_bound_device_side": t_cp_exe / dev_us, "sum_isolated_us": sum(t_exe),
                          "kernels_run": sum(1 for t in t_exe if t > 0),
                          "note": "weights = the kernels the replay mode really runs, fused variants timed as themselves, tasks "
                                  "without a kernel of their own weigh 0: the harder of the two, the one the 0.80 target is judged on"},
          "launch_and_wait_floor_us": floor_us,
          "fraction_as_executed_above_floor": t_cp_exe / max(t_e2e - floor_us, 1e-9)}
    if name == "chain50":
        cp["overhead_us_per_task"] = (t_e2e - sum(t_exe)) / max(sum(1 for t in t_exe if t > 0), 1)
    else:
        cp["overhead_us_per_task"] = (t_e2e - t_cp_exe) / max(cp_tasks_exe, 1)
    if headline and not args.no_chain_check:
        # cross-check without any clock inside the kernel: chains of dependent launches
        c_empty = B.ng_time_chain(runner.g, -1, 200)
        c_raw = [B.ng_time_chain(runner.g, v, 20) for v in range(n_nodes)]
        lo, _ = longest_path(preds, [max(c - c_empty, 0.0) if c > 0 else 0.0 for c in c_raw])
        hi, _ = longest_path(preds, c_raw)
        cp["all_tasks"]["cross_check_chain_of_launches"] = {
            "t_cp_if_only_time_above_an_empty_kernel_counts_us": lo, "t_cp_if_chain_time_counts_as_duration_us": hi,
            "empty_kernel_chain_us_per_node": c_empty,
            "note": "per node of a chain of dependent launches of the same kernel: the lower figure subtracts the same for an empty "
                    "kernel (dispatch gap + empty execution), the upper one subtracts nothing (gap included)"}

    # ---- roofline of the kernel that dominates the replay ------------------------------------------
    per_kernel = {}
    all_bytes = all_flops = 0.0
    for v in range(n_nodes):
        nbytes, flops = B.ng_task_work(runner.g, v)
        if w.nodes[v].op != "input":
            all_bytes += nbytes
            all_flops += flops
        if t_exe[v] <= 0:
            continue
        k = per_kernel.setdefault(exe_name[v], {"launches": 0, "us": 0.0, "bytes": 0.0, "flops": 0.0})
        k["launches"] += 1
        k["us"] += t_exe[v]
        k["bytes"] += nbytes
        k["flops"] += flops
    if mode_name == "device_resident":
        achieved = all_bytes / dev_us * 1e-3
        roofline = {"kernel": "resident_kernel", "bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS,
                    "unit": "GB/s", "frac": achieved / PEAK_HBM_GBS,
                    "traffic": MEASURED_TRAFFIC_BYTES.get((label(name, batch), "resident_kernel")),
                    "launches_per_step": 1, "avg_launch_us": dev_us, "algorithmic_bytes_per_launch": all_bytes,
                    "algorithmic_flops_per_launch": all_flops,
                    "timing": "HIP events on the stream of the launch, around back-to-back replays",
                    "note": "one launch runs every task; latency-bound by construction: the bound that matters is critical_path"}
    else:
        dom = max(per_kernel, key=lambda kn: per_kernel[kn]["us"])
        d = per_kernel[dom]
        avg_us = d["us"] / d["launches"]
        intensity = d["flops"] / max(d["bytes"], 1.0)
        if intensity >= RIDGE_FLOP_PER_BYTE:
            achieved = d["flops"] / d["us"] * 1e-6
            roofline = {"kernel": dom, "bound": "mfma_f32", "achieved": achieved, "peak": PEAK_MFMA_F32_TFLOPS, "unit": "TFLOP/s",
                        "frac": achieved / PEAK_MFMA_F32_TFLOPS}
        else:
            achieved = d["bytes"] / d["us"] * 1e-3
            roofline = {"kernel": dom, "bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                        "frac": achieved / PEAK_HBM_GBS}
        roofline.update({"traffic": MEASURED_TRAFFIC_BYTES.get((label(name, batch), dom)), "launches_per_step": d["launches"],
                         "avg_launch_us": avg_us, "flop_per_byte": intensity, "share_of_isolated_time": d["us"] / max(sum(t_exe), 1e-9),
                         "algorithmic_bytes_per_launch": d["bytes"] / d["launches"], "algorithmic_flops_per_launch": d["flops"] / d["launches"],
                         "timing": "device clock read inside the kernel, each launch alone (kernels inside a graph launch cannot be "
                                   "bracketed by events); work = the tasks' own algorithmic bytes and flops, fused epilogues not counted"})
    if args.per_task:
        print(f"--- {label(name, batch)}: kernels as executed in mode {mode_name}", file=sys.stderr)
        for kn, k in sorted(per_kernel.items(), key=lambda kv: -kv[1]["us"]):
            print(f"{kn:24s} launches {k['launches']:4d}  isolated total {k['us']:9.1f} us  avg {k['us'] / k['launches']:7.2f} us"
                  f"  {k['bytes'] / k['us'] * 1e-3:8.1f} GB/s  {k['flops'] / k['us'] * 1e-6:8.3f} TFLOP/s", file=sys.stderr)

    timeline = resident_timeline(runner, B, w, n_nodes, args.timeline) if mode_name == "device_resident" else None
    n_wg, n_entries, xcds, est_us = B.ng_resident_sizes(runner.g)
    fusion = B.ng_resident_fusion(runner.g)
    out = {
        "workload": label(name, batch), "input_shape": list(w.input.shape), "tasks": n_tasks, "streams": sched["n_streams"],
        "sync_edges": sched["n_sync"], "events": sched["n_events"], "replay": mode_name, "steps": steps, "warmup": warmup,
        "capture_s": t_prep, "tolerance": "1e-4 of max|ref| per tensor (max-norm), checked by tests/test_gpu_parity.py",
        "latency_us": {"median": t_e2e, "p10": percentile(lat, 0.10), "p90": percentile(lat, 0.90), "device_side": dev_us,
                       "mean_over_timed_region": ms_per_step * 1e3},
        "throughput_replays_per_s": thr, "throughput_images_per_s": thr * batch,
        "us_per_task": t_e2e / n_tasks,
        "critical_path": cp,
        "modes_median_us": modes,
        "auto_mode": {"chosen": MODE_NAMES[auto_mode], "trial_us": {MODE_NAMES[k]: v for k, v in auto_trial.items()},
                      "multi_stream_graph_check": {"state": gm_state, "replays_compared": gm_checked}},
        "resident_plan": {"workgroups": n_wg, "entries": n_entries, "xcds": xcds, "planner_expected_us": est_us,
                          "tasks_inside_their_producer": sum(h >= 0 for h in fusion), "concats_in_place": sum(h == -2 for h in fusion),
                          "setting_kept": B.ng_resident_plan_kept(runner.g)},
        "roofline": roofline,
    }
    if timeline:
        out["resident_timeline"] = timeline
    if "graph_single" in modes and "graph_multi" in modes:
        out["graph_multi_vs_single_stream"] = modes["graph_single"] / modes["graph_multi"]
    if "graph_single" in modes:
        out["chosen_mode_vs_single_stream_graph"] = modes["graph_single"] / t_e2e
    if headline and not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
    out["_ms_per_step"] = ms_per_step
    runner.close()
    del runner
    torch.cuda.empty_cache()
    return out


def solo_launches(args):
    """Every task's kernel `R` times by itself, then the kernels the chosen replay mode really runs, each
    after a marker of three empty kernels; writes what was launched, in order, to the sidecar file."""
    from paper_2012_02732_amd import GraphRunner, binding as B
    name, batch = args.config, args.batch
    w = make_workload(name, batch)
    runner = GraphRunner(w, "cuda:0")
    runner.prepare()
    auto_mode, _ = B.ng_auto_mode(runner.g)
    mode_name = MODE_NAMES[auto_mode] if args.mode == "auto" else args.mode
    total, lat = time_mode(runner, B, MODES[mode_name], 50, 10)
    n = len(w.nodes)
    seq = []
    for executed in (False, True):
        for _ in range(3):
            B.ng_launch_task_solo(runner.g, -1)
        for v in range(n):
            kn = B.ng_task_kernel_executed(runner.g, v) if executed else B.ng_task_kernel(runner.g, v)
            if not kn:
                continue
            for _ in range(args.solo_launches):
                B.ng_launch_task_solo(runner.g, v, executed)
            seq.append({"task": v, "as_executed": executed, "kernel": kn, "launches": args.solo_launches})
    side = {"workload": label(name, batch), "replay": mode_name, "replay_median_us_under_the_profiler": statistics.median(lat),
            "preds": [list(nd.preds) for nd in w.nodes], "ops": [nd.op for nd in w.nodes], "sequence": seq}
    with open(args.sidecar, "w") as f:
        json.dump(side, f)
    runner.close()
    print(json.dumps({"solo_launches": len(seq) * args.solo_launches, "sidecar": args.sidecar}))


def dispatch_trace(args):
    """Critical path from a kernel trace of --solo-launches (begin-to-end timestamps of every dispatch)."""
    side = json.load(open(args.sidecar))
    rows = []
    with open(args.dispatch_trace, newline="") as f:
        for r in csv.DictReader(f):
            rows.append((int(r["Start_Timestamp"]), int(r["End_Timestamp"]), r["Kernel_Name"]))
    rows.sort()
    # the two sequences start after the last two markers: three empty kernels in a row
    marks = [i for i in range(len(rows) - 2) if all("empty_kernel" in rows[i + j][2] for j in range(3))]
    starts = [m + 3 for m in marks if m + 3 >= len(rows) or "empty_kernel" not in rows[m + 3][2]]
    assert len(starts) >= 2, "markers not found in the trace"
    n = len(side["preds"])
    t = {False: [0.0] * n, True: [0.0] * n}
    per_kernel = {}
    empty = [(e - s) / 1000.0 for s, e, k in rows if "empty_kernel" in k]
    for executed, at in zip((False, True), starts[-2:]):
        i = at
        for item in side["sequence"]:
            if item["as_executed"] != executed:
                continue
            durs = []
            for _ in range(item["launches"]):
                s, e, k = rows[i]
                assert "standalone_kernel" in k, (i, k, item)
                durs.append((e - s) / 1000.0)
                i += 1
            t[executed][item["task"]] = statistics.median(durs)
            pk = per_kernel.setdefault((executed, item["kernel"]), [])
            pk.append(statistics.median(durs))
    out = {"workload": side["workload"], "replay": side["replay"], "source": "rocprofv3 --kernel-trace: End_Timestamp - Start_Timestamp of solo dispatches, median per task",
           "empty_kernel_dispatch_us": statistics.median(empty) if empty else None,
           "replay_median_us_under_the_profiler": side["replay_median_us_under_the_profiler"]}
    for executed, key in ((False, "all_tasks"), (True, "as_executed")):
        total, path = longest_path(side["preds"], t[executed])
        out[key] = {"t_cp_us": total, "tasks_on_path_with_a_kernel": sum(1 for v in path if t[executed][v] > 0), "sum_isolated_us": sum(t[executed])}
    print(json.dumps(out))
    print(f"{'kernel':28s} {'variant':12s} {'tasks':>5s} {'median us':>10s} {'min':>7s} {'max':>7s}", file=sys.stderr)
    for (executed, kn), v in sorted(per_kernel.items(), key=lambda kv: (kv[0][0], -sum(kv[1]))):
        print(f"{kn:28s} {'as executed' if executed else 'per task':12s} {len(v):5d} {statistics.median(v):10.2f} {min(v):7.2f} {max(v):7.2f}", file=sys.stderr)


def replay_only(args):
    """A few replays in one launch-based mode and nothing else after the marker: for a kernel trace from outside."""
    from paper_2012_02732_amd import GraphRunner, binding as B
    w = make_workload(args.config, args.batch)
    runner = GraphRunner(w, "cuda:0")
    runner.prepare(plan_trials=1)
    mode = MODES[args.mode]
    total, lat = time_mode(runner, B, mode, 20, 5)
    for _ in range(3):
        B.ng_launch_task_solo(runner.g, -1)
    for _ in range(args.replay_only):
        B.ng_replay(runner.g)
        B.ng_sync(runner.g)
    for _ in range(3):
        B.ng_launch_task_solo(runner.g, -1)
    runner.close()
    print(json.dumps({"workload": label(args.config, args.batch), "replay": args.mode, "replays_after_marker": args.replay_only,
                      "replay_median_us_under_the_profiler": statistics.median(lat)}))


def overlap_trace(args):
    """Kernel overlap and idle gaps of launch-based replays, from the begin / end timestamps of a kernel trace of
    --replay-only (no GPU needed): between the two markers (three empty kernels each), per replay."""
    rows = []
    with open(args.overlap_trace, newline="") as f:
        for r in csv.DictReader(f):
            rows.append((int(r["Start_Timestamp"]), int(r["End_Timestamp"]), r["Kernel_Name"]))
    rows.sort()
    marks = [i for i in range(len(rows) - 2) if all("empty_kernel" in rows[i + j][2] for j in range(3))]
    assert len(marks) >= 2, "markers not found in the trace"
    body = rows[marks[-2] + 3:marks[-1]]
    assert body and args.replay_only > 0 and len(body) % args.replay_only == 0, (len(body), args.replay_only)
    per = len(body) // args.replay_only
    hist, spans, busy_any, sum_dur, gaps = {}, [], [], [], []
    for rep in range(args.replay_only):
        ks = body[rep * per:(rep + 1) * per]
        t0, t1 = min(k[0] for k in ks), max(k[1] for k in ks)
        ev = sorted([(k[0], 1) for k in ks] + [(k[1], -1) for k in ks])
        level, last = 0, t0
        local = {}
        for t, d in ev:
            local[level] = local.get(level, 0) + (t - last)
            if level == 0 and t > last:
                gaps.append((t - last) / 1000.0)
            level += d
            last = t
        for k, v in local.items():
            hist[k] = hist.get(k, 0.0) + v / 1000.0
        spans.append((t1 - t0) / 1000.0)
        busy_any.append(((t1 - t0) - local.get(0, 0)) / 1000.0)
        sum_dur.append(sum(k[1] - k[0] for k in ks) / 1000.0)
    n = args.replay_only
    out = {"kernels_per_replay": per, "replays": n, "first_start_to_last_end_us": statistics.median(spans),
           "some_kernel_executing_us": statistics.median(busy_any), "no_kernel_executing_us": statistics.median(spans) - statistics.median(busy_any),
           "sum_of_kernel_durations_us": statistics.median(sum_dur),
           "kernels_executing_on_average_while_any_is": statistics.median(sum_dur) / statistics.median(busy_any),
           "time_with_k_kernels_executing_us": {str(k): hist[k] / n for k in sorted(hist)},
           "idle_gaps": {"count_per_replay": len(gaps) / n, "median_us": statistics.median(gaps) if gaps else 0.0,
                         "p90_us": percentile(gaps, 0.9) if gaps else 0.0, "max_us": max(gaps) if gaps else 0.0}}
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--config", default="all", help="all (default: the headline workload's line with every configuration under 'configs') or one configuration")
    ap.add_argument("--batch", type=int, default=1, help="only for inception_style")
    ap.add_argument("--mode", default="auto", choices=sorted(MODES) + ["auto"],
                    help="auto = the mode the library's own trial at capture time found fastest")
    ap.add_argument("--isolated-reps", type=int, default=30, help="solo launches per task for the isolated times")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-modes", action="store_true")
    ap.add_argument("--no-chain-check", action="store_true")
    ap.add_argument("--per-task", action="store_true", help="also print a per-kernel table to stderr")
    ap.add_argument("--timeline", action="store_true",
                    help="device-resident mode: print how many tasks execute at the same time during one traced replay (stderr)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 256 MiB device copy (scale reference for HBM traffic counters)")
    ap.add_argument("--solo-launches", type=int, default=0)
    ap.add_argument("--sidecar", default="solo_sidecar.json")
    ap.add_argument("--dispatch-trace", default=None)
    ap.add_argument("--replay-only", type=int, default=0, help="with --config and --mode: that many replays between two markers, for a kernel trace")
    ap.add_argument("--overlap-trace", default=None, help="kernel trace (csv) of a --replay-only run: overlap histogram and idle gaps (give the same --replay-only)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the path has no multi-GPU part); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.dispatch_trace:
        return dispatch_trace(args)
    if args.overlap_trace:
        return overlap_trace(args)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    if args.solo_launches > 0 or args.replay_only > 0:
        if args.config == "all":
            args.config = HEADLINE[0]
        if args.replay_only > 0:
            if args.mode in ("auto", "device_resident"):
                print("bench.py: --replay-only is for the launch-based modes (give --mode)", file=sys.stderr)
                sys.exit(2)
            return replay_only(args)
        return solo_launches(args)

    if args.copy_probe:
        src = torch.ones(64 << 20, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.config == "all":
        todo, head = ALL_CONFIGS, HEADLINE
    else:
        head = (args.config, args.batch if args.config in ("inception_style", "nas_cell_cifar_training") else 1)
        todo = [head]
    results = {}
    for name, batch in todo:
        is_head = (name, batch) == head
        if is_head:
            steps, warmup = args.steps, args.warmup
        else:                                   # the other configurations: their own K, sized to a few seconds each
            steps, warmup = (500, 50) if batch == 1 else (50, 10)
        t0 = time.perf_counter()
        results[label(name, batch)] = measure(name, batch, steps, warmup, args, is_head)
        print(f"[bench] {label(name, batch)}: {results[label(name, batch)]['latency_us']['median']:.1f} us per replay "
              f"({results[label(name, batch)]['replay']}), measured in {time.perf_counter() - t0:.1f} s", file=sys.stderr, flush=True)

    h = results[label(*head)]
    ms_per_step = h.pop("_ms_per_step")
    for r in results.values():
        r.pop("_ms_per_step", None)
    out = {
        "metric": "DAG latency (µs) at batch 1; % of critical-path bound; µs overhead/task",
        "metric_note": "value = wall time of the K timed steps (each: replay + wait) / K on the headline workload, input resident in HBM; "
                       "the other two parts of the metric are critical_path.as_executed.fraction_of_bound (the harder of the two bounds) "
                       "and critical_path.overhead_us_per_task; every configuration is under 'configs'",
        "value": ms_per_step * 1e3, "unit": "us",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": h["workload"], "input_shape": h["input_shape"], "tasks": h["tasks"], "streams": h["streams"],
                   "sync_edges": h["sync_edges"], "events": h["events"], "replay": h["replay"]},
        "latency_us": h["latency_us"],
        "throughput_replays_per_s": h["throughput_replays_per_s"],
        "critical_path": h["critical_path"],
        "modes_median_us": h["modes_median_us"],
        "roofline": h["roofline"],
    }
    if "resident_timeline" in h:
        out["resident_timeline"] = h["resident_timeline"]
    if "cpu_baseline" in h:
        out["cpu_baseline"] = h.pop("cpu_baseline")
    out["configs"] = results
    print(json.dumps(out))


if __name__ == "__main__":
    main()
