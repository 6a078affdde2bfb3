#!/usr/bin/env python3
"""Benchmark of the stitched-kernel hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 3] [--no-extras] [--no-cpu] [--copy-sweep | --survey [--filter NAME]]

A step is one fs_plan_run of the whole fused subgraph on one batch of seeded synthetic input
already resident in HBM.  The headline line is workload 3 of the benchmark spec, the largest of the five
(20-op elementwise DAG over 4 fp32 [65536,1024] inputs, 1.5 GiB per step); the other four, the two
backward-pass subgraphs and two row-sweep end points ride along under `other_workloads`, each with
the same `roofline` block.  `value` is effective HBM GB/s = minimal bytes (every plan input read once
+ every plan output written once) / time per step.

Timing protocol: steps cycle through enough distinct buffer sets (>= 1.5 GiB in total, at least two)
that the 256 MB last-level cache cannot serve them; the warm-up touches every set and lasts at least
50 ms (the device needs tens of milliseconds of work to reach its steady clocks); the K timed steps
are cut into consecutive blocks with a HIP event at every block boundary, on the stream the kernels
are launched on, so the line carries the mean over all K steps (`ms_per_step`) and the median,
minimum and 90th percentile of the per-block means.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MAX_SETS = 1024


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def build_sets(plan, graph, host_inputs, device, total_bytes_target):
    """Distinct device buffer sets of one workload (same seeded content, different addresses)."""
    import torch
    from paper_1811_05213_amd.runner import DeviceRun
    from workloads import min_hbm_bytes
    per_set = max(1, min_hbm_bytes(graph))
    n_sets = max(2 if total_bytes_target else 1, min(MAX_SETS, -(-total_bytes_target // per_set)))
    in_nodes = [graph.nodes[i] for i in graph.input_ids()]
    first = DeviceRun(plan, device)
    first.set_inputs(host_inputs)
    runs = [first]
    for _ in range(n_sets - 1):
        r = DeviceRun(plan, device)
        # small vectors are shared, large tensors get their own copy
        r.set_device_inputs([t.clone() if n.rows * n.cols > 65536 else t for t, n in zip(first.inputs, in_nodes)])
        runs.append(r)
    torch.cuda.synchronize()
    return runs


def time_launches(launchers, steps, warmup, min_warm_ms=50.0, blocks=10):
    """`steps` launches cycling through `launchers`, timed with events on the launch stream in `blocks` consecutive blocks.

    Untimed first: max(warmup, len(launchers)) launches (every buffer set is touched), repeated until `min_warm_ms` of
    wall time have passed.  Returns ms per step: mean over all steps, and median / min / p90 of the block means."""
    import torch
    n = len(launchers)
    t_warm = time.perf_counter()
    while True:
        for i in range(max(warmup, n)):
            launchers[i % n]()
        torch.cuda.synchronize()
        if (time.perf_counter() - t_warm) * 1e3 >= min_warm_ms:
            break
    blocks = max(1, min(blocks, steps))
    bounds = [round(b * steps / blocks) for b in range(blocks + 1)]
    events = [torch.cuda.Event(enable_timing=True) for _ in range(blocks + 1)]
    order = [launchers[i % n] for i in range(steps)]
    t0 = time.perf_counter()
    events[0].record()
    for b in range(blocks):
        for launch in order[bounds[b]:bounds[b + 1]]:
            launch()
        events[b + 1].record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    per_block = sorted(events[b].elapsed_time(events[b + 1]) / (bounds[b + 1] - bounds[b]) for b in range(blocks))
    return {"ms": events[0].elapsed_time(events[-1]) / steps, "ms_median": statistics.median(per_block), "ms_min": per_block[0],
            "ms_p90": per_block[min(len(per_block) - 1, int(0.9 * len(per_block)))], "blocks": blocks, "wall_ms_per_step": wall_ms / steps}


def time_plan(runs, steps, warmup, min_warm_ms=50.0):
    return time_launches([r.prepare() for r in runs], steps, warmup, min_warm_ms)


def time_graph_replay(plan, graph, host_inputs, steps):
    """The plan's launches of one step captured into a HIP graph and replayed: ms per replay, and whether every replay
    reproduced the eager result bit for bit (checked on three replays with eager work and synchronisation in between)."""
    import torch
    from paper_1811_05213_amd.runner import DeviceRun
    r = DeviceRun(plan, "cuda:0")
    r.set_inputs(host_inputs)
    plan.load()          # nothing may be loaded (allocated) while the stream is being captured
    r.launch()
    eager = [t.clone() for t in r.outputs]
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        r.launch()       # fs_plan_run on the capturing stream: kernel launches only, no memset nodes
    same = True
    for _ in range(3):
        for t in r.outputs:
            t.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        same &= all(torch.equal(a, b) for a, b in zip(r.outputs, eager))
    res = time_launches([g.replay], steps, max(4, steps // 10))
    res["replays_match_eager"] = bool(same)
    del g
    return res


def time_copy_probe(nbytes, reps=20, shape=None):
    """GB/s (read + write) of the library's plain copy kernel moving nbytes -> nbytes, rotating buffers.
    shape = (vectors in flight per lane, workgroups) selects fs_copy_probe_shape instead of the one-shot kernel."""
    import torch
    from paper_1811_05213_amd import copy_probe, copy_probe_shape
    n_sets = max(3, min(24, (3 << 30) // (2 * nbytes)))
    srcs = [torch.empty(nbytes, dtype=torch.uint8, device="cuda:0").random_(0, 255) for _ in range(n_sets)]
    dsts = [torch.empty(nbytes, dtype=torch.uint8, device="cuda:0") for _ in range(n_sets)]
    stream = torch.cuda.current_stream().cuda_stream
    if shape is None:
        launchers = [(lambda s=s, d=d: copy_probe(s.data_ptr(), d.data_ptr(), nbytes, stream)) for s, d in zip(srcs, dsts)]
    else:
        launchers = [(lambda s=s, d=d: copy_probe_shape(s.data_ptr(), d.data_ptr(), nbytes, shape[0], shape[1], stream)) for s, d in zip(srcs, dsts)]
    res = time_launches(launchers, reps, 4, min_warm_ms=30.0, blocks=5)
    return 2 * nbytes / res["ms_median"] / 1e6  # GB/s (read + write)


def time_empty_launch(steps=2000):
    """Microseconds per launch of an empty kernel: back to back on the stream, and one at a time with a synchronisation each."""
    import torch
    from paper_1811_05213_amd import launch_probe
    stream = torch.cuda.current_stream().cuda_stream
    res = time_launches([lambda: launch_probe(stream)], steps, 200, min_warm_ms=20.0)
    singles = []
    for _ in range(50):
        torch.cuda.synchronize()
        t = time.perf_counter()
        launch_probe(stream)
        torch.cuda.synchronize()
        singles.append((time.perf_counter() - t) * 1e6)
    return {"back_to_back_us": res["ms_median"] * 1e3, "launch_and_sync_us": statistics.median(singles)}


def time_alu_probe(reps=5):
    """What the vector ALUs sustain on chains of dependent fp32 FMAs (8 wavefronts per SIMD, no memory traffic): the clock
    that figure implies (one wavefront FMA occupies a 16-lane SIMD for 4 cycles) and the fp32 rate without packed instructions."""
    import torch
    from paper_1811_05213_amd import alu_probe, device_limits
    cus = device_limits()["compute_units"]
    workgroups, iters = cus * 32, 2000          # 32 workgroups of 256 lanes per CU: four rounds of 8 wavefronts per SIMD; 256000 FMAs per lane
    out = torch.empty(workgroups * 256, dtype=torch.float32, device="cuda:0")
    stream = torch.cuda.current_stream().cuda_stream
    best = None
    for _ in range(reps + 1):                   # (the first launch also warms the clocks)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        alu_probe(out.data_ptr(), workgroups, iters, stream)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1)
        best = ms if best is None else min(best, ms)
    fma_per_simd = iters * 128 * (workgroups * 4) // (cus * 4)   # wavefront-FMAs one SIMD issues: 4 wavefronts per workgroup, 4 SIMDs per CU
    return {"ms": best, "implied_clock_ghz": fma_per_simd * 4 / (best * 1e-3) / 1e9,
            "fp32_tflops": 2.0 * iters * 128 * 256 * workgroups / (best * 1e-3) / 1e12, "wavefronts_per_simd": 8}


def measured_traffic(workload_name):
    """HBM bytes per launch (per step for multi-kernel plans) of the workload's stitched kernels, from the committed
    rocprofv3 counter summary (FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0, scale factors calibrated on the copy probe), or None."""
    path = os.path.join(ROOT, "profiles", workload_name + "_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def measure_workload(cfg, steps, warmup, with_unfused=True, rows=None, graph_leg=False):
    import torch
    from paper_1811_05213_amd import Plan, FS_MODE_UNFUSED, FS_MODE_LAYERED
    from workloads import workload, min_hbm_bytes
    g, ins, name = workload(cfg, rows)
    out = {"workload": name}
    target = int(1.5 * 2 ** 30)
    for mode, label in ((0, "stitched"),) + (((FS_MODE_UNFUSED, "unfused"),) if with_unfused else ()):
        plan = Plan(g, mode=mode)
        st = plan.stats()
        # (the unfused executor of the largest workload moves 13 GB per step: it runs on the first buffer sets only)
        runs = build_sets(plan, g, ins, "cuda:0", target if mode == 0 or st["launched_hbm_bytes"] < 2 ** 31 else 0)
        res = time_plan(runs, steps if mode == 0 else max(5, steps // 4), warmup if mode == 0 else max(2, warmup // 4))
        hot = time_plan(runs[:1], max(5, steps // 4), 2, min_warm_ms=0.0)
        res.update({"ms_hot": hot["ms_median"], "launches": st["num_launches"], "launched_hbm_bytes": st["launched_hbm_bytes"],
                    "buffer_sets": len(runs)})
        out[label] = res
        if mode == 0:
            ms = res["ms"]
            out["min_hbm_bytes"] = st["min_hbm_bytes"]
            out["unfused_hbm_bytes"] = st["unfused_hbm_bytes"]
            out["gbs"] = st["min_hbm_bytes"] / ms / 1e6
            out["frac_of_peak"] = out["gbs"] / HBM_PEAK_GBS
            out["groups"] = [plan.group_info(i) for i in range(min(st["num_groups"], 4))]
            out["kernels"] = [plan.group_kernel_name(i) for i in range(st["num_groups"])]
            # the roofline of the step: algorithmic bytes of the plan over the measured time of its launches
            out["roofline"] = {"bound": "hbm", "achieved": out["gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": out["frac_of_peak"],
                               "traffic": measured_traffic(name), "kernel": plan.group_kernel_name(0) if st["num_groups"] == 1 else out["kernels"],
                               "algorithmic_bytes_per_launch": st["min_hbm_bytes"], "avg_launch_us": ms * 1e3,
                               "median_us": res["ms_median"] * 1e3, "min_us": res["ms_min"] * 1e3, "p90_us": res["ms_p90"] * 1e3,
                               "frac_at_median": st["min_hbm_bytes"] / res["ms_median"] / 1e6 / HBM_PEAK_GBS}
            if graph_leg:
                out["stitched"]["hip_graph"] = time_graph_replay(plan, g, ins, steps)
        elif graph_leg:
            out["unfused"]["hip_graph"] = time_graph_replay(plan, g, ins, max(5, steps // 4))
        del runs
        plan.destroy()
        torch.cuda.empty_cache()
    if cfg == 5:
        # the same DAG grouped by the layered planner exactly as the paper states it (Section 3.2)
        plan = Plan(g, mode=FS_MODE_LAYERED)
        runs = build_sets(plan, g, ins, "cuda:0", target)
        res = time_plan(runs, steps, warmup)
        out["layered_planner"] = {"ms": res["ms"], "ms_median": res["ms_median"], "launches": plan.stats()["num_launches"],
                                  "launched_hbm_bytes": plan.stats()["launched_hbm_bytes"]}
        del runs
        plan.destroy()
        torch.cuda.empty_cache()
    if with_unfused:
        out["speedup_vs_unfused"] = out["unfused"]["ms"] / out["stitched"]["ms"]
        out["launch_ratio"] = out["stitched"]["launches"] / out["unfused"]["launches"]
    assert min_hbm_bytes(g) == out["min_hbm_bytes"]
    return out


def cpu_baseline(cfg):
    """The CPU oracle as it stands, timed on the host cores of this machine on a bounded sample of the workload."""
    import oracle
    from workloads import workload, min_hbm_bytes
    # a row sample keeps the oracle's work to seconds: every workload here is a set of independent rows (column reductions
    # aside, whose cost per row is the same), so bytes / time on the sample is the rate of the whole workload
    sample_rows = {3: 8192}.get(cfg)
    g, ins, name = workload(cfg, sample_rows)
    cores = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "0") or 0) or (os.cpu_count() or 1))
    oracle.run(g, ins, cores)  # warm the pages
    times = []
    for _ in range(3):
        t = time.perf_counter()
        oracle.run(g, ins, cores)
        times.append(time.perf_counter() - t)
    dt = statistics.median(times)
    what = f"{name}" + (f" (the first {sample_rows} rows' worth: 1/{65536 // sample_rows} of the workload)" if sample_rows else " (the whole workload)")
    return {"value": min_hbm_bytes(g) / dt / 1e9, "unit": "GB/s", "cores": cores, "kind": "oracle",
            "sample": f"{what}, median of 3 runs, {dt * 1e3:.0f} ms each"}


def copy_sweep(sizes):
    """Plain copies of the given sizes in every launch shape of fs_copy_probe_shape: what the fastest copy of that size reaches."""
    rows = []
    for nbytes in sizes:
        best = None
        for u in (1, 2, 4, 8):
            for wgs in (0, 256, 512, 1024, 2048, 4096):
                gbs = time_copy_probe(nbytes, reps=200 if nbytes < (1 << 28) else 20, shape=(u, wgs))
                rows.append({"bytes_each_way": nbytes, "vectors_in_flight": u, "workgroups": wgs, "gbs": gbs, "frac_of_peak": gbs / HBM_PEAK_GBS})
                log(f"copy {nbytes} B each way, {u} vectors in flight, {wgs or 'one-shot'} workgroups: {gbs:.0f} GB/s ({100 * gbs / HBM_PEAK_GBS:.1f} %)")
                if best is None or gbs > best["gbs"]:
                    best = rows[-1]
        log(f"best at {nbytes} B: {best}")
    return rows


def survey(steps, name_filter):
    """Common fused patterns over a range of shapes, each as ONE stitched plan: the schedule the planner chose and the
    measured time, effective GB/s and fraction of peak, one text line per case (the table kept in profiles/shape_survey.txt)."""
    import numpy as np
    import torch
    from paper_1811_05213_amd import Plan
    from workloads import f32_to_bf16_bits, min_hbm_bytes
    from workloads.patterns import cases, more_cases
    rng = np.random.default_rng(181105213)
    print("%-30s %9s x %-9s %2s  %5s %3s %5s %7s %6s | %9s %9s %7s %6s" % ("pattern", "rows", "cols", "k", "L", "E", "WG", "grid", "LDS", "us", "median us", "GB/s", "% peak"))
    for name, g, r, c in cases() + more_cases():
        if name_filter and name_filter not in name:
            continue
        ins = []
        for i in g.input_ids():
            n = g.nodes[i]
            a = rng.standard_normal((n.rows, n.cols), dtype=np.float32)
            ins.append(f32_to_bf16_bits(a) if n.dtype == "bf16" else (a > -1.28).astype(np.uint8) if n.dtype == "u8" else a)
        plan = Plan(g)
        gi = plan.group_info(0)
        runs = build_sets(plan, g, ins, "cuda:0", 2 << 30)
        res = time_plan(runs, steps, 5)
        if res["ms_median"] < 0.03:  # short kernels: a longer loop (30 launches are over before the clocks have settled)
            res = time_plan(runs, 400, 40)
        gbs = min_hbm_bytes(g) / res["ms_median"] / 1e6
        print("%-30s %9d x %-9d %2d  %5d %3d %5d %7d %6d | %9.1f %9.1f %7.0f %6.1f" % (
            name, r, c, plan.stats()["num_launches"], gi["lanes_per_row"], gi["elems_per_lane"], gi["wg_threads"], gi["grid"],
            gi["lds_bytes"], res["ms"] * 1e3, res["ms_median"] * 1e3, gbs, gbs / 80.0), flush=True)
        del runs
        plan.destroy()
        torch.cuda.empty_cache()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=400, help="untimed launches before the timed ones (repeated until 50 ms have passed: steady clocks)")
    ap.add_argument("--workload", type=int, default=3, help="BASELINE.json config number (1-5; 6-7 are extra backward-pass subgraphs) for the headline line")
    ap.add_argument("--no-extras", action="store_true", help="skip the other workloads")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline")
    ap.add_argument("--copy-sweep", action="store_true", help="only sweep the plain-copy launch shapes at the workloads' sizes and print that")
    ap.add_argument("--survey", action="store_true", help="only time the common fused patterns of workloads/patterns.py (a text table, not the JSON line)")
    ap.add_argument("--filter", default="", help="with --survey: only patterns whose name contains this")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1")
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        log("bench.py: no GPU visible; the stitched kernels only run on a MI355X")
        sys.exit(3)
    from paper_1811_05213_amd import lib, device_limits
    lib()  # fails loudly if libfs.so is missing

    if args.survey:
        survey(min(args.steps, 30), args.filter)
        return
    if args.copy_sweep:
        print(json.dumps({"copy_sweep": copy_sweep([1 << 20, 33560576, 67239936, 1 << 28, 805310464])}), flush=True)
        return

    head = measure_workload(args.workload, args.steps, args.warmup, graph_leg=args.workload == 5)
    log("headline", json.dumps(head))
    extras = {}
    copy_gbs = time_copy_probe(1 << 29)
    # the same number of bytes as the headline workload moves, as a plain copy: the practical ceiling at that size
    same = max(1 << 20, (head["min_hbm_bytes"] // 2) // 4096 * 4096)
    copy_same_gbs = time_copy_probe(same, reps=200 if same < (1 << 28) else 20)
    empty = time_empty_launch()
    alu = time_alu_probe()
    log(f"alu probe: {alu}")
    if not args.no_extras:
        for cfg in (1, 2, 3, 4, 5, 6, 7):  # 6, 7: backward-pass subgraphs (LayerNorm, softmax), not benchmark configurations
            if cfg == args.workload:
                continue
            steps = {1: 2000, 2: 2000, 3: 100, 4: 1000, 5: 400, 6: 500, 7: 500}[cfg]
            extras[f"cfg{cfg}"] = measure_workload(cfg, steps, steps, graph_leg=cfg == 5)
            log(f"cfg{cfg}", json.dumps(extras[f"cfg{cfg}"]))
        # the same stitched kernels on more rows: where the launch stops dominating (row sweep end points)
        for cfg, rows in ((1, 65536), (2, 262144)):
            extras[f"cfg{cfg}_rows{rows}"] = measure_workload(cfg, 100, 20, with_unfused=False, rows=rows)
            log(f"cfg{cfg}_rows{rows}", json.dumps(extras[f"cfg{cfg}_rows{rows}"]))
    cpu = None if args.no_cpu else cpu_baseline(args.workload)

    st = head["stitched"]
    # every workload's roofline block under the headline's (algorithmic bytes, live-measured launch time, counter traffic)
    per_workload = {f"cfg{args.workload}": dict(head["roofline"], workload=head["workload"], launches=st["launches"],
                                               speedup_vs_unfused=head.get("speedup_vs_unfused"))}
    for key, w in extras.items():
        per_workload[key] = dict(w["roofline"], workload=w["workload"], launches=w["stitched"]["launches"], speedup_vs_unfused=w.get("speedup_vs_unfused"))
    head["roofline"] = dict(head["roofline"], workloads=per_workload)
    line = {
        "metric": "effective HBM GB/s (% of peak) per fused subgraph; fused vs unfused speedup",
        "value": head["gbs"],
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": st["ms"],
        "ms_per_step_median": st["ms_median"],
        "ms_per_step_min": st["ms_min"],
        "ms_per_step_p90": st["ms_p90"],
        "timed_blocks": st["blocks"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": head["workload"], "mode": "stitched", "launches_per_step": st["launches"],
                   "buffer_sets": st["buffer_sets"], "min_hbm_bytes": head["min_hbm_bytes"]},
        "pct_of_hbm_peak": 100.0 * head["frac_of_peak"],
        "speedup_vs_unfused": head.get("speedup_vs_unfused"),
        "launch_ratio": head.get("launch_ratio"),
        "unfused_ms_per_step": head.get("unfused", {}).get("ms"),
        "roofline": head["roofline"],
        "cpu_baseline": cpu,
        "copy_probe_gbs": copy_gbs,
        "copy_probe_same_bytes_gbs": copy_same_gbs,
        "empty_kernel_launch": empty,
        "alu_probe": alu,
        "device": device_limits(),
        "other_workloads": extras,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
