#!/usr/bin/env python3
"""Benchmark of the NoLoCo outer step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

One "step" = one whole outer step of the method (arxiv 2506.10911, Eq. 1-3 + restart):
noloco_plan_groups on the host, then noloco_outer_step over the whole arena, all W worker
replicas resident in HBM. Between steps an UNTIMED fake inner phase re-draws the fast weights
(theta = cast(phi + sigma z)), so every timed step sees the workload's input distribution.
The timed region of a step is bracketed by torch.cuda.synchronize() on both sides; the kernel
itself is additionally timed with HIP events on the stream it is launched on.

Prints ONE JSON line: throughput in worker-parameter updates per second, the HBM roofline
fraction of the kernel, and the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E peak
DEFAULT_WORKLOAD = "stage6p8b"  # the configuration the target is quoted on (fits one GPU: 257.8 GB)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD,
                    choices=["tiny", "gpt125m", "stage1p3b", "stage6p8b", "ragged_tight", "ragged_gapped"])
    ap.add_argument("--op", default="outer_step", choices=["outer_step", "replica_spread"],
                    help="outer_step (the headline path) or the read-only replica-spread pass over phi")
    ap.add_argument("--workers", type=int, default=0, help="override W (0 = the workload's own)")
    ap.add_argument("--subgroup", type=int, default=0, help="override the subgroup size n (0 = the workload's schedule)")
    ap.add_argument("--vectors-per-thread", type=int, default=-1)
    ap.add_argument("--nontemporal", type=int, default=-1)
    ap.add_argument("--group-major", type=int, default=-1)
    ap.add_argument("--xcd-map", type=int, default=-1)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-inner-phase", action="store_true",
                    help="skip the untimed re-draw of theta between steps (for profiler runs)")
    return ap.parse_args()


def recorded_traffic(workload):
    """HBM bytes per launch measured with rocprofv3 --pmc, if a summary for this workload is committed."""
    path = os.path.join(ROOT, "profiles", f"outer_step_{workload}_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def cpu_baseline(wl, n, hp):
    """The oracle, as it stands, on a bounded column sample of the same workload (all W rows)."""
    import concurrent.futures as cf
    import oracle
    import workloads
    cores = max(1, min(len(os.sched_getaffinity(0)), int(os.environ.get("OMP_NUM_THREADS", "16"))))
    W = wl.W
    cols = max(1 << 16, min((1 << 26) // W, wl.P))          # about 64M worker-params per step
    cols -= cols % cores
    phi = np.tile(workloads.phi0_cpu(cols, wl.seed, wl.init_std), (W, 1))
    delta = np.zeros((W, cols), dtype=np.float32)
    theta = workloads.fake_inner_phase_cpu(phi, wl.seed, 0, wl.sigma, wl.theta_dtype)
    members, offsets = oracle.plan_groups(wl.seed, 0, W, n)
    oracle.outer_step_f32(phi, delta, theta, hp, members, offsets, segments=[(0, 1 << 12)])   # page in, warm up

    def timed(fn, min_seconds):
        reps, t0 = 0, time.perf_counter()
        while True:
            fn()
            reps += 1
            dt = time.perf_counter() - t0
            if dt >= min_seconds:
                return reps, dt

    one = lambda: oracle.outer_step_f32(phi, delta, theta, hp, members, offsets)
    reps1, dt1 = timed(one, 5.0)
    chunk = cols // cores
    parts = [[(i * chunk, chunk)] for i in range(cores)]
    pool = cf.ThreadPoolExecutor(cores)

    def many():
        list(pool.map(lambda seg: oracle.outer_step_f32(phi, delta, theta, hp, members, offsets, segments=seg), parts))

    repsN, dtN = timed(many, 8.0)
    pool.shutdown()
    return {
        "value": W * cols * repsN / dtN, "unit": "worker-param updates/s", "cores": cores,
        "kind": "oracle",
        "sample": f"{cols} columns x all {W} workers of {wl.name} (n={n}, theta {wl.theta_dtype}), "
                  f"{repsN} steps on {cores} threads (disjoint column ranges of the same single-threaded routine)",
        "single_core_value": W * cols * reps1 / dt1,
        "implied_dram_GBps": W * cols * repsN / dtN * wl.bytes_per_update / 1e9,
    }


def spread_cpu_baseline(wl):
    """oracle.replica_spread (binary64 definition) on a bounded column sample, all W rows."""
    import concurrent.futures as cf
    import oracle
    import workloads
    cores = max(1, min(len(os.sched_getaffinity(0)), int(os.environ.get("OMP_NUM_THREADS", "16"))))
    W = wl.W
    cols = max(1 << 16, min((1 << 26) // W, wl.P))
    cols -= cols % cores
    x = np.tile(workloads.phi0_cpu(cols, wl.seed, wl.init_std), (W, 1)) + workloads.drift_cpu((W, cols), wl.seed, 0, wl.sigma)
    x = np.ascontiguousarray(x, dtype=np.float32)
    chunk = cols // cores
    parts = [[(i * chunk, chunk)] for i in range(cores)]
    pool = cf.ThreadPoolExecutor(cores)
    oracle.replica_spread(x, [(0, 1 << 12)])
    reps, t0 = 0, time.perf_counter()
    while time.perf_counter() - t0 < 8.0:
        list(pool.map(lambda seg: oracle.replica_spread(x, seg), parts))
        reps += 1
    dt = time.perf_counter() - t0
    pool.shutdown()
    return {"value": W * cols * reps / dt, "unit": "worker-params/s", "cores": cores, "kind": "oracle",
            "sample": f"{cols} columns x all {W} workers of {wl.name}, {reps} passes on {cores} threads "
                      "(disjoint column ranges of the same single-threaded routine)"}


def run_replica_spread(args, wl, torch, nl, workloads, dev):
    """K timed passes of noloco_replica_spread over the slow weights of the workload."""
    W, S = wl.W, wl.stride
    phi = torch.empty((W, S), dtype=torch.float32, device=dev)
    workloads.fill_phi0_device(phi, wl.seed, wl.init_std)
    workloads.fake_inner_phase_device(phi, phi, wl.seed, 0, wl.sigma)      # replicas drift apart
    plan = nl.LaunchPlan(phi, phi, phi, S, W, nl.F32, wl.segments)
    out = torch.zeros(len(wl.segments) + 1, dtype=torch.float64, device=dev)
    kernel_ms, host_s = [], []
    for t in range(args.warmup + args.steps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record()
        nl.replica_spread(plan, phi, nl.F32, out)
        e1.record()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        if t >= args.warmup:
            host_s.append(t1 - t0)
            kernel_ms.append(e0.elapsed_time(e1))
    elems = W * wl.P
    total_s = sum(host_s)
    avg_s = sum(kernel_ms) / len(kernel_ms) / 1e3
    achieved = elems * 4 / avg_s / 1e9
    res = {
        "metric": "replica-spread worker-params/s", "value": elems * args.steps / total_s,
        "unit": "worker-params/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": total_s / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.name, "W": W, "params_per_worker": wl.P, "tensors": len(wl.tensors),
                   "array": "phi (f32)", "resident_GB": W * S * 4 / 1e9,
                   "overall_std": float(out[-1]), "device": torch.cuda.get_device_name(0)},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": None,
                     "kernel": "replica_spread_tiles (+ replica_spread_finish)",
                     "algorithmic_bytes_per_launch": elems * 4, "bytes_per_update": 4,
                     "avg_kernel_ms": avg_s * 1e3, "min_kernel_ms": min(kernel_ms), "max_kernel_ms": max(kernel_ms)},
    }
    del phi
    torch.cuda.empty_cache()
    res["cpu_baseline"] = None if args.no_cpu_baseline else spread_cpu_baseline(wl)
    print(json.dumps(res))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the W worker replicas are stacked in one GPU's "
              "HBM; there is no multi-GPU path). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads
    import paper_2506_10911_amd as nl          # raises if libnoloco.so is missing: no fallback

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    wl = workloads.make(args.workload)
    note = None
    if args.workers:
        wl.W = args.workers
    free, total = torch.cuda.mem_get_info()
    per_worker = wl.stride * (8 + wl.theta_bytes)
    reserve = 3 << 30                                     # inner-phase scratch, allocator slack
    if wl.W * per_worker + reserve > free:
        fit = int((free - reserve) // per_worker) // 2 * 2
        note = f"W reduced from {wl.W} to {fit}: {wl.W * per_worker / 1e9:.1f} GB does not fit in {free / 1e9:.1f} GB free"
        wl.W = fit
    W, S = wl.W, wl.stride
    hp = (wl.alpha, wl.beta, wl.gamma)
    if args.op == "replica_spread":
        run_replica_spread(args, wl, torch, nl, workloads, dev)
        return

    tdt = torch.float32 if wl.theta_dtype == "f32" else torch.bfloat16
    phi = torch.empty((W, S), dtype=torch.float32, device=dev)
    delta = torch.zeros((W, S), dtype=torch.float32, device=dev)
    theta = torch.empty((W, S), dtype=tdt, device=dev)
    workloads.fill_phi0_device(phi, wl.seed, wl.init_std)
    plan = nl.LaunchPlan(phi, delta, theta, S, W, nl.F32 if wl.theta_dtype == "f32" else nl.BF16, wl.segments)
    plan.tune(args.vectors_per_thread, args.nontemporal, args.group_major, args.xcd_map)
    n_of = (lambda t: args.subgroup) if args.subgroup else wl.n_at

    ev0 = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    ev1 = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    host_s, plan_us = [], []
    workloads.fake_inner_phase_device(theta, phi, wl.seed, 0, wl.sigma)
    for t in range(args.warmup + args.steps):
        if t > 0 and not args.no_inner_phase:
            workloads.fake_inner_phase_device(theta, phi, wl.seed, t, wl.sigma)   # untimed
        timed = t >= args.warmup
        k = t - args.warmup
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        members, offsets = nl.plan_groups(wl.seed, t, W, n_of(t))
        t_plan = time.perf_counter()
        if timed:
            ev0[k].record()
        nl.outer_step(plan, phi, delta, theta, hp, members, offsets)
        if timed:
            ev1[k].record()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        if timed:
            host_s.append(t1 - t0)
            plan_us.append((t_plan - t0) * 1e6)

    updates = W * wl.P                                    # worker-parameter updates per step
    total_s = sum(host_s)
    ms_per_step = total_s / args.steps * 1e3
    kernel_ms = [a.elapsed_time(b) for a, b in zip(ev0, ev1)]
    avg_kernel_s = sum(kernel_ms) / len(kernel_ms) / 1e3
    alg_bytes = updates * wl.bytes_per_update             # per launch: one launch covers the whole arena
    achieved = alg_bytes / avg_kernel_s / 1e9

    # yardsticks: plain streaming kernels over the momentum array (its contents are no longer needed)
    half = (W // 2) * S * 4 // 16 * 16
    probes = {"copy": None, "read": None, "fill": None}
    if half >= (1 << 24):
        sink = torch.zeros(4, dtype=torch.float32, device=dev)
        runs = {
            "copy": (lambda: nl.copy_probe(delta.data_ptr() + half, delta, half), 2 * half),
            "read": (lambda: nl.read_probe(delta, 2 * half, sink), 2 * half),
            "fill": (lambda: nl.fill_probe(delta, 2 * half, 0.0), 2 * half),
        }
        for name, (fn, nbytes) in runs.items():
            c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            fn()
            c0.record()
            for _ in range(3):
                fn()
            c1.record()
            torch.cuda.synchronize()
            probes[name] = 3 * nbytes / (c0.elapsed_time(c1) / 1e3) / 1e9

    out = {
        "metric": "outer-step worker-param updates/s",
        "value": updates * args.steps / total_s,
        "unit": "worker-param updates/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {
            "workload": wl.name, "W": W, "params_per_worker": wl.P, "tensors": len(wl.tensors),
            "theta_dtype": wl.theta_dtype, "subgroup_n": sorted({n_of(t) for t in range(args.warmup, args.warmup + args.steps)}),
            "alpha": wl.alpha, "beta": wl.beta, "gamma": wl.gamma, "drift_sigma": wl.sigma,
            "resident_GB": W * per_worker / 1e9, "device": torch.cuda.get_device_name(0),
            "launch": plan.info(), "note": note,
        },
        "roofline": {
            "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBPS, "traffic": recorded_traffic(wl.name),
            "kernel": ("outer_step_fixed" if n_of(args.warmup) in (1, 2, 4, 8, 16) else
                       "outer_step_phi_resident" if n_of(args.warmup) in (32, 64) else "outer_step_generic"),
            "algorithmic_bytes_per_launch": alg_bytes,
            "bytes_per_update": wl.bytes_per_update,
            "avg_kernel_ms": avg_kernel_s * 1e3, "median_kernel_ms": float(np.median(kernel_ms)),
            "min_kernel_ms": min(kernel_ms), "max_kernel_ms": max(kernel_ms),
            "copy_probe_GBps": probes["copy"], "read_probe_GBps": probes["read"],
            "fill_probe_GBps": probes["fill"],
        },
        "host": {"plan_groups_us": float(np.median(plan_us)),
                 "step_minus_kernel_ms": ms_per_step - avg_kernel_s * 1e3},
    }
    del phi, delta, theta
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, n_of(args.warmup), hp)
    else:
        out["cpu_baseline"] = None
    print(json.dumps(out))


if __name__ == "__main__":
    main()
