#!/usr/bin/env python3
"""Benchmark of the NoLoCo outer step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

One "step" = one whole outer step of the method (arxiv 2506.10911, Eq. 1-3 + restart):
noloco_plan_groups on the host, then noloco_outer_step over the whole arena, all W worker
replicas resident in HBM. Between steps an UNTIMED fake inner phase re-draws the fast weights
(theta = cast(phi + sigma z)), so every timed step sees the workload's input distribution.
The timed region of a step is bracketed by torch.cuda.synchronize() on both sides; the kernel
itself is additionally timed with HIP events on the stream it is launched on.

Prints ONE JSON line: throughput in worker-parameter updates per second on the benchmark
workload, the HBM roofline fraction of its kernel, and the CPU oracle timed on a bounded sample
of the same workload. With no --workload the same line also carries, under "extra", a few steps of
every other configuration (per subgroup size), of the larger-subgroup modes and of the
replica-spread pass.

    python bench.py --summarize KIND --from DIR [DIR] --out profiles/NAME.txt --command "..."

reduces a rocprofv3 output directory (CSV format) to the short text summaries kept under profiles/.
"""
import argparse
import csv
import glob
import json
import os
import statistics
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E peak
DEFAULT_WORKLOAD = "stage6p8b"  # the configuration the target is quoted on (fits one GPU: 257.8 GB)
WORKLOADS = ["tiny", "gpt125m", "stage1p3b", "stage6p8b", "ragged_tight", "ragged_gapped"]
REGION_BYTES = 96 << 30         # the GPU's memory behaves as three such regions, see class Arena


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default=None, choices=WORKLOADS,
                    help=f"default: {DEFAULT_WORKLOAD}, followed by the other configurations under 'extra'")
    ap.add_argument("--op", default="outer_step", choices=["outer_step", "replica_spread"],
                    help="outer_step (the headline path) or the read-only replica-spread pass over phi")
    ap.add_argument("--workers", type=int, default=0, help="override W (0 = the workload's own)")
    ap.add_argument("--subgroup", type=int, default=0, help="override the subgroup size n (0 = the workload's schedule)")
    ap.add_argument("--vectors-per-thread", type=int, default=-1)
    ap.add_argument("--nontemporal", type=int, default=-1)
    ap.add_argument("--group-major", type=int, default=-1)
    ap.add_argument("--xcd-map", type=int, default=-1)
    ap.add_argument("--placement", default="spread", choices=["spread", "plain"],
                    help="spread: small arenas get their three arrays in different thirds of the GPU memory")
    ap.add_argument("--no-extra", action="store_true", help="headline workload only")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-inner-phase", action="store_true",
                    help="skip the untimed re-draw of theta between steps (for profiler runs)")
    ap.add_argument("--summarize", default=None, choices=["kernel_stats", "hbm_traffic", "counters"])
    ap.add_argument("--from", dest="src", nargs="+", default=[])
    ap.add_argument("--out", default=None)
    ap.add_argument("--command", action="append", default=[])
    ap.add_argument("--title", default="")
    ap.add_argument("--bench-log", default=None, help="with --summarize kernel_stats: the profiled run's own output")
    return ap.parse_args()


# ----------------------------------------------------------------------------------------------
# profiles/: stored counter summaries and the code that writes them
# ----------------------------------------------------------------------------------------------

def recorded_traffic(name):
    """HBM bytes per launch measured with rocprofv3 --pmc, if a summary of that name is committed."""
    path = os.path.join(ROOT, "profiles", f"{name}_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def short_kernel_name(name):
    for junk in ("noloco::(anonymous namespace)::", "void ", "noloco::"):
        name = name.replace(junk, "")
    return name.split("(")[0]


def _find(dirs, suffix):
    hits = []
    for d in dirs:
        hits += sorted(glob.glob(os.path.join(d, "**", "*" + suffix), recursive=True))
    if not hits:
        sys.exit(f"bench.py --summarize: no *{suffix} under {dirs}")
    return hits


def _counter_rows(dirs):
    rows = []
    for path in _find(dirs, "counter_collection.csv"):
        rows += list(csv.DictReader(open(path)))
    return rows


def is_ours(kernel_name):
    return any(k in kernel_name for k in ("outer_step_", "replica_spread_tiles", "copy_probe_kernel",
                                          "read_probe_kernel", "fill_probe_kernel"))


def summarize(args):
    """rocprofv3 CSV output -> the text under profiles/ (figures only, a few KB)."""
    head = [args.title or f"rocprofv3 {args.summarize} summary", ""]
    head += ["Command(s), run on the MI355X box from /tmp with TMPDIR=/tmp:"] + [f"  {c}" for c in args.command] + [""]
    head += [f"Reduced with: python bench.py --summarize {args.summarize} --from <output dirs> --out {args.out}", ""]
    lines = []
    if args.summarize == "kernel_stats":
        rows = []
        for path in _find(args.src, "kernel_stats.csv"):
            rows += list(csv.DictReader(open(path)))
        rows.sort(key=lambda r: -float(r["TotalDurationNs"]))
        lines.append(f"{'kernel':<70}{'calls':>7}{'avg ms':>11}{'min ms':>11}{'max ms':>11}{'% time':>8}")
        for r in rows[:10]:
            lines.append(f"{short_kernel_name(r['Name'])[:68]:<70}{r['Calls']:>7}{float(r['AverageNs']) / 1e6:>11.4f}"
                         f"{float(r['MinNs']) / 1e6:>11.4f}{float(r['MaxNs']) / 1e6:>11.4f}{r['Percentage']:>8}")
        lines.append("")
        for r in rows:
            if is_ours(r["Name"]):
                lines.append(f"avg_kernel_ms[{short_kernel_name(r['Name'])}]: {float(r['AverageNs']) / 1e6:.4f}")
        lines.append("(at::native kernels are the untimed fake inner phase between steps and the arena set-up)")
        if args.bench_log:
            line = [l for l in open(args.bench_log) if l.startswith("{")][0]
            r = json.loads(line)["roofline"]
            lines += ["", "bench.py's own figures in the same run (HIP events on the launch stream, the 10 timed steps):",
                      f"  avg_kernel_ms {r['avg_kernel_ms']:.4f}  min {r['min_kernel_ms']:.4f}  max {r['max_kernel_ms']:.4f}",
                      f"  algorithmic bytes per launch {r['algorithmic_bytes_per_launch']}  ->  {r['achieved']:.0f} GB/s = "
                      f"{100 * r['frac']:.1f} % of the {r['peak']:.0f} GB/s HBM peak"]
    elif args.summarize == "hbm_traffic":
        rows = _counter_rows(args.src)
        per = {}                                   # (kernel, counter) -> values in KiB per dispatch
        for r in rows:
            if is_ours(r["Kernel_Name"]):
                per.setdefault((short_kernel_name(r["Kernel_Name"]), r["Counter_Name"]), []).append(float(r["Counter_Value"]))
        copies = {c: v for (k, c), v in per.items() if k.startswith("copy_probe_kernel")}
        if "FETCH_SIZE" not in copies or "WRITE_SIZE" not in copies:
            sys.exit("bench.py --summarize hbm_traffic: the runs must include the copy probe (calibration)")
        grid = [int(r["Grid_Size"]) for r in rows if "copy_probe_kernel" in r["Kernel_Name"]][0]
        copy_bytes = grid * 4 * 16                  # each thread of the copy probe moves 4 x 16 bytes each way
        fcal = copy_bytes / 1024 / statistics.mean(copies["FETCH_SIZE"])
        wcal = copy_bytes / 1024 / statistics.mean(copies["WRITE_SIZE"])
        lines.append("Counter values per dispatch (KiB), mean over the launches of each kernel:")
        lines.append(f"  {'kernel':<58}{'launches':>9}{'FETCH_SIZE':>16}{'WRITE_SIZE':>16}")
        kernels = sorted({k for k, _ in per})
        for k in kernels:
            f, w = per.get((k, "FETCH_SIZE"), []), per.get((k, "WRITE_SIZE"), [])
            lines.append(f"  {k[:56]:<58}{max(len(f), len(w)):>9}{statistics.mean(f) if f else float('nan'):>16.1f}"
                         f"{statistics.mean(w) if w else float('nan'):>16.1f}")
        lines += ["", f"Calibration against the plain copy kernel of the same runs, which reads and writes {copy_bytes} bytes each:",
                  f"  FETCH_SIZE scale factor {fcal:.5f}", f"  WRITE_SIZE scale factor {wcal:.5f}", ""]
        main = [k for k in kernels if k.startswith(("outer_step_", "replica_spread_tiles"))]
        for k in main:
            f = statistics.mean(per[(k, "FETCH_SIZE")]) * 1024 * fcal
            w = statistics.mean(per.get((k, "WRITE_SIZE"), [0.0])) * 1024 * wcal
            lines.append(f"{k}: fetched {f:.6g} bytes, written {w:.6g} bytes per launch")
        k = main[0]
        total = (statistics.mean(per[(k, "FETCH_SIZE")]) * fcal + statistics.mean(per.get((k, "WRITE_SIZE"), [0.0])) * wcal) * 1024
        lines.append(f"traffic_bytes_per_launch: {total:.0f}")
    else:
        rows = _counter_rows(args.src)
        per, dur = {}, {}
        for r in rows:
            if is_ours(r["Kernel_Name"]):
                k = short_kernel_name(r["Kernel_Name"])
                per.setdefault((k, r["Counter_Name"]), []).append(float(r["Counter_Value"]))
                dur.setdefault(k, []).append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e6)
        counters = sorted({c for _, c in per})
        kernels = sorted({k for k, _ in per})
        lines.append("Counter values per dispatch (mean over the launches of each kernel; sums over all L2 channels / shader engines):")
        for k in kernels:
            lines.append(f"{k}   ({len(dur[k]) // max(len(counters), 1)} launches, {statistics.mean(dur[k]):.3f} ms each under the profiler)")
            mean = {c: statistics.mean(per[(k, c)]) for c in counters if (k, c) in per}
            for c in counters:
                if c in mean:
                    lines.append(f"    {c:<44}{mean[c]:>22.1f}")
            # derived figures (TCC = L2 channel, EA = its port towards the fabric and HBM)
            if mean.get("TCC_EA0_RDREQ_sum"):
                lines.append(f"    -> EA read latency  {mean['TCC_EA0_RDREQ_LEVEL_sum'] / mean['TCC_EA0_RDREQ_sum']:.0f} L2 cycles "
                             f"(RDREQ_LEVEL / RDREQ)")
            if mean.get("TCC_EA0_WRREQ_sum"):
                lines.append(f"    -> EA write latency {mean['TCC_EA0_WRREQ_LEVEL_sum'] / mean['TCC_EA0_WRREQ_sum']:.0f} L2 cycles "
                             f"(WRREQ_LEVEL / WRREQ)")
            if mean.get("TCC_CYCLE_sum"):
                for c in ("TCC_EA0_RDREQ_DRAM_CREDIT_STALL_sum", "TCC_EA0_WRREQ_DRAM_CREDIT_STALL_sum", "TCC_TAG_STALL_sum"):
                    if c in mean:
                        lines.append(f"    -> {c} / TCC_CYCLE_sum = {100 * mean[c] / mean['TCC_CYCLE_sum']:.1f} % of L2-channel cycles")
    text = "\n".join(head + lines) + "\n"
    with open(args.out, "w") as f:
        f.write(text)
    print(text)


# ----------------------------------------------------------------------------------------------
# CPU baseline: the oracle as it stands
# ----------------------------------------------------------------------------------------------

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


# ----------------------------------------------------------------------------------------------
# GPU side
# ----------------------------------------------------------------------------------------------

class Arena:
    """The three caller-owned arrays of one workload, allocated through torch."""

    def __init__(self, torch, wl, dev, placement, need_delta=True, need_theta=True):
        W, S = wl.W, wl.stride
        tdt = torch.float32 if wl.theta_dtype == "f32" else torch.bfloat16
        f32_bytes, theta_bytes = W * S * 4, W * S * wl.theta_bytes
        free, _ = torch.cuda.mem_get_info()
        # On MI355X an in-place stream over three arrays runs about 15 % slower when the arrays are
        # neighbours inside one 96 GiB third of the memory than when they lie in different thirds
        # (measured; consistent with the three ranks of a 12-high HBM3E stack sitting at the top of
        # the physical address). An arena that fills the memory is spread by itself. For a small one
        # the harness takes one slab of 2 x 96 GiB + theta and carves phi, delta and theta out of it
        # 96 GiB apart, so that element k of the three arrays always lies in three different thirds.
        slab_bytes = 2 * REGION_BYTES + theta_bytes
        spread = (placement == "spread" and need_delta and need_theta and (1 << 30) <= f32_bytes <= REGION_BYTES
                  and free > slab_bytes + (6 << 30))
        self.slab = None
        if spread:
            self.slab = torch.empty(slab_bytes, dtype=torch.uint8, device=dev)
            self.phi = self.slab[:f32_bytes].view(torch.float32).view(W, S)
            self.delta = self.slab[REGION_BYTES:REGION_BYTES + f32_bytes].view(torch.float32).view(W, S)
            self.delta.zero_()
            self.theta = self.slab[2 * REGION_BYTES:2 * REGION_BYTES + theta_bytes].view(tdt).view(W, S)
        else:
            self.phi = torch.empty((W, S), dtype=torch.float32, device=dev)
            self.delta = torch.zeros((W, S), dtype=torch.float32, device=dev) if need_delta else None
            self.theta = torch.empty((W, S), dtype=tdt, device=dev) if need_theta else None
        self.placement = "spread" if spread else "plain"
        self.resident_bytes = 2 * f32_bytes + theta_bytes

    def free(self, torch):
        self.phi = self.delta = self.theta = self.slab = None
        torch.cuda.empty_cache()


def kernel_of(n):
    return ("outer_step_fixed" if n in (1, 2, 4, 8, 16) else
            "outer_step_phi_resident" if n in (32, 64) else "outer_step_generic")


def run_outer_steps(torch, nl, workloads, wl, arena, plan, n_of, steps, warmup, inner_phase=True):
    """warmup + steps outer steps; returns per-step host seconds, kernel ms (HIP events), n, host call us."""
    W = wl.W
    hp = (wl.alpha, wl.beta, wl.gamma)
    ev0 = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    ev1 = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    host_s, plan_us, call_us, ns = [], [], [], []
    workloads.fake_inner_phase_device(arena.theta, arena.phi, wl.seed, 0, wl.sigma)
    for t in range(warmup + steps):
        if t > 0 and inner_phase:
            workloads.fake_inner_phase_device(arena.theta, arena.phi, wl.seed, t, wl.sigma)   # untimed
        timed = t >= warmup
        k = t - warmup
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        members, offsets = nl.plan_groups(wl.seed, t, W, n_of(t))
        t_plan = time.perf_counter()
        if timed:
            ev0[k].record()
        nl.outer_step(plan, arena.phi, arena.delta, arena.theta, hp, members, offsets)
        t_call = time.perf_counter()
        if timed:
            ev1[k].record()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        if timed:
            host_s.append(t1 - t0)
            plan_us.append((t_plan - t0) * 1e6)
            call_us.append((t_call - t_plan) * 1e6)     # includes recording the first event
            ns.append(n_of(t))
    kernel_ms = [a.elapsed_time(b) for a, b in zip(ev0, ev1)]
    return {"host_s": host_s, "kernel_ms": kernel_ms, "n": ns, "plan_us": plan_us, "call_us": call_us}


def per_n_figures(wl, run):
    """Kernel time and achieved bandwidth by subgroup size (one launch covers the whole arena)."""
    out = {}
    alg = wl.W * wl.P * wl.bytes_per_update
    for n in sorted(set(run["n"])):
        ms = [m for m, k in zip(run["kernel_ms"], run["n"]) if k == n]
        avg = sum(ms) / len(ms)
        out[str(n)] = {"kernel": kernel_of(n), "launches": len(ms), "avg_kernel_ms": avg, "min_kernel_ms": min(ms),
                       "GBps": alg / avg / 1e6, "frac": alg / avg / 1e6 / HBM_PEAK_GBPS}
    return out


def stream_probes(torch, nl, delta, W, S, dev):
    """Plain streaming kernels over the momentum array (its contents are no longer needed)."""
    half = (W // 2) * S * 4 // 16 * 16
    probes = {"copy": None, "read": None, "fill": None, "runtime_copy": None}
    if half < (1 << 20):
        return probes
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
    # the HIP runtime's own device-to-device copy of the same bytes (torch's copy_ of a contiguous
    # tensor is a hipMemcpyAsync): a yardstick that owes nothing to this library's kernels
    flat = delta.view(-1)
    n = half // 4
    dst, src = flat[n:2 * n], flat[:n]
    dst.copy_(src)
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record()
    for _ in range(3):
        dst.copy_(src)
    c1.record()
    torch.cuda.synchronize()
    probes["runtime_copy"] = 3 * 2 * half / (c0.elapsed_time(c1) / 1e3) / 1e9
    return probes


def graph_replay_us(torch, nl, wl, arena, plan, steps=20, replays=5):
    """A window of outer steps captured once into a HIP graph and replayed: microseconds per step."""
    hp = (wl.alpha, wl.beta, wl.gamma)
    plans = [nl.plan_groups(wl.seed, t, wl.W, wl.n_at(t)) for t in range(steps)]
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for members, offsets in plans:
            nl.outer_step(plan, arena.phi, arena.delta, arena.theta, hp, members, offsets)
    torch.cuda.synchronize()
    graph.replay()
    torch.cuda.synchronize()
    best = None
    for _ in range(replays):
        t0 = time.perf_counter()
        graph.replay()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / steps * 1e6
        best = dt if best is None else min(best, dt)
    return best


def eager_step_us(torch, nl, wl, arena, plan, steps=300):
    """Host-clock cost of an eager step without the event records of the timed loop: plan + launch +
    synchronize per step, and plan + launch back to back with one synchronize at the end."""
    hp = (wl.alpha, wl.beta, wl.gamma)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(steps):
        members, offsets = nl.plan_groups(wl.seed, t, wl.W, wl.n_at(t))
        nl.outer_step(plan, arena.phi, arena.delta, arena.theta, hp, members, offsets)
        torch.cuda.synchronize()
    synced = (time.perf_counter() - t0) / steps * 1e6
    t0 = time.perf_counter()
    for t in range(steps):
        members, offsets = nl.plan_groups(wl.seed, t, wl.W, wl.n_at(t))
        nl.outer_step(plan, arena.phi, arena.delta, arena.theta, hp, members, offsets)
    torch.cuda.synchronize()
    streamed = (time.perf_counter() - t0) / steps * 1e6
    return {"eager_us_per_step_synchronized": synced, "eager_us_per_step_back_to_back": streamed}


def extra_outer(torch, nl, workloads, dev, name, placement, steps, warmup, subgroup=0):
    """A few steps of one configuration for the 'extra' section."""
    wl = workloads.make(name)
    arena = Arena(torch, wl, dev, placement)
    workloads.fill_phi0_device(arena.phi, wl.seed, wl.init_std)
    plan = nl.LaunchPlan(arena.phi, arena.delta, arena.theta, wl.stride, wl.W,
                         nl.F32 if wl.theta_dtype == "f32" else nl.BF16, wl.segments)
    n_of = (lambda t: subgroup) if subgroup else wl.n_at
    run = run_outer_steps(torch, nl, workloads, wl, arena, plan, n_of, steps, warmup)
    res = extra_entry(wl, run, arena.placement, arena.resident_bytes)
    if name == "tiny":
        res.update(eager_step_us(torch, nl, wl, arena, plan))
        res["graph_replay_us_per_step"] = graph_replay_us(torch, nl, wl, arena, plan)
        res["note"] = ("cache-resident (50 MB) and launch-bound: not an HBM measurement; the kernel itself runs "
                       "18 us (rocprofv3), HIP events around so short a launch mostly time the launch")
    plan.destroy()
    arena.free(torch)
    return res


def extra_entry(wl, run, placement, resident_bytes):
    updates = wl.W * wl.P
    total_s = sum(run["host_s"])
    steps = len(run["host_s"])
    avg_ms = sum(run["kernel_ms"]) / steps
    alg = updates * wl.bytes_per_update
    return {"op": "outer_step", "workload": wl.name, "W": wl.W, "theta": wl.theta_dtype, "steps": steps,
            "resident_GB": resident_bytes / 1e9, "placement": placement,
            "ms_per_step": total_s / steps * 1e3, "updates_per_s": updates * steps / total_s,
            "avg_kernel_ms": avg_ms, "GBps": alg / avg_ms / 1e6, "frac": alg / avg_ms / 1e6 / HBM_PEAK_GBPS,
            "per_n": per_n_figures(wl, run),
            "host_plan_groups_us": float(np.median(run["plan_us"])),
            "host_outer_step_call_us": float(np.median(run["call_us"])),
            "traffic": recorded_traffic(f"outer_step_{wl.name}")}


def measure_replica_spread(torch, nl, workloads, dev, wl, placement, steps, warmup):
    """K timed passes of noloco_replica_spread over the slow weights of the workload."""
    W, S = wl.W, wl.stride
    arena = Arena(torch, wl, dev, placement, need_delta=False, need_theta=False)
    phi = arena.phi
    workloads.fill_phi0_device(phi, wl.seed, wl.init_std)
    workloads.fake_inner_phase_device(phi, phi, wl.seed, 0, wl.sigma)      # replicas drift apart
    plan = nl.LaunchPlan(phi, phi, phi, S, W, nl.F32, wl.segments)
    out = torch.zeros(len(wl.segments) + 1, dtype=torch.float64, device=dev)
    kernel_ms, host_s = [], []
    for t in range(warmup + steps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record()
        nl.replica_spread(plan, phi, nl.F32, out)
        e1.record()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        if t >= warmup:
            host_s.append(t1 - t0)
            kernel_ms.append(e0.elapsed_time(e1))
    overall = float(out[-1])
    probes = stream_probes(torch, nl, phi, W, S, dev)     # phi is no longer needed: calibration for counter runs
    plan.destroy()
    arena.free(torch)
    elems = W * wl.P
    avg_ms = sum(kernel_ms) / len(kernel_ms)
    return {"elems": elems, "host_s": host_s, "kernel_ms": kernel_ms, "avg_ms": avg_ms, "overall_std": overall,
            "GBps": elems * 4 / avg_ms / 1e6, "resident_bytes": W * S * 4, "probes": probes}


def run_replica_spread(args, wl, torch, nl, workloads, dev):
    m = measure_replica_spread(torch, nl, workloads, dev, wl, args.placement, args.steps, args.warmup)
    total_s = sum(m["host_s"])
    res = {
        "metric": "replica-spread worker-params/s", "value": m["elems"] * args.steps / total_s,
        "unit": "worker-params/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": total_s / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.name, "W": wl.W, "params_per_worker": wl.P, "tensors": len(wl.tensors),
                   "array": "phi (f32)", "resident_GB": m["resident_bytes"] / 1e9,
                   "overall_std": m["overall_std"], "device": torch.cuda.get_device_name(0)},
        "roofline": {"bound": "hbm", "achieved": m["GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": m["GBps"] / HBM_PEAK_GBPS, "traffic": recorded_traffic(f"replica_spread_{wl.name}"),
                     "kernel": "replica_spread_tiles (+ two pooling kernels)",
                     "algorithmic_bytes_per_launch": m["elems"] * 4, "bytes_per_update": 4,
                     "avg_kernel_ms": m["avg_ms"], "min_kernel_ms": min(m["kernel_ms"]), "max_kernel_ms": max(m["kernel_ms"])},
    }
    res["cpu_baseline"] = None if args.no_cpu_baseline else spread_cpu_baseline(wl)
    print(json.dumps(res))


def main():
    args = parse()
    if args.summarize:
        summarize(args)
        return
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

    with_extra = args.workload is None and not args.no_extra and args.op == "outer_step" \
        and not args.workers and not args.subgroup
    wl = workloads.make(args.workload or DEFAULT_WORKLOAD)
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

    arena = Arena(torch, wl, dev, args.placement)
    workloads.fill_phi0_device(arena.phi, wl.seed, wl.init_std)
    plan = nl.LaunchPlan(arena.phi, arena.delta, arena.theta, S, W,
                         nl.F32 if wl.theta_dtype == "f32" else nl.BF16, wl.segments)
    plan.tune(args.vectors_per_thread, args.nontemporal, args.group_major, args.xcd_map)
    n_of = (lambda t: args.subgroup) if args.subgroup else wl.n_at

    run = run_outer_steps(torch, nl, workloads, wl, arena, plan, n_of, args.steps, args.warmup,
                          inner_phase=not args.no_inner_phase)
    host_s, kernel_ms = run["host_s"], run["kernel_ms"]
    updates = W * wl.P                                    # worker-parameter updates per step
    total_s = sum(host_s)
    ms_per_step = total_s / args.steps * 1e3
    avg_kernel_s = sum(kernel_ms) / len(kernel_ms) / 1e3
    alg_bytes = updates * wl.bytes_per_update             # per launch: one launch covers the whole arena
    achieved = alg_bytes / avg_kernel_s / 1e9

    extra = []
    if with_extra:
        # the larger-subgroup modes on the same resident arena (n = W is the DiLoCo-style outer step)
        plan.tune(-1, -1, -1, -1)
        for n in (4, W):
            r = run_outer_steps(torch, nl, workloads, wl, arena, plan, lambda t, n=n: n, 3, 1)
            extra.append(extra_entry(wl, r, arena.placement, arena.resident_bytes))

    probes = stream_probes(torch, nl, arena.delta, W, S, dev)

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
            "theta_dtype": wl.theta_dtype, "subgroup_n": sorted(set(run["n"])),
            "alpha": wl.alpha, "beta": wl.beta, "gamma": wl.gamma, "drift_sigma": wl.sigma,
            "resident_GB": W * per_worker / 1e9, "placement": arena.placement,
            "device": torch.cuda.get_device_name(0), "launch": plan.info(), "note": note,
        },
        "roofline": {
            "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBPS, "traffic": recorded_traffic(f"outer_step_{wl.name}"),
            "kernel": kernel_of(run["n"][0]),
            "algorithmic_bytes_per_launch": alg_bytes,
            "bytes_per_update": wl.bytes_per_update,
            "avg_kernel_ms": avg_kernel_s * 1e3, "median_kernel_ms": float(np.median(kernel_ms)),
            "min_kernel_ms": min(kernel_ms), "max_kernel_ms": max(kernel_ms),
            "per_n": per_n_figures(wl, run),
            "copy_probe_GBps": probes["copy"], "read_probe_GBps": probes["read"],
            "fill_probe_GBps": probes["fill"], "runtime_copy_GBps": probes["runtime_copy"],
        },
        "host": {"plan_groups_us": float(np.median(run["plan_us"])),
                 "outer_step_call_us": float(np.median(run["call_us"])),
                 "step_minus_kernel_ms": ms_per_step - avg_kernel_s * 1e3},
    }
    plan.destroy()
    arena.free(torch)

    if with_extra:
        for name in ("tiny", "gpt125m", "stage1p3b", "ragged_tight", "ragged_gapped"):
            if name == wl.name:
                continue
            k = 12 if name.startswith("ragged") else 6     # the ragged schedule cycles n = 2, 4, 8
            extra.append(extra_outer(torch, nl, workloads, dev, name, args.placement, k, 3))
        if args.placement == "spread":
            # the same small arena from three neighbouring allocations, for comparison (see class Arena)
            extra.append(extra_outer(torch, nl, workloads, dev, "gpt125m", "plain", 6, 3))
        m = measure_replica_spread(torch, nl, workloads, dev, workloads.make(DEFAULT_WORKLOAD), args.placement, 5, 2)
        extra.append({"op": "replica_spread", "workload": DEFAULT_WORKLOAD, "array": "phi (f32)", "steps": 5,
                      "resident_GB": m["resident_bytes"] / 1e9, "ms_per_step": sum(m["host_s"]) / 5 * 1e3,
                      "avg_kernel_ms": m["avg_ms"], "GBps": m["GBps"], "frac": m["GBps"] / HBM_PEAK_GBPS,
                      "kernel": "replica_spread_tiles", "traffic": recorded_traffic(f"replica_spread_{DEFAULT_WORKLOAD}")})
        out["extra"] = extra

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, run["n"][0], hp)
    else:
        out["cpu_baseline"] = None
    print(json.dumps(out))


if __name__ == "__main__":
    main()
