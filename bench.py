#!/usr/bin/env python3
"""Benchmark of the WAGMA-SGD hot path on one MI355X.

A step is one wagma_step(): local momentum-SGD update of all P replicas, group model average
with the lateness rule (or the global average every tau-th iteration), send-buffer refresh
(Algorithm 2 lines 6-17 with the groups of Algorithm 1).  All inputs are resident in HBM before
the timed region.  Prints ONE JSON line on stdout; progress goes to stderr.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 1..5] [--opt NAME=VALUE ...]

The default run times the headline workload (4: P=64, S=8, 25.6M parameters) on arrays placed by
the library's allocator, then the same steps on ordinary torch allocations ("plain_alloc": what
a caller who brings its own buffers gets), then measures the HBM traffic of the group launches
with the counters (two child runs under rocprofv3: "roofline.traffic"), then the other four
seeded workloads in child processes ("workloads"), then the CPU oracle on the host cores
("cpu_baseline").  --no-extras stops after the headline run.
"""
from __future__ import annotations

import argparse
import json
import os
import subprocess
import sys
import time

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published peak

# HBM bytes per launch of the dominant kernel from two `rocprofv3 --pmc` runs (FETCH_SIZE scaled by
# 2.000, WRITE_SIZE by 1.000, the factors a plain copy of known size gave in the same runs), averaged
# over the group launches of the profiled command; valid for the launch options of PROFILE_OPTIONS
# only.  workload -> (bytes per launch, the file under profiles/ that holds the figure).
MEASURED_TRAFFIC = {
    2: (10.116e9, "group_step_S4__resnet50-25.6M_P16_S4.md"),
    3: (24.017e9, "group_step_S4__transformer-base-61.4M_P16_S4.md"),
    4: (40.94e9, "group_step_S8__resnet50-25.6M_P64_S8.md"),
    5: (166.38e9, "group_step_S8__transformer-big-210.8M_P32_S8.md"),
}
# --tensors --tensor-layout stacked (as views into rows the tensors are joined and the step is the flat one)
MEASURED_TRAFFIC_PER_TENSOR = {4: (40.939e9, "group_step_S8_per_tensor__resnet50-25.6M_P64_S8.md")}
# option number -> value the profiles were taken with (the library's defaults at that time)
PROFILE_OPTIONS = {"nontemporal": 1, "force_stream": 0, "stripe_log2": 2, "xcd_chunk_log2": -1, "map": 0}

OPTS = {"nontemporal": 2, "force_stream": 3, "stripe_log2": 7, "xcd_chunk_log2": 8, "placement": 9, "placed_shape": 10,
        "map": 11, "placed_coop_shape": 12}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def popcount(words) -> int:
    return sum(bin(int(x)).count("1") for x in words)


# ---------------------------------------------------------------- CPU oracle baseline

def oracle_slice_state(wl, columns: int, iters: int, seed_offset: int = 0):
    """Inputs of the oracle on a column slice (columns are independent, so a slice is the same
    work per replica-parameter): all P rows, the workload's gradient scale and masks."""
    import numpy as np
    import torch
    from oracle import wagma_oracle as orc
    from paper_2005_00124_amd import workloads as wk

    P = wl.P
    gen = wk.make_generator(wl.seed + seed_offset, "cpu")
    row = torch.empty(columns)
    row.normal_(0.0, 0.05, generator=gen)
    w = np.repeat(row.numpy()[None, :], P, axis=0).copy()
    m = np.zeros_like(w)
    pub = w.copy()
    g = torch.empty((P, columns)).normal_(0.0, wl.grad_std, generator=gen).numpy()
    masks = [orc.stale_mask(wl.seed, t, P, wl.stale_threshold) for t in range(iters)]
    return w, g, m, pub, masks


def oracle_run(wl, state, iters: int) -> float:
    """Seconds the oracle takes for `iters` iterations on `state` (one thread)."""
    from oracle import wagma_oracle as orc
    w, g, m, pub, masks = state
    t0 = time.perf_counter()
    for t in range(iters):
        orc.step_f32(wl.P, wl.S, wl.tau, t, w, g, m, pub, masks[t], wl.lr, wl.mu)
    return time.perf_counter() - t0


def cpu_shard_main(args) -> int:
    """Child of the all-cores leg: sets up its column shard, says "ready", waits for "go" on
    stdin, runs, prints its seconds.  CPU only."""
    from oracle import wagma_oracle as orc
    from paper_2005_00124_amd import workloads as wk
    wl = wk.workload(args.workload)
    iters = args.steps
    state = oracle_slice_state(wl, args.cpu_shard, iters, seed_offset=1000 + args.shard_index)
    w, g, m, pub, masks = state
    orc.step_f32(wl.P, wl.S, wl.tau, 0, w.copy(), g, m.copy(), pub.copy(), masks[0], wl.lr, wl.mu)  # warm
    print("ready", flush=True)
    if sys.stdin.readline().strip() != "go":
        return 1
    start = time.time()
    seconds = oracle_run(wl, state, iters)
    print(json.dumps({"seconds": seconds, "start": start, "end": time.time()}), flush=True)
    return 0


def cpu_model_name() -> str:
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(wl, columns: int, iters: int, workers: int):
    """The CPU oracle as it stands: one thread on a `columns`-column slice of the workload, and
    the same binary as `workers` column-sharded processes (fresh children, CPU only)."""
    from oracle import wagma_oracle as orc
    P = wl.P
    state = oracle_slice_state(wl, columns, iters)
    w, g, m, pub, masks = state
    orc.step_f32(P, wl.S, wl.tau, 0, w[:, :4096].copy(), g[:, :4096].copy(), m[:, :4096].copy(),
                 pub[:, :4096].copy(), masks[0], wl.lr, wl.mu)   # warm (library load, page faults of the code)
    dt = oracle_run(wl, state, iters)
    out = {"value": P * columns * iters / dt, "unit": "replica-params/s", "cores": 1, "kind": "oracle",
           "cpu_model": cpu_model_name(),
           "sample": "%d-column slice of all %d rows, %d iterations (group and global, same masks), "
                     "%.1f s single-threaded" % (columns, P, iters, dt)}
    del state, w, g, m, pub
    if workers > 1:
        shard = max(4096, columns // workers)
        cmd = [sys.executable, os.path.abspath(__file__), "--workload", str(wl.index), "--steps", str(iters),
               "--cpu-shard", str(shard)]
        env = dict(os.environ, OMP_NUM_THREADS="1", HIP_VISIBLE_DEVICES="", CUDA_VISIBLE_DEVICES="")
        kids = [subprocess.Popen(cmd + ["--shard-index", str(k)], stdin=subprocess.PIPE, stdout=subprocess.PIPE,
                                 text=True, env=env) for k in range(workers)]
        try:
            ok = all(kid.stdout.readline().strip() == "ready" for kid in kids)
            for kid in kids:
                kid.stdin.write("go\n" if ok else "stop\n")
                kid.stdin.flush()
            results = [json.loads(kid.stdout.readline()) for kid in kids] if ok else []
        except (ValueError, OSError):
            results = []
        for kid in kids:
            try:
                kid.wait(timeout=60)
            except subprocess.TimeoutExpired:
                kid.kill()
        if len(results) == workers:
            span = max(r["end"] for r in results) - min(r["start"] for r in results)
            out["all_cores"] = {
                "value": P * shard * iters * workers / span, "unit": "replica-params/s", "cores": workers,
                "cpu_model": cpu_model_name(),
                "sample": "%d processes, each the oracle on its own %d-column shard of all %d rows, %d iterations; "
                          "%.1f s from the first start to the last end" % (workers, shard, P, iters, span)}
        else:
            out["all_cores"] = {"error": "a shard process failed"}
    return out


# ---------------------------------------------------------------- HBM traffic from the counters

def measure_traffic(workload: int, K: int, W: int, array_bytes: int):
    """HBM bytes per group launch of this very command, measured now: two child runs of the
    headline part of this script under `rocprofv3 --pmc` (FETCH_SIZE, then WRITE_SIZE, each in a
    run of its own), each counter scaled by what it reads for the plain device copy of one whole
    array (`array_bytes`) in the same run.  Returns a dict, or None if the profiler is not there
    or a run fails."""
    import csv
    import glob
    import shutil
    import tempfile
    if shutil.which("rocprofv3") is None:
        return None
    per_launch, factors = {}, {}
    for counter in ("FETCH_SIZE", "WRITE_SIZE"):
        out_dir = tempfile.mkdtemp(prefix="wagma_pmc_", dir="/tmp")
        cmd = ["rocprofv3", "--kernel-trace", "--pmc", counter, "--output-format", "csv", "-d", out_dir, "--",
               sys.executable, os.path.abspath(__file__), "--workload", str(workload), "--no-extras",
               "--no-cpu-baseline", "--steps", str(K), "--warmup", str(W)]
        try:
            run = subprocess.run(cmd, cwd="/tmp", env=dict(os.environ, TMPDIR="/tmp"), capture_output=True,
                                 text=True, timeout=300)
            files = glob.glob(os.path.join(out_dir, "**", "*_counter_collection.csv"), recursive=True)
            if run.returncode != 0 or not files:
                return None
            steps, copies = [], []
            for row in csv.DictReader(open(files[0])):
                if row["Counter_Name"] != counter:
                    continue
                nbytes = float(row["Counter_Value"]) * 1024.0          # the counters are in KiB
                if "step_rows" in row["Kernel_Name"] or "step_tensors" in row["Kernel_Name"]:
                    steps.append((row["Kernel_Name"], nbytes))
                elif "copyBuffer" in row["Kernel_Name"]:
                    copies.append(nbytes)
            timed = [b for name, b in steps[-K:] if "in_registers" in name]      # the group launches
            if not timed or not copies or max(copies) <= 0:
                return None
            factors[counter] = array_bytes / max(copies)
            per_launch[counter] = sum(timed) / len(timed)
        except (OSError, subprocess.TimeoutExpired, KeyError, ValueError):
            return None
        finally:
            shutil.rmtree(out_dir, ignore_errors=True)
    return {"bytes": factors["FETCH_SIZE"] * per_launch["FETCH_SIZE"] + factors["WRITE_SIZE"] * per_launch["WRITE_SIZE"],
            "fetch_factor": factors["FETCH_SIZE"], "write_factor": factors["WRITE_SIZE"]}


# ---------------------------------------------------------------- GPU timing

def time_steps(step, stream, K, graph=False):
    """Per-step milliseconds (HIP events on the launch stream) and the wall time of K steps."""
    import torch
    starts = [torch.cuda.Event(enable_timing=True) for _ in range(K)]
    ends = [torch.cuda.Event(enable_timing=True) for _ in range(K)]
    if graph:
        # masks and iteration numbers are baked into the captured launches
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                for t in range(K):
                    step(t)
        stream.wait_stream(side)
        g.replay()                      # untimed first replay
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        starts[0].record(stream)
        g.replay()
        ends[0].record(stream)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        per_step = starts[0].elapsed_time(ends[0]) / K      # no events inside a graph: the mean
        return [per_step] * K, wall
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(K):
        starts[t].record(stream)
        step(t)
        ends[t].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return [starts[t].elapsed_time(ends[t]) for t in range(K)], wall


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", type=int, default=4, help="1..5; 4 = the headline P=64 S=8 25.6M")
    ap.add_argument("--P", type=int, default=None, help="override the workload's number of replicas")
    ap.add_argument("--S", type=int, default=None, help="override the workload's group size")
    ap.add_argument("--tau", type=int, default=None, help="override the workload's global period")
    ap.add_argument("--opt", action="append", default=[], help="launch switch NAME=VALUE (%s)" % ", ".join(OPTS))
    ap.add_argument("--ld", type=int, default=None, help="row stride override (floats)")
    ap.add_argument("--plain-alloc", action="store_true",
                    help="ordinary torch allocations instead of the library's HBM-region-aware allocator")
    ap.add_argument("--tensors", action="store_true",
                    help="time wagma_step_tensors on the workload's tensor list (views into the same rows)")
    ap.add_argument("--tensor-layout", choices=("views", "stacked", "separate"), default="views",
                    help="with --tensors, where the tensors lie: views into the rows of the flat arrays, back to "
                         "back (the library joins them); every parameter stacked to its own [P, size] torch "
                         "allocation; or every tensor of every replica a torch allocation of its own")
    ap.add_argument("--graph", action="store_true",
                    help="capture the K steps in one HIP graph and time its replay (for launch-bound sizes)")
    ap.add_argument("--lag", type=int, default=None, metavar="TOLERANCE_MS",
                    help="lateness deeper than one iteration: wagma_lag_masks with this tolerance drive "
                         "wagma_step_lag instead of the workload's Bernoulli mask")
    ap.add_argument("--use-memory-first", action="store_true",
                    help="before anything is allocated, make the GPU's memory one that has been in use: 120 "
                         "allocations of 0.2 to 3.5 GiB, half of them freed in random order, 20 more, then all "
                         "given back (what ordinary allocations return afterwards is mixed over the HBM regions)")
    ap.add_argument("--no-extras", action="store_true",
                    help="the headline run only: no plain-allocation leg, no other workloads")
    ap.add_argument("--no-counters", action="store_true",
                    help="do not run the two rocprofv3 child runs that measure roofline.traffic (the figure "
                         "stored under profiles/ is reported instead)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-columns", type=int, default=1048576)
    ap.add_argument("--cpu-workers", type=int, default=None,
                    help="processes of the all-cores oracle leg (default: the host's cores, at most OMP_NUM_THREADS)")
    ap.add_argument("--cpu-shard", type=int, default=None, help=argparse.SUPPRESS)
    ap.add_argument("--shard-index", type=int, default=0, help=argparse.SUPPRESS)
    args = ap.parse_args()

    if args.cpu_shard is not None:
        return cpu_shard_main(args)
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU only (the P workers are rows in one GPU's HBM); "
            "--gpus %d is not supported" % args.gpus)
        return 2

    import numpy as np
    import torch
    from paper_2005_00124_amd import wagma as lw
    from paper_2005_00124_amd import workloads as wk

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible; the HIP path has no CPU fallback")
        return 2
    if not os.path.exists(lw.LIB_PATH):
        from paper_2005_00124_amd import build
        build.build()

    wl = wk.workload(args.workload)
    custom = {k: v for k, v in (("P", args.P), ("S", args.S), ("tau", args.tau)) if v is not None}
    if custom:
        import dataclasses
        wl = dataclasses.replace(wl, **custom)
        wl = dataclasses.replace(wl, name="%s with %s" % (wl.name, ", ".join("%s=%d" % kv for kv in custom.items())))
    variant = bool(custom or args.opt or args.ld or args.tensors or args.graph or args.lag is not None
                   or args.plain_alloc or args.use_memory_first)
    extras = not args.no_extras and not variant and args.workload == 4
    K = wl.iters if args.steps is None else args.steps
    W = args.warmup
    P, S, n = wl.P, wl.S, wl.n
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.use_memory_first:
        import random
        rnd = random.Random(1)
        free_bytes = torch.cuda.mem_get_info()[0]
        held, total = [], 0
        for _ in range(120):
            size = int(rnd.uniform(0.2, 3.5) * 2 ** 30)
            if total + size > 0.8 * free_bytes:
                break
            held.append(torch.empty(size, dtype=torch.uint8, device=dev).fill_(1))
            total += size
        rnd.shuffle(held)
        del held[:len(held) // 2]
        more = [torch.empty(int(rnd.uniform(0.2, 3.5) * 2 ** 30), dtype=torch.uint8, device=dev).fill_(2)
                for _ in range(20)]
        torch.cuda.synchronize()
        del held, more
        torch.cuda.empty_cache()
        log("the GPU's memory has been used: %.0f GB allocated, freed in random order" % (total / 1e9))

    ctx = lw.Wagma(P, S, n, wl.tau)
    if args.ld:
        ctx.set_row_stride(args.ld)
    defaults_match = all(ctx.debug_get_option(OPTS[k]) == v for k, v in PROFILE_OPTIONS.items())
    for kv in args.opt:
        k, v = kv.split("=")
        ctx.debug_set_option(OPTS[k], int(v, 0))
    ld = ctx.ld
    log("workload %d: %s  n=%d ld=%d  buffers 4 x %.2f GB" % (wl.index, wl.name, n, ld, P * ld * 4 / 1e9))
    busy_masks = None
    if args.lag is None:
        masks = [ctx.stale_mask(wl.seed, t, wl.stale_threshold) for t in range(max(K, W))]
    else:
        both = [ctx.lag_masks(wl.seed, t, args.lag) for t in range(max(K, W))]
        masks = [late for late, _ in both]
        busy_masks = [busy for _, busy in both]
    stream = torch.cuda.current_stream()
    is_global = [ctx.is_global(t) for t in range(K)]
    grp = [t for t in range(K) if not is_global[t]]
    glb = [t for t in range(K) if is_global[t]]
    late = [0 if is_global[t] else popcount(masks[t]) for t in range(K)]
    busy = [0 if is_global[t] or busy_masks is None else popcount(busy_masks[t]) for t in range(K)]
    # algorithmic bytes: read w, g, m and write w, m, pub for every replica-parameter
    # (24 B), plus a 4 B send-buffer read for every late replica-parameter; of a process
    # that is still computing only the send buffer is read (4 B)
    bytes_of = [n * (24 * (P - busy[t]) + 4 * late[t] + 4 * busy[t]) for t in range(K)]

    def run_on(w, g, m, pub, steps):
        """Fill the arrays, warm up, time `steps` steps; returns (per-step ms, wall seconds)."""
        wk.fill_initial_state(wl, w, m, pub)
        wk.fill_gradients(wl, 0, g)       # one gradient slab, reused: generating it is not part of the path
        plan = None
        if args.tensors:
            import math
            sizes = [math.prod(t[1]) for t in wl.tensors()]

            def views(buf):
                out = []
                for p in range(P):
                    at, row = 0, []
                    for size in sizes:
                        row.append(buf[p, at:at + size])
                        at += size
                    out.append(row)
                return out
            if args.tensor_layout == "views":
                lists = [views(w), views(g), views(m), views(pub)]
            else:
                # the tensors live in torch allocations of their own (the flat arrays stay unused);
                # the bandwidth does not depend on the values: small normal numbers, as in the rows
                lists = []
                for scale in (0.05, 0.01, 0.01, 0.05):
                    if args.tensor_layout == "stacked":
                        stacks = [torch.empty((P, size + (-size) % 4), device="cuda").normal_(0.0, scale)
                                  for size in sizes]
                        lists.append([[stack[p, :size] for stack, size in zip(stacks, sizes)] for p in range(P)])
                    else:
                        per = [[torch.empty(size, device="cuda") for size in sizes] for p in range(P)]
                        every = [t for row in per for t in row]
                        torch._foreach_zero_(every)          # P x T allocations, filled by a few launches
                        torch._foreach_add_(every, scale)
                        lists.append(per)
            plan = ctx.tensor_plan(*lists)
            log("per-tensor layout (%s): %d tensors per replica" % (args.tensor_layout, len(sizes)))

        def step(t):
            b = None if busy_masks is None else busy_masks[t]
            if plan is not None:
                plan.step(masks[t], wl.lr, wl.mu, t, busy_mask=b)
            else:
                ctx.step(w, g, m, pub, masks[t], wl.lr, wl.mu, t, busy_mask=b)

        for t in range(W):
            step(t)
        torch.cuda.synchronize()
        ms, wall = time_steps(step, stream, steps, graph=args.graph)
        assert torch.isfinite(w[:, :n]).all()
        if plan is not None:
            plan.destroy()
        return ms, wall

    if args.plain_alloc:
        bufs = ctx.alloc()
        placement = "torch allocations"
    else:
        bufs = ctx.alloc_placed()     # w, m, pub in different HBM regions
        info = ctx.placement_info()
        placement = "wagma_alloc_buffers: %(mode)s placement, %(candidates)d memory blocks examined" % info
        if info["mode"] == "chunks":   # which of the three chunk patterns: pub apart 2, one region 1, three regions 3
            placement += ", w, m and pub in %d region%s" % (info["regions"], "" if info["regions"] == 1 else "s")
        placement += ", launch shapes %d (group rows in registers) and %d (rows over a workgroup) measured best on them" % (
            ctx.debug_get_option(lw.WAGMA_DEBUG_PLACED_SHAPE), ctx.debug_get_option(lw.WAGMA_DEBUG_PLACED_COOP_SHAPE))
        log("placement:", info)
    ms, wall = run_on(*bufs, K)
    grp_ms = sum(ms[t] for t in grp)
    glb_ms = sum(ms[t] for t in glb)

    if grp:
        dom, dom_ts = "group step (S=%d member rows %s%s)" % (
            S, "in registers" if S <= 8 else "dealt out to the wavefronts of a workgroup" if S <= 64 else "streamed",
            ", per-tensor layout" if args.tensors else ""), grp
    else:
        dom, dom_ts = "global step (all P rows one group)", glb
    dom_ms = sum(ms[t] for t in dom_ts)
    achieved = sum(bytes_of[t] for t in dom_ts) / (dom_ms * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                "avg_launch_ms": dom_ms / len(dom_ts), "launches": len(dom_ts),
                "algorithmic_bytes_per_launch": sum(bytes_of[t] for t in dom_ts) / len(dom_ts),
                "traffic": None, "traffic_source": None}
    if args.tensors:
        stored = MEASURED_TRAFFIC_PER_TENSOR.get(wl.index) if args.tensor_layout == "stacked" else None
    else:
        stored = MEASURED_TRAFFIC.get(wl.index)
    if (stored and grp and defaults_match and not args.opt and not args.ld and args.lag is None
            and not custom and not args.graph):
        # HBM bytes of such a launch as the counters measured them in the profiled run; stale
        # (hence left out) as soon as the library's launch defaults differ from that run's
        roofline["traffic"] = stored[0]
        roofline["traffic_source"] = "profiles/" + stored[1] + " (counter runs of that file, not of this run)"
    out = {
        "metric": "replica-params averaged/sec", "value": P * n * K / wall, "unit": "replica-params/s",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": wall * 1e3 / K,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.name, "P": P, "S": S, "n": n, "ld": ld, "tau": wl.tau,
                   "late_probability": wl.q if args.lag is None else None,
                   "lateness": "Bernoulli mask per iteration" if args.lag is None else
                   "steps back to back, tolerance %d ms: %.3f of the process-iterations late, %.3f still computing"
                   % (args.lag, sum(late) / max(1, P * len(grp)), sum(busy) / max(1, P * len(grp))),
                   "global_steps_in_run": len(glb),
                   "options": args.opt, "allocation": placement,
                   "layout": "per-tensor (%s)" % args.tensor_layout if args.tensors else "flat rows",
                   "launch": "one HIP graph of K steps" if args.graph else "one launch per step"},
        "hbm_gbs_all_steps": sum(bytes_of) / ((grp_ms + glb_ms) * 1e-3) / 1e9,
        "group_step_ms": (grp_ms / len(grp)) if grp else None,
        "group_step_ms_median": float(np.median([ms[t] for t in grp])) if grp else None,
        "group_step_ms_min": min(ms[t] for t in grp) if grp else None,
        "global_step_ms": (glb_ms / len(glb)) if glb else None,
        "global_step_gbs": (sum(bytes_of[t] for t in glb) / (glb_ms * 1e-3) / 1e9) if glb else None,
        "roofline": roofline,
    }
    del bufs
    if not args.plain_alloc:
        ctx.free_placed()

    if extras:
        # the boundary's own configuration: the caller owns w, g, m, pub (torch allocations)
        log("the same steps on torch allocations ...")
        bufs = ctx.alloc()
        pms, _ = run_on(*bufs, K)
        del bufs
        p_ms = sum(pms[t] for t in dom_ts)
        p_gbs = sum(bytes_of[t] for t in dom_ts) / (p_ms * 1e-3) / 1e9
        out["plain_alloc"] = {"allocation": "torch allocations (caller-owned buffers)", "kernel": dom,
                              "group_step_ms": p_ms / len(dom_ts), "achieved": p_gbs, "unit": "GB/s",
                              "frac": p_gbs / HBM_PEAK_GBS, "launches": len(dom_ts)}
    ctx.destroy()
    torch.cuda.empty_cache()

    if extras and not args.no_counters:
        log("HBM traffic of the group launches from the counters (two profiler runs of this command) ...")
        measured = measure_traffic(wl.index, K, W, P * ld * 4)
        if measured is not None:
            roofline["traffic"] = measured["bytes"]
            roofline["traffic_source"] = (
                "measured now: rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE, each in a child run of this command "
                "(--no-extras), average over its %d group launches, scaled by %.3f and %.3f (what each counter "
                "reads for the device copy of one %d-byte array in the same run)"
                % (len(dom_ts), measured["fetch_factor"], measured["write_factor"], P * ld * 4))
            roofline["traffic_gbs"] = measured["bytes"] / (roofline["avg_launch_ms"] * 1e-3) / 1e9

    if extras:
        summary = {wl.index: {"workload": wl.name, "value": out["value"], "ms_per_step": out["ms_per_step"],
                              "group_step_gbs": roofline["achieved"], "frac": roofline["frac"],
                              "global_step_gbs": out["global_step_gbs"]}}
        # the largest first: how much of a box's memory earlier processes have used and given back
        # shows in the rates (workload 5 as the first process on a box: 0.82; after the others: 0.79)
        for k in range(len(wk.WORKLOADS), 0, -1):
            if k == wl.index:
                continue
            log("workload %d ..." % k)
            try:
                child = subprocess.run([sys.executable, os.path.abspath(__file__), "--workload", str(k),
                                        "--no-cpu-baseline", "--no-extras", "--warmup", str(W)],
                                       capture_output=True, text=True, timeout=240)
                line = [x for x in child.stdout.splitlines() if x.startswith("{")]
                if child.returncode != 0 or not line:
                    raise RuntimeError(child.stderr[-300:])
                o = json.loads(line[-1])
                summary[k] = {"workload": o["config"]["workload"], "value": o["value"], "ms_per_step": o["ms_per_step"],
                              "group_step_gbs": o["roofline"]["achieved"], "frac": o["roofline"]["frac"],
                              "global_step_gbs": o["global_step_gbs"], "allocation": o["config"]["allocation"]}
            except (RuntimeError, subprocess.TimeoutExpired, ValueError) as e:
                summary[k] = {"error": str(e)[-300:]}
        out["workloads"] = {str(k): summary[k] for k in sorted(summary)}
    if not args.no_cpu_baseline:
        log("timing the CPU oracle on a slice ...")
        workers = args.cpu_workers
        if workers is None:
            workers = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "16") or 16))
        out["cpu_baseline"] = cpu_baseline(wl, args.cpu_columns, min(K, wl.iters), workers)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
