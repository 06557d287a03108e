#!/usr/bin/env python3
"""Benchmark of the WAGMA-SGD hot path on one MI355X.

A step is one wagma_step(): local momentum-SGD update of all P replicas, group model average
with the lateness rule (or the global average every tau-th iteration), send-buffer refresh
(Algorithm 2 lines 6-17 with the groups of Algorithm 1).  All inputs are resident in HBM before
the timed region.  Prints ONE JSON line on stdout; progress goes to stderr.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 1..5] [--opt NAME=VALUE ...]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published peak

# HBM bytes per launch of the dominant kernel from two `rocprofv3 --pmc` runs (FETCH_SIZE scaled by
# 2.000, WRITE_SIZE by 1.000, the factors a plain copy of known size gave in the same runs), averaged
# over the group launches of `bench.py --steps 20` (10 for workload 5); valid for the default launch
# options only.  Source: the files under profiles/ for these kernels and workloads.
MEASURED_TRAFFIC_BYTES = {2: 10.116e9, 3: 24.016e9, 4: 40.92e9, 5: 166.41e9}
MEASURED_TRAFFIC_BYTES_PER_TENSOR = {4: 40.94e9}

OPTS = {"block": 1, "nontemporal": 2, "force_stream": 3, "xcd_swizzle": 4, "tile_major": 5, "waves": 6,
        "stripe_log2": 7, "xcd_chunk_log2": 8, "placement": 9}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def popcount(words) -> int:
    return sum(bin(int(x)).count("1") for x in words)


def cpu_baseline(wl, columns: int, iters: int):
    """The CPU oracle as it stands, one thread, on a column slice of the same workload
    (columns are independent, so a slice is the same work per replica-parameter)."""
    import numpy as np
    import torch
    from oracle import wagma_oracle as orc
    from paper_2005_00124_amd import workloads as wk

    P = wl.P
    gen = wk.make_generator(wl.seed, "cpu")
    row = torch.empty(columns)
    row.normal_(0.0, 0.05, generator=gen)
    w = np.repeat(row.numpy()[None, :], P, axis=0).copy()
    m = np.zeros_like(w)
    pub = w.copy()
    g = torch.empty((P, columns)).normal_(0.0, wl.grad_std, generator=gen).numpy()
    masks = [orc.stale_mask(wl.seed, t, P, wl.stale_threshold) for t in range(iters)]
    orc.step_f32(P, wl.S, wl.tau, 0, w.copy(), g, m.copy(), pub.copy(), masks[0], wl.lr, wl.mu)  # warm
    t0 = time.perf_counter()
    for t in range(iters):
        orc.step_f32(P, wl.S, wl.tau, t, w, g, m, pub, masks[t], wl.lr, wl.mu)
    dt = time.perf_counter() - t0
    return {"value": P * columns * iters / dt, "unit": "replica-params/s", "cores": 1,
            "kind": "oracle",
            "sample": "%d-column slice of all %d rows, %d iterations (group and global, same masks), "
                      "%.1f s single-threaded" % (columns, P, iters, dt)}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", type=int, default=4, help="1..5; 4 = the headline P=64 S=8 25.6M")
    ap.add_argument("--P", type=int, default=None, help="override the workload's number of replicas")
    ap.add_argument("--S", type=int, default=None, help="override the workload's group size")
    ap.add_argument("--tau", type=int, default=None, help="override the workload's global period")
    ap.add_argument("--opt", action="append", default=[], help="tuning knob NAME=VALUE (%s)" % ", ".join(OPTS))
    ap.add_argument("--ld", type=int, default=None, help="row stride override (floats)")
    ap.add_argument("--plain-alloc", action="store_true",
                    help="ordinary torch allocations instead of the library's HBM-region-aware allocator")
    ap.add_argument("--tensors", action="store_true",
                    help="time wagma_step_tensors on the workload's tensor list (views into the same rows)")
    ap.add_argument("--graph", action="store_true",
                    help="capture the K steps in one HIP graph and time its replay (for launch-bound sizes)")
    ap.add_argument("--lag", type=int, default=None, metavar="TOLERANCE_MS",
                    help="lateness deeper than one iteration: wagma_lag_masks with this tolerance drive "
                         "wagma_step_lag instead of the workload's Bernoulli mask")
    ap.add_argument("--all-workloads", action="store_true",
                    help="afterwards run the other four seeded workloads too (child processes of this "
                         "script) and attach their throughput and bandwidth as \"workloads\"")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-columns", type=int, default=131072)
    args = ap.parse_args()

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
    K = wl.iters if args.steps is None else args.steps
    W = args.warmup
    P, S, n = wl.P, wl.S, wl.n
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    ctx = lw.Wagma(P, S, n, wl.tau)
    if args.ld:
        ctx.set_row_stride(args.ld)
    for kv in args.opt:
        k, v = kv.split("=")
        ctx.set_option(OPTS[k], int(v))
    ld = ctx.ld
    log("workload %d: %s  n=%d ld=%d  buffers 4 x %.2f GB" % (wl.index, wl.name, n, ld, P * ld * 4 / 1e9))
    if args.plain_alloc:
        w, g, m, pub = ctx.alloc()
        placement = "torch allocations"
    else:
        w, g, m, pub = ctx.alloc_placed()     # w, m, pub in different HBM regions
        info = ctx.placement_info()
        placement = "wagma_alloc_buffers: %(mode)s placement, %(candidates)d memory blocks examined" % info
        log("placement:", info)
    wk.fill_initial_state(wl, w, m, pub)
    wk.fill_gradients(wl, 0, g)       # one gradient slab, reused: generating it is not part of the path
    busy_masks = None
    if args.lag is None:
        masks = [ctx.stale_mask(wl.seed, t, wl.stale_threshold) for t in range(max(K, W))]
    else:
        both = [ctx.lag_masks(wl.seed, t, args.lag) for t in range(max(K, W))]
        masks = [late for late, _ in both]
        busy_masks = [busy for _, busy in both]
    stream = torch.cuda.current_stream()

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
        plan = ctx.tensor_plan(views(w), views(g), views(m), views(pub))
        log("per-tensor layout: %d tensors per replica" % len(sizes))

    def step(t):
        busy = None if busy_masks is None else busy_masks[t]
        if plan is not None:
            plan.step(masks[t], wl.lr, wl.mu, t, busy_mask=busy)
        else:
            ctx.step(w, g, m, pub, masks[t], wl.lr, wl.mu, t, busy_mask=busy)

    for t in range(W):
        step(t)
    torch.cuda.synchronize()

    starts = [torch.cuda.Event(enable_timing=True) for _ in range(K)]
    ends = [torch.cuda.Event(enable_timing=True) for _ in range(K)]
    if args.graph:
        # masks and iteration numbers are baked into the captured launches
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                for t in range(K):
                    step(t)
        stream.wait_stream(side)
        graph.replay()                      # untimed first replay
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        starts[0].record(stream)
        graph.replay()
        ends[0].record(stream)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        per_step = starts[0].elapsed_time(ends[0]) / K      # no events inside a graph: the mean
        ms = [per_step] * K
    else:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for t in range(K):
            starts[t].record(stream)
            step(t)
            ends[t].record(stream)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        ms = [starts[t].elapsed_time(ends[t]) for t in range(K)]
    is_global = [ctx.is_global(t) for t in range(K)]
    grp = [t for t in range(K) if not is_global[t]]
    glb = [t for t in range(K) if is_global[t]]
    late = [0 if is_global[t] else popcount(masks[t]) for t in range(K)]
    busy = [0 if is_global[t] or busy_masks is None else popcount(busy_masks[t]) for t in range(K)]
    # algorithmic bytes: read w, g, m and write w, m, pub for every replica-parameter
    # (24 B), plus a 4 B send-buffer read for every late replica-parameter; of a process
    # that is still computing only the send buffer is read (4 B)
    bytes_of = [n * (24 * (P - busy[t]) + 4 * late[t] + 4 * busy[t]) for t in range(K)]
    grp_ms = sum(ms[t] for t in grp)
    glb_ms = sum(ms[t] for t in glb)
    assert torch.isfinite(w[:, :n]).all()

    if grp:
        dom, dom_ts = "group step (S=%d member rows %s%s)" % (
            S, "in registers" if S <= 8 else "streamed", ", per-tensor layout" if plan is not None else ""), grp
    else:
        dom, dom_ts = "global step (rows streamed)", glb
    dom_ms = sum(ms[t] for t in dom_ts)
    achieved = sum(bytes_of[t] for t in dom_ts) / (dom_ms * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                "avg_launch_ms": dom_ms / len(dom_ts), "launches": len(dom_ts),
                "algorithmic_bytes_per_launch": sum(bytes_of[t] for t in dom_ts) / len(dom_ts),
                "traffic": (MEASURED_TRAFFIC_BYTES if plan is None else MEASURED_TRAFFIC_BYTES_PER_TENSOR).get(wl.index)
                if grp and not args.opt and not args.ld and args.lag is None and not custom else None}
    if roofline["traffic"]:
        # counter-based rate: the measured HBM bytes of such a launch over this run's launch time
        roofline["traffic_gbs"] = roofline["traffic"] / (roofline["avg_launch_ms"] * 1e-3) / 1e9
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
                   "layout": "per-tensor" if plan is not None else "flat rows",
                   "launch": "one HIP graph of K steps" if args.graph else "one launch per step"},
        "hbm_gbs_all_steps": sum(bytes_of) / ((grp_ms + glb_ms) * 1e-3) / 1e9,
        "group_step_ms": (grp_ms / len(grp)) if grp else None,
        "group_step_ms_median": float(np.median([ms[t] for t in grp])) if grp else None,
        "group_step_ms_min": min(ms[t] for t in grp) if grp else None,
        "global_step_ms": (glb_ms / len(glb)) if glb else None,
        "global_step_gbs": (sum(bytes_of[t] for t in glb) / (glb_ms * 1e-3) / 1e9) if glb else None,
        "roofline": roofline,
    }
    if plan is not None:
        plan.destroy()
    del w, g, m, pub
    ctx.destroy()
    torch.cuda.empty_cache()
    if args.all_workloads:
        import subprocess
        summary = {wl.index: {"workload": wl.name, "value": out["value"], "ms_per_step": out["ms_per_step"],
                              "group_step_gbs": roofline["achieved"], "frac": roofline["frac"]}}
        for k in range(1, len(wk.WORKLOADS) + 1):
            if k == wl.index:
                continue
            log("workload %d ..." % k)
            child = subprocess.run([sys.executable, os.path.abspath(__file__), "--workload", str(k),
                                    "--no-cpu-baseline", "--warmup", str(W)], capture_output=True, text=True)
            line = [x for x in child.stdout.splitlines() if x.startswith("{")]
            if child.returncode != 0 or not line:
                summary[k] = {"error": child.stderr[-300:]}
                continue
            o = json.loads(line[-1])
            summary[k] = {"workload": o["config"]["workload"], "value": o["value"], "ms_per_step": o["ms_per_step"],
                          "group_step_gbs": o["roofline"]["achieved"], "frac": o["roofline"]["frac"]}
        out["workloads"] = {str(k): summary[k] for k in sorted(summary)}
    if not args.no_cpu_baseline:
        log("timing the CPU oracle on a slice ...")
        out["cpu_baseline"] = cpu_baseline(wl, args.cpu_columns, min(K, wl.iters))
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
