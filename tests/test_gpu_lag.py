"""GPU parity of the path for lateness deeper than one iteration (wagma_step_lag,
wagma_step_tensors_lag, wagma_lag_masks) against the CPU oracle, through the C-ABI.

Bar: masks bit-exact; w, m and pub bit-exact (same order of operations), rows of processes
that are still computing untouched bit for bit, the gradient never written.
"""
import numpy as np
import pytest
import torch

from oracle import wagma_oracle as orc
from paper_2005_00124_amd import wagma as lw

from test_gpu_parity import LR, MU, assert_same_bits, random_state, say

pytestmark = pytest.mark.gpu


def words(flags):
    return orc.mask_words(np.asarray(flags, dtype=bool))


def random_masks(rng, P, t):
    """Late and busy sets of one iteration; every fourth iteration an extreme."""
    late = rng.random(P) < 0.25
    busy = rng.random(P) < 0.3
    if t % 8 == 3:
        busy[:] = True                 # nobody finishes anything
    if t % 8 == 7:
        busy[:] = False
        late[:] = True
    return late, busy


@pytest.mark.parametrize("P,S,n,tau", [
    (1, 1, 300, 0), (4, 2, 1000, 5), (8, 1, 515, 0), (16, 4, 70001, 10), (64, 8, 40000, 16),
    (32, 8, 9999, 8), (64, 16, 5000, 0), (64, 64, 3001, 7), (256, 32, 2049, 6), (1024, 128, 1100, 0),
])
def test_step_lag_random_masks(P, S, n, tau):
    say("lag case P=%d S=%d n=%d tau=%d" % (P, S, n, tau))
    rng = np.random.default_rng(P * 131 + S)
    with lw.Wagma(P, S, n, tau) as ctx:
        ld = ctx.ld
        w, g, m, pub, gen = random_state(P, ld, n, 99 + P + S)
        ow, om, opub = (x.cpu().numpy().copy() for x in (w, m, pub))
        for t in range(10):
            g.normal_(0.0, 1e-2, generator=gen)
            og = g.cpu().numpy()
            late, busy = random_masks(rng, P, t)
            before = [x.clone() for x in (w, m, pub)]
            ctx.step(w, g, m, pub, words(late), LR, MU, t, busy_mask=words(busy))
            orc.step_lag_f32(P, S, tau, t, ow, og, om, opub, late, busy, LR, MU, n=n)
            torch.cuda.synchronize()
            for have, want, what in ((w, ow, "w"), (m, om, "m"), (pub, opub, "pub")):
                assert_same_bits(have.cpu().numpy()[:, :n], want[:, :n], "%s at t=%d" % (what, t))
            if not ctx.is_global(t):
                rows = torch.from_numpy(np.nonzero(busy)[0]).cuda()
                for x, b in zip((w, m, pub), before):
                    assert torch.equal(x[rows], b[rows]), "a busy process was written at t=%d" % t
        assert torch.equal(g.cpu(), torch.from_numpy(og)), "g was written"


@pytest.mark.parametrize("options", [
    ((lw.WAGMA_OPT_NONTEMPORAL, 1),),
    ((lw.WAGMA_OPT_NONTEMPORAL, 0), (lw.WAGMA_DEBUG_STRIPE_LOG2, 0), (lw.WAGMA_DEBUG_XCD_CHUNK_LOG2, 0)),
    ((lw.WAGMA_DEBUG_FORCE_STREAM, 1), (lw.WAGMA_DEBUG_STRIPE_LOG2, 3)),
])
def test_step_lag_launch_options(options):
    """The other launch shapes of the same kernels, S = 8 (in registers and streamed)."""
    P, S, n, tau = 32, 8, 33333, 6
    say("lag options", options)
    rng = np.random.default_rng(17)
    with lw.Wagma(P, S, n, tau) as ctx:
        for opt, val in options:
            ctx.debug_set_option(opt, val)
        w, g, m, pub, gen = random_state(P, ctx.ld, n, 5)
        ow, om, opub = (x.cpu().numpy().copy() for x in (w, m, pub))
        for t in range(7):
            g.normal_(0.0, 1e-2, generator=gen)
            og = g.cpu().numpy()
            late, busy = random_masks(rng, P, t)
            ctx.step(w, g, m, pub, words(late), LR, MU, t, busy_mask=words(busy))
            orc.step_lag_f32(P, S, tau, t, ow, og, om, opub, late, busy, LR, MU, n=n)
            torch.cuda.synchronize()
            for have, want, what in ((w, ow, "w"), (m, om, "m"), (pub, opub, "pub")):
                assert_same_bits(have.cpu().numpy()[:, :n], want[:, :n], "%s at t=%d" % (what, t))


def test_lag_masks_bit_exact():
    for P, tau in [(1, 0), (4, 5), (16, 10), (64, 16), (32, 8), (1024, 12), (128, 0)]:
        with lw.Wagma(P, 1, 16, tau) as ctx:
            for seed in (0, 200500128, 2 ** 64 - 1):
                for tol in (0, 300, 1699):
                    for window in (1, 7, 64):
                        for t in list(range(0, 3 * max(tau, 8))) + [10 ** 6 + 3]:
                            late, busy = ctx.lag_masks(seed, t, tol, window)
                            olate, obusy = orc.lag_masks(seed, t, P, tau, window, tol)
                            assert np.array_equal(late, olate), (P, tau, seed, tol, window, t)
                            assert np.array_equal(busy, obusy), (P, tau, seed, tol, window, t)
                        if tau:
                            break          # the window only matters without a global period
            with pytest.raises(lw.WagmaError):
                ctx.lag_masks(1, 0, 1700, 8)
            if tau == 0:
                with pytest.raises(lw.WagmaError):
                    ctx.lag_masks(1, 0, 10, 0)
    say("lag masks: bit-exact")


@pytest.mark.parametrize("P,S,n,tau,iters", [(16, 4, 50000, 10, 30), (64, 8, 20000, 16, 34), (32, 8, 4097, 0, 20)])
def test_training_run_with_back_to_back_steps(P, S, n, tau, iters):
    """A run in which the library's own lag masks drive the library and the oracle's own masks
    drive the oracle; the states must stay equal bit for bit, the fp32 state within
    1e-6 * max|w| of the fp64 shadow."""
    say("lag run P=%d S=%d n=%d tau=%d" % (P, S, n, tau))
    seed, tol, window = 200500124 + P, 250, 9
    with lw.Wagma(P, S, n, tau) as ctx:
        w, g, m, pub, gen = random_state(P, ctx.ld, n, seed % 1000)
        pub.copy_(w)
        ow, om, opub = (x.cpu().numpy().copy() for x in (w, m, pub))
        dw, dm, dpub = (x.astype(np.float64) for x in (ow, om, opub))
        seen_busy = seen_late = 0
        for t in range(iters):
            g.normal_(0.0, 1e-2, generator=gen)
            og = g.cpu().numpy()
            late, busy = ctx.lag_masks(seed, t, tol, window)
            olate, obusy = orc.lag_masks(seed, t, P, tau, window, tol)
            seen_busy += int(sum(bin(int(x)).count("1") for x in busy))
            seen_late += int(sum(bin(int(x)).count("1") for x in late))
            ctx.step(w, g, m, pub, late, LR, MU, t, busy_mask=busy)
            orc.step_lag_f32(P, S, tau, t, ow, og, om, opub, olate, obusy, LR, MU, n=n)
            orc.step_lag_f64(P, S, tau, t, dw, og.astype(np.float64), dm, dpub, olate, obusy,
                             float(np.float32(LR)), float(np.float32(MU)), n=n)
            torch.cuda.synchronize()
            for have, want, what in ((w, ow, "w"), (m, om, "m"), (pub, opub, "pub")):
                assert_same_bits(have.cpu().numpy()[:, :n], want[:, :n], "%s at t=%d" % (what, t))
            assert np.abs(ow[:, :n] - dw[:, :n]).max() <= 1e-6 * np.abs(dw[:, :n]).max()
        assert seen_busy > 0 and seen_late > 0
        say("  busy process-iterations %d, late %d of %d" % (seen_busy, seen_late, P * iters))


@pytest.mark.parametrize("where", ["separate", "stacked", "stacked, by place"])
@pytest.mark.parametrize("P,S", [(4, 2), (16, 8), (32, 16), (32, 32)])
def test_step_tensors_lag(P, S, where):
    """Per-tensor layout: ragged tensors between sentinels (one with a whole 256 KiB block, which the
    plan deals out by the launch shape's map), late and busy processes.  stacked: the P replicas of
    a tensor lie equally far apart in one allocation (the tile's entry names the tensor's place);
    separate: every tensor of every process is an allocation of its own (pointers laid out by
    place); stacked, by place: the first layout with the plan told to treat it like the second."""
    stacked = where.startswith("stacked")
    sizes = [1, 7, 64, 1030, 5, 4096, 333, 65536 + 4 * 70 + 3]
    n = sum(sizes)
    tau = 4
    say("lag tensors P=%d S=%d %s" % (P, S, where))
    rng = np.random.default_rng(P + S)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(3 + P)
    guard = 8
    SENTINEL = 12345.0

    def make(scale):
        stacks = [torch.full((P, guard + (size + 3) // 4 * 4 + guard), SENTINEL, device="cuda") for size in sizes]
        out = []
        for p in range(P):
            per = []
            for k, size in enumerate(sizes):
                buf = stacks[k][p] if stacked else torch.full((stacks[k].shape[1],), SENTINEL, device="cuda")
                buf[guard:guard + size] = torch.randn(size, generator=gen, device="cuda") * scale
                per.append(buf)
            out.append(per)
        return out

    bufs = {name: make(scale) for name, scale in (("w", 0.05), ("g", 0.01), ("m", 0.01), ("pub", 0.05))}
    views = {name: [[b[guard:guard + size] for b, size in zip(per, sizes)] for per in arr]
             for name, arr in bufs.items()}

    def flat(name):
        return np.stack([np.concatenate([v.cpu().numpy() for v in per]) for per in views[name]])

    ow, og, om, opub = (flat(k).copy() for k in ("w", "g", "m", "pub"))
    with lw.Wagma(P, S, n, tau) as ctx:
        if where == "stacked, by place":
            ctx.debug_set_option(lw.WAGMA_DEBUG_TENSOR_TABLES, 1)
        plan = ctx.tensor_plan(views["w"], views["g"], views["m"], views["pub"])
        try:
            for t in range(6):
                late, busy = random_masks(rng, P, t + 1)
                plan.step(words(late), LR, MU, t, busy_mask=words(busy))
                orc.step_lag_f32(P, S, tau, t, ow, og, om, opub, late, busy, LR, MU)
                torch.cuda.synchronize()
                for name, want in (("w", ow), ("m", om), ("pub", opub), ("g", og)):
                    assert_same_bits(flat(name), want, "%s at t=%d" % (name, t))
        finally:
            plan.destroy()
    for name, arr in bufs.items():
        for per in arr:
            for b, size in zip(per, sizes):
                assert bool((b[:guard] == SENTINEL).all()) and bool((b[guard + size:] == SENTINEL).all()), \
                    "wrote outside a tensor of %s" % name


def test_seeded_random_configurations():
    """Forty seeded draws of everything at once: sizes, period, row stride, grouping mode,
    launch options, late and busy sets; flat layout, bit for bit against the oracle."""
    rng = np.random.default_rng(20050012)
    sizes = [1, 2, 4, 8, 16, 32, 64, 128, 256]
    for case in range(40):
        P = int(rng.choice(sizes))
        S = int(rng.choice([s for s in sizes if s <= P]))
        n = int(rng.integers(1, 30000))
        tau = int(rng.integers(0, 6))
        fixed = bool(rng.integers(0, 2))
        options = []
        if rng.integers(0, 2):
            options.append((lw.WAGMA_OPT_NONTEMPORAL, int(rng.integers(0, 2))))
        if rng.integers(0, 2):
            options.append((lw.WAGMA_DEBUG_STRIPE_LOG2, int(rng.integers(0, 5))))
        if rng.integers(0, 2):
            options.append((lw.WAGMA_DEBUG_XCD_CHUNK_LOG2, int(rng.integers(0, 5))))
        if rng.integers(0, 3) == 0:
            options.append((lw.WAGMA_DEBUG_FORCE_STREAM, 1))
        pad = int(rng.integers(0, 3)) * 4
        say("random case %d: P=%d S=%d n=%d tau=%d fixed=%s pad=%d options=%s"
            % (case, P, S, n, tau, fixed, pad, options))
        with lw.Wagma(P, S, n, tau) as ctx:
            if pad:
                ctx.set_row_stride((n + 3) // 4 * 4 + pad)
            for opt, val in options:
                ctx.debug_set_option(opt, val)
            if fixed:
                ctx.set_grouping(lw.WAGMA_GROUPING_FIXED)
            w, g, m, pub, gen = random_state(P, ctx.ld, n, 1000 + case)
            ow, om, opub = (x.cpu().numpy().copy() for x in (w, m, pub))
            t0 = int(rng.integers(0, 1000))
            for t in range(t0, t0 + 5):
                g.normal_(0.0, 1e-2, generator=gen)
                og = g.cpu().numpy()
                late = rng.random(P) < 0.3
                busy = rng.random(P) < 0.3 if rng.integers(0, 3) else None
                ctx.step(w, g, m, pub, words(late), LR, MU, t,
                         busy_mask=None if busy is None else words(busy))
                orc.step_lag_f32(P, S, tau, t, ow, og, om, opub, late, busy, LR, MU, n=n, fixed_groups=fixed)
                torch.cuda.synchronize()
                for have, want, what in ((w, ow, "w"), (m, om, "m"), (pub, opub, "pub")):
                    assert_same_bits(have.cpu().numpy()[:, :n], want[:, :n],
                                     "%s at t=%d of case %d" % (what, t, case))


def test_lag_steps_captured_in_a_hip_graph():
    """The lag entry points launch only, like wagma_step: a run of flat and per-tensor steps with
    busy processes, captured once in a HIP graph, must reproduce the eager result on every
    replay (eager work and synchronisations in between), and the oracle's."""
    P, S, tau, iters = 16, 4, 5, 9
    sizes = [5000, 36, 1024, 2051]          # every tensor begins 16-byte aligned, the last one is ragged
    n = sum(sizes)
    seed, tol = 7, 300
    with lw.Wagma(P, S, n, tau) as ctx:
        w, g, m, pub, gen = random_state(P, ctx.ld, n, 11)
        g.normal_(0.0, 1e-2, generator=gen)
        start = [x.clone() for x in (w, m, pub)]

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
        masks = [ctx.lag_masks(seed, t, tol) for t in range(iters)]

        def run():
            for t in range(iters):
                late, busy = masks[t]
                if t % 2:
                    plan.step(late, LR, MU, t, busy_mask=busy)
                else:
                    ctx.step(w, g, m, pub, late, LR, MU, t, busy_mask=busy)
        run()
        torch.cuda.synchronize()
        want = [x.clone() for x in (w, m, pub)]
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for x, s in zip((w, m, pub), start):
                x.copy_(s)
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                run()
        torch.cuda.current_stream().wait_stream(side)
        for replay in range(4):
            for x, s in zip((w, m, pub), start):
                x.copy_(s)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            for have, ref, what in zip((w, m, pub), want, "wmp"):
                assert torch.equal(have, ref), "%s differs on replay %d" % (what, replay)
            g.add_(0.0)
            torch.cuda.synchronize()
        ow, om, opub = (s.cpu().numpy().copy() for s in start)
        og = g.cpu().numpy()
        for t in range(iters):
            late, busy = masks[t]
            orc.step_lag_f32(P, S, tau, t, ow, og, om, opub, late, busy, LR, MU, n=n)
        assert_same_bits(w.cpu().numpy()[:, :n], ow[:, :n], "w after the graph")
        plan.destroy()


def test_library_masks_equal_the_stored_ones():
    """The stored lateness masks of the five workloads (tests/golden/lateness_masks.txt, written
    from the oracle) against what the library draws."""
    import os
    from paper_2005_00124_amd import workloads as wk
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "lateness_masks.txt")
    ctxs = {wl.index: lw.Wagma(wl.P, wl.S, 16, wl.tau) for wl in wk.WORKLOADS}
    try:
        checked = 0
        for line in open(path):
            if line.startswith("#") or not line.strip():
                continue
            head, values = line.split(":")
            kind, index, t = head.split()
            wl, t = wk.workload(int(index)), int(t)
            ctx = ctxs[wl.index]
            parts = [np.array([int(x, 16) for x in part.split()], dtype=np.uint64) for part in values.split("|")]
            if kind == "bernoulli":
                have = [ctx.stale_mask(wl.seed, t, wl.stale_threshold)]
            elif kind == "stragglers2":
                have = [ctx.straggler_mask(wl.seed, t, min(2, wl.P))]
            else:
                have = list(ctx.lag_masks(wl.seed, t, 300))
            for h, want in zip(have, parts):
                assert np.array_equal(h, want), line
            checked += 1
        assert checked == 60
    finally:
        for ctx in ctxs.values():
            ctx.destroy()
