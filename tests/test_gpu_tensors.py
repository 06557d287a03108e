"""GPU parity of the per-tensor entry point (wagma_step_tensors) against the CPU oracle and
against the flat entry point, through the C-ABI."""
import numpy as np
import pytest
import torch

from oracle import wagma_oracle as orc
from paper_2005_00124_amd import wagma as lw
from paper_2005_00124_amd import workloads as wk

pytestmark = pytest.mark.gpu
LR, MU = 0.1, 0.9
GUARD = 8        # floats of sentinel before and after every tensor


def say(*a):
    print(*a, flush=True)


def bits(a):
    return np.ascontiguousarray(a).view(np.uint32)


def make_arrays(P, sizes, gen, scale, layout="separate"):
    """For every process a list of tensors, and the sentinels around them (views that must still
    hold 777 at the end).  layout "separate": every tensor of every process in an allocation of
    its own; "arena": views into one row per process with sentinels between them (rows 64
    KiB-multiples apart: a tensor then crosses the 64 KiB boundaries of the address space at the same
    place in every process); "packed": views into one row per process, back to back (a tensor whose
    size is no multiple of 4 is followed by 1..3 sentinels, the others by the next tensor: the plan
    joins those); "stacked": the P replicas of a tensor side by side in one allocation.  In the last
    three the replicas of a tensor lie equally far apart, in every array alike: the plan then finds
    its tensors without the pointer tables."""
    arrays, sentinels = [], []
    if layout in ("arena", "packed"):
        gap = GUARD if layout == "arena" else 0
        row = (sum(size + (-size) % 4 + gap for size in sizes) + 2 * GUARD + 16383) // 16384 * 16384
        slab = torch.full((P, row), 777.0, device="cuda")
        for p in range(P):
            tensors, at = [], GUARD
            for size in sizes:
                t = slab[p, at:at + size]
                t.normal_(0.0, scale, generator=gen)
                tensors.append(t)
                sentinels.append(slab[p, at - GUARD:at] if at == GUARD or gap else slab[p, at:at])
                at += size
                sentinels.append(slab[p, at:at + (-size) % 4 + gap])
                at += (-size) % 4 + gap
            sentinels.append(slab[p, at:])
            arrays.append(tensors)
        return arrays, sentinels
    stacks = [torch.full((P, size + (-size) % 4 + 2 * GUARD), 777.0, device="cuda") for size in sizes] \
        if layout == "stacked" else None
    for p in range(P):
        tensors = []
        for k, size in enumerate(sizes):
            buf = stacks[k][p] if stacks else torch.full((size + 2 * GUARD,), 777.0, device="cuda")
            t = buf[GUARD:GUARD + size]          # 32-byte offset: still 16-byte aligned
            t.normal_(0.0, scale, generator=gen)
            tensors.append(t)
            sentinels += [buf[:GUARD], buf[GUARD + size:]]
        arrays.append(tensors)
    return arrays, sentinels


def to_rows(arrays):
    """(P, n) numpy matrix: the tensors of every process side by side."""
    return np.stack([torch.cat(t).cpu().numpy() for t in arrays])


def run_tensor_case(P, S, sizes, tau, iters, q, seed, fixed_groups=False, options=(), layout="separate"):
    say("tensor case P=%d S=%d T=%d n=%d tau=%d iters=%d q=%.2f seed=%d %s" % (P, S, len(sizes), sum(sizes), tau, iters, q, seed, layout))
    n = sum(sizes)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    with lw.Wagma(P, S, n, tau) as ctx:
        if fixed_groups:
            ctx.set_grouping(lw.WAGMA_GROUPING_FIXED)
        for option, value in options:
            ctx.debug_set_option(option, value)
        (w, gw), (g, gg), (m, gm), (pub, gp) = (make_arrays(P, sizes, gen, s, layout) for s in (0.05, 0.01, 0.01, 0.05))
        ow, om, opub = to_rows(w), to_rows(m), to_rows(pub)
        thr = min(int(q * 2 ** 32), 2 ** 32 - 1)
        with ctx.tensor_plan(w, g, m, pub) as plan:
            for t in range(iters):
                for tensors in g:
                    for x in tensors:
                        x.normal_(0.0, 1e-2, generator=gen)
                og = to_rows(g)
                mask = ctx.stale_mask(seed, t, thr)
                if t % 4 == 2:
                    mask = orc.mask_words(np.ones(P, dtype=bool))
                plan.step(mask, LR, MU, t)
                orc.step_f32(P, S, tau, t, ow, og, om, opub, mask, LR, MU, fixed_groups=fixed_groups)
                torch.cuda.synchronize()
                for have, want, what in ((w, ow, "w"), (m, om, "m"), (pub, opub, "pub")):
                    h = to_rows(have)
                    assert np.array_equal(bits(h), bits(want)), "%s differs at t=%d" % (what, t)
        assert np.array_equal(bits(to_rows(g)), bits(og)), "g was written"
        for sentinel in gw + gg + gm + gp:
            assert bool((sentinel == 777.0).all()), "an element outside a tensor was written"


RAGGED = [1, 2, 3, 4, 5, 7, 64, 255, 257, 1000, 1023, 1025, 4099, 70001]


@pytest.mark.parametrize("layout", ["separate", "stacked"])
@pytest.mark.parametrize("P,S", [(1, 1), (2, 2), (4, 2), (8, 4), (16, 4), (64, 8), (32, 16), (64, 64), (128, 32)])
def test_tensors_bit_exact(P, S, layout):
    sizes = RAGGED if P <= 16 else RAGGED[:-1]
    run_tensor_case(P, S, sizes, tau=3, iters=8, q=0.3, seed=100 + P + S, layout=layout)


def test_tensors_variants():
    run_tensor_case(16, 4, [33, 1024, 9], tau=0, iters=4, q=1.0, seed=7)            # everybody late
    run_tensor_case(16, 4, [33, 1024, 9], tau=1, iters=3, q=0.5, seed=8)            # always global
    run_tensor_case(32, 8, [4097, 130], tau=0, iters=6, q=0.3, seed=9, fixed_groups=True)
    run_tensor_case(8, 1, [17], tau=2, iters=4, q=0.5, seed=10)                     # one tensor, S = 1


BLOCKS = [65536, 3, 65536 + 4 * 300 + 2, 2 * 65536 + 1, 65535, 5]   # whole 256 KiB blocks, with and without a rest


@pytest.mark.parametrize("layout", ["separate", "stacked"])
@pytest.mark.parametrize("P,S", [(16, 4), (32, 8), (16, 16), (32, 32), (8, 1)])
def test_tensors_with_mapped_blocks(P, S, layout):
    """Every whole 256 KiB of a tensor is dealt out by the launch shape's map, the rest in 4 KiB tiles."""
    run_tensor_case(P, S, BLOCKS, tau=3, iters=4, q=0.3, seed=300 + P + S, layout=layout)


@pytest.mark.parametrize("P,S", [(16, 4), (32, 8), (16, 16), (32, 32)])
def test_tensors_blocks_on_address_boundaries(P, S):
    """Tensors that are views into rows 64 KiB-multiples apart: the mapped blocks begin on a 64 KiB
    boundary of the address space, the slices before it are contiguous tiles."""
    run_tensor_case(P, S, [70001, 65536 + 8, 3, 2 * 65536 + 20000, 1000], tau=3, iters=4, q=0.3, seed=500 + P + S, layout="arena")


@pytest.mark.parametrize("P,S", [(16, 4), (32, 8), (16, 16), (32, 32)])
def test_tensors_back_to_back_are_joined(P, S):
    """Views into one row per process, back to back: the plan treats tensors without a gap between
    them as one (here 4 + 2 + 2 tensors become three), which moves the tiles and the mapped blocks
    but not a single bit of the result."""
    run_tensor_case(P, S, [1000, 64, 70000, 4097, 36864, 5, 65536 + 20, 3], tau=3, iters=4, q=0.3,
                    seed=700 + P + S, layout="packed")


def test_tensors_back_to_back_taken_one_by_one():
    """The same views with the plan told to take the tensor list as it is."""
    run_tensor_case(32, 8, [1000, 64, 70000, 4097, 36864, 5, 65536 + 20, 3], tau=3, iters=3, q=0.3, seed=777,
                    layout="packed", options=((lw.WAGMA_DEBUG_TENSOR_TABLES, 1),))


def test_tensors_spaced_alike_found_by_place():
    """Views into rows again, with the plan told to find its tensors as it does when they are not
    spaced alike: through the pointers laid out by the places of the schedule table's rows."""
    for P, S in ((32, 8), (16, 16), (32, 32), (128, 32)):
        run_tensor_case(P, S, [70001, 65536 + 8, 3, 1000], tau=3, iters=8, q=0.3, seed=600 + P + S, layout="arena",
                        options=((lw.WAGMA_DEBUG_TENSOR_TABLES, 1),))


def test_tensors_spaced_alike_but_not_in_every_array():
    """The replicas of a tensor equally far apart in w, m and pub and not in g: pointers by place."""
    P, S, sizes = 8, 4, [1000, 70001, 3]
    n = sum(sizes)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(77)
    with lw.Wagma(P, S, n, 0) as ctx:
        (w, _), (m, _), (pub, _) = (make_arrays(P, sizes, gen, s, "stacked") for s in (0.05, 0.01, 0.05))
        g, _ = make_arrays(P, sizes, gen, 0.01, "separate")
        ow, og, om, opub = (to_rows(x) for x in (w, g, m, pub))
        with ctx.tensor_plan(w, g, m, pub) as plan:
            for t in range(3):
                mask = ctx.stale_mask(5, t, 1 << 30)
                plan.step(mask, LR, MU, t)
                orc.step_f32(P, S, 0, t, ow, og, om, opub, mask, LR, MU)
                torch.cuda.synchronize()
                for have, want, what in ((w, ow, "w"), (m, om, "m"), (pub, opub, "pub")):
                    assert np.array_equal(bits(to_rows(have)), bits(want)), "%s differs at t=%d" % (what, t)


def test_tensors_block_options():
    run_tensor_case(32, 8, BLOCKS, tau=0, iters=3, q=0.3, seed=41, options=((lw.WAGMA_DEBUG_MAP, 0x5329618470),))
    run_tensor_case(16, 16, BLOCKS, tau=0, iters=3, q=0.3, seed=42, options=((lw.WAGMA_DEBUG_MAP, 0x0123456789),))
    run_tensor_case(32, 8, BLOCKS, tau=2, iters=3, q=0.3, seed=43, options=((lw.WAGMA_DEBUG_XCD_CHUNK_LOG2, 2),))   # no blocks
    run_tensor_case(32, 32, BLOCKS, tau=2, iters=3, q=0.3, seed=44, options=((lw.WAGMA_DEBUG_STRIPE_LOG2, 2),))     # no blocks


def test_plan_validation():
    P, S = 4, 2
    sizes = [10, 6]
    with lw.Wagma(P, S, 16, 0) as ctx:
        def arrs():
            return [[torch.zeros(s, device="cuda") for s in sizes] for _ in range(P)]
        w, g, m, pub = arrs(), arrs(), arrs(), arrs()
        plan = ctx.tensor_plan(w, g, m, pub)
        plan.destroy()
        with pytest.raises(lw.WagmaError):                       # sizes do not add up to n
            lw.wagma_tensors_create(ctx.ctx, [10, 5], *[[t.data_ptr() for ts in a for t in ts] for a in (w, g, m, pub)])
        bad = [t.data_ptr() for ts in w for t in ts]
        bad[3] += 4                                              # misaligned
        with pytest.raises(lw.WagmaError):
            lw.wagma_tensors_create(ctx.ctx, sizes, bad, *[[t.data_ptr() for ts in a for t in ts] for a in (g, m, pub)])
        with pytest.raises(ValueError):
            ctx.tensor_plan(w[:-1], g, m, pub)
        with lw.Wagma(P, S, 16, 0) as other:
            plan = ctx.tensor_plan(w, g, m, pub)
            assert lw.load().wagma_step_tensors(other.ctx, plan.plan, None, LR, MU, 0, None) == lw.WAGMA_EINVAL
            plan.destroy()


@pytest.mark.parametrize("where", ["views", "views, as given", "stacked", "separate"])
def test_tensors_of_workload_2_equal_the_flat_path(where):
    """ResNet-50-shaped tensor list (161 tensors): the per-tensor entry point and the flat entry
    point give the same bits on the whole model, and both match the oracle on a column sample.
    views: the tensors are views into flat rows, back to back (the plan joins them into one);
    views, as given: the same with the plan told to keep the 161 tensors and to find them through
    the pointers by place; stacked: every parameter in a [P, size] allocation of its own (161 tile
    entries name their tensor's place); separate: every tensor of every process in an allocation of
    its own (pointers by place)."""
    wl = wk.workload(2)
    P, S, n = wl.P, wl.S, wl.n
    tensors = wl.tensors()
    sizes = [int(np.prod(t[1])) for t in tensors]
    assert len(sizes) == 161 and sum(sizes) == n
    say("workload 2 per-tensor (%s) vs flat:" % where, wl.name)
    with lw.Wagma(P, S, n, wl.tau) as ctx:
        if where == "views, as given":
            ctx.debug_set_option(lw.WAGMA_DEBUG_TENSOR_TABLES, 1)
        flat = ctx.alloc()
        wk.fill_initial_state(wl, flat[0], flat[2], flat[3])

        def views(buf):
            out = []
            for p in range(P):
                at, row = 0, []
                for s in sizes:
                    row.append(buf[p, at:at + s])
                    at += s
                out.append(row)
            return out

        if where in ("stacked", "separate"):
            if where == "stacked":
                stacks = [[torch.empty((P, s + (-s) % 4), device="cuda") for s in sizes] for _ in range(4)]
            else:   # a list of P one-row tensors behaves like a [P, size] tensor in what follows
                class Rows:
                    def __init__(self, s):
                        self.rows = [torch.empty(s, device="cuda") for _ in range(P)]

                    def __getitem__(self, key):
                        p, cols = key
                        if isinstance(p, slice):
                            return Block(self.rows, cols)
                        return self.rows[p][cols]

                class Block:
                    def __init__(self, rows, cols):
                        self.rows, self.cols = rows, cols

                    def copy_(self, src):
                        for p, row in enumerate(self.rows):
                            row[self.cols].copy_(src[p])

                    def gather(self):
                        return torch.stack([row[self.cols] for row in self.rows])
                stacks = [[Rows(s) for s in sizes] for _ in range(4)]
            lists = [[[st[p, :s] for st, s in zip(per_array, sizes)] for p in range(P)] for per_array in stacks]

            def put(a):          # flat array a -> the tensors of array a
                at = 0
                for st, s in zip(stacks[a], sizes):
                    st[:, :s].copy_(flat[a][:, at:at + s])
                    at += s

            def get(a):          # the tensors of array a as a (P, n) matrix
                parts = [st[:, :s] for st, s in zip(stacks[a], sizes)]
                return torch.cat([x.gather() if where == "separate" else x for x in parts], dim=1)
            for a in (0, 2, 3):
                put(a)
        else:
            twin = [x.clone() for x in flat]
            lists = [views(x) for x in twin]

            def put(a):
                twin[a].copy_(flat[a])

            def get(a):
                return twin[a][:, :n]
        cols = wk.sample_columns(n, 20000, wl.seed).cuda()
        ow, om, opub = (np.ascontiguousarray(x[:, cols].cpu().numpy()) for x in (flat[0], flat[2], flat[3]))
        with ctx.tensor_plan(*lists) as plan:
            for t in range(12):
                wk.fill_gradients(wl, t, flat[1])
                put(1)
                mask = ctx.stale_mask(wl.seed, t, wl.stale_threshold)
                ctx.step(*flat, mask, wl.lr, wl.mu, t)
                plan.step(mask, wl.lr, wl.mu, t)
                orc.step_f32(P, S, wl.tau, t, ow, np.ascontiguousarray(flat[1][:, cols].cpu().numpy()), om, opub,
                             mask, wl.lr, wl.mu)
                torch.cuda.synchronize()
                for a, what in enumerate("wgmp"):
                    assert torch.equal(flat[a][:, :n], get(a)), "%s differs between the layouts at t=%d" % (what, t)
                assert np.array_equal(bits(get(0)[:, cols].cpu().numpy()), bits(ow))
                assert np.array_equal(bits(get(3)[:, cols].cpu().numpy()), bits(opub))
