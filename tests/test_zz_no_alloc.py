"""wagma_step_static (the entry point that allocates nothing: its schedule table is a static
device array) against wagma_step, through the C-ABI, bit for bit, on two calls in a row, the
second with a smaller input.  Collected last on purpose: a failure here must not hide the
other GPU tests.
"""
import ctypes

import numpy as np
import pytest
import torch

from paper_2005_00124_amd import wagma as lw

pytestmark = pytest.mark.gpu

LR, MU = 0.1, 0.9


def say(*a):
    print(*a, flush=True)


def state(P, ld, seed):
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    w = torch.randn((P, ld), generator=gen, device="cuda") * 0.05
    m = torch.randn((P, ld), generator=gen, device="cuda") * 0.01
    pub = torch.randn((P, ld), generator=gen, device="cuda") * 0.05
    g = torch.randn((P, ld), generator=gen, device="cuda") * 0.01
    return w, g, m, pub


def same_bits(a, b):
    return torch.equal(a.view(torch.int32), b.view(torch.int32))


def both_ways(P, S, n, tau, iters, seed):
    """Runs `iters` iterations with wagma_step on one copy of the state and with raw calls of
    wagma_step_static on another; compares w, m and pub after every iteration."""
    lib = lw.load()
    stream = torch.cuda.current_stream().cuda_stream
    with lw.Wagma(P, S, n, tau) as ctx:
        ld = ctx.ld
        w, g, m, pub = state(P, ld, seed)
        w2, m2, pub2 = w.clone(), m.clone(), pub.clone()
        g_before = g.clone()
        for t in range(iters):
            say("  wagma_step_static P=%d S=%d n=%d tau=%d ld=%d t=%d" % (P, S, n, tau, ld, t))
            mask = ctx.stale_mask(seed, t, 1 << 30)           # a quarter of the processes late
            ctx.step(w, g, m, pub, mask, LR, MU, t)
            words = np.ascontiguousarray(mask, dtype=np.uint64)
            rc = lib.wagma_step_static(P, S, n, tau, ld, w2.data_ptr(), g.data_ptr(), m2.data_ptr(),
                                       pub2.data_ptr(), words.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64)),
                                       LR, MU, t, stream)
            assert rc == lw.WAGMA_OK, rc
            torch.cuda.synchronize()
            for have, want, what in ((w2, w, "w"), (m2, m, "m"), (pub2, pub, "pub")):
                assert same_bits(have[:, :n], want[:, :n]), "%s differs at t=%d (P=%d S=%d n=%d)" % (what, t, P, S, n)
        assert torch.equal(g, g_before), "g was written"
        # ld = 0 stands for the stride wagma_create chooses
        w3, m3, pub3 = w.clone(), m.clone(), pub.clone()
        ctx.step(w, g, m, pub, None, LR, MU, iters)
        lw.wagma_step_static(P, S, n, tau, 0, w3, g, m3, pub3, None, LR, MU, iters)
        torch.cuda.synchronize()
        assert same_bits(w3[:, :n], w[:, :n]) and same_bits(m3[:, :n], m[:, :n]) and same_bits(pub3[:, :n], pub[:, :n])


def test_static_step_matches_wagma_step_twice_second_smaller():
    # first a large case (period 5, wrapped phase bits, the streamed kernel in the global iterations),
    # then smaller ones, which find the larger case's table still in the array
    both_ways(32, 8, 70001, 4, 6, seed=11)
    both_ways(8, 2, 1001, 3, 4, seed=12)
    both_ways(64, 16, 4099, 0, 3, seed=13)      # streamed kernel in group iterations
    both_ways(4, 4, 5, 2, 2, seed=14)


def test_static_step_rejects_bad_sizes():
    lib = lw.load()
    w, g, m, pub = state(4, 64, 1)
    args = (w.data_ptr(), g.data_ptr(), m.data_ptr(), pub.data_ptr(), None, LR, MU, 0, None)
    before = w.clone()
    assert lib.wagma_step_static(2 * lw.WAGMA_MAX_P, 2, 64, 0, 64, *args) == lw.WAGMA_EINVAL   # beyond the array
    assert lib.wagma_step_static(6, 2, 64, 0, 64, *args) == lw.WAGMA_EINVAL
    assert lib.wagma_step_static(4, 8, 64, 0, 64, *args) == lw.WAGMA_EINVAL
    assert lib.wagma_step_static(4, 2, 0, 0, 64, *args) == lw.WAGMA_EINVAL
    assert lib.wagma_step_static(4, 2, 64, -1, 64, *args) == lw.WAGMA_EINVAL
    assert lib.wagma_step_static(4, 2, 64, 0, 62, *args) == lw.WAGMA_EINVAL                    # stride
    assert lib.wagma_step_static(4, 2, 64, 0, 64, None, *args[1:]) == lw.WAGMA_EINVAL
    assert lib.wagma_step_static(4, 2, 64, 0, 64, *args[:7], -1, None) == lw.WAGMA_EINVAL       # iter
    torch.cuda.synchronize()
    assert torch.equal(w, before)
