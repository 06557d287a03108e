"""Pins of the oracle's model of lateness deeper than one iteration (no GPU).

Two things are pinned to something other than the oracle: what one iteration does when some
processes are still computing an earlier step (they take part through their send buffer only:
Section 4, the execution snapshot, carried on for more than one iteration), and who is on
time, late or still computing when every process runs its steps back to back and the first
arrival activates the group allreduce (Section 3.2).
"""
import heapq
import math

import numpy as np
import pytest

from oracle import wagma_oracle as orc

FRESH, LATE, BUSY = orc.FRESH, orc.LATE, orc.BUSY


def f32(x):
    return np.float32(x)


def lag_step(P, S, tau, t, w, g, m, pub, late, busy, lr, mu, dtype=np.float32):
    w, g, m, pub = (np.array(a, dtype=dtype).reshape(P, -1).copy() for a in (w, g, m, pub))
    fn = orc.step_lag_f32 if dtype == np.float32 else orc.step_lag_f64
    fn(P, S, tau, t, w, g, m, pub, None if late is None else np.array(late, dtype=bool),
       None if busy is None else np.array(busy, dtype=bool), lr, mu)
    return w, m, pub


# ------------------------------------------------------------ one iteration

def test_busy_member_hand_value():
    """S=2: P0 has W'=1; P1 is still computing, its send buffer holds 10.  W_sum = 11,
    P0 gets 11/2; nothing of P1 changes (model 77, momentum 5, send buffer 10)."""
    w, m, pub = lag_step(2, 2, 0, 0, [1, 77], [0, 3], [0, 5], [99, 10], None, [False, True], 0.0, 0.9)
    assert w.ravel().tolist() == [5.5, 77.0]
    assert m.ravel().tolist() == [0.0, 5.0]
    assert pub.ravel().tolist() == [1.0, 10.0]


def test_busy_and_late_in_one_group_hand_value():
    """S=4, W'=(1,2,-,4); P1 late with send buffer 10, P2 still computing with send buffer 20.
    W_sum = (1+10)+(20+4) = 35: P0 and P3 get 35/4, P1 gets (35+2)/5, P2 keeps 50;
    send buffers afterwards: 1, 2, 20, 4."""
    w, m, pub = lag_step(4, 4, 0, 0, [1, 2, 50, 4], [0] * 4, [0] * 4, [9, 10, 20, 9],
                         [False, True, False, False], [False, False, True, False], 0.0, 0.0)
    assert w.ravel().tolist() == [8.75, float(f32(37.0) / f32(5.0)), 50.0, 8.75]
    assert pub.ravel().tolist() == [1.0, 2.0, 20.0, 4.0]


def test_snapshot_with_a_step_spanning_two_iterations():
    """The snapshot of Section 4 (P=4, S=2) with P1's step spanning iterations 0 and 1:
    lr=1, mu=0, every gradient 1, models (0,10,20,30), send buffers equal to the models.
    t=0, groups {0,1},{2,3}: W'=(-1,-,19,29); P1 contributes its send buffer 10 -> P0 = 4.5;
         P2 = P3 = 24; P1 untouched.
    t=1, groups {0,2},{1,3}: P1 finishes (W'=9) after the allreduce took its send buffer,
         still 10: W'=(3.5,9,23,23); P0 = P2 = 13.25; W_sum{1,3} = 10+23 = 33 -> P3 = 16.5,
         P1 = (33+9)/3 = 14; send buffers (3.5, 9, 23, 23)."""
    for dtype in (np.float32, np.float64):
        w = np.array([[0.0], [10.0], [20.0], [30.0]], dtype=dtype)
        m = np.zeros_like(w)
        pub = w.copy()
        g = np.ones_like(w)
        fn = orc.step_lag_f32 if dtype == np.float32 else orc.step_lag_f64
        fn(4, 2, 0, 0, w, g, m, pub, None, np.array([False, True, False, False]), 1.0, 0.0)
        assert w.ravel().tolist() == [4.5, 10.0, 24.0, 24.0]
        assert pub.ravel().tolist() == [-1.0, 10.0, 19.0, 29.0]
        assert m.ravel().tolist() == [1.0, 0.0, 1.0, 1.0]
        fn(4, 2, 0, 1, w, g, m, pub, np.array([False, True, False, False]), None, 1.0, 0.0)
        assert w.ravel().tolist() == [13.25, 14.0, 13.25, 16.5]
        assert pub.ravel().tolist() == [3.5, 9.0, 23.0, 23.0]


def brute_force_lag_step(P, S, tau, t, w, g, m, pub, late, busy, lr, mu):
    """fp64 restatement without member lists: process i sums over every j that differs from
    it only in the iteration's phase bits."""
    G, gg = int(math.log2(P)), int(math.log2(S))
    M = sum(1 << ((t * gg + r) % G) for r in range(gg)) if G else 0
    glob = tau > 0 and (t + 1) % tau == 0
    if glob:
        late = busy = np.zeros(P, dtype=bool)
    steps = ~busy
    m_out = np.where(steps[:, None], mu * m + g, m)
    wp = w - lr * m_out                       # only meaningful where steps
    sent = np.where((late | busy)[:, None], pub, wp)
    w_out = w.copy()
    for i in range(P):
        if busy[i]:
            continue
        if glob:
            w_out[i] = sum(wp[j] for j in range(P)) / P
            continue
        total = np.zeros(w.shape[1])
        for j in range(P):
            if ((i ^ j) & ~M) == 0:
                total = total + sent[j]
        w_out[i] = (total + wp[i]) / (S + 1) if late[i] else total / S
    pub_out = np.where(steps[:, None], wp, pub)
    return w_out, m_out, pub_out


@pytest.mark.parametrize("P", [4, 8, 16])
def test_lag_step_brute_force(P):
    rng = np.random.default_rng(77 + P)
    n = 29
    for S in [s for s in (1, 2, 4, 8, 16) if s <= P]:
        for tau in (0, 4):
            w32, m32, pub32 = (rng.normal(0, s, (P, n)).astype(np.float32) for s in (1, 0.1, 1))
            for t in range(9):
                g32 = rng.normal(0, 0.5, (P, n)).astype(np.float32)
                late = rng.random(P) < 0.3
                busy = rng.random(P) < (0.0, 0.35, 1.0, 0.35)[t % 4]
                lr, mu = float(f32(0.1)), float(f32(0.9))
                w, g, m, pub = (a.astype(np.float64) for a in (w32, g32, m32, pub32))
                want_w, want_m, want_pub = brute_force_lag_step(P, S, tau, t, w, g, m, pub, late, busy, lr, mu)
                orc.step_lag_f64(P, S, tau, t, w, g, m, pub, late, busy, lr, mu)
                before = [a.copy() for a in (w32, m32, pub32)]
                orc.step_lag_f32(P, S, tau, t, w32, g32, m32, pub32, late, busy, lr, mu)
                for have, want in ((w, want_w), (m, want_m), (pub, want_pub)):
                    assert np.allclose(have, want, rtol=0, atol=1e-12)
                scale = np.abs(want_w).max()
                assert np.abs(w32 - want_w).max() <= 1e-6 * scale
                assert np.abs(m32 - want_m).max() <= 1e-6 * max(1.0, np.abs(want_m).max())
                assert np.abs(pub32 - want_pub).max() <= 1e-6 * scale
                if not (tau > 0 and (t + 1) % tau == 0):
                    for a, b in zip(before, (w32, m32, pub32)):   # bit for bit untouched
                        assert np.array_equal(a[busy].view(np.uint32), b[busy].view(np.uint32))


def test_no_busy_process_is_algorithm_2_as_printed():
    """oracle_step_lag_* with nobody busy against oracle_step_*, Algorithm 2 written out on its
    own: bit for bit on random inputs, over group and global iterations, both precisions,
    dynamic and fixed groups, with and without late processes."""
    rng = np.random.default_rng(5)
    for P, S, tau in ((16, 4, 3), (8, 8, 0), (32, 2, 2), (4, 1, 5), (64, 8, 4)):
        n = 33
        state = [rng.normal(0, 1, (P, n)).astype(np.float32) for _ in range(4)]
        for fixed in (False, True):
            for busy in (None, np.zeros(P, dtype=bool)):
                a = [x.copy() for x in state]
                b = [x.copy() for x in state]
                a64 = [x.astype(np.float64) for x in state]
                b64 = [x.astype(np.float64) for x in state]
                for t in range(7):
                    late = (rng.random(P) < 0.3) if t % 3 else None
                    g = rng.normal(0, 1e-2, (P, n)).astype(np.float32)
                    a[1], b[1] = g, g.copy()
                    a64[1], b64[1] = g.astype(np.float64), g.astype(np.float64)
                    orc.step_f32(P, S, tau, t, *a, late, 0.1, 0.9, fixed_groups=fixed)
                    orc.step_lag_f32(P, S, tau, t, *b, late, busy, 0.1, 0.9, fixed_groups=fixed)
                    orc.step_f64(P, S, tau, t, *a64, late, 0.1, 0.9, fixed_groups=fixed)
                    orc.step_lag_f64(P, S, tau, t, *b64, late, busy, 0.1, 0.9, fixed_groups=fixed)
                    for x, y in zip(a, b):
                        assert np.array_equal(x.view(np.uint32), y.view(np.uint32)), (P, S, tau, t)
                    for x, y in zip(a64, b64):
                        assert np.array_equal(x.view(np.uint64), y.view(np.uint64)), (P, S, tau, t)


def test_busy_wins_over_late_and_a_global_iteration_waits_for_everybody():
    rng = np.random.default_rng(6)
    P, S, n = 8, 4, 17
    state = [rng.normal(0, 1, (P, n)).astype(np.float32) for _ in range(4)]
    busy = np.array([0, 1, 0, 0, 1, 0, 0, 1], dtype=bool)
    late = np.array([0, 0, 1, 0, 0, 0, 1, 0], dtype=bool)
    a = [x.copy() for x in state]
    b = [x.copy() for x in state]
    orc.step_lag_f32(P, S, 0, 1, *a, late, busy, 0.1, 0.9)
    orc.step_lag_f32(P, S, 0, 1, *b, late | busy, busy, 0.1, 0.9)
    for x, y in zip(a, b):
        assert np.array_equal(x.view(np.uint32), y.view(np.uint32))
    # iteration 4 with tau = 5 is a global one: both masks are ignored
    a = [x.copy() for x in state]
    b = [x.copy() for x in state]
    orc.step_lag_f32(P, S, 5, 4, *a, late, busy, 0.1, 0.9)
    orc.step_f32(P, S, 5, 4, *b, None, 0.1, 0.9)
    for x, y in zip(a, b):
        assert np.array_equal(x.view(np.uint32), y.view(np.uint32))
    assert np.all(a[0] == a[0][0])


def test_a_group_of_busy_processes_stands_still():
    rng = np.random.default_rng(8)
    P, S, n = 4, 2, 9
    state = [rng.normal(0, 1, (P, n)).astype(np.float32) for _ in range(4)]
    a = [x.copy() for x in state]
    orc.step_lag_f32(P, S, 0, 0, *a, None, np.array([True, True, False, False]), 0.1, 0.9)
    for x, y in zip(a, state):
        assert np.array_equal(x[:2], y[:2])
    assert not np.array_equal(a[0][2:], state[0][2:])


# ------------------------------------------------- who is fresh, late, busy

def test_lag_states_hand_timeline():
    """Two processes, no tolerance: P0's steps take 2, P1's take 7.  P0 activates allreduce k
    at time 2(k+1).  P1 finishes at 7 (between allreduce 2 at 6 and allreduce 3 at 8: late in
    2), at 14 (allreduce 6 runs at 14, but P1's step was begun for allreduce 3, so it is late
    in 5 and in time for nothing), at 21 (late in 9), at 28 (late in 12)."""
    K = 14
    ms = np.tile(np.array([[2, 7]], dtype=np.uint32), (K + 1, 1))
    states = orc.lag_states(ms, 0)
    assert states[:, 0].tolist() == [FRESH] * K
    want = [BUSY] * K
    for k in (2, 5, 9, 12):
        want[k] = LATE
    assert states[:, 1].tolist() == want


def test_lag_states_hand_timeline_with_tolerance():
    """Three processes, tolerance 3, step times P0: 10, P1: 12, P2: 38.  P0 activates every
    allreduce and P1 is always within the tolerance: allreduce k is activated at 13k + 10 and
    reads at 13(k+1) (P0 and P1 go on from there and finish 10 and 12 later).
    P2 ends its first step at 38: after allreduce 2 was activated (36) but before it reads
    (39), so its send buffer is refreshed in time: busy in 0, late in 1.  Its next step ends at
    76, between the reads of allreduce 4 (65) and 5 (78, activated 75): busy in 2 and 3, late
    in 4."""
    ms = np.tile(np.array([[10, 12, 38]], dtype=np.uint32), (6, 1))
    states = orc.lag_states(ms, 3)
    assert states[:, 0].tolist() == [FRESH] * 5
    assert states[:, 1].tolist() == [FRESH] * 5
    assert states[:, 2].tolist() == [BUSY, LATE, BUSY, BUSY, LATE]


def event_queue_states(step_ms, tol):
    """The same model told as a queue of events in time: a process that ends a step begun for
    the allreduce that comes next arrives at it (the first arrival sets its read time); one
    that ends a step begun for an allreduce that has run already is late for the last one that
    ran and goes on at once; when an allreduce reads, the arrived go on together."""
    K, P = step_ms.shape[0] - 1, step_ms.shape[1]
    states = np.full((K, P), BUSY, dtype=np.uint8)
    FINISH, READ = 0, 1        # at equal times a finished step is seen by the read
    heap = [(int(step_ms[0, p]), FINISH, p, 0) for p in range(P)]
    heapq.heapify(heap)
    v = 0                      # the next allreduce to run
    arrived = []
    while True:
        time, kind, p, begun = heapq.heappop(heap)
        if kind == READ and v == K:
            break              # allreduce K reads: whoever was late for K-1 is known by now
        if kind == READ:
            for q in arrived:
                states[v, q] = FRESH
                heapq.heappush(heap, (time + int(step_ms[v + 1, q]), FINISH, q, v + 1))
            arrived = []
            v += 1
        elif begun == v:
            if not arrived:
                heapq.heappush(heap, (time + tol, READ, -1, v))
            arrived.append(p)
        else:
            assert begun < v
            states[v - 1, p] = LATE
            heapq.heappush(heap, (time + int(step_ms[v, p]), FINISH, p, v))
    return states


@pytest.mark.parametrize("P,tol,lo,hi", [(2, 0, 1, 9), (3, 2, 3, 40), (8, 5, 6, 30), (8, 0, 10, 14),
                                         (16, 100, 1700, 43500), (5, 1, 2, 200)])
def test_lag_states_against_an_event_queue(P, tol, lo, hi):
    rng = np.random.default_rng(P * 1000 + tol)
    for trial in range(40):
        K = int(rng.integers(1, 40))
        if trial % 3 == 0:     # heavy tail: a few very long steps
            ms = np.where(rng.random((K + 1, P)) < 0.15, hi, rng.integers(lo, lo + max(1, (hi - lo) // 8), (K + 1, P)))
        else:
            ms = rng.integers(lo, hi + 1, (K + 1, P))
        ms = ms.astype(np.uint32)
        have = orc.lag_states(ms, tol)
        want = event_queue_states(ms, tol)
        assert np.array_equal(have, want), (trial, ms.tolist())
        assert (have == FRESH).any(axis=1).all()          # the activator is always in time


def test_lag_states_special_cases():
    rng = np.random.default_rng(9)
    # equal step times: everybody always in time
    ms = np.full((11, 8), 2000, dtype=np.uint32)
    assert not orc.lag_states(ms, 0).any()
    # in the first iteration after a global one all start together: in time iff within the
    # tolerance of the fastest (the rule of the one-iteration clock mask)
    ms = rng.integers(1700, 43500, (2, 32)).astype(np.uint32)
    first = orc.lag_states(ms, 250)[0]
    assert np.array_equal(first == FRESH, ms[0].astype(np.int64) <= int(ms[0].min()) + 250)
    # a step 5.3 times as long as everybody else's ends at 5300, 10600, 15900, between the
    # allreduces 4 and 5, 9 and 10, 14 and 15 (allreduce k runs at 1000 (k+1))
    ms = np.full((16, 4), 1000, dtype=np.uint32)
    ms[:, 3] = 5300
    col = orc.lag_states(ms, 0)[:, 3].tolist()
    assert col == ([BUSY] * 4 + [LATE]) * 3
    # step times at or below the tolerance are refused
    with pytest.raises(ValueError):
        orc.lag_states(np.full((3, 2), 5, dtype=np.uint32), 5)


def bits(words, P):
    return np.array([(int(words[p >> 6]) >> (p & 63)) & 1 for p in range(P)], dtype=bool)


@pytest.mark.parametrize("P,tau", [(16, 10), (64, 16), (128, 0)])
def test_lag_masks_follow_the_clock_step_times(P, tau):
    seed, tol, window = 200500129, 300, 12
    length = tau if tau else window
    longest = 0
    run = np.zeros(P, dtype=int)
    for t in range(3 * length + 2):
        late, busy = (bits(x, P) for x in orc.lag_masks(seed, t, P, tau, window, tol))
        assert not (late & busy).any()
        first = t // length * length
        if tau and (t + 1) % tau == 0:
            assert not late.any() and not busy.any()       # everybody waits at the global average
            run[:] = 0
            continue
        ms = np.stack([orc.clock_mask(seed, k, P, 0)[1] for k in range(first, t + 2)])
        states = event_queue_states(ms, tol)[-1]
        assert np.array_equal(late, states == LATE) and np.array_equal(busy, states == BUSY)
        if t == first:
            assert np.array_equal(late | busy, bits(orc.clock_mask(seed, t, P, tol)[0], P))
            run[:] = 0
        run = np.where(late | busy, run + 1, 0)
        longest = max(longest, int(run.max()))
    # some steps span iterations; a send buffer is refreshed at the latest when the clocks restart
    assert 2 <= longest <= (tau - 1 if tau else window)
    with pytest.raises(ValueError):
        orc.lag_masks(seed, 0, P, tau, window, 1700)
