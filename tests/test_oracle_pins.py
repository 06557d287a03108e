"""Pins of the CPU oracle against the paper and the mathematics (no GPU).

Each test fixes the oracle to something other than itself: values the paper
prints, closed forms, invariants, hand-derived fp32 values and a brute-force
restatement on tiny inputs, chosen so that a plausible slip in the oracle
(a dropped term, a wrong sign, index, order or divisor) fails one of them.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import wagma_oracle as orc

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
POW2 = [1, 2, 4, 8, 16, 32, 64]


def f32(x):
    return np.float32(x)


def rows(*vals, dtype=np.float32):
    """One column, P rows."""
    return np.array(vals, dtype=dtype).reshape(-1, 1).copy()


def read_golden(name):
    out = []
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.strip()
            if line and not line.startswith("#"):
                out.append(line)
    return out


def groups_from_rep(rep):
    g = {}
    for p, r in enumerate(rep):
        g.setdefault(int(r), set()).add(p)
    return sorted(sorted(s) for s in g.values())


# ---------------------------------------------------------------- Algorithm 1

def test_alg1_printed_example_p8_s4():
    """Section 3.3 worked example: both printed groupings and the printed relations."""
    for line in read_golden("alg1_example_p8_s4.txt"):
        head, body = line.split(":")
        kind, P, S, t = head.split()
        P, S, t = int(P), int(S), int(t)
        if kind == "groups":
            want = sorted(sorted(int(x) for x in part.split()) for part in body.split("|"))
            assert groups_from_rep(orc.grouping_unionfind(P, S, t)) == want
            assert sorted(sorted(r) for r in orc.member_table(P, S, t).tolist()) == want
        else:
            # the printed relations, phase by phase: pairs of members e, e^(1<<r)
            table = orc.member_table(P, S, t)
            have = []
            for r in range(int(math.log2(S))):
                pairs = set()
                for grp in table:
                    for e in range(S):
                        a, b = int(grp[e]), int(grp[e ^ (1 << r)])
                        pairs.add((min(a, b), max(a, b)))
                have.extend(sorted(pairs))
            want = [tuple(int(x) for x in rel.split("=")) for rel in body.split()]
            assert have == want


def test_alg1_snapshot_p4_s2():
    """Section 4 snapshot: P0,P1 together in iteration t, P1,P3 together in t+1."""
    for line in read_golden("snapshot_p4_s2.txt"):
        head, body = line.split(":")
        _, P, S, t = head.split()
        p, q = (int(x) for x in body.split())
        rep = orc.grouping_unionfind(int(P), int(S), int(t))
        assert rep[p] == rep[q]
        table = orc.member_table(int(P), int(S), int(t))
        assert any({p, q} <= set(r) for r in table.tolist())


@pytest.mark.parametrize("P", POW2 + [128, 256, 1024])
def test_alg1_partition_and_period(P):
    """P/S groups of exactly S members for every t; the union-find partition equals
    'ranks that differ only in the phase bits'; member table = same partition;
    schedule repeats with period G/gcd(g,G)."""
    G = int(math.log2(P))
    for S in [s for s in POW2 + [128, 256, 1024] if s <= P]:
        g = int(math.log2(S))
        period = 1 if g == 0 or G == 0 else G // math.gcd(g, G)
        for t in range(0, min(4 * period, 12)):
            rep = orc.grouping_unionfind(P, S, t)
            bits = [(t * g + r) % G for r in range(g)] if G else []
            M = sum(1 << b for b in bits)
            assert len(set(bits)) == g
            # closed form: the group's smallest member clears the phase bits
            assert np.array_equal(rep, np.arange(P) & ~M)
            table = orc.member_table(P, S, t)
            assert table.shape == (P // S, S)
            assert sorted(table.ravel().tolist()) == list(range(P))
            for grp in table:
                assert len({int(rep[p]) for p in grp}) == 1
                assert int(grp[0]) == int(rep[grp[0]])     # member 0 is the smallest
            assert np.all(np.diff(table[:, 0]) > 0)         # groups by ascending smallest member
            # butterfly order: members e and e^(1<<r) are the phase-r pair
            for r, b in enumerate(bits):
                for e in range(S):
                    assert np.array_equal(table[:, e ^ (1 << r)], table[:, e] ^ (1 << b))
            assert np.array_equal(orc.member_table(P, S, t + period), table)
            if period > 1 and S < P:
                assert not np.array_equal(orc.member_table(P, S, t + 1), table)


def test_alg1_phase_bits_wrap_order():
    """P=32, S=8, t=1: phases use bits 3, 4, 0 in that order."""
    table = orc.member_table(32, 8, 1)
    assert table[0].tolist() == [0, 8, 16, 24, 1, 9, 17, 25]
    assert table[1].tolist() == [2, 10, 18, 26, 3, 11, 19, 27]


def test_alg1_rejects_bad_arguments():
    for P, S in [(6, 2), (8, 3), (4, 8), (0, 1)]:
        with pytest.raises(ValueError):
            orc.grouping_unionfind(P, S, 0)
        with pytest.raises(ValueError):
            orc.member_table(P, S, 0)


def test_global_iteration_predicate():
    """Algorithm 2 line 8: global average iff (t+1) mod tau == 0; tau = 0 never."""
    assert [t for t in range(12) if orc.is_global_iteration(5, t)] == [4, 9]
    assert [t for t in range(50) if orc.is_global_iteration(16, t)] == [15, 31, 47]
    assert all(orc.is_global_iteration(1, t) for t in range(5))
    assert not any(orc.is_global_iteration(0, t) for t in range(40))


# ------------------------------------------------------- Algorithm 2, fp32 facts

def one_step(P, S, tau, t, w, g, m, pub, stale, lr, mu):
    w, g, m, pub = (np.array(a, dtype=np.float32).reshape(P, -1).copy() for a in (w, g, m, pub))
    orc.step_f32(P, S, tau, t, w, g, m, pub, stale, lr, mu)
    return w, m, pub


def test_local_update_hand_value():
    """w=1, g=.5, m=.2, mu=.9, lr=.1: m' = .68, w' = .932 (S=1 leaves w' alone)."""
    w, m, pub = one_step(1, 1, 0, 0, [1.0], [0.5], [0.2], [7.0], None, 0.1, 0.9)
    exact_m = Fraction(float(f32(0.9))) * Fraction(float(f32(0.2))) + Fraction(float(f32(0.5)))
    m_new = f32(float(exact_m))                      # one rounding: fused
    exact_w = Fraction(1) - Fraction(float(f32(0.1))) * Fraction(float(m_new))
    assert m[0, 0] == m_new and abs(float(m[0, 0]) - 0.68) < 1e-7
    assert w[0, 0] == f32(float(exact_w)) and abs(float(w[0, 0]) - 0.932) < 1e-7
    assert pub[0, 0] == w[0, 0]                      # send buffer <- W'


def test_update_lines_are_fused():
    """mu*m is not rounded before g is added: (1+2^-12)^2 - 1 keeps its 2^-24 term."""
    a = 1.0 + 2.0 ** -12
    w, m, _ = one_step(1, 1, 0, 0, [0.0], [-1.0], [a], [0.0], None, 0.0, a)
    assert float(m[0, 0]) == 2.0 ** -11 + 2.0 ** -24
    # second line: w - lr*m' with lr = a, m' = a (mu = 0, g = a), w = 1
    w, m, _ = one_step(1, 1, 0, 0, [1.0], [a], [0.0], [0.0], None, a, 0.0)
    assert float(w[0, 0]) == -(2.0 ** -11 + 2.0 ** -24)


def test_momentum_closed_form():
    """Constant gradient, m0 = 0, S = 1: w_T = w_0 - lr*g*sum_{k=1..T}(1-mu^k)/(1-mu)."""
    P, T, lr, mu, g0, w0 = 2, 25, 0.05, 0.9, 0.3, 1.5
    w = np.full((P, 3), w0, dtype=np.float64)
    g = np.full((P, 3), g0, dtype=np.float64)
    m = np.zeros((P, 3))
    pub = w.copy()
    w32, g32, m32, pub32 = (a.astype(np.float32) for a in (w, g, m, pub))
    for t in range(T):
        orc.step_f64(P, 1, 0, t, w, g, m, pub, None, lr, mu)
        orc.step_f32(P, 1, 0, t, w32, g32, m32, pub32, None, lr, mu)
    want = w0 - lr * g0 * sum((1 - mu ** k) / (1 - mu) for k in range(1, T + 1))
    assert np.allclose(w, want, rtol=0, atol=1e-12)
    assert np.allclose(w32, want, rtol=0, atol=2e-6)
    assert np.allclose(m, g0 * (1 - mu ** T) / (1 - mu), rtol=0, atol=1e-12)


def test_mixing_example_p4_s2():
    """lr = 0: (1,2,3,4) -> t=0 (1.5,1.5,3.5,3.5) -> t=1 all 2.5: updates reach
    everybody within log_S P iterations (Section 3.3)."""
    w, g, m, pub = rows(1, 2, 3, 4), rows(0, 0, 0, 0), rows(0, 0, 0, 0), rows(1, 2, 3, 4)
    orc.step_f32(4, 2, 0, 0, w, g, m, pub, None, 0.0, 0.9)
    assert w.ravel().tolist() == [1.5, 1.5, 3.5, 3.5]
    orc.step_f32(4, 2, 0, 1, w, g, m, pub, None, 0.0, 0.9)
    assert w.ravel().tolist() == [2.5, 2.5, 2.5, 2.5]


@pytest.mark.parametrize("P,S", [(8, 2), (16, 4), (64, 8), (32, 8), (64, 4)])
def test_mixing_reaches_global_mean(P, S):
    """lr = 0, nobody late: after ceil(G/g) group iterations every replica holds the mean."""
    rng = np.random.default_rng(P * 100 + S)
    w0 = rng.integers(-64, 64, size=(P, 5)).astype(np.float64)   # exact in fp32 too
    w = w0.copy()
    g, m, pub = np.zeros_like(w), np.zeros_like(w), w.copy()
    G, gg = int(math.log2(P)), int(math.log2(S))
    for t in range(-(-G // gg)):
        orc.step_f64(P, S, 0, t, w, g, m, pub, None, 0.0, 0.9)
    assert np.allclose(w, w0.mean(axis=0, keepdims=True), rtol=0, atol=1e-12)
    w32 = w0.astype(np.float32)
    g32, m32, pub32 = np.zeros_like(w32), np.zeros_like(w32), w32.copy()
    for t in range(-(-G // gg)):
        orc.step_f32(P, S, 0, t, w32, g32, m32, pub32, None, 0.0, 0.9)
    assert np.array_equal(w32, np.broadcast_to(w0.mean(axis=0).astype(np.float32), w32.shape))


def test_stale_rule_hand_value():
    """S=2, W'=(1,2), P1 late with send buffer 10: W_sum = 11; P0 -> 11/2; P1 -> (11+2)/3;
    P1's send buffer becomes 2 (Algorithm 2 lines 11 and 13; Section 4 snapshot)."""
    stale = np.array([False, True])
    w, m, pub = one_step(2, 2, 0, 0, [1, 2], [0, 0], [0, 0], [99, 10], stale, 0.0, 0.9)
    assert w[0, 0] == f32(5.5)
    assert w[1, 0] == f32(13.0) / f32(3.0)
    assert pub.ravel().tolist() == [1.0, 2.0]


def test_stale_divisor_is_a_true_division():
    """(W_sum + W')/(S+1) is an IEEE division, not a multiply by a rounded 1/(S+1)."""
    found = 0
    for k in range(1, 400):
        x = f32(k)
        if x / f32(3.0) != x * (f32(1.0) / f32(3.0)):
            # S=2; P1 late: W_sum = pub_1 + w'_0 = 0 + 0, own w' = k => (0 + k)/3
            stale = np.array([False, True])
            w, _, _ = one_step(2, 2, 0, 0, [0, k], [0, 0], [0, 0], [0, 0], stale, 0.0, 0.0)
            assert w[1, 0] == x / f32(3.0)
            found += 1
    assert found > 10


def test_snapshot_script_p4_s2():
    """Section 4 snapshot: P1 late in iterations t and t+1 contributes W'_{t-1}, then W'_t."""
    P, S, lr, mu = 4, 2, 0.5, 0.0
    w = rows(1, 2, 3, 4, dtype=np.float64)
    pub = rows(1, 20, 3, 4, dtype=np.float64)          # P1's send buffer: W'_{t-1} = 20
    m = np.zeros_like(w)
    g = rows(2, 2, 2, 2, dtype=np.float64)             # W' = W - 1
    late = np.array([False, True, False, False])
    orc.step_f64(P, S, 0, 0, w, g, m, pub, late, lr, mu)
    # W'_0 = (0,1,2,3); groups {0,1},{2,3}; W_sum{0,1} = 0 + 20
    assert np.allclose(w.ravel(), [10.0, (20.0 + 1.0) / 3, 2.5, 2.5])
    assert np.allclose(pub.ravel(), [0, 1, 2, 3])      # send buffer of P1 <- W'_0
    w_before = w.copy()
    orc.step_f64(P, S, 0, 1, w, g, m, pub, late, lr, mu)
    wp = w_before.ravel() - 1.0                        # W'_1
    # groups {0,2},{1,3}; P1 contributes W'_0[1] = 1 again
    s13 = 1.0 + wp[3]
    assert np.allclose(w.ravel(), [(wp[0] + wp[2]) / 2, (s13 + wp[1]) / 3,
                                   (wp[0] + wp[2]) / 2, s13 / 2])
    assert np.allclose(pub.ravel(), wp)
    # a global iteration ignores lateness and the send buffers
    orc.step_f64(P, S, 3, 2, w, g, m, pub, late, lr, mu)
    assert np.allclose(w, w[0, 0]) and np.ptp(w) == 0.0


def test_snapshot_script_p4_s2_f32():
    """The same script in fp32, ending in a global iteration: all replicas get the mean of W'."""
    P, S = 4, 2
    w, pub = rows(1, 2, 3, 4), rows(1, 20, 3, 4)
    m, g = rows(0, 0, 0, 0), rows(2, 2, 2, 2)
    late = np.array([False, True, False, False])
    orc.step_f32(P, S, 0, 0, w, g, m, pub, late, 0.5, 0.0)
    assert w.ravel().tolist() == [10.0, float(f32(21.0) / f32(3.0)), 2.5, 2.5]
    before = w.astype(np.float64).ravel() - 1.0
    orc.step_f32(P, S, 2, 1, w, g, m, pub, late, 0.5, 0.0)         # (1+1) mod 2 == 0: global
    assert np.all(w == f32(before.sum() / 4)) and abs(float(w[0, 0]) - before.mean()) < 1e-6


def test_sum_is_a_pairwise_tree_in_member_order():
    """(1 + e) + (e + e) = 1 + 2e in fp32 with e = 2^-24, while a left-to-right sum gives 1."""
    e = 2.0 ** -24
    w, _, _ = one_step(4, 4, 0, 0, [1, e, e, e], [0] * 4, [0] * 4, [0] * 4, None, 0.0, 0.0)
    assert np.all(w == f32((1.0 + 2.0 ** -23) / 4))
    # global path: same tree over ranks 0..P-1
    w, _, _ = one_step(4, 2, 1, 0, [1, e, e, e], [0] * 4, [0] * 4, [0] * 4, None, 0.0, 0.0)
    assert np.all(w == f32((1.0 + 2.0 ** -23) / 4))
    # member order, not rank order, when the phase bits wrap: P=8, S=4, t=1 runs bits
    # 2 then 0, so the members are (0,4,1,5) and the sum is (c0 + c4) + (c1 + c5).
    assert orc.member_table(8, 4, 1)[0].tolist() == [0, 4, 1, 5]
    vals = [0.0] * 8
    vals[0], vals[4], vals[1], vals[5] = 1.0, -1.0, e, e
    w, _, _ = one_step(8, 4, 0, 1, vals, [0] * 8, [0] * 8, [0] * 8, None, 0.0, 0.0)
    # (1 - 1) + (e + e) = 2e; the rank-order tree (1 + e) + (-1 + e) would give e
    assert np.all(w[[0, 4, 1, 5], 0] == f32(2 * e / 4))


def test_subnormals_are_kept():
    tiny = 2.0 ** -149
    w, _, pub = one_step(2, 2, 0, 0, [3 * tiny, 5 * tiny], [0, 0], [0, 0], [0, 0], None, 0.0, 0.0)
    assert w.ravel().tolist() == [4 * tiny, 4 * tiny]
    assert pub.ravel().tolist() == [3 * tiny, 5 * tiny]


# ------------------------------------------- brute force and invariants, random data

def brute_force_step(P, S, tau, t, w, g, m, pub, stale, lr, mu):
    """fp64 restatement that never builds a member list: for every process i, add the
    contribution of every process j that differs from i only in the iteration's phase bits."""
    G, gg = int(math.log2(P)), int(math.log2(S))
    M = sum(1 << ((t * gg + r) % G) for r in range(gg)) if G else 0
    glob = tau > 0 and (t + 1) % tau == 0
    m_new = mu * m + g
    wp = w - lr * m_new
    out = np.empty_like(w)
    for i in range(P):
        if glob:
            out[i] = sum(wp[j] for j in range(P)) / P
            continue
        total = np.zeros(w.shape[1])
        for j in range(P):
            if ((i ^ j) & ~M) == 0:
                total = total + (pub[j] if stale[j] else wp[j])
        out[i] = (total + wp[i]) / (S + 1) if stale[i] else total / S
    return out, m_new, wp.copy()


@pytest.mark.parametrize("P", [4, 8])
def test_brute_force_small(P):
    """P = 4 and P = 8, every S, every schedule residue, random lateness, all-late and
    none-late included; fp64 oracle to 1e-12, fp32 oracle to 1e-6 * max|w|."""
    rng = np.random.default_rng(2005 + P)
    n = 37
    for S in [s for s in (1, 2, 4, 8) if s <= P]:
        for tau in (0, 3):
            w = rng.normal(0, 1, (P, n))
            m = rng.normal(0, 0.1, (P, n))
            pub = rng.normal(0, 1, (P, n))
            w32, m32, pub32 = (a.astype(np.float32) for a in (w, m, pub))
            w, m, pub = (a.astype(np.float64) for a in (w32, m32, pub32))
            for t in range(9):
                g32 = rng.normal(0, 0.5, (P, n)).astype(np.float32)
                g = g32.astype(np.float64)
                stale = rng.random(P) < (0.0, 0.3, 1.0)[t % 3]
                lr, mu = float(f32(0.1)), float(f32(0.9))
                want_w, want_m, want_pub = brute_force_step(P, S, tau, t, w, g, m, pub, stale, lr, mu)
                orc.step_f64(P, S, tau, t, w, g, m, pub, stale, lr, mu)
                orc.step_f32(P, S, tau, t, w32, g32, m32, pub32, stale, lr, mu)
                for have, want in ((w, want_w), (m, want_m), (pub, want_pub)):
                    assert np.allclose(have, want, rtol=0, atol=1e-12)
                scale = np.abs(want_w).max()
                assert np.abs(w32 - want_w).max() <= 1e-6 * scale
                assert np.abs(m32 - want_m).max() <= 1e-6 * max(1.0, np.abs(want_m).max())
                assert np.abs(pub32 - want_pub).max() <= 1e-6 * scale
                # carry the fp64 state forward from the fp32 one so rounding does not pile up
                w, m, pub = (a.astype(np.float64) for a in (w32, m32, pub32))


@pytest.mark.parametrize("P,S", [(4, 2), (8, 4), (16, 4), (64, 8), (32, 8), (16, 16), (8, 1)])
def test_invariants_without_lateness(P, S):
    """Nobody late: group members end bit-identical; the mean over all P replicas is
    preserved by the averaging; a global iteration makes all replicas bit-identical."""
    rng = np.random.default_rng(P * 1000 + S)
    n = 23
    w = rng.normal(0, 0.02, (P, n)).astype(np.float32)
    m = np.zeros_like(w)
    pub = w.copy()
    tau = 4
    for t in range(8):
        g = rng.normal(0, 1e-3, (P, n)).astype(np.float32)
        w_before, m_before = w.astype(np.float64), m.astype(np.float64)
        orc.step_f32(P, S, tau, t, w, g, m, pub, None, 0.1, 0.9)
        wp = w_before - float(f32(0.1)) * (float(f32(0.9)) * m_before + g.astype(np.float64))
        assert np.abs(w.astype(np.float64).mean(axis=0) - wp.mean(axis=0)).max() < 1e-8
        assert np.abs(pub - wp).max() < 1e-8
        if orc.is_global_iteration(tau, t):
            assert np.all(w == w[0:1])
        else:
            for grp in orc.member_table(P, S, t):
                assert np.all(w[grp] == w[grp[0]:grp[0] + 1])
            if S == 1:
                assert np.array_equal(w, pub)


@pytest.mark.parametrize("P", [2, 8, 64])
def test_group_of_all_equals_global(P):
    """S = P: the group path and the global path give the same bits (same tree)."""
    rng = np.random.default_rng(P)
    w0 = rng.normal(0, 1, (P, 19)).astype(np.float32)
    g = rng.normal(0, 1, (P, 19)).astype(np.float32)
    a = [w0.copy(), g, np.zeros_like(w0), w0.copy()]
    b = [w0.copy(), g, np.zeros_like(w0), w0.copy()]
    for t in range(3):
        orc.step_f32(P, P, 0, t, *a, None, 0.1, 0.9)       # always the group path
        orc.step_f32(P, 2 if P > 2 else 1, 1, t, *b, None, 0.1, 0.9)  # always the global path
        for x, y in zip(a, b):
            assert np.array_equal(x, y)


def test_padding_columns_untouched_and_columns_independent():
    """Only columns [0, n) are used; a column's result does not depend on the others."""
    rng = np.random.default_rng(5)
    P, S, ld, n = 8, 4, 11, 7
    w, g, m, pub = (rng.normal(0, 1, (P, ld)).astype(np.float32) for _ in range(4))
    stale = rng.random(P) < 0.4
    keep = [a.copy() for a in (w, m, pub)]
    sub = [np.ascontiguousarray(a[:, 2:5]) for a in (w, g, m, pub)]
    orc.step_f32(P, S, 0, 1, w, g, m, pub, stale, 0.1, 0.9, n=n)
    orc.step_f32(P, S, 0, 1, *sub, stale, 0.1, 0.9)
    for a, k in zip((w, m, pub), keep):
        assert np.array_equal(a[:, n:], k[:, n:])
    for a, s in zip((w, m, pub), (sub[0], sub[2], sub[3])):
        assert np.array_equal(a[:, 2:5], s)


def test_fp32_tracks_fp64_shadow_over_a_run():
    """Workload-1-like run (P=4, S=2, tau=5, 10 iterations): |w32 - w64| <= 1e-6 * max|w|."""
    rng = np.random.default_rng(1)
    P, S, tau, n = 4, 2, 5, 4096
    row = rng.normal(0, 0.02, (1, n)).astype(np.float32)
    w = np.repeat(row, P, axis=0)
    m, pub = np.zeros_like(w), w.copy()
    w64, m64, pub64 = (a.astype(np.float64) for a in (w, m, pub))
    for t in range(10):
        g = rng.normal(0, 1e-3, (P, n)).astype(np.float32)
        stale = rng.random(P) < 0.25
        orc.step_f32(P, S, tau, t, w, g, m, pub, stale, 0.1, 0.9)
        orc.step_f64(P, S, tau, t, w64, g.astype(np.float64), m64, pub64, stale,
                     float(f32(0.1)), float(f32(0.9)))
        assert np.abs(w - w64).max() <= 1e-6 * np.abs(w64).max()
    assert np.all(w == w[0:1])          # t = 9 is a global iteration


# ------------------------------------------------------------- seeded lateness

MASK64 = (1 << 64) - 1


def splitmix_finish(z):
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK64
    return z ^ (z >> 31)


def test_lateness_hash_against_published_splitmix64():
    """The Python restatement reproduces the published splitmix64 outputs for state 0,
    and the C oracle agrees with the restatement bit for bit."""
    want = [int(x, 16) for x in read_golden("splitmix64_seed0.txt")]
    state, have = 0, []
    for _ in want:
        state = (state + 0x9E3779B97F4A7C15) & MASK64
        have.append(splitmix_finish(state))
    assert have == want
    for seed, t, P, thr in [(0, 0, 64, 1 << 31), (200500128, 17, 64, 1073741824),
                            (2 ** 64 - 1, 123456789, 1024, 858993459), (7, 3, 5, 4294967295)]:
        per_iter = splitmix_finish((seed + 0x9E3779B97F4A7C15 * (t + 1)) & MASK64)
        bits = 0
        for p in range(P):
            h = splitmix_finish((per_iter + 0xD1B54A32D192ED03 * (p + 1)) & MASK64)
            if (h >> 32) < thr:
                bits |= 1 << p
        words = orc.stale_mask(seed, t, P, thr)
        assert [int(x) for x in words] == [(bits >> (64 * k)) & MASK64 for k in range(len(words))]


def test_lateness_rate_and_extremes():
    P = 64
    assert not orc.stale_mask(1, 0, P, 0).any()
    for q in (0.1, 0.2, 0.25):
        thr = int(q * 2 ** 32)
        late = sum(bin(int(orc.stale_mask(200500128, t, P, thr)[0])).count("1") for t in range(400))
        total = 400 * P
        assert abs(late - q * total) < 5 * math.sqrt(total * q * (1 - q))
    a = orc.stale_mask(3, 5, P, 1 << 31)
    assert not np.array_equal(a, orc.stale_mask(3, 6, P, 1 << 31))
    assert not np.array_equal(a, orc.stale_mask(4, 5, P, 1 << 31))
    assert np.array_equal(a, orc.stale_mask(3, 5, P, 1 << 31))


# ------------------------------------------------- the family of variants (Sections 4 and 6.2)

def test_fixed_groups_ablation():
    """Second ablation of Section 6.2: without the rotation the groups of iteration 0 are used
    every time, so with lr = 0 a second averaging changes nothing and the replicas never mix
    beyond their fixed group (only the global average mixes them)."""
    P, S = 16, 4
    rng = np.random.default_rng(11)
    w0 = rng.integers(-32, 32, size=(P, 7)).astype(np.float32)
    w = w0.copy()
    g, m, pub = np.zeros_like(w), np.zeros_like(w), w.copy()
    orc.step_f32(P, S, 0, 0, w, g, m, pub, None, 0.0, 0.9, fixed_groups=True)
    first = w.copy()
    groups = orc.member_table(P, S, 0)
    for grp in groups:
        assert np.array_equal(first[grp], np.broadcast_to(w0[grp].mean(axis=0), (S, 7)))
    for t in range(1, 6):
        orc.step_f32(P, S, 0, t, w, g, m, pub, None, 0.0, 0.9, fixed_groups=True)
        assert np.array_equal(w, first)
    assert len({tuple(r) for r in w.tolist()}) == P // S           # still P/S distinct models
    orc.step_f32(P, S, 3, 8, w, g, m, pub, None, 0.0, 0.9, fixed_groups=True)   # (8+1) mod 3 == 0
    assert np.all(w == w[0:1])
    # with the rotation the same start mixes completely in two group iterations
    w = w0.copy()
    pub = w.copy()
    for t in range(2):
        orc.step_f32(P, S, 0, t, w, g, m, pub, None, 0.0, 0.9)
    assert np.all(w == w[0:1])


def test_fixed_groups_brute_force():
    P, S, n = 8, 2, 9
    rng = np.random.default_rng(12)
    w = rng.normal(0, 1, (P, n)).astype(np.float32).astype(np.float64)
    m = rng.normal(0, 0.1, (P, n)).astype(np.float32).astype(np.float64)
    pub = rng.normal(0, 1, (P, n)).astype(np.float32).astype(np.float64)
    lr, mu = float(f32(0.1)), float(f32(0.9))
    for t in range(5):
        g = rng.normal(0, 0.5, (P, n)).astype(np.float32).astype(np.float64)
        stale = rng.random(P) < 0.3
        # the brute force of iteration 0's phase bits, whatever t is
        want_w, want_m, want_pub = brute_force_step(P, S, 0, 0, w, g, m, pub, stale, lr, mu)
        orc.step_f64(P, S, 0, t, w, g, m, pub, stale, lr, mu, fixed_groups=True)
        for have, want in ((w, want_w), (m, want_m), (pub, want_pub)):
            assert np.allclose(have, want, rtol=0, atol=1e-12)


def test_local_sgd_is_group_size_one():
    """First ablation of Section 6.2: no group collectives = local SGD with period tau."""
    P, n, tau = 4, 5, 3
    rng = np.random.default_rng(13)
    w = rng.normal(0, 1, (P, n))
    m = np.zeros_like(w)
    pub = w.copy()
    ref_w, ref_m = w.copy(), m.copy()
    for t in range(6):
        g = rng.normal(0, 1, (P, n))
        orc.step_f64(P, 1, tau, t, w, g, m, pub, None, 0.1, 0.9)
        ref_m = 0.9 * ref_m + g
        ref_w = ref_w - 0.1 * ref_m
        if (t + 1) % tau == 0:
            ref_w = np.broadcast_to(ref_w.mean(axis=0), ref_w.shape).copy()
        assert np.allclose(w, ref_w, rtol=0, atol=1e-12) and np.allclose(m, ref_m, rtol=0, atol=1e-12)


# ------------------------------------------------- lateness models of the experiments

def test_straggler_mask_selects_exactly_k():
    """Section 6.2 delays two randomly selected processes per step."""
    P = 64
    counts = np.zeros(P)
    for t in range(2000):
        words = orc.straggler_mask(200500128, t, P, 2)
        late = [p for p in range(P) if (int(words[p >> 6]) >> (p & 63)) & 1]
        assert len(late) == 2
        counts[late] += 1
    # every process is selected about 2/64 of the time (binomial bounds, 5 sigma)
    expect = 2000 * 2 / P
    assert np.all(np.abs(counts - expect) < 5 * math.sqrt(expect))
    assert not orc.straggler_mask(1, 0, 8, 0).any()
    assert int(orc.straggler_mask(1, 0, 8, 8)[0]) == 0xFF
    assert int(orc.straggler_mask(1, 5, 1, 1)[0]) == 1
    assert int(orc.straggler_mask(9, 3, 1024, 1024).view(np.uint8).astype(np.int64).sum()) == 128 * 255
    assert np.array_equal(orc.straggler_mask(5, 7, 64, 2), orc.straggler_mask(5, 7, 64, 2))
    assert not np.array_equal(orc.straggler_mask(5, 7, 64, 2), orc.straggler_mask(5, 8, 64, 2))
    with pytest.raises(ValueError):
        orc.straggler_mask(1, 0, 8, 9)
    # Python restatement, bit for bit
    for seed, t, P, k in [(0, 0, 16, 3), (2 ** 64 - 1, 99, 64, 2), (77, 5, 1024, 17)]:
        bits_per_rank = int(math.log2(P))
        per_iter = splitmix_finish(((seed ^ 0x5354524147474C52) + 0x9E3779B97F4A7C15 * (t + 1)) & MASK64)
        chosen, j = set(), 0
        while len(chosen) < k:
            h = splitmix_finish((per_iter + 0xD1B54A32D192ED03 * (j + 1)) & MASK64)
            chosen.add(h >> (64 - bits_per_rank))
            j += 1
        words = orc.straggler_mask(seed, t, P, k)
        have = {p for p in range(P) if (int(words[p >> 6]) >> (p & 63)) & 1}
        assert have == chosen


def test_clock_mask_distribution_and_activator():
    """Section 6.4: step times from 1.7 s to 43.5 s with a median below 2 s; Section 3.2: the
    process that arrives first (the activator) is never late."""
    P = 64
    all_ms = []
    for t in range(300):
        words, ms = orc.clock_mask(200500128, t, P, 500)
        all_ms.append(ms)
        late = np.array([(int(words[p >> 6]) >> (p & 63)) & 1 for p in range(P)], dtype=bool)
        assert not late[np.argmin(ms)]
        assert np.array_equal(late, ms.astype(np.int64) > int(ms.min()) + 500)
    all_ms = np.concatenate(all_ms)
    assert all_ms.min() >= 1700 and all_ms.max() == 43500
    assert np.median(all_ms) < 2000
    assert 0.40 < np.mean(all_ms >= 2000) < 0.475          # seven steps in sixteen are in the tail
    # an infinite tolerance makes nobody late; zero tolerance leaves only the ties with the fastest
    assert not orc.clock_mask(3, 0, P, 2 ** 32 - 1)[0].any()
    words, ms = orc.clock_mask(3, 0, P, 0)
    assert bin(int(words[0])).count("1") == int(np.sum(ms > ms.min()))
