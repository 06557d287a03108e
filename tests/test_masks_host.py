"""The library's host-side lateness generators (csrc/wagma_masks.h) against the oracle's, on the
CPU: the header has no HIP in it, so a small driver (tests/masks_host.cpp, built with the address
and undefined-behaviour sanitizers) runs it here.  Bit-exact, as the parity bar demands."""
import os
import subprocess

import numpy as np
import pytest

from oracle import wagma_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    exe = tmp_path_factory.mktemp("masks") / "masks_host"
    subprocess.run(["g++", "-std=c++17", "-O1", "-Wall", "-Wextra", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=all", "-I", os.path.join(ROOT, "paper_2005_00124_amd", "csrc"),
                    "-o", str(exe), os.path.join(ROOT, "tests", "masks_host.cpp")], check=True)

    def ask(requests):
        out = subprocess.run([str(exe)], input="\n".join(requests) + "\n", capture_output=True, text=True,
                             timeout=120)
        assert out.returncode == 0, out.stderr
        lines = out.stdout.strip().split("\n")
        assert len(lines) == len(requests)
        return [np.array(line.split(), dtype=np.uint64) for line in lines]
    return ask


SEEDS = (0, 200500128, 2 ** 64 - 1)


def test_global_iteration_predicate(driver):
    cases = [(tau, t) for tau in (0, 1, 2, 5, 16) for t in list(range(40)) + [10 ** 12, 2 ** 62]]
    have = driver(["global %d %d" % c for c in cases])
    for (tau, t), h in zip(cases, have):
        assert int(h[0]) == int(orc.is_global_iteration(tau, t)), (tau, t)


def test_bernoulli_masks(driver):
    cases = [(P, seed, t, thr) for P in (1, 4, 16, 64, 128, 1024) for seed in SEEDS
             for t in (0, 1, 49, 10 ** 9) for thr in (0, 1 << 30, 858993459, 2 ** 32 - 1)]
    have = driver(["bernoulli %d %d %d %d" % c for c in cases])
    for (P, seed, t, thr), h in zip(cases, have):
        assert np.array_equal(h, orc.stale_mask(seed, t, P, thr)), (P, seed, t, thr)


def test_straggler_masks(driver):
    cases = [(P, seed, t, k) for P in (1, 8, 64, 1024) for seed in SEEDS for t in (0, 7, 10 ** 9)
             for k in sorted({k for k in (0, 1, 2, P // 2, P) if k <= P})]
    have = driver(["stragglers %d %d %d %d" % c for c in cases])
    for (P, seed, t, k), h in zip(cases, have):
        assert np.array_equal(h, orc.straggler_mask(seed, t, P, k)), (P, seed, t, k)


def test_clock_masks(driver):
    cases = [(P, seed, t, tol) for P in (1, 8, 64, 1024) for seed in SEEDS for t in (0, 7, 10 ** 9)
             for tol in (0, 300, 5000, 2 ** 32 - 1)]
    have = driver(["clock %d %d %d %d" % c for c in cases])
    for (P, seed, t, tol), h in zip(cases, have):
        words, ms = orc.clock_mask(seed, t, P, tol)
        k = (P + 63) // 64
        assert np.array_equal(h[:k], words), (P, seed, t, tol)
        assert np.array_equal(h[k:], ms.astype(np.uint64)), (P, seed, t, tol)


def test_lag_masks(driver):
    cases = []
    for P, tau in [(1, 0), (4, 5), (16, 10), (64, 16), (32, 8), (1024, 12), (128, 0)]:
        for seed in SEEDS:
            for tol in (0, 300, 1699):
                for window in ((1, 7, 64) if tau == 0 else (1,)):
                    for t in list(range(0, 3 * max(tau, 8))) + [10 ** 6 + 3]:
                        cases.append((P, tau, window, seed, t, tol))
    have = driver(["lag %d %d %d %d %d %d" % c for c in cases])
    for (P, tau, window, seed, t, tol), h in zip(cases, have):
        late, busy = orc.lag_masks(seed, t, P, tau, window, tol)
        k = (P + 63) // 64
        assert np.array_equal(h[:k], late) and np.array_equal(h[k:], busy), (P, tau, window, seed, t, tol)
