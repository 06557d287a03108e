"""Writes tests/golden/lateness_masks.txt: the lateness masks of the five seeded workloads for
their first iterations, as the CPU oracle computes them (this script calls nothing but the oracle
and the workload constants).  A regression pin: the file must change only when the generators'
definition changes.  Run from the repository root: python tests/golden/make_lateness_masks.py"""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import wagma_oracle as orc                      # noqa: E402
from paper_2005_00124_amd import workloads as wk            # noqa: E402  (constants only)


def lines():
    yield "# kind workload iteration : mask words (hex, word 0 first)"
    for wl in wk.WORKLOADS:
        for t in range(4):
            words = orc.stale_mask(wl.seed, t, wl.P, wl.stale_threshold)
            yield "bernoulli %d %d : %s" % (wl.index, t, " ".join("%016x" % int(x) for x in words))
        for t in range(4):
            words = orc.straggler_mask(wl.seed, t, wl.P, min(2, wl.P))
            yield "stragglers2 %d %d : %s" % (wl.index, t, " ".join("%016x" % int(x) for x in words))
        for t in range(4):
            late, busy = orc.lag_masks(wl.seed, t, wl.P, wl.tau, 64, 300)
            yield "lag300 %d %d : %s | %s" % (wl.index, t, " ".join("%016x" % int(x) for x in late),
                                              " ".join("%016x" % int(x) for x in busy))


if __name__ == "__main__":
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "lateness_masks.txt")
    with open(out, "w") as fh:
        fh.write("\n".join(lines()) + "\n")
    print("wrote", out)
