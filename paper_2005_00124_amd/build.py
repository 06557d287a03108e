"""Builds libwagma.so (gfx950) in-tree with hipcc.  `python -m paper_2005_00124_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
# wagma.hip: the step (kernels in wagma_kernels.h, lateness generators in wagma_masks.h);
# wagma_alloc.hip: the optional allocator (searches in wagma_placement.h and wagma_chunks.h)
SOURCES = [os.path.join(PKG, "csrc", "wagma.hip"), os.path.join(PKG, "csrc", "wagma_alloc.hip")]
SRC = SOURCES[0]
LIB = os.path.join(PKG, "libwagma.so")

# IEEE fp32 throughout: no contraction (the two fused multiply-adds are explicit), no
# fast-math, correctly rounded division, denormals kept.  Packed-fp32 instruction
# selection is switched off.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off", "-fno-fast-math", "-fhip-fp32-correctly-rounded-divide-sqrt",
    "-fno-gpu-flush-denormals-to-zero",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
    "-I" + os.path.join(ROOT, "include"),
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def build(verbose: bool = False) -> str:
    """Compile csrc/*.hip into paper_2005_00124_amd/libwagma.so; returns the path."""
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [hipcc(), *HIPCC_FLAGS, "-o", tmp, *SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-q" not in sys.argv))
