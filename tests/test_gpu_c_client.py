"""The boundary is usable without the Python binding: a C99 program (tests/c_client.c) built
against include/wagma.h and the HIP runtime's C API runs a few iterations on the GPU, and its
output bytes equal the CPU oracle's."""
import os
import struct
import subprocess

import numpy as np
import pytest

from oracle import wagma_oracle as orc
from paper_2005_00124_amd import wagma as lw

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


def build_c_client(tmp_path):
    exe = tmp_path / "c_client"
    lib_dir = os.path.dirname(lw.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-O1", "-Wall", "-Wextra", "-Werror", "-D__HIP_PLATFORM_AMD__",
                    "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROCM, "include"),
                    "-o", str(exe), os.path.join(ROOT, "tests", "c_client.c"),
                    "-L", lib_dir, "-lwagma", "-L", os.path.join(ROCM, "lib"), "-lamdhip64",
                    "-Wl,-rpath," + lib_dir, "-Wl,-rpath," + os.path.join(ROCM, "lib")],
                   check=True, timeout=300)
    return exe


def test_c_client_compiles_as_c99_and_links(tmp_path):
    if not os.path.exists(lw.LIB_PATH):
        from paper_2005_00124_amd import build
        build.build()
    assert os.path.exists(build_c_client(tmp_path))


@pytest.mark.gpu
@pytest.mark.parametrize("P,S,n,tau,iters", [(8, 4, 1001, 3, 3), (64, 8, 5000, 4, 5), (32, 16, 777, 0, 2)])
def test_c_client_matches_the_oracle(tmp_path, P, S, n, tau, iters):
    print("c client P=%d S=%d n=%d tau=%d iters=%d" % (P, S, n, tau, iters), flush=True)
    exe = build_c_client(tmp_path)
    rng = np.random.default_rng(P * 1000 + n)
    lr, mu = np.float32(0.1), np.float32(0.9)
    w = rng.normal(0, 0.05, (P, n)).astype(np.float32)
    m = rng.normal(0, 0.01, (P, n)).astype(np.float32)
    pub = rng.normal(0, 0.05, (P, n)).astype(np.float32)
    masks, grads = [], []
    for t in range(iters):
        late = rng.random(P) < (0.3 if t % 2 else 0.0)       # t = 1: some processes late
        masks.append(orc.mask_words(late))
        grads.append(rng.normal(0, 1e-2, (P, n)).astype(np.float32))
    problem = tmp_path / "problem.bin"
    with open(problem, "wb") as f:
        f.write(struct.pack("<4iq2f", P, S, tau, iters, n, float(lr), float(mu)))
        for a in (w, m, pub):
            f.write(a.tobytes())
        for t in range(iters):
            f.write(np.ascontiguousarray(masks[t], dtype=np.uint64).tobytes())
            f.write(grads[t].tobytes())
    result = tmp_path / "result.bin"
    run = subprocess.run([str(exe), str(problem), str(result)], capture_output=True, text=True, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "c client: done" in run.stdout
    ow, om, opub = w.copy(), m.copy(), pub.copy()
    for t in range(iters):
        orc.step_f32(P, S, tau, t, ow, grads[t], om, opub, masks[t], float(lr), float(mu))
        first = orc.member_table(P, S, t).ravel()[:min(S, 8)] if not orc.is_global_iteration(tau, t) else range(min(S, 8))
        assert ("t=%d" % t) in run.stdout and " ".join(str(int(r)) for r in first) in run.stdout.splitlines()[t]
    got = np.fromfile(result, dtype=np.float32).reshape(3, P, n)
    for have, want, what in zip(got, (ow, om, opub), ("w", "m", "pub")):
        assert np.array_equal(have.view(np.uint32), want.view(np.uint32)), what
