"""The tile table of the per-tensor layout (csrc/wagma_tiles.h: which workgroup takes which slices of
which tensor) on the CPU: the header has no HIP in it, so a small driver (tests/tiles_host.cpp, built
with the address and undefined-behaviour sanitizers) checks here that for mixes of tensor sizes,
address phases, maps and XCD run lengths every element of every tensor belongs to exactly one lane, and
that tensors are joined, and taken as spaced alike, exactly when their pointers say so."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_tile_table_covers_every_element_once(tmp_path):
    exe = tmp_path / "tiles_host"
    subprocess.run(["g++", "-std=c++17", "-O1", "-Wall", "-Wextra", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=all", "-I", os.path.join(ROOT, "paper_2005_00124_amd", "csrc"),
                    "-o", str(exe), os.path.join(ROOT, "tests", "tiles_host.cpp")], check=True)
    out = subprocess.run([str(exe)], capture_output=True, text=True, timeout=300)
    assert out.returncode == 0 and out.stdout.strip().endswith("ok"), out.stdout + out.stderr
