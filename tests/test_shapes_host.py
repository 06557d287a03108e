"""The launch shapes (csrc/wagma_shapes.h: which slices of a row the lanes of a workgroup take) on the
CPU: the header has no HIP in it, so a small driver (tests/shapes_host.cpp, built with the address
and undefined-behaviour sanitizers) checks here that every shape the library uses, and the stripes,
runs and maps that can be forced, deal every slice of a padded row out exactly once."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_launch_shape_is_a_bijection(tmp_path):
    exe = tmp_path / "shapes_host"
    subprocess.run(["g++", "-std=c++17", "-O1", "-Wall", "-Wextra", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=all", "-I", os.path.join(ROOT, "paper_2005_00124_amd", "csrc"),
                    "-o", str(exe), os.path.join(ROOT, "tests", "shapes_host.cpp")], check=True)
    out = subprocess.run([str(exe)], capture_output=True, text=True, timeout=300)
    assert out.returncode == 0 and out.stdout.strip().endswith("ok"), out.stdout + out.stderr
