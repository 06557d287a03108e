"""The HBM-region search (host logic of wagma_alloc_buffers) against a simulated memory, on the CPU."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_region_search_on_simulated_memory(tmp_path):
    exe = tmp_path / "placement_sim"
    subprocess.run(["g++", "-std=c++17", "-O1", "-Wall", "-fsanitize=address,undefined",
                    "-I", os.path.join(ROOT, "paper_2005_00124_amd", "csrc"),
                    "-o", str(exe), os.path.join(ROOT, "tests", "placement_sim.cpp")], check=True)
    out = subprocess.run([str(exe)], capture_output=True, text=True, timeout=600)
    print(out.stdout)
    print(out.stderr)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "all scenarios hold" in out.stdout


def test_chunk_placement_on_simulated_memory(tmp_path):
    exe = tmp_path / "chunks_sim"
    subprocess.run(["g++", "-std=c++17", "-O1", "-Wall", "-fsanitize=address,undefined",
                    "-I", os.path.join(ROOT, "paper_2005_00124_amd", "csrc"),
                    "-o", str(exe), os.path.join(ROOT, "tests", "chunks_sim.cpp")], check=True)
    out = subprocess.run([str(exe)], capture_output=True, text=True, timeout=600)
    print(out.stdout)
    print(out.stderr)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "all scenarios hold" in out.stdout
