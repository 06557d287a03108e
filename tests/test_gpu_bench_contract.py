"""bench.py keeps its output contract: one JSON line with the agreed keys (small workload, GPU)."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_bench(*extra):
    out = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "1", "--steps", "10",
                          "--warmup", "2", "--cpu-columns", "8192", "--cpu-workers", "2", *extra],
                         capture_output=True, text=True, cwd=ROOT, timeout=600)
    assert out.returncode == 0, out.stderr[-2000:]
    lines = [l for l in out.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, "exactly one line on stdout"
    return json.loads(lines[0])


def test_bench_json_contract():
    d = run_bench()
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better",
                "scaling", "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 10 and d["warmup"] == 2 and d["higher_is_better"] is True
    assert d["dtype"] == "f32" and d["data"] == "synthetic" and d["vs_baseline"] is None
    assert "workload" in d["config"] and "model" not in d["config"]
    assert d["value"] > 0 and d["ms_per_step"] > 0
    r = d["roofline"]
    assert r["bound"] == "hbm" and r["peak"] == 8000.0 and r["unit"] == "GB/s"
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-9
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["cores"] == 1 and c["value"] > 0 and c["sample"] and c["cpu_model"]
    a = c["all_cores"]
    assert a["cores"] == 2 and a["value"] > 0 and a["sample"] and a["cpu_model"]
    assert r["traffic"] is None and r["traffic_source"] is None      # no counter run stored for workload 1


@pytest.mark.parametrize("layout", ["views", "stacked", "separate"])
def test_bench_per_tensor_layouts(layout):
    """--tensors on the 161-tensor model of workload 2, in each of the three places the tensors can lie."""
    out = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "2", "--steps", "4",
                          "--warmup", "1", "--no-cpu-baseline", "--no-extras", "--tensors", "--tensor-layout", layout],
                         capture_output=True, text=True, cwd=ROOT, timeout=600)
    assert out.returncode == 0, out.stderr[-2000:]
    d = json.loads([l for l in out.stdout.splitlines() if l.strip()][-1])
    assert d["config"]["layout"] == "per-tensor (%s)" % layout
    assert d["value"] > 0 and 0.3 < d["roofline"]["frac"] < 1.0
    assert d["roofline"]["traffic"] is None      # the stored counter figure is workload 4's, stacked
