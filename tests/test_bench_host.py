"""Host logic of bench.py that needs no GPU: the parsing of the profiler's counter files."""
import os
import stat
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

FAKE = r'''#!/usr/bin/env python3
# stands in for rocprofv3: writes the counter file bench.measure_traffic() reads
import os, sys
a = sys.argv
counter = a[a.index("--pmc") + 1]
out = os.path.join(a[a.index("-d") + 1], "host", "1_counter_collection.csv")
os.makedirs(os.path.dirname(out))
K = int(a[a.index("--steps") + 1])
rows = [("__amd_rocclr_copyBuffer", 10.0), ("__amd_rocclr_copyBuffer", 500.0 if counter == "FETCH_SIZE" else 1000.0)]
rows += [("void step_rows_in_registers<8, true, false>(StepParams)", 7777.0)] * 5        # search and warm-up
for t in range(K):
    if t == K - 1:
        rows.append(("void step_rows_streamed<true, false>(StepParams)", 999.0))           # a global iteration
    else:
        rows.append(("void step_rows_in_registers<8, true, false>(StepParams)", 100.0 + t if counter == "FETCH_SIZE" else 300.0))
with open(out, "w") as f:
    f.write('"Dispatch_Id","Kernel_Name","Counter_Name","Counter_Value"\n')
    for i, (k, v) in enumerate(rows):
        f.write('%d,"%s","%s",%f\n' % (i + 1, k, counter, v))
        f.write('%d,"%s","OTHER",%f\n' % (i + 1, k, 5.0))
'''


def test_measure_traffic_reads_the_timed_group_launches(tmp_path, monkeypatch):
    import bench
    tool = tmp_path / "rocprofv3"
    tool.write_text(FAKE)
    tool.chmod(tool.stat().st_mode | stat.S_IEXEC)
    monkeypatch.setenv("PATH", str(tmp_path) + os.pathsep + os.environ["PATH"])
    K = 6
    got = bench.measure_traffic(4, K, 2, array_bytes=1000 * 1024)
    # the copy of 1000 KiB reads 500 KiB in FETCH_SIZE (factor 2) and 1000 KiB in WRITE_SIZE (factor 1);
    # the timed group launches are the last K step launches minus the streamed one: 100..104 KiB and 300 KiB
    assert got is not None
    assert got["fetch_factor"] == 2.0 and got["write_factor"] == 1.0
    assert got["bytes"] == (2.0 * 102.0 + 300.0) * 1024


def test_measure_traffic_without_the_profiler(monkeypatch, tmp_path):
    import bench
    monkeypatch.setenv("PATH", str(tmp_path))
    assert bench.measure_traffic(4, 6, 2, array_bytes=1 << 20) is None
