"""The synthetic workloads reproduce the paper's model sizes (Section 6) and are seeded."""
import torch

from paper_2005_00124_amd import workloads as wk


def test_parameter_counts():
    assert wk.count_params(wk.resnet50_tensors()) == 25557032
    # Section 6.2 prints 25,559,081 for ResNet-50: the 1001-class classifier
    assert wk.count_params(wk.resnet50_tensors(1001)) == 25559081
    # Section 6.3 prints 61,362,176 (245 MB) for the Transformer
    assert wk.count_params(wk.transformer_tensors(512, 2048)) == 61362176
    assert wk.count_params(wk.transformer_tensors(1024, 4096)) == 210804736
    assert [w.n for w in wk.WORKLOADS] == [1048576, 25557032, 61362176, 25557032, 210804736]
    assert [(w.P, w.S, w.tau, w.iters) for w in wk.WORKLOADS] == [
        (4, 2, 5, 10), (16, 4, 10, 50), (16, 4, 10, 50), (64, 8, 16, 50), (32, 8, 8, 20)]


def test_resnet_tensor_list_shape():
    t = wk.resnet50_tensors()
    assert t[0][1] == (7, 7, 3, 64) and t[-2][1] == (2048, 1000)
    assert sum(1 for x in t if x[2] == "he_normal") == 54      # 53 convolutions + fc


def test_seeded_and_distributed_as_stated():
    wl = wk.workload(1)
    P, n = wl.P, wl.n
    a = [torch.empty(P, n) for _ in range(3)]
    b = [torch.empty(P, n) for _ in range(3)]
    wk.fill_initial_state(wl, *a)
    wk.fill_initial_state(wl, *b)
    for x, y in zip(a, b):
        assert torch.equal(x, y)
    w, m, pub = a
    assert torch.equal(w[0], w[3]) and torch.equal(pub, w) and not m.any()
    assert abs(float(w[0].std()) - 0.02) < 1e-3
    g0, g1 = torch.empty(P, n), torch.empty(P, n)
    wk.fill_gradients(wl, 0, g0)
    wk.fill_gradients(wl, 1, g1)
    assert not torch.equal(g0, g1) and not torch.equal(g0[0], g0[1])
    assert abs(float(g0.std()) - 1e-3) < 1e-4
    g0b = torch.empty(P, n)
    wk.fill_gradients(wl, 0, g0b)
    assert torch.equal(g0, g0b)


def test_init_kinds_small():
    tensors = [("c", (3, 3, 8, 16), "he_normal", 72, 16), ("bn.g", (16,), "ones", 0, 0),
               ("bn.b", (16,), "zeros", 0, 0), ("x", (64, 32), "xavier_uniform", 64, 32),
               ("e", (100, 16), "embedding", 16, 0)]
    n = wk.count_params(tensors)
    row = torch.full((n,), 7.0)
    wk.init_model_row(tensors, row, wk.make_generator(3, "cpu"))
    assert torch.all(row[1152:1168] == 1) and torch.all(row[1168:1184] == 0)
    x = row[1184:1184 + 2048]
    assert float(x.abs().max()) <= (6 / 96) ** 0.5
    assert abs(float(row[:1152].std()) - (2 / 72) ** 0.5) < 0.02


def test_sample_columns_cover_both_ends():
    cols = wk.sample_columns(25557032, 5000, 1)
    assert cols[0] == 0 and cols[-1] == 25557031 and len(cols) >= 5000
    assert torch.all(cols[1:] > cols[:-1])
    assert wk.workload(4).stale_threshold == 1 << 30


def test_lateness_masks_of_the_workloads_are_frozen():
    """The masks the five workloads draw in their first iterations equal the stored ones
    (tests/golden/lateness_masks.txt, written by tests/golden/make_lateness_masks.py from the
    oracle): a change of a seed, a threshold or a generator shows up here."""
    import importlib.util
    import os
    here = os.path.dirname(os.path.abspath(__file__))
    spec = importlib.util.spec_from_file_location("make_lateness_masks",
                                                  os.path.join(here, "golden", "make_lateness_masks.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    stored = open(os.path.join(here, "golden", "lateness_masks.txt")).read().split("\n")
    assert [x for x in stored if x] == list(mod.lines())


def test_stored_traffic_figures_are_those_of_the_profiles():
    """bench.py's roofline.traffic constants are copies of figures under profiles/: each must
    equal the number its file states, and the launch options they were taken with likewise."""
    import os
    import re
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    sys.path.insert(0, root)
    import bench
    for table in (bench.MEASURED_TRAFFIC, bench.MEASURED_TRAFFIC_PER_TENSOR):
        for index, (nbytes, name) in table.items():
            text = open(os.path.join(root, "profiles", name)).read()
            stated = re.search(r"traffic_bytes_per_launch = ([0-9.e+]+)", text)
            assert stated and float(stated.group(1)) == nbytes, name
            options = re.search(r"launch options of these runs: ([a-z0-9_= -]+)\)", text)
            assert options, name
            have = dict(kv.split("=") for kv in options.group(1).split())
            assert {k: int(v) for k, v in have.items()} == bench.PROFILE_OPTIONS, name
            assert set(bench.PROFILE_OPTIONS) <= set(bench.OPTS)
