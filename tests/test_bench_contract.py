"""Host-side checks of bench.py's command-line contract (CPU only; nothing here touches a GPU)."""
import json
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    """This build runs on one GPU: --gpus N with N > 1 must exit non-zero and say why, before importing torch."""
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=60)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_metric_and_workloads_follow_the_baseline_file():
    base = json.load(open(os.path.join(ROOT, "BASELINE.json")))
    src = open(os.path.join(ROOT, "bench.py")).read()
    assert "candidates" in base["metric"].lower() and "candidates/s" in src
    for name in ("C1", "C2", "C3", "C4", "C5"):
        assert re.search(rf'"{name}":', src), name
    # the default workload is the one the metric is quoted on: cached path vs full recompute at 4096 x 512
    assert re.search(r'--config", default="C3"', src)


def test_every_workload_named_by_bench_exists_in_the_generator():
    import synth
    src = open(os.path.join(ROOT, "bench.py")).read()
    names = set(re.findall(r'^    "([CX]\d)": "', src, flags=re.M))
    assert names == set(synth.WORKLOADS), (names, set(synth.WORKLOADS))


def test_algorithmic_work_per_launch_at_c3():
    """The figures the rooflines divide by, for one C3 rank launch with every prefix cached: 4 d visible keys per
    candidate (FLOP), K and V once + q + the candidates' own k and v + fp32 sums (attention bytes), 8 d^2 per row
    (projection), 4 d e per row (layer tail; 8 KB per row as built)."""
    import types
    import numpy as np
    sys.path.insert(0, ROOT)
    import bench
    import synth
    wl = synth.WORKLOADS["C3"]
    n, L0, M0, d, e = wl.n_users, wl.prefix_len, wl.n_cands, wl.model.d_model, 2
    stub = types.SimpleNamespace(cfg=wl.model, n=n, handles=[[1] * n],
                                 shapes=[(np.full(n, L0), np.zeros(n, dtype=int), np.full(n, M0), np.ones(n, bool))])
    w = bench.Loaded.layer_work(stub, 0)
    rows = n * M0
    assert w["attn"][0][0] == 4.0 * d * n * M0 * L0 == 68719476736.0
    assert w["attn"][1][0] == 2 * n * L0 * d * e + rows * d * e + 2 * rows * d * e + rows * d * 4 == 176160768
    assert w["f1"][0][0] == 8.0 * d * d * rows
    assert w["f2"][1][0] == 4 * rows * d * e == 33554432 and w["f2"][2][0] == 2 * w["f2"][1][0]
    # an uncached user adds its causal prefix visits to every layer but the last (whose prefix rows only supply K and V)
    stub.handles = [[0] + [1] * (n - 1)]
    w2 = bench.Loaded.layer_work(stub, 0)
    assert w2["attn"][0][0] - w["attn"][0][0] == 4.0 * d * (L0 * (L0 + 1) // 2) and w2["attn"][0][-1] == w["attn"][0][-1]
