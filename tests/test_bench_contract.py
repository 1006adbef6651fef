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
