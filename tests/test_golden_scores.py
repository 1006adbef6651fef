"""The stored oracle scores the full-size GPU tests compare against (tests/golden/full_size_scores.npz)
are what the oracle computes today: the script that wrote them imports only `oracle` and `synth`, and the
cheapest stored users are recomputed here on every CPU run."""
import os
import re

import numpy as np

import oracle
import synth
from synth.generator import user_slices

HERE = os.path.dirname(__file__)
GOLDEN = os.path.join(HERE, "golden", "full_size_scores.npz")
SCRIPT = os.path.join(HERE, "golden", "make_full_size_scores.py")


def test_the_script_imports_nothing_of_the_hip_path():
    src = open(SCRIPT).read()
    imports = re.findall(r"^\s*(?:import|from)\s+([\w\.]+)", src, flags=re.M)
    assert "oracle" in imports and "synth" in imports
    assert not any(m.startswith("paper_2601_01712_amd") for m in imports)
    assert "librelaygr" not in src and "ctypes" not in src


def test_stored_users_cover_what_the_gpu_tests_need():
    with np.load(GOLDEN, allow_pickle=False) as z:
        users = {}
        for k in z.files:
            if k.endswith("/shape"):
                continue
            wl, u = k.split("/u")
            users.setdefault(wl, []).append(int(u))
            assert z[k].dtype == np.float64 and np.isfinite(z[k]).all()
            assert z[k].shape == (int(z[k + "/shape"][2]),)
    assert sorted(users["C3"]) == list(range(16)) and len(users["C4"]) >= 8 and len(users["C5"]) >= 8
    L, S, M, cached = synth.make_lengths(synth.WORKLOADS["C5"], 0)
    assert any(L[u] >= 16000 for u in users["C5"]) and any(not cached[u] for u in users["C5"])


def test_cheapest_stored_users_equal_a_fresh_oracle_run():
    wl = synth.WORKLOADS["C5"]
    weights = synth.make_weights(wl.model, wl.seed)
    batch = synth.make_batch(wl, 0)
    with np.load(GOLDEN, allow_pickle=False) as z:
        for u in (32, 4):
            p, s, c = user_slices(batch, u)
            assert list(z[f"C5/u{u}/shape"]) == [len(p), len(s), len(c)]
            fresh = oracle.full_recompute(wl.model, weights, p, s, c)
            assert np.array_equal(fresh, z[f"C5/u{u}"]) or float(np.abs(fresh - z[f"C5/u{u}"]).max()) < 1e-12
