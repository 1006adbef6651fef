"""GPU parity at the benchmark's full sizes (C3, C4, C5 and the X variants), in the launch configuration bench.py times.

Users are independent, so the oracle checks whole users of the batch: every candidate of those users,
element by element, to the same tolerance as the small cases.  The float64 oracle takes 20 s (C3) to five
minutes (a 16 384-token prefix) per user on eight cores, so its scores are computed once, by
tests/golden/make_full_size_scores.py (which imports only `oracle` and `synth`), and stored in
tests/golden/full_size_scores.npz: every user of C3, eight users of C4, nine users of C5 (both users at
the 16 384-token clip, one of them uncached; the shortest cached and uncached users; uncached users of
middle length; the longest suffixes), one user of each X variant.  For the remaining users the test checks
what holds at any size: ranking on the cached prefix and full recompute, two different kernel sequences,
must agree (Section 2.3 of the paper), scores must be finite, and a second call must reproduce the first
bit for bit.
"""
import os
import time

import numpy as np
import pytest
import torch

import paper_2601_01712_amd as rg
import synth
from gpu_util import Harness, TOL

pytestmark = pytest.mark.gpu

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "full_size_scores.npz")


def stored_scores(name, batch):
    """user -> float64 oracle scores stored for workload `name`; checks that the stored shapes are this batch's."""
    out = {}
    with np.load(GOLDEN, allow_pickle=False) as z:
        for key in z.files:
            wl, rest = key.split("/", 1)
            if wl != name or rest.endswith("/shape"):
                continue
            u = int(rest[1:])
            L = int(batch["prefix_off"][u + 1] - batch["prefix_off"][u])
            S = int(batch["suffix_off"][u + 1] - batch["suffix_off"][u])
            M = int(batch["cand_off"][u + 1] - batch["cand_off"][u])
            assert list(z[key + "/shape"]) == [L, S, M], f"{key}: stored for another batch shape"
            out[u] = z[key]
    return out


def run_full(name, min_users, page_tokens=256):
    wl = synth.WORKLOADS[name]
    cfg = wl.model
    t0 = time.time()
    weights = synth.make_weights(cfg, wl.seed)
    batch = synth.make_batch(wl, 0)
    L, S, M, cached = synth.make_lengths(wl, 0)
    want = stored_scores(name, batch)
    assert len(want) >= min_users
    print(f"\n  {name}: inputs in {time.time() - t0:.1f}s; users {wl.n_users}, prefix tokens {int(L.sum())}, "
          f"candidates {int(M.sum())}, uncached {int((~cached).sum())}; oracle scores stored for users {sorted(want)}", flush=True)
    h = Harness(cfg, weights, batch, page_tokens)
    try:
        h.prefill([u for u in range(wl.n_users) if cached[u]])
        got_cached = h.rank_cached()
        again = h.rank_cached()
        got_full = h.rank_full()
        assert np.isfinite(got_cached).all() and np.isfinite(got_full).all()
        assert np.array_equal(got_cached, again), "two identical calls must give identical bits"
        scale = max(1.0, float(np.abs(got_full).max()))
        diff = float(np.abs(got_cached - got_full).max())
        assert diff <= 2 * TOL[cfg.dtype] * scale, f"cached vs full recompute differ by {diff:.3e}"
        e1 = h.check(got_cached, want, f"{name} rank_with_cache")
        e2 = h.check(got_full, want, f"{name} rank_full_recompute")
        print(f"  {name}: max err vs stored oracle scores: cached {e1:.2e}, full {e2:.2e} (bound {TOL[cfg.dtype]:.1e}); "
              f"cached vs full over all users {diff:.2e}", flush=True)
        return L, S, M, cached, want
    finally:
        h.close()


def test_c3_every_user_against_the_oracle():
    run_full("C3", min_users=16)


def test_c4_eight_users_against_the_oracle_and_kv_footprint():
    run_full("C4", min_users=8)
    cfg = rg.make_config(8, 512, 8, "bf16")
    assert rg.relaygr_kv_footprint_bytes(cfg, 8192) == 134217728     # per-user KV bytes of this workload


def test_x1_width_1024():
    """Section 4.4's width axis: d = 1024 (d_head = 128)."""
    run_full("X1", min_users=1)


def test_x2_depth_16_layers():
    """Section 4.4's depth axis: 16 layers."""
    run_full("X2", min_users=1)


def test_x3_fp16():
    """The half precision the paper mentions (Section 4.2): C3's shape in IEEE fp16."""
    run_full("X3", min_users=1)


def test_x4_softmax_attention():
    """The backbone variant that differs only in its attention computation (Section 4.4), read as a
    softmax over the visible keys: C3's shape."""
    run_full("X4", min_users=1)


def test_c5_jagged_batch_nine_users_against_the_oracle():
    L, S, M, cached, want = run_full("C5", min_users=8)
    users = sorted(want)
    assert any(not cached[u] for u in users), "an uncached user (recomputed inside the call) must be among the checked"
    assert any(L[u] >= 16000 and cached[u] for u in users) and any(L[u] >= 16000 and not cached[u] for u in users)
    assert int(L[users].min()) <= 800 and int(S[users].max()) >= 60
