"""Input generator: determinism, storage rounding, shape recipes (CPU only)."""
import numpy as np
import torch

import synth
from synth.generator import user_slices


def test_normal_is_counter_based_and_seeded():
    a = synth.normal(7, "x", 1000)
    b = synth.normal(7, "x", 2000)
    assert np.array_equal(a, b[:1000])          # element i depends on (seed, tag, i) only
    assert not np.array_equal(a, synth.normal(8, "x", 1000))
    assert not np.array_equal(a, synth.normal(7, "y", 1000))


def test_normal_moments():
    z = synth.normal(1, "moments", 400000)
    assert abs(z.mean()) < 0.01
    assert abs(z.std() - 1.0) < 0.01
    assert abs((z ** 3).mean()) < 0.03
    assert abs((z ** 4).mean() - 3.0) < 0.08


def test_bf16_rounding_matches_library_rne():
    x = synth.normal(3, "r", 100000).astype(np.float32)
    x[:4] = [1.0, 1.00390625, 1.01171875, -3.0e-40]   # exact ties round to even
    ours = synth.round_to_bf16(x)
    lib = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(ours, lib)


def test_uniform_int_range():
    v = synth.uniform_int(5, "u", 20000, 200, 2000)
    assert v.min() == 200 and v.max() == 2000


def test_fixed_workload_shapes():
    wl = synth.WORKLOADS["C2"]
    L, S, M, cached = synth.make_lengths(wl)
    assert (L == 2048).all() and (S == 16).all() and (M == 256).all() and cached.all()
    assert wl.model.d_head == 64 and wl.model.elem_bytes == 2


def test_jagged_workload_recipe():
    wl = synth.WORKLOADS["C5"]
    L, S, M, cached = synth.make_lengths(wl, 0)
    assert len(L) == 64
    assert L.min() >= 512 and L.max() <= 16384
    assert M.min() >= 200 and M.max() <= 2000
    assert S.min() >= 0 and S.max() <= 64
    assert 0 < (~cached).sum() < 64
    L2, _, _, _ = synth.make_lengths(wl, 1)
    assert not np.array_equal(L, L2)
    # over many batches about 30 % of users are uncached
    frac = np.mean([(~synth.make_lengths(wl, b)[3]).mean() for b in range(40)])
    assert 0.25 < frac < 0.35


def test_batch_layout_and_storage_type():
    wl = synth.WORKLOADS["C1"]
    b = synth.make_batch(wl)
    assert b["prefix_emb"].shape == (256, 64) and b["cand_emb"].shape == (16, 64)
    assert b["suffix_emb"].shape == (0, 64)
    assert list(b["prefix_off"]) == [0, 256] and list(b["cand_off"]) == [0, 16]
    p, s, c = user_slices(b, 0)
    assert p.shape == (256, 64) and s.shape == (0, 64) and c.shape == (16, 64)
    import dataclasses
    small = dataclasses.replace(synth.WORKLOADS["C2"], n_users=2, prefix_len=70, n_cands=5, n_suffix=3)
    bb = synth.make_batch(small)
    e = bb["prefix_emb"]
    assert np.array_equal(e, synth.round_to_bf16(e))     # already bf16-representable
    w = synth.make_weights(small.model, small.seed)
    assert w["layers"][0]["w1"].shape == (1024, 256)
    assert np.array_equal(w["layers"][0]["w1"], synth.round_to_bf16(w["layers"][0]["w1"]))
    assert abs(w["layers"][0]["ln_in_g"].mean() - 1.0) < 0.01
