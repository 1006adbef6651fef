"""Pins for the CPU oracle (CPU only).

The paper prints no model outputs, so the oracle is pinned to what the paper
and the mathematics fix: the relay-race identity (Section 2.3), the
candidate-independence of psi (Section 3.1), the printed KV-cache size
(Section 4.1 / table "KV caches"), a scalar brute-force evaluator on tiny
inputs, closed forms for degenerate weights and degenerate sequences, and
library routines for LayerNorm and SiLU.  The last group plants plausible
mistakes in a copy of the oracle and checks that a pin catches each.
"""
import dataclasses
import math
import os

import numpy as np
import pytest
import torch

import oracle
import synth
from oracle import relaygr_oracle as ro

F64 = torch.float64
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def tiny_model(n_layers=2, d=8, heads=2, seed=11, wstd_boost=1.0):
    cfg = synth.ModelConfig(n_layers, d, heads, "fp32")
    w = synth.make_weights(cfg, seed)
    if wstd_boost != 1.0:   # larger weights make every term matter at tiny d
        for lw in w["layers"]:
            for k_ in ("w1", "b1", "w2", "b2", "ln_in_b", "ln_at_b"):
                lw[k_] = (lw[k_] * wstd_boost).astype(np.float32)
        w["w_score"] = (w["w_score"] * wstd_boost).astype(np.float32)
    return cfg, w


def tokens(seed, tag, n, d, std=1.0):
    return synth.normal(seed, tag, n * d, 0.0, std).reshape(n, d).astype(np.float32)


# ---------------------------------------------------------------- brute force
@pytest.mark.parametrize("L,S,M,heads,layers", [
    (5, 2, 3, 2, 2), (0, 0, 1, 1, 1), (0, 3, 2, 2, 2), (4, 0, 4, 1, 2),
    (7, 1, 1, 2, 1), (1, 1, 1, 2, 2), (12, 4, 8, 2, 2), (3, 0, 0, 2, 1),
])
def test_oracle_equals_scalar_brute_force(L, S, M, heads, layers):
    cfg, w = tiny_model(layers, 8, heads, seed=100 + L + S + M, wstd_boost=15.0)
    p, s, c = tokens(1, "p", L, 8), tokens(1, "s", S, 8), tokens(1, "c", M, 8)
    got = oracle.full_recompute(cfg, w, p, s, c)
    want = np.array(oracle.brute_force_scores(cfg, w, p, s, c))
    assert got.shape == (M,)
    if M:
        assert np.abs(want).max() > 1e-3
        np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-12)


# ------------------------------------------------- relay-race identity (S2.3)
@pytest.mark.parametrize("L,S,M", [(40, 6, 9), (64, 0, 5), (1, 0, 1), (33, 7, 1)])
def test_cached_prefix_equals_full_inference(L, S, M):
    cfg, w = tiny_model(3, 16, 2, seed=5, wstd_boost=8.0)
    p, s, c = tokens(2, "p", L, 16), tokens(2, "s", S, 16), tokens(2, "c", M, 16)
    psi = oracle.prefix_kv(cfg, w, p)
    assert len(psi) == cfg.n_layers and psi[0][0].shape == (L, 16)
    two_phase = oracle.rank_with_kv(cfg, w, psi, s, c)
    one_shot = oracle.full_recompute(cfg, w, p, s, c)
    np.testing.assert_allclose(two_phase, one_shot, rtol=1e-11, atol=1e-13)


def test_psi_does_not_depend_on_candidates_or_suffix():
    """Section 3.1: psi is a function of the prefix tokens and weights only."""
    cfg, w = tiny_model(3, 16, 2, seed=6, wstd_boost=8.0)
    L, S, M = 20, 4, 6
    p, s, c = tokens(3, "p", L, 16), tokens(3, "s", S, 16), tokens(3, "c", M, 16)
    psi = oracle.prefix_kv(cfg, w, p)
    x = torch.from_numpy(np.concatenate([p, s, c])).to(F64)
    mask = oracle.visibility_mask(L, S, M)
    for l, lw in enumerate(w["layers"]):
        x, k, v = oracle.backbone_layer(x, lw, mask, cfg.n_heads, 1 / math.sqrt(8), cfg.ln_eps)
        np.testing.assert_allclose(k[:L].numpy(), psi[l][0].numpy(), rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(v[:L].numpy(), psi[l][1].numpy(), rtol=1e-12, atol=1e-14)


def test_candidates_never_see_each_other():
    cfg, w = tiny_model(2, 16, 2, seed=7, wstd_boost=8.0)
    p, s, c = tokens(4, "p", 30, 16), tokens(4, "s", 3, 16), tokens(4, "c", 10, 16)
    full = oracle.full_recompute(cfg, w, p, s, c)
    perm = np.array([3, 1, 9, 0, 7, 2, 8, 6, 5, 4])
    np.testing.assert_allclose(oracle.full_recompute(cfg, w, p, s, c[perm]), full[perm], rtol=1e-12)
    one_by_one = np.concatenate([oracle.full_recompute(cfg, w, p, s, c[i:i + 1]) for i in range(10)])
    np.testing.assert_allclose(one_by_one, full, rtol=1e-12)
    dup = np.concatenate([c[:4], c[:4]])
    r = oracle.full_recompute(cfg, w, p, s, dup)
    np.testing.assert_allclose(r[:4], r[4:], rtol=1e-12)


def test_moving_prefix_tokens_into_the_suffix_changes_nothing():
    """The mask depends on L + S only, so where the cache boundary sits is immaterial."""
    cfg, w = tiny_model(2, 16, 2, seed=8, wstd_boost=8.0)
    p, s, c = tokens(5, "p", 24, 16), tokens(5, "s", 2, 16), tokens(5, "c", 5, 16)
    base = oracle.full_recompute(cfg, w, p, s, c)
    for t in (1, 7, 24):
        p2, s2 = p[:24 - t], np.concatenate([p[24 - t:], s])
        np.testing.assert_allclose(oracle.full_recompute(cfg, w, p2, s2, c), base, rtol=1e-12)
        psi = oracle.prefix_kv(cfg, w, p2) if t < 24 else [(torch.zeros(0, 16, dtype=F64),) * 2] * cfg.n_layers
        np.testing.assert_allclose(oracle.rank_with_kv(cfg, w, psi, s2, c), base, rtol=1e-11)


# ------------------------------------------------------------- closed forms
def test_zero_projection_closed_form():
    """W1 = 0, b1 = 0 => u = v = q = k = 0, the gated term vanishes, x_c = x_c0 + NL * b2."""
    cfg, w = tiny_model(3, 16, 2, seed=9, wstd_boost=8.0)
    for lw in w["layers"]:
        lw["w1"] = np.zeros_like(lw["w1"])
        lw["b1"] = np.zeros_like(lw["b1"])
        lw["b2"] = w["layers"][0]["b2"]
    p, s, c = tokens(6, "p", 9, 16), tokens(6, "s", 2, 16), tokens(6, "c", 4, 16)
    got = oracle.full_recompute(cfg, w, p, s, c)
    b2 = w["layers"][0]["b2"].astype(np.float64)
    want = []
    for row in c.astype(np.float64):
        z = row + 3 * b2
        zn = (z - z.mean()) / math.sqrt(z.var() + cfg.ln_eps)
        want.append(float(np.dot(zn * w["ln_out_g"] + w["ln_out_b"], w["w_score"]) + w["b_score"]))
    np.testing.assert_allclose(got, want, rtol=1e-12)


def test_lone_candidate_is_a_per_token_mlp():
    """L = S = 0: a candidate sees only itself with n = 1, o^h = SiLU(alpha <q^h,k^h>) v^h."""
    cfg, w = tiny_model(1, 16, 2, seed=10, wstd_boost=8.0)
    c = tokens(7, "c", 3, 16)
    got = oracle.full_recompute(cfg, w, np.zeros((0, 16)), np.zeros((0, 16)), c)
    lw = w["layers"][0]
    F = torch.nn.functional
    want = []
    for row in c:
        x = torch.tensor(row, dtype=F64)
        xh = F.layer_norm(x, (16,), torch.tensor(lw["ln_in_g"], dtype=F64), torch.tensor(lw["ln_in_b"], dtype=F64), cfg.ln_eps)
        z = F.silu(torch.tensor(lw["w1"], dtype=F64) @ xh + torch.tensor(lw["b1"], dtype=F64))
        u, v, q, k = z[0:16], z[16:32], z[32:48], z[48:64]
        o = torch.cat([F.silu((q[h * 8:h * 8 + 8] @ k[h * 8:h * 8 + 8]) / math.sqrt(8)) * v[h * 8:h * 8 + 8] for h in range(2)])
        y = F.layer_norm(o, (16,), torch.tensor(lw["ln_at_g"], dtype=F64), torch.tensor(lw["ln_at_b"], dtype=F64), cfg.ln_eps) * u
        x = x + torch.tensor(lw["w2"], dtype=F64) @ y + torch.tensor(lw["b2"], dtype=F64)
        zf = F.layer_norm(x, (16,), torch.tensor(w["ln_out_g"], dtype=F64), torch.tensor(w["ln_out_b"], dtype=F64), cfg.ln_eps)
        want.append(float(zf @ torch.tensor(w["w_score"], dtype=F64) + w["b_score"]))
    np.testing.assert_allclose(got, want, rtol=1e-12)


def test_identical_tokens_fix_the_normaliser():
    """If every token is the same vector, every visible key contributes the same term, so the
    length-normalised sum equals that single term: the score equals the lone-candidate score
    whatever L and S are.  Any normaliser other than the count of visible keys breaks this."""
    cfg, w = tiny_model(2, 16, 2, seed=12, wstd_boost=8.0)
    t = tokens(8, "t", 1, 16)
    lone = oracle.full_recompute(cfg, w, np.zeros((0, 16)), np.zeros((0, 16)), t)
    for L, S in ((5, 0), (9, 3), (1, 1)):
        got = oracle.full_recompute(cfg, w, np.repeat(t, L, 0), np.repeat(t, S, 0), np.repeat(t, 2, 0))
        np.testing.assert_allclose(got, [lone[0], lone[0]], rtol=1e-12)


def test_visibility_mask_by_enumeration():
    m = oracle.visibility_mask(3, 2, 2).numpy()
    want = np.array([
        [1, 0, 0, 0, 0, 0, 0],
        [1, 1, 0, 0, 0, 0, 0],
        [1, 1, 1, 0, 0, 0, 0],
        [1, 1, 1, 1, 0, 0, 0],
        [1, 1, 1, 1, 1, 0, 0],
        [1, 1, 1, 1, 1, 1, 0],
        [1, 1, 1, 1, 1, 0, 1],
    ], dtype=bool)
    assert np.array_equal(m, want)
    assert list(m.sum(1)) == [1, 2, 3, 4, 5, 6, 6]


# ------------------------------------------------------- library primitives
def test_layer_norm_and_silu_match_library():
    z = torch.from_numpy(synth.normal(13, "z", 5 * 32).reshape(5, 32)) * 3 + 1
    g = torch.from_numpy(synth.normal(13, "g", 32, 1.0, 0.1))
    b = torch.from_numpy(synth.normal(13, "b", 32, 0.0, 0.1))
    lib = torch.nn.functional.layer_norm(z, (32,), g, b, 1e-5)
    torch.testing.assert_close(oracle.layer_norm(z, g, b, 1e-5), lib, rtol=1e-12, atol=1e-13)
    torch.testing.assert_close(oracle.silu(z), torch.nn.functional.silu(z), rtol=1e-13, atol=1e-14)
    # a constant row normalises to the offset alone (variance 0, eps keeps it finite)
    flat = torch.full((1, 32), 2.5, dtype=F64)
    torch.testing.assert_close(oracle.layer_norm(flat, g, b, 1e-5), b.unsqueeze(0))


# --------------------------------------------------------- printed footprint
def test_kv_footprint_matches_the_papers_table():
    with open(os.path.join(GOLDEN, "kv_cache_size.txt")) as f:
        rows = [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]
    assert rows
    for L, nl, d, e, want in rows:
        assert oracle.kv_footprint_bytes(int(nl), int(L), int(d), int(e)) == int(want)
    assert int(rows[0][4]) == 32 * 1024 * 1024
    # the long-sequence benchmark shape: 8192 tokens, 8 layers, d 512, bf16
    assert oracle.kv_footprint_bytes(8, 8192, 512, 2) == 134217728
    # psi as the oracle actually builds it has exactly that many elements
    cfg, w = tiny_model(2, 8, 2)
    psi = oracle.prefix_kv(cfg, w, tokens(1, "p", 6, 8))
    assert sum(k.numel() + v.numel() for k, v in psi) * 4 == oracle.kv_footprint_bytes(2, 6, 8, 4)


# ----------------------------------------------- planted mistakes are caught
def _brute_vs_oracle(cfg, w, p, s, c):
    return np.abs(oracle.full_recompute(cfg, w, p, s, c) - np.array(oracle.brute_force_scores(cfg, w, p, s, c))).max()


def _case():
    cfg, w = tiny_model(2, 8, 2, seed=21, wstd_boost=15.0)
    return cfg, w, tokens(9, "p", 6, 8), tokens(9, "s", 2, 8), tokens(9, "c", 3, 8)


def test_pin_catches_candidates_seeing_each_other(monkeypatch):
    def wrong(L, S, M):
        N = L + S + M
        i = torch.arange(N).unsqueeze(1)
        j = torch.arange(N).unsqueeze(0)
        return j <= i
    assert _brute_vs_oracle(*_case()) < 1e-12
    monkeypatch.setattr(ro, "visibility_mask", wrong)
    assert _brute_vs_oracle(*_case()) > 1e-6


def test_pin_catches_wrong_block_order(monkeypatch):
    orig = ro._project

    def wrong(x, lw, eps, d):
        u, v, q, k = orig(x, lw, eps, d)
        return u, v, k, q          # q and k swapped (a transposed score matrix)
    monkeypatch.setattr(ro, "_project", wrong)
    assert _brute_vs_oracle(*_case()) > 1e-6


def test_pin_catches_dropped_bias_and_missing_scale(monkeypatch):
    cfg, w, p, s, c = _case()
    orig = ro._finish_layer

    def no_b2(x, o, u, lw, eps):
        lw2 = dict(lw)
        lw2["b2"] = np.zeros_like(lw["b2"])
        return orig(x, o, u, lw2, eps)
    monkeypatch.setattr(ro, "_finish_layer", no_b2)
    assert _brute_vs_oracle(cfg, w, p, s, c) > 1e-6
    monkeypatch.setattr(ro, "_finish_layer", orig)
    orig_att = ro._attend
    monkeypatch.setattr(ro, "_attend", lambda q, k, v, m, h, a: orig_att(q, k, v, m, h, 1.0))
    assert _brute_vs_oracle(cfg, w, p, s, c) > 1e-6


def test_pin_catches_sequence_length_normaliser(monkeypatch):
    """Normalising by the total length N instead of the visible count breaks both the
    identical-token closed form and the candidate-independence of psi."""
    def wrong(q, k_all, v_all, mask, n_heads, alpha):
        R, d = q.shape
        dh = d // n_heads
        o = torch.empty((R, d), dtype=F64)
        for h in range(n_heads):
            cs = slice(h * dh, (h + 1) * dh)
            o[:, cs] = (ro.silu(alpha * (q[:, cs] @ k_all[:, cs].T)) * mask.to(F64) / k_all.shape[0]) @ v_all[:, cs]
        return o
    monkeypatch.setattr(ro, "_attend", wrong)
    cfg, w = tiny_model(2, 16, 2, seed=12, wstd_boost=8.0)
    t = tokens(8, "t", 1, 16)
    lone = oracle.full_recompute(cfg, w, np.zeros((0, 16)), np.zeros((0, 16)), t)
    got = oracle.full_recompute(cfg, w, np.repeat(t, 5, 0), np.zeros((0, 16)), np.repeat(t, 2, 0))
    assert abs(got[0] - lone[0]) > 1e-6
    p, s, c = tokens(2, "p", 20, 16), tokens(2, "s", 3, 16), tokens(2, "c", 4, 16)
    two = oracle.rank_with_kv(cfg, w, oracle.prefix_kv(cfg, w, p), s, c)
    assert np.abs(two - oracle.full_recompute(cfg, w, p, s, c)).max() > 1e-6
