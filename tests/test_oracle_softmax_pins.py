"""Pins for the oracle's second attention form (CPU only).

Section 4.4 of the paper evaluates a backbone variant that differs from the
first only in its attention computation and prints neither a formula nor an
output for it, so the reading (a softmax over the visible keys in place of
SiLU(.)/n) is pinned to what the mathematics fixes: a library attention
routine on the same mask, a scalar brute-force evaluator on tiny inputs, the
relay-race identity (Section 2.3), closed forms for degenerate inputs, and
invariances of a softmax.  The last group plants plausible mistakes in a copy
of the oracle and checks that a pin catches each.
"""
import dataclasses
import math

import numpy as np
import pytest
import torch

import oracle
import synth
from oracle import relaygr_oracle as ro

F64 = torch.float64


def tiny_model(n_layers=2, d=8, heads=2, seed=11, boost=1.0, attention="softmax"):
    cfg = synth.ModelConfig(n_layers, d, heads, "fp32", attention=attention)
    w = synth.make_weights(cfg, seed)
    if boost != 1.0:
        for lw in w["layers"]:
            for k_ in ("w1", "b1", "w2", "b2", "ln_in_b", "ln_at_b"):
                lw[k_] = (lw[k_] * boost).astype(np.float32)
        w["w_score"] = (w["w_score"] * boost).astype(np.float32)
    return cfg, w


def tokens(seed, tag, n, d, std=1.0):
    return synth.normal(seed, tag, n * d, 0.0, std).reshape(n, d).astype(np.float32)


def rand(seed, tag, shape, std=1.0):
    return torch.from_numpy(synth.normal(seed, tag, int(np.prod(shape)), 0.0, std).reshape(shape))


# ------------------------------------------------------------ library routine
@pytest.mark.parametrize("L,S,M,heads", [(9, 3, 4, 2), (0, 0, 3, 1), (17, 0, 5, 4), (1, 2, 1, 2)])
def test_softmax_attention_matches_library_attention(L, S, M, heads):
    """Per head, step 3 is textbook masked scaled-dot-product attention."""
    d = 8 * heads
    N = L + S + M
    q, k, v = rand(1, "q", (N, d), 2.0), rand(1, "k", (N, d), 2.0), rand(1, "v", (N, d))
    mask = oracle.visibility_mask(L, S, M)
    alpha = 1.0 / math.sqrt(8)
    got = ro._attend_softmax(q, k, v, mask, heads, alpha)
    split = lambda t: t.reshape(N, heads, 8).transpose(0, 1)     # [heads, N, 8]
    lib = torch.nn.functional.scaled_dot_product_attention(split(q), split(k), split(v), attn_mask=mask, scale=alpha)
    torch.testing.assert_close(got, lib.transpose(0, 1).reshape(N, d), rtol=1e-12, atol=1e-13)


# ---------------------------------------------------------------- brute force
@pytest.mark.parametrize("L,S,M,heads,layers", [
    (5, 2, 3, 2, 2), (0, 0, 1, 1, 1), (0, 3, 2, 2, 2), (4, 0, 4, 1, 2), (7, 1, 1, 2, 1), (12, 4, 8, 2, 2),
])
def test_oracle_equals_scalar_brute_force(L, S, M, heads, layers):
    cfg, w = tiny_model(layers, 8, heads, seed=200 + L + S + M, boost=15.0)
    p, s, c = tokens(1, "p", L, 8), tokens(1, "s", S, 8), tokens(1, "c", M, 8)
    got = oracle.full_recompute(cfg, w, p, s, c)
    want = np.array(oracle.brute_force_scores(cfg, w, p, s, c))
    assert np.abs(want).max() > 1e-3
    np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-12)


def test_the_two_forms_differ():
    """The form switch is live: same weights and tokens, different scores."""
    cfg, w = tiny_model(2, 16, 2, seed=3, boost=8.0)
    p, s, c = tokens(2, "p", 12, 16), tokens(2, "s", 2, 16), tokens(2, "c", 4, 16)
    a = oracle.full_recompute(cfg, w, p, s, c)
    b = oracle.full_recompute(dataclasses.replace(cfg, attention="silu"), w, p, s, c)
    assert np.abs(a - b).max() > 1e-3
    with pytest.raises(ValueError):
        oracle.full_recompute(dataclasses.replace(cfg, attention="other"), w, p, s, c)


# ------------------------------------------------- relay-race identity (S2.3)
@pytest.mark.parametrize("L,S,M", [(40, 6, 9), (64, 0, 5), (1, 0, 1), (33, 7, 1)])
def test_cached_prefix_equals_full_inference(L, S, M):
    cfg, w = tiny_model(3, 16, 2, seed=5, boost=8.0)
    p, s, c = tokens(2, "p", L, 16), tokens(2, "s", S, 16), tokens(2, "c", M, 16)
    psi = oracle.prefix_kv(cfg, w, p)
    two_phase = oracle.rank_with_kv(cfg, w, psi, s, c)
    one_shot = oracle.full_recompute(cfg, w, p, s, c)
    np.testing.assert_allclose(two_phase, one_shot, rtol=1e-11, atol=1e-13)


def test_candidates_never_see_each_other():
    cfg, w = tiny_model(2, 16, 2, seed=7, boost=8.0)
    p, s, c = tokens(4, "p", 30, 16), tokens(4, "s", 3, 16), tokens(4, "c", 10, 16)
    full = oracle.full_recompute(cfg, w, p, s, c)
    one_by_one = np.concatenate([oracle.full_recompute(cfg, w, p, s, c[i:i + 1]) for i in range(10)])
    np.testing.assert_allclose(one_by_one, full, rtol=1e-12)


# ------------------------------------------------------------- closed forms
def test_identical_tokens_give_the_lone_candidate_score():
    """Identical tokens have identical values, and softmax weights sum to one over the visible
    keys, so every attention output equals that value whatever L and S are.  A denominator that
    counts invisible keys, or misses the candidate's own key, breaks this."""
    cfg, w = tiny_model(2, 16, 2, seed=12, boost=8.0)
    t = tokens(8, "t", 1, 16)
    lone = oracle.full_recompute(cfg, w, np.zeros((0, 16)), np.zeros((0, 16)), t)
    for L, S in ((5, 0), (9, 3), (1, 1)):
        got = oracle.full_recompute(cfg, w, np.repeat(t, L, 0), np.repeat(t, S, 0), np.repeat(t, 2, 0))
        np.testing.assert_allclose(got, [lone[0], lone[0]], rtol=1e-12)


def test_weights_are_a_convex_combination_and_shift_invariant():
    N, d, heads = 11, 16, 2
    q, k = rand(5, "q", (N, d), 3.0), rand(5, "k", (N, d), 3.0)
    mask = oracle.visibility_mask(6, 2, 3)
    alpha = 1 / math.sqrt(8)
    # constant values come back unchanged, row by row
    const = rand(5, "c", (1, d)).expand(N, d).contiguous()
    torch.testing.assert_close(ro._attend_softmax(q, k, const, mask, heads, alpha), const, rtol=1e-13, atol=1e-14)
    # the output lies inside the range of the visible values
    v = rand(5, "v", (N, d))
    o = ro._attend_softmax(q, k, v, mask, heads, alpha)
    for i in range(N):
        vis = v[mask[i]]
        assert torch.all(o[i] <= vis.max(0).values + 1e-12) and torch.all(o[i] >= vis.min(0).values - 1e-12)
    # one-hot values read the weights out: they are positive on visible keys, zero elsewhere, sum to 1
    eye = torch.eye(N, dtype=F64)
    wts = ro._attend_softmax(q[:, :8], k[:, :8], eye[:, :8], mask, 1, alpha)      # weights of keys 0..7
    assert torch.all(wts[mask[:, :8]] > 0) and torch.all(wts[~mask[:, :8]] == 0)
    # a key direction added to every key shifts each row's scores by a constant: nothing changes
    shift = rand(5, "s", (1, d), 2.0)
    torch.testing.assert_close(ro._attend_softmax(q, k + shift, v, mask, heads, alpha), o, rtol=1e-10, atol=1e-12)
    big = ro._attend_softmax(q * 40.0, k, v, mask, heads, alpha)       # large scores stay finite (max subtracted)
    assert torch.isfinite(big).all()


def test_sharp_scores_select_the_best_visible_key():
    """As the scores grow the softmax tends to the argmax over VISIBLE keys."""
    N, d = 7, 8
    q, k, v = rand(6, "q", (N, d)), rand(6, "k", (N, d)), rand(6, "v", (N, d))
    mask = oracle.visibility_mask(4, 1, 2)
    o = ro._attend_softmax(q * 2000.0, k, v, mask, 1, 1.0)
    s = (q @ k.T).masked_fill(~mask, -math.inf)
    torch.testing.assert_close(o, v[s.argmax(dim=1)], rtol=1e-9, atol=1e-9)


# ----------------------------------------------- planted mistakes are caught
def _gap(cfg, w, p, s, c):
    return np.abs(oracle.full_recompute(cfg, w, p, s, c) - np.array(oracle.brute_force_scores(cfg, w, p, s, c))).max()


def _case():
    cfg, w = tiny_model(2, 8, 2, seed=21, boost=15.0)
    return cfg, w, tokens(9, "p", 6, 8), tokens(9, "s", 2, 8), tokens(9, "c", 3, 8)


def test_pin_catches_mask_applied_after_the_softmax(monkeypatch):
    def wrong(q, k_all, v_all, mask, n_heads, alpha):
        R, d = q.shape
        dh = d // n_heads
        o = torch.empty((R, d), dtype=F64)
        for h in range(n_heads):
            c = slice(h * dh, (h + 1) * dh)
            a = torch.softmax(alpha * (q[:, c] @ k_all[:, c].T), dim=1) * mask.to(F64)   # denominator counts invisible keys
            o[:, c] = a @ v_all[:, c]
        return o
    assert _gap(*_case()) < 1e-12
    monkeypatch.setattr(ro, "_attend_softmax", wrong)
    assert _gap(*_case()) > 1e-6
    # and the identical-token closed form catches it on its own
    cfg, w = tiny_model(2, 16, 2, seed=12, boost=8.0)
    t = tokens(8, "t", 1, 16)
    lone = oracle.full_recompute(cfg, w, np.zeros((0, 16)), np.zeros((0, 16)), t)
    got = oracle.full_recompute(cfg, w, np.repeat(t, 5, 0), np.zeros((0, 16)), np.repeat(t, 2, 0))
    assert abs(got[0] - lone[0]) > 1e-6


def test_pin_catches_missing_scale_and_transposed_scores(monkeypatch):
    orig = ro._attend_softmax
    monkeypatch.setattr(ro, "_attend_softmax", lambda q, k, v, m, h, a: orig(q, k, v, m, h, 1.0))
    assert _gap(*_case()) > 1e-6
    orig_proj = ro._project

    def swapped(x, lw, eps, d):
        u, v, q, k = orig_proj(x, lw, eps, d)
        return u, v, k, q          # q and k swapped (a transposed score matrix)
    monkeypatch.setattr(ro, "_attend_softmax", orig)
    monkeypatch.setattr(ro, "_project", swapped)
    assert _gap(*_case()) > 1e-6


def test_pin_catches_softmax_over_the_query_axis():
    """Normalising over rows instead of keys fails the library pin."""
    N, d = 6, 8
    q, k, v = rand(7, "q", (N, d), 2.0), rand(7, "k", (N, d), 2.0), rand(7, "v", (N, d))
    mask = oracle.visibility_mask(3, 1, 2)
    s = (q @ k.T / math.sqrt(d)).masked_fill(~mask, -math.inf)
    wrong = torch.nan_to_num(torch.softmax(s, dim=0)) @ v
    right = ro._attend_softmax(q, k, v, mask, 1, 1 / math.sqrt(d))
    assert (wrong - right).abs().max() > 1e-3
