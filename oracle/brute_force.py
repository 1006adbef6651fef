"""Per-token, per-key scalar evaluation of the ranking model.  TEST INFRASTRUCTURE ONLY.

A second, independent statement of the same definition as relaygr_oracle.py,
written with Python scalars and explicit loops over tokens, keys, heads and
features -- no matrix products, no array masks -- so that a transposed
operand, a wrong block order or an off-by-one in the visibility rule in the
array version shows up as a mismatch on tiny inputs.  Only practical for a few
dozen tokens.

Sequence: [prefix | suffix | candidates] (Section 2.3).  Token i may use key j
when j <= i and j is not another candidate.  With cfg.attention == "softmax"
(the reading of the backbone variant of Section 4.4) the weight of key j is
exp(alpha q.k_j) over the sum of the same over the visible keys, instead of
SiLU(alpha q.k_j) / n_i.
"""
from __future__ import annotations

import math
from typing import List


def _silu(t: float) -> float:
    return t / (1.0 + math.exp(-t))


def _layer_norm(z: List[float], g, b, eps: float) -> List[float]:
    d = len(z)
    mean = sum(z) / d
    var = sum((t - mean) ** 2 for t in z) / d
    r = 1.0 / math.sqrt(var + eps)
    return [(z[f] - mean) * r * float(g[f]) + float(b[f]) for f in range(d)]


def _affine(x: List[float], w, bias) -> List[float]:
    """out[o] = sum_i x[i] * w[o][i] + bias[o] (output-major weight)."""
    return [sum(x[i] * float(w[o][i]) for i in range(len(x))) + float(bias[o]) for o in range(len(bias))]


def brute_force_scores(cfg, weights: dict, prefix, suffix, cands) -> List[float]:
    d = cfg.d_model
    H = cfg.n_heads
    dh = d // H
    alpha = 1.0 / math.sqrt(dh)
    eps = cfg.ln_eps
    softmax = getattr(cfg, "attention", "silu") == "softmax"
    rows = [[float(t) for t in r] for seg in (prefix, suffix, cands) for r in seg]
    L, S, M = len(prefix), len(suffix), len(cands)
    N = L + S + M
    first_cand = L + S

    def visible(i: int, j: int) -> bool:
        if j > i:
            return False
        if j >= first_cand and j != i:
            return False
        return True

    x = rows
    for lw in weights["layers"]:
        u, v, q, k = [], [], [], []
        for i in range(N):
            xh = _layer_norm(x[i], lw["ln_in_g"], lw["ln_in_b"], eps)
            z = [_silu(t) for t in _affine(xh, lw["w1"], lw["b1"])]
            u.append(z[0:d])
            v.append(z[d:2 * d])
            q.append(z[2 * d:3 * d])
            k.append(z[3 * d:4 * d])
        new_x = []
        for i in range(N):
            keys = [j for j in range(N) if visible(i, j)]
            n_i = len(keys)
            o = [0.0] * d
            for h in range(H):
                lo = h * dh
                dots = []
                for j in keys:
                    dot = 0.0
                    for f in range(lo, lo + dh):
                        dot += q[i][f] * k[j][f]
                    dots.append(alpha * dot)
                if softmax:
                    total = sum(math.exp(t) for t in dots)
                    wts = [math.exp(t) / total for t in dots]
                else:
                    wts = [_silu(t) / n_i for t in dots]
                for j, a in zip(keys, wts):
                    for f in range(lo, lo + dh):
                        o[f] += a * v[j][f]
            y = _layer_norm(o, lw["ln_at_g"], lw["ln_at_b"], eps)
            y = [y[f] * u[i][f] for f in range(d)]
            delta = _affine(y, lw["w2"], lw["b2"])
            new_x.append([x[i][f] + delta[f] for f in range(d)])
        x = new_x

    scores = []
    for c in range(first_cand, N):
        z = _layer_norm(x[c], weights["ln_out_g"], weights["ln_out_b"], eps)
        scores.append(sum(z[f] * float(weights["w_score"][f]) for f in range(d)) + float(weights["b_score"]))
    return scores
