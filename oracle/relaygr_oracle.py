"""Plain float64 CPU evaluation of the ranking model.  TEST INFRASTRUCTURE ONLY.

This is the slow, obviously-correct definition the HIP path is compared with.
It is imported only by tests, the smoke check and the benchmark's cpu_baseline
leg; it shares no code with the HIP path.

What the paper fixes (Section 2.3, the relay-race identity, and Section 3.1,
"Cache object"): the model f scores candidate items from the sequence
[long-term prefix | short-term / cross tokens | candidates]; psi is the
per-layer K/V of the backbone over the long-term prefix, a deterministic
function of the prefix tokens and the weights that does not depend on the
candidates; and f evaluated on the incremental tokens with psi must equal f
evaluated on the whole sequence up to a small deviation.  Section 4.1 ("Models
and workloads", "Cache semantics") names the backbone family (HSTU-style) and
fixes the cache as one K and one V of width d per layer and token.

The paper never prints the layer equations.  The reading used here, for one
user with sequence X = [p_0..p_{L-1} | s_0..s_{S-1} | c_0..c_{M-1}], N = L+S+M:

  visibility  m_ij = 1  iff  j <= i  and  (j < L+S  or  j == i)
              (causal over prefix and suffix; a candidate sees the whole prefix,
               the whole suffix and itself, never another candidate)
              n_i = sum_j m_ij
  per layer   xh_i            = LN(x_i; g_in, b_in)
              [u|v|q|k]_i     = SiLU(xh_i W1^T + b1)          (four blocks of width d)
              a_ij^h          = m_ij SiLU(alpha <q_i^h, k_j^h>) / n_i,  alpha = 1/sqrt(d_head)
              o_i^h           = sum_j a_ij^h v_j^h
              y_i             = LN(o_i; g_at, b_at) * u_i
              x_i            <- x_i + y_i W2^T + b2
  head        score_c         = <w_s, LN(x_c; g_out, b_out)> + b_s   for candidate rows

  LN(z) = (z - mean z) / sqrt(var z + eps) * g + b  with the biased variance
  over the d features; SiLU(t) = t / (1 + exp(-t)).

Under this mask row i < L of every layer depends on p_0..p_i only, so the
prefix K/V are candidate-independent and the identity holds with zero deviation
in exact arithmetic.

Second attention form.  Section 4.4 evaluates a variant of the backbone that
differs from the first only in how attention is computed and gives no formula
for it.  The reading used here (cfg.attention == "softmax") replaces the
pointwise activation and the 1/n_i by a softmax over the visible keys,

              a_ij^h          = m_ij exp(alpha <q_i^h, k_j^h>) / sum_j' m_ij' exp(alpha <q_i^h, k_j'^h>)

with everything else (projections, mask, gate, residual, head, and therefore
the cached K/V) unchanged.  The mask alone makes psi candidate-independent, so
the relay-race identity holds for this form too.

All arithmetic is float64 with no intermediate rounding; inputs arrive already
rounded to their storage type by the input generator.
"""
from __future__ import annotations

import math
from typing import List, Sequence, Tuple

import numpy as np
import torch

_F64 = torch.float64


def _t(a) -> torch.Tensor:
    if isinstance(a, torch.Tensor):
        return a.to(_F64)
    return torch.from_numpy(np.ascontiguousarray(a)).to(_F64)


def layer_norm(z: torch.Tensor, gain: torch.Tensor, offset: torch.Tensor, eps: float) -> torch.Tensor:
    """LayerNorm over the last axis with the biased variance (reading: three sites, eps 1e-5)."""
    mean = z.mean(dim=-1, keepdim=True)
    centred = z - mean
    var = (centred * centred).mean(dim=-1, keepdim=True)
    return centred / torch.sqrt(var + eps) * gain + offset


def silu(t: torch.Tensor) -> torch.Tensor:
    """SiLU(t) = t / (1 + exp(-t))."""
    return t / (1.0 + torch.exp(-t))


def visibility_mask(L: int, S: int, M: int) -> torch.Tensor:
    """Dense N x N mask m_ij of the sequence [prefix | suffix | candidates] (bool)."""
    N = L + S + M
    i = torch.arange(N).unsqueeze(1)
    j = torch.arange(N).unsqueeze(0)
    return (j <= i) & ((j < L + S) | (j == i))


def _project(x: torch.Tensor, lw: dict, eps: float, d: int):
    """Steps 1-2 of a layer: input LayerNorm and the four SiLU-activated projections."""
    xh = layer_norm(x, _t(lw["ln_in_g"]), _t(lw["ln_in_b"]), eps)
    z = silu(xh @ _t(lw["w1"]).T + _t(lw["b1"]))
    u, v, q, k = z[:, 0:d], z[:, d:2 * d], z[:, 2 * d:3 * d], z[:, 3 * d:4 * d]
    return u, v, q, k


def _attend(q, k_all, v_all, mask, n_heads: int, alpha: float) -> torch.Tensor:
    """Step 3: o_i^h = sum_j m_ij SiLU(alpha <q_i^h, k_j^h>) v_j^h / n_i, heads concatenated.

    q is [R, d] (the rows being evaluated); k_all, v_all are [J, d] (every key
    those rows may see); mask is [R, J] bool.
    """
    R, d = q.shape
    dh = d // n_heads
    n = mask.sum(dim=1, keepdim=True).to(_F64)
    mf = mask.to(_F64)
    o = torch.empty((R, d), dtype=_F64)
    for h in range(n_heads):
        c = slice(h * dh, (h + 1) * dh)
        a = silu(alpha * (q[:, c] @ k_all[:, c].T)) * mf / n
        o[:, c] = a @ v_all[:, c]
    return o


def _attend_softmax(q, k_all, v_all, mask, n_heads: int, alpha: float) -> torch.Tensor:
    """Step 3 in the second form: o_i^h = sum_j softmax_j(alpha <q_i^h, k_j^h> over visible j) v_j^h.

    Same arguments as _attend.  Every row must see at least one key (each token
    sees itself under the visibility rule).
    """
    R, d = q.shape
    dh = d // n_heads
    o = torch.empty((R, d), dtype=_F64)
    for h in range(n_heads):
        c = slice(h * dh, (h + 1) * dh)
        s = alpha * (q[:, c] @ k_all[:, c].T)
        s = torch.where(mask, s, torch.full_like(s, -math.inf))
        e = torch.exp(s - s.max(dim=1, keepdim=True).values)     # invisible keys: exp(-inf) = 0
        o[:, c] = (e / e.sum(dim=1, keepdim=True)) @ v_all[:, c]
    return o


def _attention_of(cfg):
    form = getattr(cfg, "attention", "silu")
    if form not in ("silu", "softmax"):
        raise ValueError(f"unknown attention form {form!r}")
    return form


def _finish_layer(x, o, u, lw: dict, eps: float) -> torch.Tensor:
    """Step 4: gated, normalised attention output through W2, plus the residual."""
    y = layer_norm(o, _t(lw["ln_at_g"]), _t(lw["ln_at_b"]), eps) * u
    return x + y @ _t(lw["w2"]).T + _t(lw["b2"])


def backbone_layer(x: torch.Tensor, lw: dict, mask: torch.Tensor, n_heads: int, alpha: float, eps: float,
                   form: str = "silu"):
    """One layer over a whole sequence; returns (new x, k, v)."""
    d = x.shape[1]
    u, v, q, k = _project(x, lw, eps, d)
    o = (_attend_softmax if form == "softmax" else _attend)(q, k, v, mask, n_heads, alpha)
    return _finish_layer(x, o, u, lw, eps), k, v


def score_head(x_c: torch.Tensor, weights: dict, eps: float) -> torch.Tensor:
    """score_c = <w_s, LN(x_c; g_out, b_out)> + b_s."""
    z = layer_norm(x_c, _t(weights["ln_out_g"]), _t(weights["ln_out_b"]), eps)
    return z @ _t(weights["w_score"]) + float(weights["b_score"])


def full_recompute(cfg, weights: dict, prefix, suffix, cands) -> np.ndarray:
    """Scores of one user's candidates by full inference over the whole sequence, no cache.

    cfg needs n_layers, n_heads, d_model, ln_eps.  prefix [L,d], suffix [S,d],
    cands [M,d] (any of L, S may be 0).  Returns float64 [M].
    """
    d = cfg.d_model
    prefix, suffix, cands = _t(prefix).reshape(-1, d), _t(suffix).reshape(-1, d), _t(cands).reshape(-1, d)
    L, S, M = prefix.shape[0], suffix.shape[0], cands.shape[0]
    x = torch.cat([prefix, suffix, cands], dim=0)
    mask = visibility_mask(L, S, M)
    alpha = 1.0 / math.sqrt(d // cfg.n_heads)
    form = _attention_of(cfg)
    for lw in weights["layers"]:
        x, _, _ = backbone_layer(x, lw, mask, cfg.n_heads, alpha, cfg.ln_eps, form)
    return score_head(x[L + S:], weights, cfg.ln_eps).numpy()


def prefix_kv(cfg, weights: dict, prefix) -> List[Tuple[torch.Tensor, torch.Tensor]]:
    """psi: per-layer (K [L,d], V [L,d]) of the backbone run over the prefix alone (Section 3.1)."""
    d = cfg.d_model
    x = _t(prefix).reshape(-1, d)
    L = x.shape[0]
    mask = visibility_mask(L, 0, 0)
    alpha = 1.0 / math.sqrt(d // cfg.n_heads)
    psi = []
    form = _attention_of(cfg)
    for lw in weights["layers"]:
        x, k, v = backbone_layer(x, lw, mask, cfg.n_heads, alpha, cfg.ln_eps, form)
        psi.append((k, v))
    return psi


def rank_with_kv(cfg, weights: dict, psi: Sequence[Tuple[torch.Tensor, torch.Tensor]], suffix, cands) -> np.ndarray:
    """Scores from the incremental tokens only, reading the prefix K/V from psi.

    The second leg of the relay-race identity (Section 2.3): rows are
    [suffix | candidates]; keys are [cached prefix | suffix | candidates] under
    the same visibility rule as full inference.
    """
    d = cfg.d_model
    suffix, cands = _t(suffix).reshape(-1, d), _t(cands).reshape(-1, d)
    S, M = suffix.shape[0], cands.shape[0]
    L = psi[0][0].shape[0] if len(psi) else 0
    x = torch.cat([suffix, cands], dim=0)
    mask = visibility_mask(L, S, M)[L:, :]
    alpha = 1.0 / math.sqrt(d // cfg.n_heads)
    form = _attention_of(cfg)
    for lw, (kp, vp) in zip(weights["layers"], psi):
        u, v, q, k = _project(x, lw, cfg.ln_eps, d)
        o = (_attend_softmax if form == "softmax" else _attend)(
            q, torch.cat([kp, k], dim=0), torch.cat([vp, v], dim=0), mask, cfg.n_heads, alpha)
        x = _finish_layer(x, o, u, lw, cfg.ln_eps)
    return score_head(x[S:], weights, cfg.ln_eps).numpy()


def kv_footprint_bytes(n_layers: int, prefix_len: int, d_model: int, elem_bytes: int) -> int:
    """Bytes of psi for one user: K and V, every layer, every prefix token (Section 4.1, Table 'KV caches')."""
    return 2 * n_layers * prefix_len * d_model * elem_bytes
