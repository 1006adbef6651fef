"""Counter-based seeded generator of model weights and ranking batches.

Every value is a pure function of (seed, tensor tag, element index), so a
tensor can be regenerated anywhere, in any order, on any backend:

    bits(seed, tag, i) = splitmix64_finalise(key(seed, tag) + (i + 1) * GOLDEN)
    normal             = Box-Muller over two such 53-bit uniforms

Values are rounded ONCE to the workload's storage type (bf16 by
round-to-nearest-even, or fp32) and returned as float32 arrays holding exactly
representable values, so the CPU oracle and the GPU path consume identical
numbers.  Nothing in this module evaluates any part of the model.

Workload shapes follow the paper's evaluation ranges (Section 4.1, "Models and
workloads": lengths from 1K to tens of thousands of tokens, widths 128-1024,
several to tens of layers; Section 4.4: about 512 candidates per query, up to
2048) and the five benchmark configurations this repository is measured on.
"""
from __future__ import annotations

import dataclasses
import math
import os
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, List, Optional

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 22  # elements generated per pass (bounds temporary memory)


def _mix(z: np.ndarray) -> np.ndarray:
    """splitmix64 output function on a uint64 array (wrapping arithmetic)."""
    z = z.copy()
    z ^= z >> np.uint64(30)
    z *= _M1
    z ^= z >> np.uint64(27)
    z *= _M2
    z ^= z >> np.uint64(31)
    return z


def _tag_key(seed: int, tag: str) -> np.uint64:
    """64-bit stream key from an integer seed and a tensor tag (FNV-1a, then mixed)."""
    h = 0xCBF29CE484222325
    for b in tag.encode("utf-8"):
        h = ((h ^ b) * 0x100000001B3) & 0xFFFFFFFFFFFFFFFF
    h = (h ^ ((seed & 0xFFFFFFFFFFFFFFFF) * 0x9E3779B97F4A7C15)) & 0xFFFFFFFFFFFFFFFF
    return _mix(np.array([h], dtype=np.uint64))[0]


def _bits(key: np.uint64, start: int, count: int, lane: int) -> np.ndarray:
    """Raw 64-bit words for counters start..start+count-1 of sub-stream `lane` (0 or 1)."""
    idx = np.arange(start, start + count, dtype=np.uint64)
    with np.errstate(over="ignore"):
        ctr = (idx * np.uint64(2) + np.uint64(lane + 1)) * _GOLDEN + key
        return _mix(ctr)


def _uniform01(key: np.uint64, start: int, count: int, lane: int) -> np.ndarray:
    """Uniform doubles in the open interval (0, 1) with 53 random bits."""
    r = _bits(key, start, count, lane) >> np.uint64(11)
    return (r.astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def normal(seed: int, tag: str, n: int, mean: float = 0.0, std: float = 1.0) -> np.ndarray:
    """n draws of N(mean, std^2) as float64, element i depending only on (seed, tag, i)."""
    key = _tag_key(seed, tag)
    out = np.empty(n, dtype=np.float64)

    def fill(s):
        c = min(_CHUNK, n - s)
        u1 = _uniform01(key, s, c, 0)
        u2 = _uniform01(key, s, c, 1)
        out[s:s + c] = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * math.pi * u2)

    starts = range(0, n, _CHUNK)
    if len(starts) > 2:
        # element i depends on (seed, tag, i) only, so chunks can be filled in any order: a few threads
        # (numpy releases the interpreter lock) cut the generation time of the large workloads
        with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
            list(pool.map(fill, starts))
    else:
        for s in starts:
            fill(s)
    out *= std
    out += mean
    return out


def uniform_int(seed: int, tag: str, n: int, lo: int, hi: int) -> np.ndarray:
    """n integers uniform in [lo, hi] (inclusive) as int64."""
    key = _tag_key(seed, tag)
    u = _uniform01(key, 0, n, 0)
    return (lo + np.floor(u * (hi - lo + 1))).astype(np.int64).clip(lo, hi)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float values to the nearest bfloat16 (ties to even); returns float32."""
    f = np.ascontiguousarray(x, dtype=np.float32)
    b = f.view(np.uint32)
    with np.errstate(over="ignore"):
        rounded = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32).reshape(f.shape)


def _store(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return round_to_bf16(x)
    if dtype == "fp16":
        return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16).astype(np.float32)   # round to nearest even
    if dtype == "fp32":
        return np.ascontiguousarray(x, dtype=np.float32)
    raise ValueError(f"unknown storage dtype {dtype!r}")


# ----------------------------------------------------------------------------
# shapes
# ----------------------------------------------------------------------------

@dataclasses.dataclass(frozen=True)
class ModelConfig:
    n_layers: int
    d_model: int
    n_heads: int
    dtype: str  # "fp32", "bf16" or "fp16": storage type of weights, embeddings and cached K/V
    ln_eps: float = 1e-5
    attention: str = "silu"  # "silu": pointwise SiLU attention; "softmax": the second attention form

    @property
    def d_head(self) -> int:
        return self.d_model // self.n_heads

    @property
    def qk_scale(self) -> float:
        return 1.0 / math.sqrt(self.d_head)

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "fp32" else 2


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    model: ModelConfig
    seed: int
    n_users: int
    prefix_len: Optional[int]        # fixed prefix length, or None for the jagged recipe
    n_cands: Optional[int]           # fixed candidate count, or None for U{200..2000}
    n_suffix: Optional[int]          # fixed suffix length, or None for U{0..64}
    miss_tenths: int = 0             # users whose hash mod 10 < miss_tenths have no cached prefix
    prefix_clip: tuple = (512, 16384)
    prefix_median: int = 4096
    prefix_sigma: float = 0.7
    cand_range: tuple = (200, 2000)
    suffix_range: tuple = (0, 64)


WORKLOADS: Dict[str, Workload] = {
    "C1": Workload("C1", ModelConfig(2, 64, 2, "fp32"), seed=0, n_users=1,
                   prefix_len=256, n_cands=16, n_suffix=0),
    "C2": Workload("C2", ModelConfig(4, 256, 4, "bf16"), seed=2, n_users=8,
                   prefix_len=2048, n_cands=256, n_suffix=16),
    "C3": Workload("C3", ModelConfig(8, 512, 8, "bf16"), seed=3, n_users=16,
                   prefix_len=4096, n_cands=512, n_suffix=0),
    "C4": Workload("C4", ModelConfig(8, 512, 8, "bf16"), seed=4, n_users=32,
                   prefix_len=8192, n_cands=1000, n_suffix=0),
    "C5": Workload("C5", ModelConfig(8, 512, 8, "bf16"), seed=5, n_users=64,
                   prefix_len=None, n_cands=None, n_suffix=None, miss_tenths=3),
    # the paper's extensibility axes (Section 4.4): embedding width up to 1024, depth 8 -> 16 layers
    "X1": Workload("X1", ModelConfig(8, 1024, 8, "bf16"), seed=6, n_users=16,
                   prefix_len=4096, n_cands=512, n_suffix=0),
    "X2": Workload("X2", ModelConfig(16, 512, 8, "bf16"), seed=7, n_users=16,
                   prefix_len=4096, n_cands=512, n_suffix=0),
    # the half precision the paper mentions as lowering the rank stage (Section 4.2): C3 in IEEE fp16
    "X3": Workload("X3", ModelConfig(8, 512, 8, "fp16"), seed=8, n_users=16,
                   prefix_len=4096, n_cands=512, n_suffix=0),
    # the backbone variant that differs only in its attention computation (Section 4.4): C3 with
    # softmax attention over the visible keys
    "X4": Workload("X4", ModelConfig(8, 512, 8, "bf16", attention="softmax"), seed=9, n_users=16,
                   prefix_len=4096, n_cands=512, n_suffix=0),
}


def make_lengths(wl: Workload, batch_index: int = 0):
    """Per-user (prefix L, suffix S, candidates M, cached?) for one batch of a workload.

    Fixed-shape workloads repeat their shape for every user.  The jagged recipe
    draws L = clip(round(exp(N(ln median, sigma^2)))), M ~ U{cand_range},
    S ~ U{suffix_range}; a user is uncached when hash(seed, user) mod 10 < miss_tenths.
    """
    n = wl.n_users
    seed = wl.seed + 1000003 * batch_index
    if wl.prefix_len is not None:
        L = np.full(n, wl.prefix_len, dtype=np.int64)
    else:
        z = normal(seed, "prefix_len", n, math.log(wl.prefix_median), wl.prefix_sigma)
        L = np.clip(np.rint(np.exp(z)), wl.prefix_clip[0], wl.prefix_clip[1]).astype(np.int64)
    if wl.n_cands is not None:
        M = np.full(n, wl.n_cands, dtype=np.int64)
    else:
        M = uniform_int(seed, "n_cands", n, wl.cand_range[0], wl.cand_range[1])
    if wl.n_suffix is not None:
        S = np.full(n, wl.n_suffix, dtype=np.int64)
    else:
        S = uniform_int(seed, "n_suffix", n, wl.suffix_range[0], wl.suffix_range[1])
    if wl.miss_tenths > 0:
        h = uniform_int(seed, "miss_hash", n, 0, 9)
        cached = h >= wl.miss_tenths
    else:
        cached = np.ones(n, dtype=bool)
    return L, S, M, cached


# ----------------------------------------------------------------------------
# tensors
# ----------------------------------------------------------------------------

_W_STD = 0.02


def make_weights(cfg: ModelConfig, seed: int) -> dict:
    """Random-initialised parameters, rounded to the storage type.

    Layout (all float32 arrays of storage-representable values):
      layers[l]: ln_in_g, ln_in_b [d]; w1 [4d, d] (output-major: y = x @ w1.T + b1,
                 output blocks in the order u | v | q | k); b1 [4d];
                 ln_at_g, ln_at_b [d]; w2 [d, d] (output-major); b2 [d]
      ln_out_g, ln_out_b, w_score [d]; b_score (python float)
    Matrices, biases, LayerNorm offsets and the score head are N(0, 0.02^2);
    LayerNorm gains are 1 + N(0, 0.02^2).
    """
    d = cfg.d_model
    dt = cfg.dtype

    def n(tag, shape, mean=0.0):
        cnt = int(np.prod(shape))
        return _store(normal(seed, tag, cnt, mean, _W_STD).reshape(shape), dt)

    layers = []
    for l in range(cfg.n_layers):
        p = f"layer{l}."
        layers.append({
            "ln_in_g": n(p + "ln_in_g", (d,), 1.0),
            "ln_in_b": n(p + "ln_in_b", (d,)),
            "w1": n(p + "w1", (4 * d, d)),
            "b1": n(p + "b1", (4 * d,)),
            "ln_at_g": n(p + "ln_at_g", (d,), 1.0),
            "ln_at_b": n(p + "ln_at_b", (d,)),
            "w2": n(p + "w2", (d, d)),
            "b2": n(p + "b2", (d,)),
        })
    return {
        "layers": layers,
        "ln_out_g": n("ln_out_g", (d,), 1.0),
        "ln_out_b": n("ln_out_b", (d,)),
        "w_score": n("w_score", (d,)),
        "b_score": float(_store(normal(seed, "b_score", 1, 0.0, _W_STD), dt)[0]),
    }


def make_embeddings(cfg: ModelConfig, seed: int, tag: str, rows: int, std: float = _W_STD) -> np.ndarray:
    """[rows, d] token embeddings ~ N(0, std^2), rounded to the storage type."""
    return _store(normal(seed, tag, rows * cfg.d_model, 0.0, std).reshape(rows, cfg.d_model), cfg.dtype)


def make_batch(wl: Workload, batch_index: int = 0, lengths=None, emb_std: float = _W_STD) -> dict:
    """One ranking batch: concatenated per-user embeddings with int32 offsets.

    Returns a dict with
      n_users, user_ids [n] uint64, cached [n] bool,
      prefix_emb [sum L, d], prefix_off [n+1] int32,
      suffix_emb [sum S, d], suffix_off [n+1] int32,
      cand_emb   [sum M, d], cand_off   [n+1] int32.
    `lengths` = (L, S, M, cached) overrides the workload's own shape recipe.
    """
    cfg = wl.model
    L, S, M, cached = lengths if lengths is not None else make_lengths(wl, batch_index)
    L = np.asarray(L, dtype=np.int64)
    S = np.asarray(S, dtype=np.int64)
    M = np.asarray(M, dtype=np.int64)
    n = len(L)
    seed = wl.seed + 1000003 * batch_index

    def off(x):
        o = np.zeros(n + 1, dtype=np.int64)
        np.cumsum(x, out=o[1:])
        assert o[-1] < 2**31
        return o.astype(np.int32)

    return {
        "n_users": n,
        "user_ids": (np.arange(n, dtype=np.uint64) + np.uint64(1000 * (batch_index + 1))),
        "cached": np.asarray(cached, dtype=bool),
        "prefix_emb": make_embeddings(cfg, seed, "prefix_emb", int(L.sum()), emb_std),
        "prefix_off": off(L),
        "suffix_emb": make_embeddings(cfg, seed, "suffix_emb", int(S.sum()), emb_std),
        "suffix_off": off(S),
        "cand_emb": make_embeddings(cfg, seed, "cand_emb", int(M.sum()), emb_std),
        "cand_off": off(M),
    }


def user_slices(batch: dict, u: int):
    """(prefix [L,d], suffix [S,d], cands [M,d]) views of user u of a batch."""
    po, so, co = batch["prefix_off"], batch["suffix_off"], batch["cand_off"]
    return (batch["prefix_emb"][po[u]:po[u + 1]],
            batch["suffix_emb"][so[u]:so[u + 1]],
            batch["cand_emb"][co[u]:co[u + 1]])
