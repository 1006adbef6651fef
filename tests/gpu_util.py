"""Helpers shared by the GPU parity tests: drive the C ABI on seeded inputs and compare with the
CPU oracle user by user.  (The oracle is imported here, in test code only.)"""
from __future__ import annotations

import dataclasses

import numpy as np
import torch

import oracle
import paper_2601_01712_amd as rg
import synth
from synth.generator import user_slices

# max-abs error relative to max(1, max|reference|).  fp32 and bf16: the stated targets.  fp16 has three more
# mantissa bits than bf16 (unit roundoff 2^-11 against 2^-8), so its bound is the bf16 one divided by 8.
TOL = {"fp32": 1e-4, "bf16": 2e-2, "fp16": 2.5e-3}


def make_workload(name, cfg: synth.ModelConfig, seed: int, n_users: int) -> synth.Workload:
    return synth.Workload(name, cfg, seed=seed, n_users=n_users, prefix_len=1, n_cands=1, n_suffix=0)


def oracle_scores(cfg, weights, batch, users=None) -> dict:
    """user -> float64 scores by full recompute on the CPU."""
    out = {}
    for u in (range(batch["n_users"]) if users is None else users):
        p, s, c = user_slices(batch, u)
        out[u] = oracle.full_recompute(cfg, weights, p, s, c)
    return out


def assert_close(got: np.ndarray, want: np.ndarray, dtype: str, what: str = ""):
    assert got.shape == want.shape, (what, got.shape, want.shape)
    if want.size == 0:
        return 0.0
    assert np.isfinite(got).all(), f"{what}: non-finite scores"
    err = float(np.abs(got.astype(np.float64) - want).max())
    bound = TOL[dtype] * max(1.0, float(np.abs(want).max()))
    assert err <= bound, f"{what}: max abs error {err:.3e} > {bound:.3e}"
    return err


class Harness:
    """One model + pool on cuda:0, sized for a given batch."""

    def __init__(self, cfg: synth.ModelConfig, weights: dict, batch: dict, page_tokens: int = 64, pool_extra_pages: int = 4):
        self.cfg, self.weights, self.batch = cfg, weights, batch
        n = batch["n_users"]
        L = np.diff(batch["prefix_off"]).astype(np.int64)
        new = int(batch["suffix_off"][-1]) + int(batch["cand_off"][-1])
        self.ctx = rg.Context(cfg, weights, max(1, n), int(L.sum()), new)
        ccfg = self.ctx.cfg
        pages = int(sum((int(l) + page_tokens - 1) // page_tokens for l in L)) + pool_extra_pages
        page_bytes = rg.relaygr_kv_pool_bytes_for(ccfg, page_tokens, page_tokens)
        self.pool = rg.KvPool(ccfg, cfg.dtype, max(1, pages) * page_bytes, page_tokens)
        # poison the slab so that a kernel reading a slot nobody wrote is noticed
        self.pool.slab.view(torch.int16).fill_(0x7FC1 if cfg.dtype != "fp32" else -1)   # a NaN in bf16 and in fp16
        self.dbatch = rg.Batch(batch, cfg.dtype)
        self.handles = np.zeros(n, dtype=np.uint64)

    def prefill(self, users=None):
        """Allocates pool entries for the given users (default: all with L > 0) and pre-infers them."""
        b = self.batch
        L = np.diff(b["prefix_off"])
        users = [u for u in range(b["n_users"]) if L[u] > 0] if users is None else list(users)
        for u in users:
            self.handles[u] = rg.relaygr_kv_pool_alloc(self.pool, int(b["user_ids"][u]), int(L[u]))
        sub = self.sub_batch(users)
        sub.set_handles([self.handles[u] for u in users])
        rg.relaygr_prefill_prefix(self.ctx, self.pool, sub)
        torch.cuda.synchronize()

    def sub_batch(self, users) -> rg.Batch:
        """A batch holding only the listed users (embeddings re-concatenated on the host)."""
        b = self.batch
        segs = {"prefix": [], "suffix": [], "cand": []}
        for u in users:
            p, s, c = user_slices(b, u)
            segs["prefix"].append(p); segs["suffix"].append(s); segs["cand"].append(c)
        d = self.cfg.d_model

        def cat(lst):
            return np.concatenate(lst, axis=0) if lst else np.zeros((0, d), np.float32)

        def off(lst):
            return np.concatenate([[0], np.cumsum([len(x) for x in lst])]).astype(np.int32)
        nb = {"n_users": len(users), "user_ids": np.asarray([b["user_ids"][u] for u in users], dtype=np.uint64),
              "prefix_emb": cat(segs["prefix"]), "prefix_off": off(segs["prefix"]),
              "suffix_emb": cat(segs["suffix"]), "suffix_off": off(segs["suffix"]),
              "cand_emb": cat(segs["cand"]), "cand_off": off(segs["cand"])}
        return rg.Batch(nb, self.cfg.dtype)

    def rank_cached(self) -> np.ndarray:
        self.dbatch.set_handles(self.handles)
        s = rg.relaygr_rank_with_cache(self.ctx, self.pool, self.dbatch)
        torch.cuda.synchronize()
        return s.cpu().numpy()

    def rank_full(self) -> np.ndarray:
        s = rg.relaygr_rank_full_recompute(self.ctx, self.dbatch)
        torch.cuda.synchronize()
        return s.cpu().numpy()

    def check(self, scores: np.ndarray, want: dict, what: str) -> float:
        co = self.batch["cand_off"]
        worst = 0.0
        for u, w in want.items():
            worst = max(worst, assert_close(scores[co[u]:co[u + 1]], w, self.cfg.dtype, f"{what} user {u}"))
        return worst

    def close(self):
        self.ctx.close()
        self.pool.close()


def store(x: np.ndarray, dtype: str) -> np.ndarray:
    """x rounded once to the storage type, returned as float32."""
    if dtype == "bf16":
        return synth.round_to_bf16(x.astype(np.float32))
    if dtype == "fp16":
        return x.astype(np.float16).astype(np.float32)
    return x.astype(np.float32)


# With the benchmark's N(0, 0.02^2) weights the attention output reaches the scores only through two small
# matrices: measured on the oracle, an attention that loses a whole key tile out of ten moves the scores by
# 5e-5, far inside every tolerance.  Boosting q/k rows 4x and u/v rows, W2 and the score head 5x makes the same
# mistake move them by 0.56 (ten times the bf16 bound) while plain bf16 rounding of the projections stays
# at 7e-3; the boosted cases are the ones that hold the attention kernels to the tolerance.
BOOST = (4.0, 5.0, 5.0, 5.0)


def boost_weights(weights: dict, cfg: synth.ModelConfig, factors=BOOST) -> dict:
    bqk, buv, b2, bs = factors
    d = cfg.d_model
    for lw in weights["layers"]:
        w1 = lw["w1"].copy()
        w1[2 * d:4 * d] *= bqk
        w1[:2 * d] *= buv
        lw["w1"] = store(w1, cfg.dtype)
        lw["w2"] = store(lw["w2"] * b2, cfg.dtype)
    weights["w_score"] = store(weights["w_score"] * bs, cfg.dtype)
    return weights


def build_case(cfg: synth.ModelConfig, seed: int, L, S, M, emb_std: float = 0.02, boost=None):
    wl = make_workload("case", cfg, seed, len(L))
    cached = np.ones(len(L), dtype=bool)
    batch = synth.make_batch(wl, 0, lengths=(L, S, M, cached), emb_std=emb_std)
    weights = synth.make_weights(cfg, seed)
    if boost is not None:
        boost_weights(weights, cfg, boost)
    return weights, batch
