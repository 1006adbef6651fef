"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Tolerance: max-abs error <= tol * max(1, max|oracle|), tol 1e-4 (fp32) / 2e-2 (bf16).

Small cases span several key tiles (64 tokens), several row tiles (64 rows fp32 / 128 rows bf16)
and ragged tails; the named benchmark shapes C1 and C2 run in full.  Each case checks the three
routes to the same scores: ranking on the cached prefix, full recompute, and (where stated) a
batch mixing cached and uncached users -- the paper's relay-race identity (Section 2.3) and miss
fallback (Section 3.1, invariant I1).
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2601_01712_amd as rg
import synth
from gpu_util import BOOST, Harness, assert_close, build_case, oracle_scores, TOL
from synth.generator import user_slices

pytestmark = pytest.mark.gpu


def run_three_routes(cfg, seed, L, S, M, page_tokens=64, miss=(), boost=None):
    weights, batch = build_case(cfg, seed, L, S, M, boost=boost)
    want = oracle_scores(cfg, weights, batch)
    h = Harness(cfg, weights, batch, page_tokens)
    try:
        hit = [u for u in range(len(L)) if L[u] > 0 and u not in miss]
        if hit:
            h.prefill(hit)
        e1 = h.check(h.rank_cached(), want, "rank_with_cache")
        e2 = h.check(h.rank_full(), want, "rank_full_recompute")
        print(f"\n  {cfg.dtype} d={cfg.d_model} H={cfg.n_heads} NL={cfg.n_layers} L={list(L)} S={list(S)} M={list(M)}: "
              f"max err cached {e1:.2e} full {e2:.2e} (tolerance {TOL[cfg.dtype]:.1e} of max(1, max|oracle|))", flush=True)
    finally:
        h.close()


# ------------------------------------------------- weights boosted so that attention reaches the scores
@pytest.mark.parametrize("dtype", ["fp32", "bf16", "fp16"])
@pytest.mark.parametrize("attention", ["silu", "softmax"])
@pytest.mark.parametrize("L,S,M", [([640], [5], [140]), ([65, 300, 0], [0, 70, 3], [3, 129, 40]), ([1000], [17], [400])])
def test_boosted_weights(dtype, attention, L, S, M):
    """Same shapes as the small cases with the boosted weights of gpu_util.BOOST: here a lost key tile, a
    wrong normaliser or a mis-scaled partial sum in the attention kernels exceeds the tolerance many times."""
    d, H = (64, 2) if dtype == "fp32" else (128, 2)
    run_three_routes(synth.ModelConfig(2, d, H, dtype, attention=attention), 500 + len(L), L, S, M, boost=BOOST)


@pytest.mark.parametrize("attention", ["silu", "softmax"])
@pytest.mark.parametrize("dtype", ["bf16", "fp16"])
def test_ragged_batch_on_256_row_work_items(dtype, attention):
    """Enough candidate rows (37 work items x 8 heads) that the MFMA attention kernel takes two row blocks per
    wavefront, the launch shape of the benchmark, here with ragged prefixes, suffixes and candidate counts
    and one uncached user.  At d = 512 the benchmark's own weight scale already lets a lost key tile move
    the scores by twenty times the tolerance (measured on the oracle)."""
    run_three_routes(synth.ModelConfig(2, 512, 8, dtype, attention=attention), 520,
                     [130, 300, 0, 64, 513, 77], [0, 70, 3, 0, 5, 64], [2000, 1500, 900, 1025, 1300, 1600],
                     page_tokens=128, miss=(4,))


# ------------------------------------------------------------------------------------ fp32
def test_c1_fp32_full():
    wl = synth.WORKLOADS["C1"]
    L, S, M, _ = synth.make_lengths(wl)
    run_three_routes(wl.model, wl.seed, L, S, M)


@pytest.mark.parametrize("L,S,M", [
    ([1], [0], [1]), ([63], [0], [5]), ([64], [3], [70]), ([65, 130], [0, 7], [3, 64]),
    ([200, 0, 77], [66, 2, 0], [65, 9, 129]),
])
def test_fp32_small_shapes(L, S, M):
    run_three_routes(synth.ModelConfig(2, 64, 2, "fp32"), 40 + len(L), L, S, M)


@pytest.mark.parametrize("d,H", [(128, 2), (128, 1), (256, 8)])
def test_fp32_head_sizes(d, H):
    run_three_routes(synth.ModelConfig(2, d, H, "fp32"), 50 + H, [150, 70], [5, 0], [20, 66])


# ------------------------------------------------------------------------------------ bf16
@pytest.mark.parametrize("L,S,M", [
    ([1], [0], [1]), ([63], [0], [5]), ([64], [3], [130]), ([65, 300], [0, 70], [3, 129]),
    ([513, 0, 128], [64, 2, 0], [257, 9, 1]), ([1000], [17], [400]),
])
def test_bf16_small_shapes(L, S, M):
    run_three_routes(synth.ModelConfig(3, 128, 2, "bf16"), 60 + len(L), L, S, M)


@pytest.mark.parametrize("d,H", [(128, 4), (256, 2), (256, 4), (512, 8), (1024, 8)])
def test_bf16_head_sizes(d, H):
    run_three_routes(synth.ModelConfig(2, d, H, "bf16"), 70 + H, [300, 129], [5, 0], [140, 66])


@pytest.mark.parametrize("dtype", ["bf16", "fp16"])
@pytest.mark.parametrize("d,H,boost", [(128, 2, BOOST), (256, 4, BOOST), (512, 8, None)])
def test_launches_of_thousands_of_rows_take_the_weight_stationary_projection(dtype, d, H, boost):
    """Row counts above 4096 per projection launch (the persistent, weight-stationary form of the u|v|q|k
    GEMM) with everything its epilogue has to place: prefix rows of three users with ragged last tiles and
    filler rows between them, K and V tiles of the pool (cached users) and of scratch (the uncached user),
    suffix rows scattered into suffix tiles, candidate rows, a last unit that ends inside a 64-row block;
    ranking on the cache runs the same launch over new rows only, full recompute over prefix and new rows
    in one row space.  Boosted weights at the small widths, so that a misplaced K/V element shows."""
    run_three_routes(synth.ModelConfig(2, d, H, dtype), 530 + d, [2500, 1300, 700], [70, 5, 0], [2100, 1900, 301],
                     page_tokens=128, miss=(1,), boost=boost)


@pytest.mark.parametrize("attention", ["silu", "softmax"])
@pytest.mark.parametrize("dtype", ["bf16", "fp16"])
@pytest.mark.parametrize("d,H,boost", [(256, 4, BOOST), (512, 8, None)])
def test_one_user_calls_take_the_eight_row_layer_tail(dtype, attention, d, H, boost):
    """One user per call: the key range is cut into 8 splits, and the layer tail of a launch of at most 1024
    rows runs with 8 rows per workgroup, every split of a row in flight at once; 342 new rows end inside an
    8-row group.  The full-recompute route of the same user (1442 rows) takes the 32-row tail."""
    cfg = synth.ModelConfig(2, d, H, dtype, attention=attention)
    run_three_routes(cfg, 810 + d, [1100], [9], [333], boost=boost)


@pytest.mark.parametrize("attention", ["silu", "softmax"])
@pytest.mark.parametrize("dtype", ["bf16", "fp16"])
def test_two_key_splits_added_inside_one_workgroup(dtype, attention):
    """32 work items of up to 256 rows x 8 heads of 64: ranking on the cache cuts the key range in two, and the two
    halves go to the two wavefront groups of ONE workgroup, which add their sums in LDS (in the softmax form after
    bringing them to a common reference score).  Prefix lengths give odd
    and even tile counts (the groups then walk different numbers of tiles), two users bring suffix tiles, the second
    work item of every user ends inside a row block."""
    L = [130, 200, 257, 320, 385, 450, 513, 577, 640, 705, 150, 330, 460, 590, 720, 260]
    S = [0, 0, 70, 0, 0, 0, 0, 3, 0, 0, 0, 0, 0, 0, 0, 0]
    M = [300, 300, 230, 300, 300, 300, 300, 297, 300, 300, 300, 300, 300, 300, 300, 300]
    assert sum((s + m + 255) // 256 for s, m in zip(S, M)) * 8 == 256      # the shape that selects that kernel
    run_three_routes(synth.ModelConfig(2, 512, 8, dtype, attention=attention), 611, L, S, M)


@pytest.mark.parametrize("attention", ["silu", "softmax"])
def test_four_key_splits_on_128_row_items_pair_up_inside_workgroups(attention):
    """One user with 2048 candidates: 16 work items of 128 rows x 8 heads and four key splits, which the two
    wavefront groups of a workgroup take in pairs (two partial sums reach the layer tail instead of four); 18
    key tiles over four splits leave the last group with fewer tiles than its partner."""
    run_three_routes(synth.ModelConfig(2, 512, 8, "bf16", attention=attention), 613, [1100], [0], [2048])


# ------------------------------------------------------------------------------------ fp16
@pytest.mark.parametrize("L,S,M", [
    ([1], [0], [1]), ([65, 300], [0, 70], [3, 129]), ([513, 0, 128], [64, 2, 0], [257, 9, 1]), ([1000], [17], [400]),
])
def test_fp16_small_shapes(L, S, M):
    run_three_routes(synth.ModelConfig(3, 128, 2, "fp16"), 160 + len(L), L, S, M)


@pytest.mark.parametrize("d,H", [(128, 4), (256, 2), (512, 8), (1024, 8)])
def test_fp16_head_sizes(d, H):
    run_three_routes(synth.ModelConfig(2, d, H, "fp16"), 170 + H, [300, 129], [5, 0], [140, 66])


def test_fp16_mixed_hits_and_misses_in_one_batch():
    cfg = synth.ModelConfig(3, 256, 4, "fp16")
    run_three_routes(cfg, 181, [400, 130, 64, 700, 257], [0, 30, 64, 3, 0], [200, 50, 129, 7, 300],
                     page_tokens=128, miss=(1, 3))


def test_bf16_mixed_hits_and_misses_in_one_batch():
    cfg = synth.ModelConfig(3, 256, 4, "bf16")
    run_three_routes(cfg, 81, [400, 130, 64, 700, 257], [0, 30, 64, 3, 0], [200, 50, 129, 7, 300],
                     page_tokens=128, miss=(1, 3))


def test_c2_bf16_full():
    wl = synth.WORKLOADS["C2"]
    L, S, M, _ = synth.make_lengths(wl)
    run_three_routes(wl.model, wl.seed, L, S, M, page_tokens=256)


# ------------------------------------------------------------------- psi, independence, determinism
@pytest.mark.parametrize("dtype", ["fp32", "bf16", "fp16"])
def test_pool_contents_equal_oracle_psi(dtype):
    """The cached object itself (Section 3.1): every layer's K and V of the prefix."""
    cfg = synth.ModelConfig(3, 128, 2, dtype)
    weights, batch = build_case(cfg, 91, [150, 64], [0, 0], [1, 1])
    h = Harness(cfg, weights, batch, page_tokens=64)
    try:
        h.prefill()
        el = h.pool.elements().float().cpu().numpy()
        for u in range(2):
            p, _, _ = user_slices(batch, u)
            psi = oracle.prefix_kv(cfg, weights, p)
            toks = sorted({0, 1, 62, 63, 64, len(p) - 1} & set(range(len(p))))
            for l, (k, v) in enumerate(psi):
                for t in toks:
                    idx = [rg.relaygr_kv_pool_locate(h.pool, int(h.handles[u]), l, t, f) for f in range(cfg.d_model)]
                    gk = el[[i[0] for i in idx]]
                    gv = el[[i[1] for i in idx]]
                    tol = {"fp32": 1e-5, "bf16": 1e-2, "fp16": 1.5e-3}[dtype]
                    np.testing.assert_allclose(gk, k[t].numpy(), rtol=tol, atol=tol * 0.3)
                    np.testing.assert_allclose(gv, v[t].numpy(), rtol=tol, atol=tol * 0.3)
    finally:
        h.close()


def test_prefill_is_deterministic_and_reranking_reuses_psi():
    cfg = synth.ModelConfig(2, 256, 4, "bf16")
    weights, batch = build_case(cfg, 93, [700, 300], [10, 0], [150, 40])
    h = Harness(cfg, weights, batch, page_tokens=128)
    try:
        h.prefill()
        snap = h.pool.slab.clone()
        a = h.rank_cached()
        b = h.rank_cached()
        assert np.array_equal(a, b), "same inputs, same cache: scores must be bit-identical"
        # pre-infer again into the same entries: the pool contents must not change by a bit
        sub = h.sub_batch([0, 1])
        sub.set_handles(h.handles)
        rg.relaygr_prefill_prefix(h.ctx, h.pool, sub)
        torch.cuda.synchronize()
        assert torch.equal(snap, h.pool.slab)
        # one cached prefix, a different candidate set (Section 3.1: psi does not depend on candidates)
        wl2 = synth.Workload("other", cfg, seed=94, n_users=2, prefix_len=1, n_cands=1, n_suffix=0)
        other = synth.make_batch(wl2, 0, lengths=([700, 300], [10, 0], [33, 90], np.ones(2, bool)))
        mixed = dict(batch)
        mixed["cand_emb"], mixed["cand_off"] = other["cand_emb"], other["cand_off"]
        want = oracle_scores(cfg, weights, mixed)
        db = rg.Batch(mixed, cfg.dtype, handles=h.handles)
        got = rg.relaygr_rank_with_cache(h.ctx, h.pool, db).cpu().numpy()
        for u in range(2):
            assert_close(got[mixed["cand_off"][u]:mixed["cand_off"][u + 1]], want[u], "bf16", f"new candidates user {u}")
    finally:
        h.close()


def test_candidates_and_users_are_independent_on_the_gpu():
    cfg = synth.ModelConfig(2, 128, 2, "bf16")
    weights, batch = build_case(cfg, 95, [200, 90], [4, 0], [70, 30])
    h = Harness(cfg, weights, batch)
    try:
        h.prefill()
        full = h.rank_cached()
        # user 1 alone, and user 0's candidates in reversed order
        only1 = h.sub_batch([1]); only1.set_handles([h.handles[1]])
        s1 = rg.relaygr_rank_with_cache(h.ctx, h.pool, only1).cpu().numpy()
        np.testing.assert_allclose(s1, full[70:], rtol=0, atol=1e-6)
        rev = dict(batch)
        ce = batch["cand_emb"].copy(); ce[:70] = ce[:70][::-1]
        rev["cand_emb"] = ce
        sr = rg.relaygr_rank_with_cache(h.ctx, h.pool, rg.Batch(rev, cfg.dtype, handles=h.handles)).cpu().numpy()
        np.testing.assert_allclose(sr[:70][::-1], full[:70], rtol=0, atol=2e-3)
    finally:
        h.close()


# ---------------------------------------------------------------------------- failure handling
def test_stale_handle_is_reported_and_fallback_gives_the_same_scores():
    """Section 3.3: when the cache is gone the instance falls back to inference without cache."""
    cfg = synth.ModelConfig(2, 128, 2, "bf16")
    weights, batch = build_case(cfg, 97, [130, 260], [0, 5], [20, 40])
    want = oracle_scores(cfg, weights, batch)
    h = Harness(cfg, weights, batch)
    try:
        h.prefill()
        stale = int(h.handles[0])
        rg.relaygr_kv_pool_free(h.pool, stale)
        with pytest.raises(rg.RelayGRError) as e:
            h.rank_cached()
        assert e.value.code == rg.RELAYGR_ENOENT
        assert rg.relaygr_kv_pool_lookup(h.pool, int(batch["user_ids"][0])) == rg.RELAYGR_NO_CACHE
        h.handles[0] = rg.RELAYGR_NO_CACHE          # the caller's fallback
        h.check(h.rank_cached(), want, "after fallback")
        # a pool that is full says so; ranking that user uncached still works
        with pytest.raises(rg.RelayGRError) as e:
            rg.relaygr_kv_pool_alloc(h.pool, 424242, 100000)
        assert e.value.code == rg.RELAYGR_ENOSPC
        # wrong prefix length for a live handle is an argument error
        bad = dict(batch); po = batch["prefix_off"].copy(); po[2] -= 1; bad["prefix_off"] = po
        with pytest.raises(rg.RelayGRError) as e:
            rg.relaygr_rank_with_cache(h.ctx, h.pool, rg.Batch(bad, cfg.dtype, handles=h.handles))
        assert e.value.code == rg.RELAYGR_EINVAL
    finally:
        h.close()


def test_scratch_too_small_is_an_error_not_a_fault():
    cfg = synth.ModelConfig(2, 128, 2, "bf16")
    weights, batch = build_case(cfg, 98, [6000], [0], [500])
    ctx = rg.Context(cfg, weights, 1, 64, 64)     # sized for a much smaller call
    try:
        with pytest.raises(rg.RelayGRError) as e:
            rg.relaygr_rank_full_recompute(ctx, rg.Batch(batch, cfg.dtype))
        assert e.value.code == rg.RELAYGR_ENOSPC
    finally:
        ctx.close()
