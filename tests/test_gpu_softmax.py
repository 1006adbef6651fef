"""GPU parity for the second attention form (softmax over the visible keys; the backbone variant
of the paper's Section 4.4, whose formula the paper does not give): the HIP path, called through the
C ABI with relaygr_ctx_set_attention(RELAYGR_ATTN_SOFTMAX), against the CPU oracle on the same seeded
inputs, to the same tolerances as the first form (1e-4 fp32, 2e-2 bf16, 2.5e-3 fp16 of
max(1, max|oracle|)).  Cases span several key tiles, row tiles and key splits, ragged tails, suffixes,
empty prefixes and batches mixing cached and uncached users; one case makes the scores grow along
the sequence so that the kernels' running reference maximum has to move after partial sums exist.
"""
import dataclasses
import math

import numpy as np
import pytest
import torch

import paper_2601_01712_amd as rg
import synth
from gpu_util import Harness, assert_close, build_case, oracle_scores, store, TOL
from oracle import relaygr_oracle as ro
from test_gpu_parity import run_three_routes

pytestmark = pytest.mark.gpu


def sm(n_layers, d, heads, dtype):
    return synth.ModelConfig(n_layers, d, heads, dtype, attention="softmax")


@pytest.mark.parametrize("L,S,M", [
    ([1], [0], [1]), ([63], [0], [5]), ([64], [3], [70]), ([65, 130], [0, 7], [3, 64]), ([200, 0, 77], [66, 2, 0], [65, 9, 129]),
])
def test_fp32_small_shapes(L, S, M):
    run_three_routes(sm(2, 64, 2, "fp32"), 340 + len(L), L, S, M)


@pytest.mark.parametrize("L,S,M", [
    ([1], [0], [1]), ([63], [0], [5]), ([64], [3], [130]), ([65, 300], [0, 70], [3, 129]),
    ([513, 0, 128], [64, 2, 0], [257, 9, 1]), ([1000], [17], [400]),
])
def test_bf16_small_shapes(L, S, M):
    run_three_routes(sm(3, 128, 2, "bf16"), 360 + len(L), L, S, M)


@pytest.mark.parametrize("L,S,M", [([1], [0], [1]), ([65, 300], [0, 70], [3, 129]), ([1000], [17], [400])])
def test_fp16_small_shapes(L, S, M):
    run_three_routes(sm(3, 128, 2, "fp16"), 460 + len(L), L, S, M)


@pytest.mark.parametrize("d,H,dtype", [(128, 4, "bf16"), (256, 2, "bf16"), (256, 4, "bf16"), (512, 8, "bf16"), (1024, 8, "bf16"),
                                       (512, 8, "fp16"), (128, 2, "fp32"), (128, 1, "fp32")])
def test_head_sizes(d, H, dtype):
    run_three_routes(sm(2, d, H, dtype), 370 + H, [300, 129], [5, 0], [140, 66])


@pytest.mark.parametrize("dtype", ["bf16", "fp16", "fp32"])
def test_mixed_hits_and_misses_in_one_batch(dtype):
    run_three_routes(sm(3, 256, 4, dtype), 381, [400, 130, 64, 700, 257], [0, 30, 64, 3, 0], [200, 50, 129, 7, 300],
                     page_tokens=128, miss=(1, 3))


def test_forms_can_be_switched_on_one_context():
    """The setter takes effect for later calls; switching back restores the first form's scores."""
    cfg = synth.ModelConfig(2, 128, 2, "bf16")
    weights, batch = build_case(cfg, 391, [200], [3], [70])
    want_silu = oracle_scores(cfg, weights, batch)
    want_soft = oracle_scores(dataclasses.replace(cfg, attention="softmax"), weights, batch)
    h = Harness(cfg, weights, batch)
    try:
        first = h.rank_full()
        h.check(first, want_silu, "silu")
        rg.relaygr_ctx_set_attention(h.ctx, "softmax")
        h.check(h.rank_full(), want_soft, "softmax")
        rg.relaygr_ctx_set_attention(h.ctx, "silu")
        assert np.array_equal(h.rank_full(), first)
        with pytest.raises(rg.RelayGRError):
            rg.relaygr_ctx_set_attention(h.ctx, "other")
    finally:
        h.close()


@pytest.mark.parametrize("dtype", ["bf16", "fp16", "fp32"])
def test_reference_maximum_moves_along_the_sequence(dtype):
    """Two blocks of near-identical prefix tokens, the second the negative of the first, and boosted
    q/k projections: for a third of the (row, head) pairs the later block scores far above the earlier
    one, so the running maximum has to rise (and sums already gathered have to be rescaled) many tiles
    into the key loop -- in the candidate pass, in the causal prefix pass, and across key splits.
    The other weights are boosted too, so that an attention output that lost or mis-scaled the later
    block would move the scores by about 70 times the tolerance (measured on the oracle)."""
    d, H, L, S, M = 128, 2, 640, 5, 140
    cfg = sm(2, d, H, dtype)
    weights, batch = build_case(cfg, 395, [L], [S], [M], emb_std=1.0)
    for lw in weights["layers"]:
        w1 = lw["w1"].copy()
        w1[2 * d:4 * d] *= 14.0          # q and k rows
        w1[:2 * d] *= 5.0                # u and v rows
        lw["w1"] = store(w1, dtype)
        lw["w2"] = store(lw["w2"] * 5.0, dtype)
    weights["w_score"] = store(weights["w_score"] * 5.0, dtype)
    a = synth.normal(395, "a", d)
    noise = synth.normal(395, "n", L * d).reshape(L, d) * 0.1
    emb = np.where(np.arange(L)[:, None] < 256, a[None, :], -a[None, :]) + noise
    batch["prefix_emb"] = store(emb, dtype)

    # the case does what it says: in layer 1 many (candidate, head) pairs find their best key
    # more than 8 binary orders of magnitude above the best key of the first 32
    x = torch.from_numpy(np.concatenate([batch["prefix_emb"], batch["suffix_emb"], batch["cand_emb"]])).double()
    _, _, q, k = ro._project(x, weights["layers"][0], cfg.ln_eps, d)
    moved = 0
    for hd in range(H):
        c = slice(hd * (d // H), (hd + 1) * (d // H))
        s = (q[L + S:, c] @ k[:L, c].T) / math.sqrt(d // H) / math.log(2.0)
        moved += int(((s.max(dim=1).values - s[:, :32].max(dim=1).values) > 8.0).sum())
    assert moved > 0.2 * M * H, moved

    want = oracle_scores(cfg, weights, batch)
    h = Harness(cfg, weights, batch)
    try:
        h.prefill()
        e1 = h.check(h.rank_cached(), want, "rank_with_cache")
        e2 = h.check(h.rank_full(), want, "rank_full_recompute")
        print(f"\n  {dtype}: {moved} of {M * H} (candidate, head) pairs move their maximum late; max err cached {e1:.2e} "
              f"full {e2:.2e} (tolerance {TOL[dtype]:.1e} of max(1, max|oracle|))", flush=True)
    finally:
        h.close()


def test_pool_contents_do_not_depend_on_the_form_in_layer_one_only():
    """K and V of the first layer are projections of the embeddings alone, so both forms write the
    same first-layer tiles; from the second layer on the inputs differ and so must the tiles."""
    cfg = synth.ModelConfig(2, 128, 2, "bf16")
    weights, batch = build_case(cfg, 397, [130], [0], [4])
    slabs = []
    for form in ("silu", "softmax"):
        h = Harness(dataclasses.replace(cfg, attention=form), weights, batch)
        try:
            h.prefill()
            idx = [[rg.relaygr_kv_pool_locate(h.pool, int(h.handles[0]), layer, t, f)[0] for t in (0, 64, 129) for f in (0, 77)]
                   for layer in (0, 1)]
            flat = h.pool.slab.view(torch.int16).cpu().numpy()
            slabs.append([flat[np.asarray(ix)] for ix in idx])
        finally:
            h.close()
    assert np.array_equal(slabs[0][0], slabs[1][0])
    assert not np.array_equal(slabs[0][1], slabs[1][1])
