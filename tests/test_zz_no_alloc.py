"""relaygr_rank_with_cache_static, the entry point for callers that cannot allocate: same scores as
relaygr_rank_with_cache on two calls in a row (the second smaller, so that it runs over what the first
left in the library's scratch), an oversized call refused, and the oracle as the outside check."""
import numpy as np
import pytest
import torch

import paper_2601_01712_amd as rg
import synth
from gpu_util import Harness, assert_close, build_case, oracle_scores

pytestmark = pytest.mark.gpu


def _both(h, users, scores_buf):
    """Scores of the listed users by the existing entry point and by the static one (same batch object)."""
    sub = h.sub_batch(users)
    sub.set_handles([h.handles[u] for u in users])
    want = rg.relaygr_rank_with_cache(h.ctx, h.pool, sub).cpu().numpy()
    out = scores_buf[:sub.n_cands]
    out.fill_(float("nan"))
    rg.relaygr_rank_with_cache_static(h.ctx, h.pool, sub, out)
    torch.cuda.synchronize()
    return want, out.cpu().numpy()


@pytest.mark.parametrize("dtype,d,heads", [("bf16", 256, 4), ("fp32", 64, 2), ("fp16", 128, 2)])
def test_static_scratch_entry_point_matches_the_existing_one(dtype, d, heads):
    cfg = synth.ModelConfig(3, d, heads, dtype)
    weights, batch = build_case(cfg, 171, [700, 300, 129], [5, 0, 64], [300, 130, 7])
    h = Harness(cfg, weights, batch, 64)
    try:
        h.prefill()
        buf = torch.empty(int(batch["cand_off"][-1]), dtype=torch.float32, device="cuda:0")
        oracle = oracle_scores(cfg, weights, batch)
        co = batch["cand_off"]
        # first call: all three users; second call, right after it: one short user (a smaller row space laid
        # out over the first call's leftovers); third: the first again
        for users in ([0, 1, 2], [2], [0, 1, 2]):
            want, got = _both(h, users, buf)
            assert np.isfinite(got).all()
            assert np.array_equal(got, want), f"users {users}: static and context scratch disagree"
            ref = np.concatenate([oracle[u] for u in users])
            assert_close(got, ref, dtype, f"static entry point, users {users}")
        # a user without a cached prefix is recomputed inside the call, as in the existing entry point
        h.handles[1] = 0
        want, got = _both(h, [0, 1], buf)
        assert np.array_equal(got, want)
        assert_close(got, np.concatenate([oracle[0], oracle[1]]), dtype, "static entry point with a miss user")
        assert co[-1] == 437
    finally:
        h.close()


def test_static_scratch_refuses_what_does_not_fit():
    cfg = synth.ModelConfig(2, 256, 4, "bf16")
    M = 24000                                           # about 4.6 KB of buffers per row: beyond 64 MiB
    weights, batch = build_case(cfg, 173, [64], [0], [M])
    h = Harness(cfg, weights, batch, 64)
    try:
        h.prefill()
        assert rg.relaygr_static_scratch_bytes() == 64 << 20
        want = h.rank_cached()                           # fits the context's own buffer
        assert np.isfinite(want).all()
        out = torch.full((M,), 7.0, dtype=torch.float32, device="cuda:0")
        h.dbatch.set_handles(h.handles)
        with pytest.raises(rg.RelayGRError) as ei:
            rg.relaygr_rank_with_cache_static(h.ctx, h.pool, h.dbatch, out)
        assert ei.value.code == rg.RELAYGR_ENOSPC and "rank_with_cache_static" in str(ei.value)
        torch.cuda.synchronize()
        assert bool((out == 7.0).all().item())           # nothing was enqueued
        # a call that fits still works afterwards
        weights2, batch2 = build_case(cfg, 173, [64], [0], [50])
        h2 = Harness(cfg, weights2, batch2, 64)
        try:
            h2.prefill()
            buf = torch.empty(50, dtype=torch.float32, device="cuda:0")
            w2, g2 = _both(h2, [0], buf)
            assert np.array_equal(w2, g2)
        finally:
            h2.close()
    finally:
        h.close()


def test_static_scratch_calls_on_two_streams_are_kept_apart():
    """Two contexts use the library's scratch from two streams with no synchronisation between them, the first held
    up behind other work on its stream: the second call is ordered behind the first by the library (an event), so
    both give the scores of the existing entry point."""
    cfg = synth.ModelConfig(2, 256, 4, "bf16")
    weights, batch = build_case(cfg, 177, [700, 200], [3, 0], [260, 90])
    h = Harness(cfg, weights, batch, 64)
    ctx2 = rg.Context(cfg, weights, 2, 900, 353)
    try:
        h.prefill()
        a = h.sub_batch([0]); a.set_handles([h.handles[0]])
        b = h.sub_batch([1]); b.set_handles([h.handles[1]])
        want_a = rg.relaygr_rank_with_cache(h.ctx, h.pool, a).cpu().numpy()
        want_b = rg.relaygr_rank_with_cache(ctx2, h.pool, b).cpu().numpy()
        out_a = torch.full((a.n_cands,), float("nan"), dtype=torch.float32, device="cuda:0")
        out_b = torch.full((b.n_cands,), float("nan"), dtype=torch.float32, device="cuda:0")
        s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
        torch.cuda.synchronize()
        with torch.cuda.stream(s1):
            torch.cuda._sleep(100_000_000)
        rg.relaygr_rank_with_cache_static(h.ctx, h.pool, a, out_a, stream=s1)
        rg.relaygr_rank_with_cache_static(ctx2, h.pool, b, out_b, stream=s2)
        torch.cuda.synchronize()
        assert np.array_equal(out_a.cpu().numpy(), want_a)
        assert np.array_equal(out_b.cpu().numpy(), want_b)
    finally:
        ctx2.close()
        h.close()
