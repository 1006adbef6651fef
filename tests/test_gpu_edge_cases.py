"""GPU edge cases of the compute calls: empty batches and segments, degenerate shapes, and the argument
errors the header promises (RELAYGR_EINVAL / RELAYGR_ENOENT / RELAYGR_ENOSPC instead of a fault).
Where scores come out they are checked against the CPU oracle."""
import ctypes as C

import numpy as np
import pytest
import torch

import paper_2601_01712_amd as rg
import synth
from gpu_util import Harness, build_case, oracle_scores

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_calls_with_nothing_to_do_succeed(dtype):
    d = 64 if dtype == "fp32" else 128
    cfg = synth.ModelConfig(2, d, 2, dtype)
    weights, batch = build_case(cfg, 701, [70, 0], [0, 0], [0, 0])          # no suffix, no candidates at all
    h = Harness(cfg, weights, batch)
    try:
        h.prefill([0])
        for scores in (h.rank_cached(), h.rank_full()):
            assert scores.shape == (0,)
        # a batch of zero users
        empty = {"n_users": 0, "user_ids": np.zeros(0, np.uint64), "prefix_emb": np.zeros((0, d), np.float32),
                 "prefix_off": np.zeros(1, np.int32), "suffix_emb": np.zeros((0, d), np.float32), "suffix_off": np.zeros(1, np.int32),
                 "cand_emb": np.zeros((0, d), np.float32), "cand_off": np.zeros(1, np.int32)}
        eb = rg.Batch(empty, dtype)
        rg.relaygr_prefill_prefix(h.ctx, h.pool, eb)
        assert rg.relaygr_rank_with_cache(h.ctx, h.pool, eb).numel() == 0
        assert rg.relaygr_rank_full_recompute(h.ctx, eb).numel() == 0
        torch.cuda.synchronize()
    finally:
        h.close()


@pytest.mark.parametrize("dtype", ["fp32", "bf16", "fp16"])
@pytest.mark.parametrize("attention", ["silu", "softmax"])
def test_suffix_without_candidates_and_candidates_without_history(dtype, attention):
    """User 0 has a prefix and a suffix but nothing to score, user 1 only candidates (no history at all: each sees
    itself alone), user 2 a suffix and candidates but no prefix, user 3 one prefix token and one candidate."""
    d = 64 if dtype == "fp32" else 128
    cfg = synth.ModelConfig(2, d, 2, dtype, attention=attention)
    weights, batch = build_case(cfg, 703, [130, 0, 0, 1], [5, 0, 66, 0], [0, 70, 3, 1])
    want = oracle_scores(cfg, weights, batch)
    h = Harness(cfg, weights, batch)
    try:
        h.prefill([0, 3])
        h.check(h.rank_cached(), want, "rank_with_cache")
        h.check(h.rank_full(), want, "rank_full_recompute")
    finally:
        h.close()


def test_argument_errors_are_reported_not_faulted():
    cfg = synth.ModelConfig(2, 128, 2, "bf16")
    weights, batch = build_case(cfg, 705, [100, 64], [2, 0], [5, 9])
    h = Harness(cfg, weights, batch)
    try:
        h.prefill()
        good = h.rank_cached()
        lib = rg.load_library()

        def rc_of(mutate, call="cached"):
            db = rg.Batch(batch, cfg.dtype, handles=[int(x) for x in h.handles])
            bc = db.c_struct()
            keep = mutate(db, bc)                                  # keeps replacement arrays alive
            scores = torch.empty(db.n_cands, dtype=torch.float32, device="cuda:0")
            if call == "cached":
                rc = lib.relaygr_rank_with_cache(h.ctx.handle, h.pool.handle, C.byref(bc), scores.data_ptr(), None)
            elif call == "prefill":
                rc = lib.relaygr_prefill_prefix(h.ctx.handle, h.pool.handle, C.byref(bc), None)
            else:
                rc = lib.relaygr_rank_full_recompute(h.ctx.handle, C.byref(bc), scores.data_ptr(), None)
            del keep
            return rc, rg.relaygr_last_error()

        def bad_offsets(db, bc):
            off = np.array([0, 9, 5], dtype=np.int32)              # not monotone
            bc.cand_off = off.ctypes.data_as(C.POINTER(C.c_int32))
            return off
        rc, msg = rc_of(bad_offsets)
        assert rc == rg.RELAYGR_EINVAL and "monotone" in msg

        def offsets_not_from_zero(db, bc):
            off = np.array([1, 5, 14], dtype=np.int32)
            bc.cand_off = off.ctypes.data_as(C.POINTER(C.c_int32))
            return off
        rc, msg = rc_of(offsets_not_from_zero)
        assert rc == rg.RELAYGR_EINVAL and "start at 0" in msg

        def wrong_prefix_length(db, bc):
            off = np.array([0, 99, 163], dtype=np.int32)           # user 0's cached entry holds 100 tokens
            bc.prefix_off = off.ctypes.data_as(C.POINTER(C.c_int32))
            return off
        rc, msg = rc_of(wrong_prefix_length)
        assert rc == rg.RELAYGR_EINVAL and "differs from the cached entry" in msg

        def null_candidates(db, bc):
            bc.cand_emb = None
        rc, msg = rc_of(null_candidates)
        assert rc == rg.RELAYGR_EINVAL and "cand_emb" in msg

        def null_prefix_for_recompute(db, bc):
            bc.prefix_emb = None
        rc, msg = rc_of(null_prefix_for_recompute, call="full")
        assert rc == rg.RELAYGR_EINVAL and "prefix_emb" in msg

        def negative_users(db, bc):
            bc.n_users = -1
        rc, msg = rc_of(negative_users)
        assert rc == rg.RELAYGR_EINVAL

        def no_handle_in_prefill(db, bc):
            hs = np.zeros(2, dtype=np.uint64)
            bc.handles = hs.ctypes.data_as(C.POINTER(C.c_uint64))
            return hs
        rc, msg = rc_of(no_handle_in_prefill, call="prefill")
        assert rc == rg.RELAYGR_EINVAL and "no handle" in msg

        assert lib.relaygr_rank_with_cache(None, h.pool.handle, None, None, None) == rg.RELAYGR_EINVAL
        assert lib.relaygr_prefill_prefix(h.ctx.handle, None, None, None) == rg.RELAYGR_EINVAL

        # a pool made for another model shape is refused
        other = rg.make_config(2, 256, 2, "bf16")
        pool2 = rg.KvPool(other, "bf16", 4 * rg.relaygr_kv_pool_bytes_for(other, 64, 64), 64)
        db = rg.Batch(batch, cfg.dtype, handles=[int(x) for x in h.handles])
        with pytest.raises(rg.RelayGRError) as ei:
            rg.relaygr_rank_with_cache(h.ctx, pool2, db)
        assert ei.value.code == rg.RELAYGR_EINVAL and "different model shapes" in str(ei.value)
        pool2.close()

        # after all the refused calls the context still works and gives the same bits
        assert np.array_equal(h.rank_cached(), good)
    finally:
        h.close()
