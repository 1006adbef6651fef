"""Sequence-aware trigger, host side (Section 3.2, Eq. 1-3): the budgets against the paper's worked
example and the oracle's formulae, and the admission gate against the bounds it must keep."""
import os

import numpy as np
import pytest

import paper_2601_01712_amd as rg
from oracle import admission as oadm

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "admission_example.txt")
GB = 1e9


def _example():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    ms, q_m, m, kv, hbm, r1, n, r2 = (float(x) for x in rows[0])
    want = [float(x) for x in rows[1]]
    return dict(ms=ms, q_m=q_m, m=int(m), kv=kv * GB, hbm=hbm * GB, r1=r1, n=int(n), r2=r2), want


def test_oracle_reproduces_the_printed_example():
    p, (L, q_life, q_cap, q_max) = _example()
    b = oadm.budgets(p["q_m"], p["m"], p["kv"], p["hbm"], p["r1"], p["n"], p["r2"], 1.0)
    assert b["max_live_caches"] == L
    assert b["q_admit_hbm"] == q_life          # T_life = 1 s: the bound is L itself
    assert b["q_admit_compute"] == q_cap
    assert b["q_max"] == pytest.approx(q_max, rel=1e-12)
    # Eq. 1 with another window: 160 live caches over 0.4 s allow 400 queries/s, so compute (150) binds
    b2 = oadm.budgets(p["q_m"], p["m"], p["kv"], p["hbm"], p["r1"], p["n"], p["r2"], 0.4)
    assert b2["q_admit_hbm"] == pytest.approx(400.0) and b2["q_admit"] == 150.0
    # and over 2 s only 80 queries/s survive: HBM binds
    b3 = oadm.budgets(p["q_m"], p["m"], p["kv"], p["hbm"], p["r1"], p["n"], p["r2"], 2.0)
    assert b3["q_admit"] == pytest.approx(80.0)


def test_library_reproduces_the_printed_example():
    p, (L, q_life, q_cap, q_max) = _example()
    b = rg.relaygr_admission_budget_compute(p["q_m"], p["m"], p["kv"], p["hbm"], p["r1"], p["n"], p["r2"], 1.0)
    assert b["max_live_caches"] == L and b["q_admit_hbm"] == q_life
    assert b["q_admit_compute"] == q_cap and b["q_admit"] == min(q_life, q_cap)
    assert b["q_max"] == pytest.approx(q_max, rel=1e-12)
    # floor(1000/35) is 28; the example rounds it to "about 30"
    assert rg.relaygr_slot_throughput(p["ms"]) == 28.0
    assert rg.relaygr_slot_throughput(0.0) == 0.0


def test_library_budgets_equal_oracle_on_random_parameters():
    rng = np.random.default_rng(5)
    for _ in range(200):
        q_m = float(rng.uniform(1, 500)); m = int(rng.integers(1, 16))
        kv = float(rng.uniform(1e6, 4e9)); hbm = float(rng.choice([32e9, 64e9, 288e9]))
        r1 = float(rng.uniform(0.05, 1.0)); n = int(rng.integers(1, 2000)); r2 = float(rng.uniform(0.01, 1.0))
        t = float(rng.uniform(0.05, 3.0))
        got = rg.relaygr_admission_budget_compute(q_m, m, kv, hbm, r1, n, r2, t)
        want = oadm.budgets(q_m, m, kv, hbm, r1, n, r2, t)
        for k in want:
            assert got[k] == pytest.approx(want[k], rel=1e-12), k
        # Eq. 2 as an inequality: L caches fit in the reserved share, L + 1 do not
        L = got["max_live_caches"]
        assert L * kv <= r1 * hbm * (1 + 1e-9) and (L + 1) * kv > r1 * hbm * (1 - 1e-9)


def test_live_cache_bound_at_exact_quotients():
    """Eq. 2 where r1 * HBM / kv_p99 is an integer: once exactly representable in binary (0.5 * 32 / 0.125 = 128),
    once only in decimal (the paper's 0.5 * 32 / 0.1 = 160, whose double quotient need not be 160.0), in GB and in
    bytes; one byte more per cache must cost one cache.  The oracle works in exact rationals of the decimal text,
    the library in doubles with a slack: two different routes to the same integers."""
    for kv_gb, hbm_gb, r1, want in ((0.125, 32.0, 0.5, 128), (0.1, 32.0, 0.5, 160), (0.3, 288.0, 0.25, 240), (0.7, 64.0, 0.7, 64)):
        for unit in (1.0, 1e9):
            kv, hbm = kv_gb * unit, hbm_gb * unit
            assert oadm.live_cache_bound(kv, hbm, r1) == want, (kv_gb, unit)
            got = rg.relaygr_admission_budget_compute(30.0, 5, kv, hbm, r1, 100, 0.1, 1.0)
            assert got["max_live_caches"] == want, (kv_gb, unit)
        assert oadm.live_cache_bound(kv_gb * 1e9 + 1, hbm_gb * 1e9, r1) == want - 1
        assert rg.relaygr_admission_budget_compute(30.0, 5, kv_gb * 1e9 + 1, hbm_gb * 1e9, r1, 100, 0.1, 1.0)["max_live_caches"] == want - 1
    # brute force over small integers: the bound is floor(a / b)
    for a in range(1, 40):
        for b in range(1, 12):
            assert oadm.live_cache_bound(float(b), float(a), 1.0) == a // b


def test_failures_leave_their_text_in_last_error():
    with pytest.raises(rg.RelayGRError) as ei:
        rg.relaygr_admission_budget_compute(30.0, 5, 1e8, 32e9, 1.5, 100, 0.1, 1.0)
    assert "admission_budget_compute" in str(ei.value) and "r1" in str(ei.value)
    t = _trigger(10.0, 3)
    with pytest.raises(rg.RelayGRError) as ei:
        rg.relaygr_trigger_release(t)
    assert ei.value.code == rg.RELAYGR_ENOENT and "trigger_release" in str(ei.value)
    t.close()
    with pytest.raises(rg.RelayGRError) as ei:
        _trigger(0.0, 10)
    assert "trigger_create" in str(ei.value)


@pytest.mark.parametrize("bad", [dict(q_m=0.0), dict(model_slots=0), dict(kv_p99_bytes=0.0), dict(hbm_bytes=-1.0),
                                 dict(r1=0.0), dict(r1=1.5), dict(n_instances=0), dict(r2=0.0), dict(t_life_s=0.0)])
def test_budget_rejects_out_of_range_parameters(bad):
    args = dict(q_m=30.0, model_slots=5, kv_p99_bytes=1e8, hbm_bytes=32e9, r1=0.5, n_instances=100, r2=0.1, t_life_s=1.0)
    args.update(bad)
    with pytest.raises(rg.RelayGRError) as ei:
        rg.relaygr_admission_budget_compute(**args)
    assert ei.value.code == rg.RELAYGR_EINVAL


def _trigger(q_admit, max_live, thr=4096):
    budget = dict(max_live_caches=float(max_live), q_admit_hbm=q_admit, q_admit_compute=q_admit, q_admit=q_admit, q_max=q_admit)
    return rg.Trigger(budget, thr)


def test_short_prefixes_cost_nothing():
    t = _trigger(100.0, 10)
    for i in range(1000):
        assert rg.relaygr_trigger_admit(t, i * 1e-3, 4095) == rg.RELAYGR_TRIGGER_NOT_AT_RISK
    s = rg.relaygr_trigger_stats(t)
    assert s == {"live": 0, "admitted": 0, "refused": 0, "not_at_risk": 1000}
    assert rg.relaygr_trigger_admit(t, 1.0, 4096) == rg.RELAYGR_TRIGGER_ADMIT
    t.close()


def test_live_cache_bound_is_never_exceeded():
    """Eq. 2: with nothing released, at most max_live_caches requests are admitted however slowly they come."""
    t = _trigger(1000.0, 7)
    out = [rg.relaygr_trigger_admit(t, 0.01 * i, 8000) for i in range(50)]
    assert out.count(rg.RELAYGR_TRIGGER_ADMIT) == 7 and out[:7] == [rg.RELAYGR_TRIGGER_ADMIT] * 7
    assert rg.relaygr_trigger_stats(t)["live"] == 7
    rg.relaygr_trigger_release(t)
    assert rg.relaygr_trigger_admit(t, 1.0, 8000) == rg.RELAYGR_TRIGGER_ADMIT
    assert rg.relaygr_trigger_admit(t, 1.0, 8000) == rg.RELAYGR_TRIGGER_REFUSED
    for _ in range(7):
        rg.relaygr_trigger_release(t)
    with pytest.raises(rg.RelayGRError):
        rg.relaygr_trigger_release(t)
    t.close()


def test_admitted_rate_stays_within_the_budget():
    """Eq. 1/3: over any window of T seconds at most q_admit * T + q_admit (the bucket's depth) are admitted."""
    q = 150.0
    t = _trigger(q, 10 ** 6)
    rng = np.random.default_rng(9)
    now, times = 0.0, []
    for _ in range(20000):
        now += float(rng.exponential(1.0 / 600.0))       # offered load 4x the budget
        if rg.relaygr_trigger_admit(t, now, 5000) == rg.RELAYGR_TRIGGER_ADMIT:
            times.append(now)
            rg.relaygr_trigger_release(t)
    times = np.array(times)
    for T in (0.5, 1.0, 5.0):
        hi = np.searchsorted(times, times + T, side="left") - np.arange(len(times))
        assert hi.max() <= q * T + q + 1
    # and the budget is actually used: beyond the initially full bucket, the long-run rate is q_admit
    assert (len(times) - q) / now == pytest.approx(q, rel=0.02)
    s = rg.relaygr_trigger_stats(t)
    assert s["admitted"] == len(times) and s["admitted"] + s["refused"] == 20000
    t.close()


def test_clock_going_backwards_grants_nothing():
    t = _trigger(2.0, 100)
    assert rg.relaygr_trigger_admit(t, 10.0, 9000) == rg.RELAYGR_TRIGGER_ADMIT
    assert rg.relaygr_trigger_admit(t, 10.0, 9000) == rg.RELAYGR_TRIGGER_ADMIT
    assert rg.relaygr_trigger_admit(t, 5.0, 9000) == rg.RELAYGR_TRIGGER_REFUSED
    assert rg.relaygr_trigger_admit(t, 10.4, 9000) == rg.RELAYGR_TRIGGER_REFUSED    # 0.8 of a token
    assert rg.relaygr_trigger_admit(t, 10.5, 9000) == rg.RELAYGR_TRIGGER_ADMIT
    t.close()


def test_trigger_create_rejects_bad_budgets():
    with pytest.raises(rg.RelayGRError):
        _trigger(0.0, 10)
    with pytest.raises(rg.RelayGRError):
        _trigger(10.0, 0)
    with pytest.raises(rg.RelayGRError):
        _trigger(10.0, 10, thr=-1)
