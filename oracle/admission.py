"""TEST INFRASTRUCTURE ONLY: the admission budgets of the sequence-aware trigger, written out from
Section 3.2, Eq. 1-3.  Pinned by the paper's worked example (tests/golden/admission_example.txt).
Imported by tests only; shares no code with the library.
"""
import math


def live_cache_bound(kv_p99_bytes: float, hbm_bytes: float, r1: float) -> int:
    """Eq. 2: the largest integer L with L * kv_p99 <= r1 * HBM."""
    return int(math.floor(r1 * hbm_bytes / kv_p99_bytes + 1e-9))


def budgets(q_m, model_slots, kv_p99_bytes, hbm_bytes, r1, n_instances, r2, t_life_s) -> dict:
    L = live_cache_bound(kv_p99_bytes, hbm_bytes, r1)
    q_hbm = L / t_life_s                      # Eq. 1: L = Q_admit * T_life
    q_compute = q_m * model_slots             # Eq. 3, per instance
    return {
        "max_live_caches": float(L),
        "q_admit_hbm": q_hbm,
        "q_admit_compute": q_compute,
        "q_admit": min(q_hbm, q_compute),
        "q_max": q_compute * (r2 * n_instances),   # Eq. 3, pool-wide
    }
