"""TEST INFRASTRUCTURE ONLY: the admission budgets of the sequence-aware trigger, written out from
Section 3.2, Eq. 1-3.  Pinned by the paper's worked example (tests/golden/admission_example.txt).
Imported by tests only; shares no code with the library.
"""
from fractions import Fraction


def _exact(x) -> Fraction:
    """The number a caller wrote: the shortest decimal that reads back as the float x (0.1 is one tenth, not the
    binary value next to it), as an exact rational."""
    return Fraction(repr(float(x)))


def live_cache_bound(kv_p99_bytes: float, hbm_bytes: float, r1: float) -> int:
    """Eq. 2: the largest integer L with L * kv_p99 <= r1 * HBM, in exact rational arithmetic."""
    budget, per_cache = _exact(r1) * _exact(hbm_bytes), _exact(kv_p99_bytes)
    L = int(budget / per_cache)          # truncation of an exact quotient, then checked both ways
    while (L + 1) * per_cache <= budget:
        L += 1
    while L > 0 and L * per_cache > budget:
        L -= 1
    return L


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
