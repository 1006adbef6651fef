// Sequence-aware trigger, host side (Section 3.2): the admission budgets of Eq. 1-3 and a small
// admission gate that applies them.  Pure host arithmetic; no GPU work.
#include <cmath>
#include <mutex>
#include <new>

#include "../../include/relaygr.h"
#include "errors.h"

using relaygr::fail;

extern "C" int relaygr_admission_budget_compute(const relaygr_admission_params* p, relaygr_admission_budget* out) {
  if (!p || !out) return fail(RELAYGR_EINVAL, "admission_budget_compute: null argument");
  if (!(p->q_m > 0) || p->model_slots < 1 || !(p->kv_p99_bytes > 0) || !(p->hbm_bytes > 0) || !(p->r1 > 0 && p->r1 <= 1) ||
      p->n_instances < 1 || !(p->r2 > 0 && p->r2 <= 1) || !(p->t_life_s > 0))
    return fail(RELAYGR_EINVAL, "admission_budget_compute: parameter out of range (rates, sizes and the window must be positive, "
                                "r1 and r2 in (0, 1], at least one slot and one instance)");
  // Eq. 2: L * kv_p99 <= r1 * HBM.  The quotient of two doubles may land a rounding error below the integer the
  // caller's decimal figures give exactly (0.5 * 32 GB / 0.1 GB), hence the slack of 1e-9 of a cache before the floor.
  out->max_live_caches = std::floor(p->r1 * p->hbm_bytes / p->kv_p99_bytes + 1e-9);
  // Eq. 1: L = Q_admit * T_life  =>  Q_admit <= L_max / T_life
  out->q_admit_hbm = out->max_live_caches / p->t_life_s;
  // Eq. 3, first inequality: Q_admit <= Q_m * M
  out->q_admit_compute = p->q_m * p->model_slots;
  out->q_admit = std::fmin(out->q_admit_hbm, out->q_admit_compute);
  // Eq. 3, second inequality: Q_max <= (Q_m * M) * (r2 * N)
  out->q_max = out->q_admit_compute * (p->r2 * p->n_instances);
  return RELAYGR_OK;
}

extern "C" double relaygr_slot_throughput(double pre_infer_ms) {
  return pre_infer_ms > 0 ? std::floor(1000.0 / pre_infer_ms) : 0.0;
}

// Admission gate of one special instance: admits a request only if it is at risk (prefix at least
// len_threshold tokens), the live-cache count stays within Eq. 2's bound, and the admitted rate
// stays within min(Eq. 1, Eq. 3) (a token bucket refilled at q_admit, one second deep).
struct relaygr_trigger {
  relaygr_admission_budget budget;
  int32_t len_threshold;
  double tokens, last_s;
  int64_t live, admitted, refused_rate, refused_live, not_at_risk;
  std::mutex mu;
};

extern "C" int relaygr_trigger_create(const relaygr_admission_budget* b, int32_t len_threshold, relaygr_trigger** out) {
  if (!b || !out) return fail(RELAYGR_EINVAL, "trigger_create: null argument");
  if (len_threshold < 0 || !(b->q_admit > 0) || !(b->max_live_caches >= 1))
    return fail(RELAYGR_EINVAL, "trigger_create: needs len_threshold >= 0, q_admit > 0 and max_live_caches >= 1");
  relaygr_trigger* t = new (std::nothrow) relaygr_trigger();
  if (!t) return fail(RELAYGR_EINVAL, "trigger_create: out of host memory");
  t->budget = *b;
  t->len_threshold = len_threshold;
  t->tokens = std::fmax(1.0, b->q_admit);
  t->last_s = -1.0;
  t->live = t->admitted = t->refused_rate = t->refused_live = t->not_at_risk = 0;
  *out = t;
  return RELAYGR_OK;
}

extern "C" void relaygr_trigger_destroy(relaygr_trigger* t) { delete t; }

extern "C" int relaygr_trigger_admit(relaygr_trigger* t, double now_s, int32_t prefix_len) {
  if (!t) return fail(RELAYGR_EINVAL, "trigger_admit: null trigger");
  std::lock_guard<std::mutex> lk(t->mu);
  if (prefix_len < t->len_threshold) { t->not_at_risk += 1; return RELAYGR_TRIGGER_NOT_AT_RISK; }
  const double cap = std::fmax(1.0, t->budget.q_admit);
  if (t->last_s >= 0 && now_s > t->last_s) t->tokens = std::fmin(cap, t->tokens + (now_s - t->last_s) * t->budget.q_admit);
  if (t->last_s < 0 || now_s > t->last_s) t->last_s = now_s;
  if ((double)t->live + 1 > t->budget.max_live_caches) { t->refused_live += 1; return RELAYGR_TRIGGER_REFUSED; }
  if (t->tokens < 1.0) { t->refused_rate += 1; return RELAYGR_TRIGGER_REFUSED; }
  t->tokens -= 1.0;
  t->live += 1;
  t->admitted += 1;
  return RELAYGR_TRIGGER_ADMIT;
}

extern "C" int relaygr_trigger_release(relaygr_trigger* t) {
  if (!t) return fail(RELAYGR_EINVAL, "trigger_release: null trigger");
  std::lock_guard<std::mutex> lk(t->mu);
  if (t->live <= 0) return fail(RELAYGR_ENOENT, "trigger_release: no live cache to release");
  t->live -= 1;
  return RELAYGR_OK;
}

extern "C" int relaygr_trigger_stats(relaygr_trigger* t, int64_t* live, int64_t* admitted, int64_t* refused, int64_t* not_at_risk) {
  if (!t) return fail(RELAYGR_EINVAL, "trigger_stats: null trigger");
  std::lock_guard<std::mutex> lk(t->mu);
  if (live) *live = t->live;
  if (admitted) *admitted = t->admitted;
  if (refused) *refused = t->refused_rate + t->refused_live;
  if (not_at_risk) *not_at_risk = t->not_at_risk;
  return RELAYGR_OK;
}
