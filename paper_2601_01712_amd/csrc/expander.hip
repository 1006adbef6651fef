// DRAM tier of the psi cache (Section 3.4, "memory-aware expander"): spill / reload of pool
// extents, and the expander that keeps consumed entries in pinned host memory behind a two-level
// lookup HBM -> DRAM with bounded reload concurrency and one live copy per user and tier.
// A pool extent is position independent (its layout depends only on the tile index inside the
// extent), so its byte image can be reloaded anywhere in a pool of the same shape and page size.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <deque>
#include <mutex>
#include <new>
#include <unordered_map>
#include <vector>

#include "../../include/relaygr.h"
#include "errors.h"
#include "kv_pool.h"

using namespace relaygr;

#define HIP_TRY(expr)                                                                          \
  do {                                                                                         \
    hipError_t e_ = (expr);                                                                    \
    if (e_ != hipSuccess) return fail(RELAYGR_EHIP, "%s: %s", #expr, hipGetErrorString(e_));   \
  } while (0)

static size_t page_bytes(const KvPool* p) {
  return (size_t)2 * p->cfg.n_layers * p->page_tokens * p->cfg.d_model * elem_bytes(p->cfg);
}
static char* extent_ptr(const KvPool* p, const PoolEntry& e) { return (char*)p->slab + (size_t)e.page0 * page_bytes(p); }

extern "C" size_t relaygr_kv_pool_entry_bytes(relaygr_kv_pool* pool, relaygr_kv_handle h) {
  KvPool* p = reinterpret_cast<KvPool*>(pool);
  PoolEntry e;
  if (!p || p->resolve(h, &e) != RELAYGR_OK) return 0;
  return (size_t)e.npages * page_bytes(p);
}

extern "C" int relaygr_kv_pool_spill(relaygr_kv_pool* pool, relaygr_kv_handle h, void* host_dst, size_t host_bytes, void* stream) {
  KvPool* p = reinterpret_cast<KvPool*>(pool);
  if (!p || !host_dst) return fail(RELAYGR_EINVAL, "kv_pool_spill: null argument");
  PoolEntry e;
  if (p->resolve(h, &e) != RELAYGR_OK) return fail(RELAYGR_ENOENT, "kv_pool_spill: stale or unknown handle");
  size_t bytes = (size_t)e.npages * page_bytes(p);
  if (host_bytes != bytes) return fail(RELAYGR_EINVAL, "kv_pool_spill: buffer is %zu bytes, the entry's extent is %zu", host_bytes, bytes);
  HIP_TRY(hipMemcpyAsync(host_dst, extent_ptr(p, e), bytes, hipMemcpyDeviceToHost, (hipStream_t)stream));
  return RELAYGR_OK;
}

extern "C" int relaygr_kv_pool_reload(relaygr_kv_pool* pool, uint64_t user_id, int32_t prefix_len, const void* host_src,
                                      size_t host_bytes, void* stream, relaygr_kv_handle* out) {
  KvPool* p = reinterpret_cast<KvPool*>(pool);
  if (!p || !host_src || !out) return fail(RELAYGR_EINVAL, "kv_pool_reload: null argument");
  *out = RELAYGR_NO_CACHE;
  if (prefix_len < 1) return fail(RELAYGR_EINVAL, "kv_pool_reload: prefix_len < 1");
  size_t pages = ((size_t)prefix_len + p->page_tokens - 1) / p->page_tokens;
  if (host_bytes != pages * page_bytes(p))
    return fail(RELAYGR_EINVAL, "kv_pool_reload: image is %zu bytes, a prefix of %d tokens takes %zu", host_bytes, prefix_len, pages * page_bytes(p));
  relaygr_kv_handle h;
  int rc = p->alloc(user_id, prefix_len, &h);
  if (rc == RELAYGR_ENOSPC) return fail(rc, "kv_pool_reload: no free extent for %d tokens", prefix_len);
  if (rc != RELAYGR_OK) return fail(rc, "kv_pool_reload: user %llu already has a live entry", (unsigned long long)user_id);
  PoolEntry e;
  p->resolve(h, &e);
  hipError_t he = hipMemcpyAsync(extent_ptr(p, e), host_src, host_bytes, hipMemcpyHostToDevice, (hipStream_t)stream);
  if (he != hipSuccess) { p->release(h); return fail(RELAYGR_EHIP, "kv_pool_reload: %s", hipGetErrorString(he)); }
  *out = h;
  return RELAYGR_OK;
}

// ---- the expander ------------------------------------------------------------------------------
// The DRAM tier is a second pool of the same page geometry whose slab is one pinned host arena
// allocated at creation: no allocation happens on the serving path.  Spills (HBM -> DRAM) and
// reloads (DRAM -> HBM) run on two streams of the expander's own, so that the two directions of
// the host link overlap and a reload -- which sits on a ranking request's critical path (the
// `load` step) -- never queues behind other users' spills or behind the ranking stream a spill
// waits for.  The arena is kept consistent with events instead of stream order: a reload waits
// for the spills still in flight into the pages it reads, a spill waits for the reloads still in
// flight out of the pages it overwrites.  HBM extents are read by the caller's streams, so an extent becomes
// reclaimable only after the event that follows its spill has completed.  Reclaimable entries stay
// in HBM (a repeat request still hits them) until an allocation needs their pages: the HBM pool is
// then a sliding window over users, consumed entries leaving it oldest retirement first (Section
// 3.3, "HBM as a lifecycle window"), while an entry that was never retired is never displaced
// (Section 3.1, invariant I2).
namespace {
struct PendingFree {
  relaygr_kv_handle handle;
  hipEvent_t spilled;
  bool cancelled;
  int64_t dram_page0, dram_pages;   // arena pages the spill writes (0 pages: no image)
};
struct Reload {
  relaygr_kv_handle handle;   // the HBM entry being filled
  hipEvent_t done;
  int64_t dram_page0, dram_pages;   // arena pages the reload reads
};
inline bool overlap(int64_t a0, int64_t an, int64_t b0, int64_t bn) { return an > 0 && bn > 0 && a0 < b0 + bn && b0 < a0 + an; }
}  // namespace

struct relaygr_expander {
  KvPool* hbm = nullptr;
  KvPool dram;                          // page allocator over the pinned arena
  void* arena = nullptr;
  int max_inflight = 1;
  hipStream_t spill_stream = nullptr, reload_stream = nullptr;   // default priority, one per direction
  std::unordered_map<uint64_t, uint64_t> last_use;   // DRAM-resident user -> LRU stamp
  std::vector<PendingFree> pending_free;        // retired, spill not yet known to be complete
  std::deque<relaygr_kv_handle> reclaimable;    // retired and spilled: still in HBM, oldest first
  std::vector<Reload> reloads;          // reloads that may still be in flight
  std::vector<hipEvent_t> spare_events;
  uint64_t clock = 0;
  // reload rate limit: a token bucket in bytes (rate 0 = unlimited), refilled on the host's monotonic clock
  double rate_bps = 0.0, burst_bytes = 0.0, tokens = 0.0;
  std::chrono::steady_clock::time_point refilled;
  int64_t stats[6] = {};
  int64_t hbm_evictions = 0;
  std::mutex mu;
};

static hipEvent_t get_event(relaygr_expander* ex) {
  hipEvent_t e = nullptr;
  if (!ex->spare_events.empty()) { e = ex->spare_events.back(); ex->spare_events.pop_back(); return e; }
  if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) return nullptr;
  return e;
}

// Retires what has completed: entries whose spill has landed become reclaimable, finished reloads are forgotten.
static void poll(relaygr_expander* ex) {
  for (size_t i = 0; i < ex->pending_free.size();) {
    PendingFree& pf = ex->pending_free[i];
    if (hipEventQuery(pf.spilled) == hipSuccess) {
      if (!pf.cancelled) ex->reclaimable.push_back(pf.handle);
      ex->spare_events.push_back(pf.spilled);
      ex->pending_free[i] = ex->pending_free.back();
      ex->pending_free.pop_back();
    } else {
      ++i;
    }
  }
  for (size_t i = 0; i < ex->reloads.size();) {
    if (hipEventQuery(ex->reloads[i].done) == hipSuccess) {
      ex->spare_events.push_back(ex->reloads[i].done);
      ex->reloads[i] = ex->reloads.back();
      ex->reloads.pop_back();
    } else {
      ++i;
    }
  }
}

// A DRAM slot for the user's image: reuses the user's slot when the length matches, else allocates,
// dropping least-recently-used images of other users until the extent fits.
static bool dram_slot(relaygr_expander* ex, uint64_t user, int32_t prefix_len, PoolEntry* slot) {
  if (!ex->arena) return false;
  relaygr_kv_handle h;
  if (ex->dram.lookup(user, &h) == RELAYGR_OK) {
    ex->dram.resolve(h, slot);
    if (slot->prefix_len == prefix_len) return true;
    ex->dram.release(h);
    ex->last_use.erase(user);
  }
  for (;;) {
    int rc = ex->dram.alloc(user, prefix_len, &h);
    if (rc == RELAYGR_OK) break;
    if (rc != RELAYGR_ENOSPC) return false;
    uint64_t victim = 0, best = ~0ull;
    bool found = false;
    for (auto& kv : ex->last_use)
      if (kv.second < best) { best = kv.second; victim = kv.first; found = true; }
    if (!found) return false;
    relaygr_kv_handle vh;
    if (ex->dram.lookup(victim, &vh) == RELAYGR_OK) ex->dram.release(vh);
    ex->last_use.erase(victim);
    ex->stats[5] += 1;
  }
  ex->dram.resolve(h, slot);
  return true;
}

static void forget_reclaimable(relaygr_expander* ex, relaygr_kv_handle h) {
  auto it = std::find(ex->reclaimable.begin(), ex->reclaimable.end(), h);
  if (it != ex->reclaimable.end()) ex->reclaimable.erase(it);
}

// Pool allocation under the sliding-window policy: when nothing fits, reclaimable entries are
// released oldest first until the extent fits or none is left.
static int alloc_in_window(relaygr_expander* ex, uint64_t user, int32_t prefix_len, relaygr_kv_handle* h) {
  for (;;) {
    int rc = ex->hbm->alloc(user, prefix_len, h);
    if (rc != RELAYGR_ENOSPC) return rc;
    bool freed = false;
    while (!freed && !ex->reclaimable.empty()) {
      relaygr_kv_handle v = ex->reclaimable.front();
      ex->reclaimable.pop_front();
      if (ex->hbm->release(v) == RELAYGR_OK) { ex->hbm_evictions += 1; freed = true; }   // stale: the caller freed it itself
    }
    if (!freed) return RELAYGR_ENOSPC;
  }
}

extern "C" int relaygr_expander_create(relaygr_kv_pool* pool, size_t dram_budget_bytes, int32_t max_inflight_reloads,
                                       relaygr_expander** out) {
  if (!out) return fail(RELAYGR_EINVAL, "expander_create: out is null");
  *out = nullptr;
  if (!pool || max_inflight_reloads < 1) return fail(RELAYGR_EINVAL, "expander_create: null pool or max_inflight_reloads < 1");
  relaygr_expander* ex = new (std::nothrow) relaygr_expander();
  if (!ex) return fail(RELAYGR_EINVAL, "expander_create: out of host memory");
  ex->hbm = reinterpret_cast<KvPool*>(pool);
  ex->max_inflight = max_inflight_reloads;
  const size_t pb = page_bytes(ex->hbm);
  const int64_t pages = (int64_t)(dram_budget_bytes / pb);
  if (pages * (int64_t)ex->hbm->page_tokens >= (1ll << 31)) { delete ex; return fail(RELAYGR_EINVAL, "expander_create: DRAM budget holds 2^31 tokens or more"); }
  hipError_t e = hipStreamCreateWithFlags(&ex->spill_stream, hipStreamNonBlocking);   // default priority
  if (e == hipSuccess) {
    e = hipStreamCreateWithFlags(&ex->reload_stream, hipStreamNonBlocking);
    if (e != hipSuccess) (void)hipStreamDestroy(ex->spill_stream);
  }
  if (e != hipSuccess) { delete ex; return fail(RELAYGR_EHIP, "expander_create: %s", hipGetErrorString(e)); }
  if (pages > 0) {
    e = hipHostMalloc(&ex->arena, (size_t)pages * pb, hipHostMallocDefault);
    if (e != hipSuccess) {
      (void)hipStreamDestroy(ex->spill_stream);
      (void)hipStreamDestroy(ex->reload_stream);
      delete ex;
      return fail(RELAYGR_EHIP, "expander_create: pinning %zu bytes of host memory: %s", (size_t)pages * pb, hipGetErrorString(e));
    }
  }
  ex->dram.cfg = ex->hbm->cfg;
  ex->dram.slab = ex->arena;
  ex->dram.slab_bytes = (size_t)pages * pb;
  ex->dram.page_tokens = ex->hbm->page_tokens;
  ex->dram.n_pages = pages;
  ex->dram.layer_stride = ex->hbm->layer_stride;
  ex->dram.tile_stride = ex->hbm->tile_stride;
  if (pages > 0) ex->dram.free_extents[0] = pages;
  *out = ex;
  return RELAYGR_OK;
}

extern "C" void relaygr_expander_destroy(relaygr_expander* ex) {
  if (!ex) return;
  (void)hipStreamSynchronize(ex->spill_stream);
  (void)hipStreamSynchronize(ex->reload_stream);
  poll(ex);
  for (auto& pf : ex->pending_free) (void)hipEventDestroy(pf.spilled);
  for (auto& r : ex->reloads) (void)hipEventDestroy(r.done);
  for (auto e : ex->spare_events) (void)hipEventDestroy(e);
  (void)hipStreamDestroy(ex->spill_stream);
  (void)hipStreamDestroy(ex->reload_stream);
  if (ex->arena) (void)hipHostFree(ex->arena);
  delete ex;
}

extern "C" int relaygr_expander_retire(relaygr_expander* ex, relaygr_kv_handle h, void* stream) {
  if (!ex) return fail(RELAYGR_EINVAL, "expander_retire: null expander");
  std::lock_guard<std::mutex> lk(ex->mu);
  poll(ex);
  PoolEntry e;
  if (ex->hbm->resolve(h, &e) != RELAYGR_OK) return fail(RELAYGR_ENOENT, "expander_retire: stale or unknown handle");
  // An earlier retire of this entry may still be pending; the caller has used the entry since, so
  // that release would come too early.  This retire supersedes it.
  for (auto& pf : ex->pending_free)
    if (pf.handle == h) pf.cancelled = true;
  forget_reclaimable(ex, h);
  const size_t bytes = (size_t)e.npages * page_bytes(ex->hbm);
  hipEvent_t consumed = get_event(ex), spilled = get_event(ex);
  if (!consumed || !spilled) {
    if (consumed) ex->spare_events.push_back(consumed);
    if (spilled) ex->spare_events.push_back(spilled);
    return fail(RELAYGR_EHIP, "expander_retire: cannot create events");
  }
  HIP_TRY(hipEventRecord(consumed, (hipStream_t)stream));
  HIP_TRY(hipStreamWaitEvent(ex->spill_stream, consumed, 0));
  ex->spare_events.push_back(consumed);   // the wait is enqueued; the event may be recorded again later
  int rc = RELAYGR_OK;
  PoolEntry slot;
  int64_t dp0 = 0, dpn = 0;
  if (dram_slot(ex, e.user_id, e.prefix_len, &slot)) {
    dp0 = slot.page0; dpn = slot.npages;
    // the slot may be recycled pages that a reload still reads (the image that lived there was displaced after
    // its reload was queued): the spill overwrites them only after that reload
    for (auto& r : ex->reloads)
      if (overlap(dp0, dpn, r.dram_page0, r.dram_pages)) HIP_TRY(hipStreamWaitEvent(ex->spill_stream, r.done, 0));
    HIP_TRY(hipMemcpyAsync(extent_ptr(&ex->dram, slot), extent_ptr(ex->hbm, e), bytes, hipMemcpyDeviceToHost, ex->spill_stream));
    ex->last_use[e.user_id] = ++ex->clock;
    ex->stats[4] += 1;
  } else {
    // no DRAM for it: the entry still becomes reclaimable once the stream has consumed it
    rc = fail(RELAYGR_ENOSPC, "expander_retire: no DRAM for %zu bytes; the entry has no image", bytes);
  }
  HIP_TRY(hipEventRecord(spilled, ex->spill_stream));
  ex->pending_free.push_back({h, spilled, false, dp0, dpn});
  return rc;
}

extern "C" int relaygr_expander_lookup(relaygr_expander* ex, uint64_t user_id, void* stream, relaygr_kv_handle* out, int32_t* source) {
  if (!ex || !out) return fail(RELAYGR_EINVAL, "expander_lookup: null argument");
  *out = RELAYGR_NO_CACHE;
  std::lock_guard<std::mutex> lk(ex->mu);
  poll(ex);
  relaygr_kv_handle h;
  if (ex->hbm->lookup(user_id, &h) == RELAYGR_OK) {         // level 1: HBM
    for (auto& pf : ex->pending_free)
      if (pf.handle == h) pf.cancelled = true;              // keep it live; its DRAM copy still completes
    forget_reclaimable(ex, h);                              // live again until it is retired again
    // a reload of this very entry may still be in flight on the reload stream: order the caller behind
    // it, and behind nothing else (a hit does not wait for other users' spills and reloads)
    for (auto& r : ex->reloads)
      if (r.handle == h) HIP_TRY(hipStreamWaitEvent((hipStream_t)stream, r.done, 0));
    auto it = ex->last_use.find(user_id);
    if (it != ex->last_use.end()) it->second = ++ex->clock;
    ex->stats[0] += 1;
    *out = h;
    if (source) *source = 0;
    return RELAYGR_OK;
  }
  relaygr_kv_handle dh;                                      // level 2: server-local DRAM
  PoolEntry slot;
  if (!ex->arena || ex->dram.lookup(user_id, &dh) != RELAYGR_OK || ex->dram.resolve(dh, &slot) != RELAYGR_OK) {
    ex->stats[2] += 1;
    return fail(RELAYGR_ENOENT, "expander_lookup: user %llu is in neither tier", (unsigned long long)user_id);
  }
  if ((int)ex->reloads.size() >= ex->max_inflight) { ex->stats[3] += 1; return fail(RELAYGR_EBUSY, "expander_lookup: %d reloads already in flight", ex->max_inflight); }
  const double image_bytes = (double)slot.npages * (double)page_bytes(ex->hbm);
  if (ex->rate_bps > 0.0) {
    const auto now = std::chrono::steady_clock::now();
    ex->tokens = std::min(ex->burst_bytes, ex->tokens + std::chrono::duration<double>(now - ex->refilled).count() * ex->rate_bps);
    ex->refilled = now;
    // an image larger than the bucket goes through when the bucket is full; the debt it leaves is paid off first
    if (ex->tokens < std::min(image_bytes, ex->burst_bytes)) {
      ex->stats[3] += 1;
      return fail(RELAYGR_EBUSY, "expander_lookup: reload rate limit (%.0f bytes/s) reached", ex->rate_bps);
    }
  }
  int rc = alloc_in_window(ex, user_id, slot.prefix_len, &h);
  if (rc != RELAYGR_OK) return fail(rc, "expander_lookup: no free or reclaimable extent to reload %d tokens", slot.prefix_len);
  PoolEntry e;
  ex->hbm->resolve(h, &e);
  hipEvent_t done = get_event(ex);
  if (!done) { ex->hbm->release(h); return fail(RELAYGR_EHIP, "expander_lookup: cannot create an event"); }
  // a spill into these arena pages that is still in flight (this image's own, most likely) finishes first;
  // spills of other pages, and whatever ranking streams they wait for, do not hold the reload up
  hipError_t he = hipSuccess;
  for (auto& pf : ex->pending_free)
    if (he == hipSuccess && overlap(slot.page0, slot.npages, pf.dram_page0, pf.dram_pages)) he = hipStreamWaitEvent(ex->reload_stream, pf.spilled, 0);
  if (he == hipSuccess)
    he = hipMemcpyAsync(extent_ptr(ex->hbm, e), extent_ptr(&ex->dram, slot), (size_t)slot.npages * page_bytes(ex->hbm),
                        hipMemcpyHostToDevice, ex->reload_stream);
  if (he != hipSuccess) { ex->hbm->release(h); ex->spare_events.push_back(done); return fail(RELAYGR_EHIP, "expander_lookup: %s", hipGetErrorString(he)); }
  HIP_TRY(hipEventRecord(done, ex->reload_stream));
  HIP_TRY(hipStreamWaitEvent((hipStream_t)stream, done, 0));
  ex->reloads.push_back({h, done, slot.page0, slot.npages});
  if (ex->rate_bps > 0.0) ex->tokens -= image_bytes;
  ex->last_use[user_id] = ++ex->clock;
  ex->stats[1] += 1;
  *out = h;
  if (source) *source = 1;
  return RELAYGR_OK;
}

extern "C" int relaygr_expander_alloc(relaygr_expander* ex, uint64_t user_id, int32_t prefix_len, relaygr_kv_handle* out) {
  if (!ex || !out) return fail(RELAYGR_EINVAL, "expander_alloc: null argument");
  *out = RELAYGR_NO_CACHE;
  std::lock_guard<std::mutex> lk(ex->mu);
  poll(ex);
  // a reclaimable entry of the same user is superseded by the new pre-inference
  relaygr_kv_handle old;
  if (ex->hbm->lookup(user_id, &old) == RELAYGR_OK) {
    auto it = std::find(ex->reclaimable.begin(), ex->reclaimable.end(), old);
    if (it == ex->reclaimable.end()) return fail(RELAYGR_EINVAL, "expander_alloc: user %llu already has a live entry", (unsigned long long)user_id);
    ex->reclaimable.erase(it);
    ex->hbm->release(old);
    ex->hbm_evictions += 1;
  }
  int rc = alloc_in_window(ex, user_id, prefix_len, out);
  if (rc == RELAYGR_ENOSPC) return fail(rc, "expander_alloc: live entries leave no extent for %d tokens", prefix_len);
  if (rc != RELAYGR_OK) return fail(rc, "expander_alloc: prefix_len < 1");
  return RELAYGR_OK;
}

extern "C" int relaygr_expander_set_reload_rate(relaygr_expander* ex, double bytes_per_second, double burst_bytes) {
  if (!ex || !(bytes_per_second >= 0.0) || !(burst_bytes >= 0.0) || (bytes_per_second > 0.0 && !(burst_bytes > 0.0)))
    return fail(RELAYGR_EINVAL, "expander_set_reload_rate: null expander, negative rate, or a rate without a burst size");
  std::lock_guard<std::mutex> lk(ex->mu);
  ex->rate_bps = bytes_per_second;
  ex->burst_bytes = burst_bytes;
  ex->tokens = burst_bytes;
  ex->refilled = std::chrono::steady_clock::now();
  return RELAYGR_OK;
}

extern "C" int relaygr_expander_trim(relaygr_expander* ex, int32_t keep) {
  if (!ex || keep < 0) return fail(RELAYGR_EINVAL, "expander_trim: null expander or keep < 0");
  std::lock_guard<std::mutex> lk(ex->mu);
  poll(ex);
  while ((int64_t)ex->reclaimable.size() > keep) {
    relaygr_kv_handle v = ex->reclaimable.front();
    ex->reclaimable.pop_front();
    if (ex->hbm->release(v) == RELAYGR_OK) ex->hbm_evictions += 1;
  }
  return RELAYGR_OK;
}

extern "C" int relaygr_expander_stats(relaygr_expander* ex, int64_t stats[10]) {
  if (!ex || !stats) return fail(RELAYGR_EINVAL, "expander_stats: null argument");
  std::lock_guard<std::mutex> lk(ex->mu);
  poll(ex);
  for (int i = 0; i < 6; ++i) stats[i] = ex->stats[i];
  int64_t total = 0, free_pages = 0, live = 0;
  ex->dram.stats(&total, &free_pages, &live, nullptr);
  stats[6] = (total - free_pages) * (int64_t)page_bytes(ex->hbm);
  stats[7] = live;
  stats[8] = ex->hbm_evictions;
  stats[9] = (int64_t)ex->reclaimable.size();
  return RELAYGR_OK;
}
