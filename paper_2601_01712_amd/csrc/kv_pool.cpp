#include "kv_pool.h"

namespace relaygr {

static inline bool split_handle(relaygr_kv_handle h, uint32_t* slot, uint32_t* gen) {
  uint32_t lo = (uint32_t)(h & 0xFFFFFFFFu);
  if (lo == 0) return false;
  *slot = lo - 1;
  *gen = (uint32_t)(h >> 32);
  return true;
}

int KvPool::alloc(uint64_t user_id, int32_t prefix_len, relaygr_kv_handle* out) {
  if (!out || prefix_len < 1) return RELAYGR_EINVAL;
  *out = RELAYGR_NO_CACHE;
  std::lock_guard<std::mutex> lk(mu);
  if (by_user.count(user_id)) return RELAYGR_EINVAL;
  int64_t need = ((int64_t)prefix_len + page_tokens - 1) / page_tokens;
  auto it = free_extents.begin();
  for (; it != free_extents.end(); ++it)
    if (it->second >= need) break;
  if (it == free_extents.end()) return RELAYGR_ENOSPC;
  int64_t start = it->first, len = it->second;
  free_extents.erase(it);
  if (len > need) free_extents[start + need] = len - need;
  uint32_t slot;
  if (!free_slots.empty()) { slot = free_slots.back(); free_slots.pop_back(); }
  else { slot = (uint32_t)entries.size(); entries.emplace_back(); }
  PoolEntry& e = entries[slot];
  e.generation += 1;            // a slot's handles differ across reuse, so old ones go stale
  e.live = true;
  e.user_id = user_id;
  e.page0 = start;
  e.npages = need;
  e.prefix_len = prefix_len;
  by_user[user_id] = slot;
  *out = ((uint64_t)e.generation << 32) | (uint64_t)(slot + 1);
  return RELAYGR_OK;
}

int KvPool::release(relaygr_kv_handle h) {
  uint32_t slot, gen;
  if (!split_handle(h, &slot, &gen)) return RELAYGR_ENOENT;
  std::lock_guard<std::mutex> lk(mu);
  if (slot >= entries.size()) return RELAYGR_ENOENT;
  PoolEntry& e = entries[slot];
  if (!e.live || e.generation != gen) return RELAYGR_ENOENT;
  e.live = false;
  by_user.erase(e.user_id);
  free_slots.push_back(slot);
  // return the extent, merging with its address neighbours
  int64_t start = e.page0, len = e.npages;
  auto next = free_extents.lower_bound(start);
  if (next != free_extents.begin()) {
    auto prev = std::prev(next);
    if (prev->first + prev->second == start) { start = prev->first; len += prev->second; free_extents.erase(prev); }
  }
  if (next != free_extents.end() && start + len == next->first) { len += next->second; free_extents.erase(next); }
  free_extents[start] = len;
  return RELAYGR_OK;
}

int KvPool::lookup(uint64_t user_id, relaygr_kv_handle* out) {
  if (!out) return RELAYGR_EINVAL;
  *out = RELAYGR_NO_CACHE;
  std::lock_guard<std::mutex> lk(mu);
  auto it = by_user.find(user_id);
  if (it == by_user.end()) return RELAYGR_ENOENT;
  const PoolEntry& e = entries[it->second];
  *out = ((uint64_t)e.generation << 32) | (uint64_t)(it->second + 1);
  return RELAYGR_OK;
}

int KvPool::resolve(relaygr_kv_handle h, PoolEntry* out) {
  uint32_t slot, gen;
  if (!split_handle(h, &slot, &gen)) return RELAYGR_ENOENT;
  std::lock_guard<std::mutex> lk(mu);
  if (slot >= entries.size()) return RELAYGR_ENOENT;
  const PoolEntry& e = entries[slot];
  if (!e.live || e.generation != gen) return RELAYGR_ENOENT;
  *out = e;
  return RELAYGR_OK;
}

void KvPool::stats(int64_t* total, int64_t* free_pages, int64_t* live, int64_t* largest) {
  std::lock_guard<std::mutex> lk(mu);
  int64_t f = 0, big = 0;
  for (auto& kv : free_extents) { f += kv.second; if (kv.second > big) big = kv.second; }
  if (total) *total = n_pages;
  if (free_pages) *free_pages = f;
  if (live) *live = (int64_t)by_user.size();
  if (largest) *largest = big;
}

}  // namespace relaygr
