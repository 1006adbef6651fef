// Host-side allocator of the HBM pool of psi objects (Section 3.3, "HBM as a lifecycle window":
// entries are inserted by pre-inference, consumed by ranking and released as new users arrive).
// A user's psi is one contiguous extent of pages in a caller-owned device slab; the allocator is
// first-fit over an address-ordered free list with coalescing.  It never evicts by itself
// (invariant I2 of Section 3.1: the live footprint is capped, a live cache is never silently
// dropped): when nothing fits, the caller is told so.
#pragma once

#include <stdint.h>

#include <map>
#include <mutex>
#include <unordered_map>
#include <vector>

#include "../../include/relaygr.h"

namespace relaygr {

struct PoolEntry {
  uint32_t generation = 0;
  bool live = false;
  uint64_t user_id = 0;
  int64_t page0 = 0;
  int64_t npages = 0;
  int32_t prefix_len = 0;
};

struct KvPool {
  relaygr_model_config cfg;
  void* slab = nullptr;
  size_t slab_bytes = 0;
  int32_t page_tokens = 0;
  int64_t n_pages = 0;
  int64_t tile_stride = 0;    // elements per 64-token tile block (all layers)
  int64_t layer_stride = 0;   // elements per layer inside a tile block
  std::mutex mu;
  std::map<int64_t, int64_t> free_extents;   // first page -> page count
  std::vector<PoolEntry> entries;
  std::vector<uint32_t> free_slots;
  std::unordered_map<uint64_t, uint32_t> by_user;

  // All four return RELAYGR_* codes and are thread-safe.
  int alloc(uint64_t user_id, int32_t prefix_len, relaygr_kv_handle* out);
  int release(relaygr_kv_handle h);
  int lookup(uint64_t user_id, relaygr_kv_handle* out);
  // Copies the live entry of h into *e (RELAYGR_ENOENT if stale).
  int resolve(relaygr_kv_handle h, PoolEntry* e);
  void stats(int64_t* total, int64_t* free_pages, int64_t* live, int64_t* largest);
};

inline int elem_bytes(const relaygr_model_config& c) { return c.dtype == RELAYGR_DTYPE_FP32 ? 4 : 2; }

}  // namespace relaygr
