// C-ABI entry points and the host side of the relay-race path: validation, the per-call row
// plan, scratch carving and the fixed kernel sequence of a layer.  Declarations and argument
// contracts are in include/relaygr.h.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <type_traits>
#include <vector>

#include "../../include/relaygr.h"
#include "attention.h"
#include "common.h"
#include "errors.h"
#include "gemm.h"
#include "gemm_bf16.h"
#include "kv_pool.h"
#include "rowwise.h"

using namespace relaygr;

// ---- errors -----------------------------------------------------------------------------------
static thread_local char g_err[512] = "";

int relaygr::fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

#define HIP_TRY(expr)                                                                          \
  do {                                                                                         \
    hipError_t e_ = (expr);                                                                    \
    if (e_ != hipSuccess) return fail(RELAYGR_EHIP, "%s: %s", #expr, hipGetErrorString(e_));   \
  } while (0)

#define LAUNCH_CHECK(name)                                                                     \
  do {                                                                                         \
    hipError_t e_ = hipGetLastError();                                                         \
    if (e_ != hipSuccess) return fail(RELAYGR_EHIP, "launch %s: %s", name, hipGetErrorString(e_)); \
  } while (0)

extern "C" const char* relaygr_last_error(void) { return g_err; }

// ---- config -----------------------------------------------------------------------------------
static inline bool is_half16(const relaygr_model_config& c) { return c.dtype == RELAYGR_DTYPE_BF16 || c.dtype == RELAYGR_DTYPE_FP16; }

static bool config_ok(const relaygr_model_config* c) {
  if (!c) return false;
  if (c->n_layers < 1 || c->n_heads < 1 || c->d_model < 64) return false;
  if (c->dtype != RELAYGR_DTYPE_FP32 && c->dtype != RELAYGR_DTYPE_BF16 && c->dtype != RELAYGR_DTYPE_FP16) return false;
  int d = c->d_model;
  if (d != 64 && d != 128 && d != 256 && d != 512 && d != 1024) return false;
  if (d % c->n_heads) return false;
  int dh = d / c->n_heads;
  if (dh != 32 && dh != 64 && dh != 128) return false;
  if (dh < d / 64) return false;                       // a head must span at least one lane in row-wise kernels
  if (is_half16(*c) && d < 128) return false;  // the MFMA GEMM tiles 128 output columns
  if (!(c->ln_eps > 0.f)) return false;
  return true;
}

static inline size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

extern "C" size_t relaygr_kv_footprint_bytes(const relaygr_model_config* cfg, int32_t prefix_len) {
  if (!config_ok(cfg) || prefix_len < 0) return 0;
  return (size_t)2 * cfg->n_layers * (size_t)prefix_len * cfg->d_model * elem_bytes(*cfg);
}

extern "C" size_t relaygr_kv_pool_bytes_for(const relaygr_model_config* cfg, int32_t prefix_len, int32_t page_tokens) {
  if (!config_ok(cfg) || prefix_len < 0 || page_tokens < kTile || page_tokens % kTile) return 0;
  size_t pages = ((size_t)prefix_len + page_tokens - 1) / page_tokens;
  return pages * (size_t)2 * cfg->n_layers * page_tokens * cfg->d_model * elem_bytes(*cfg);
}

// ---- per-call plan ----------------------------------------------------------------------------
struct Plan {
  int n_users = 0;
  int n_prows = 0, n_nrows = 0, n_rows = 0;
  int64_t sfx_tiles = 0, kvs_tiles = 0;   // suffix tiles / recomputed-prefix tiles held in scratch
  int n_tiles_new = 0, n_tiles_prefix = 0;
  int nsplit = 1;
  int gs = 1;           // key splits added inside an attention workgroup (AttnParams::gs)
  // byte offsets into scratch
  size_t off_x, off_xh, off_u, off_q, off_knew, off_vnew, off_sfx, off_kvs, off_part, off_ml, off_rows, off_blob;
  size_t blob_bytes = 0;
  size_t total = 0;
};

// Rows per attention work item: 64 (fp32), or 128 * nq for the MFMA kernel, nq in {1, 2}.
static int rows_per_attn_tile(const relaygr_model_config& c, int nq) { return c.dtype == RELAYGR_DTYPE_FP32 ? 64 : 128 * nq; }

// Lays the call's buffers out in scratch.  Everything is a function of the counts already in p.
// Bytes at the start of scratch that hold the weights re-packed into MFMA panels (bf16 only).
static size_t wpack_bytes(const relaygr_model_config& c) {
  if (!is_half16(c)) return 0;
  const size_t d = c.d_model;
  return align_up((size_t)c.n_layers * 5 * d * d * 2);
}

// Prefix rows of a user start at a multiple of this in the row space (bf16: GEMM tiles of 256 rows
// never straddle users, and 32-row MFMA blocks coincide with 32-token halves of K/V tiles).
static int prefix_row_align(const relaygr_model_config& c) { return is_half16(c) ? kPrefixRowAlign : 1; }

static void carve(const relaygr_model_config& c, Plan& p) {
  const size_t d = c.d_model, e = elem_bytes(c), R = p.n_rows;
  const size_t Rp = (R + 255) / 256 * 256;     // the bf16 GEMMs read whole 256-row tiles of xh
  size_t o = 0;   // offsets are relative to the call scratch, which follows the packed weights in a context's buffer
  auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes); return at; };
  p.off_x = take(R * d * 4);
  p.off_xh = take(Rp * d * e);
  p.off_u = take(R * d * e);
  p.off_q = take(R * d * e);
  p.off_knew = take((size_t)p.n_nrows * d * e);
  p.off_vnew = take((size_t)p.n_nrows * d * e);
  p.off_sfx = take((size_t)p.sfx_tiles * 2 * kTile * d * e);
  p.off_kvs = take((size_t)p.kvs_tiles * 2 * kTile * d * e);
  p.off_part = take((size_t)p.nsplit * R * d * 4);
  p.off_ml = take((size_t)p.nsplit * R * c.n_heads * 2 * 4);   // softmax form: (m, l) per row, head and split
  p.off_rows = take(5 * align_up(R * 4));
  size_t n_tiles = (size_t)p.n_tiles_new + p.n_tiles_prefix;
  p.blob_bytes = align_up((size_t)p.n_users * sizeof(UserDesc)) + 2 * align_up((size_t)(p.n_users + 1) * 4) +
                 align_up(n_tiles * sizeof(AttnTile));
  p.off_blob = take(p.blob_bytes);
  p.total = o;
}

// Key-range splits wanted so that the attention launch fills the chip: workgroups = tiles * heads
// * splits, as many as give every compute unit at most two (one more split and some units get a third
// workgroup, which the whole launch then waits for), never more splits than a row tile has key tiles.
static int wanted_splits(int n_tiles, int n_heads, int min_key_tiles) {
  if (n_tiles <= 0) return 1;
  int wgs = n_tiles * n_heads;
  int s = 512 / wgs;
  s = std::min(s, 8);
  s = std::min(s, std::max(1, min_key_tiles));
  return std::max(s, 1);
}

extern "C" size_t relaygr_scratch_bytes(const relaygr_model_config* cfg, int32_t max_users,
                                        int64_t max_prefix_tokens, int64_t max_new_tokens) {
  if (!config_ok(cfg) || max_users < 1 || max_prefix_tokens < 0 || max_new_tokens < 0) return 0;
  if (max_prefix_tokens + max_new_tokens >= (1ll << 31)) return 0;
  Plan p;
  p.n_users = max_users;
  int64_t padded = max_prefix_tokens + (int64_t)max_users * (prefix_row_align(*cfg) - 1);
  if (padded + max_new_tokens >= (1ll << 31)) return 0;
  p.n_prows = (int)padded;
  p.n_nrows = (int)max_new_tokens;
  p.n_rows = p.n_prows + p.n_nrows;
  p.sfx_tiles = max_new_tokens / kTile + max_users;
  p.kvs_tiles = max_prefix_tokens / kTile + max_users;
  int rpt = rows_per_attn_tile(*cfg, 1);
  p.n_tiles_new = (int)(max_new_tokens / rpt) + max_users;
  p.n_tiles_prefix = (int)(padded / rpt) + max_users;
  p.nsplit = 1;
  carve(*cfg, p);
  size_t base = wpack_bytes(*cfg) + p.total;
  // head-room so that small calls may split their key range 8 ways
  size_t small_rows = std::min<size_t>((size_t)p.n_rows, 8192);
  return base + align_up(small_rows * 7 * ((size_t)cfg->d_model * 4 + (size_t)cfg->n_heads * 8));
}

// ---- scratch that lives in the library (for callers that cannot allocate) ----------------------
// relaygr_rank_with_cache_static lays its call out here instead of in the context's buffer.  Each GPU holds
// its own copy of the array at its own address; in host code the array's name is only a stand-in, so the
// device address is looked up once per device (hipGetSymbolAddress, with that device current) and that
// pointer is what kernels, copies and fills are given.
constexpr size_t kStaticScratchBytes = RELAYGR_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_static_mu;
static char* g_static_ptr[kMaxDevices] = {};
// Calls on the shared array are kept apart on the GPU like a context's calls on its own scratch: a call on another
// stream than the last one waits for what that stream holds (order_behind; the event is created with the address).
static hipEvent_t g_static_done[kMaxDevices] = {};
static hipStream_t g_static_last_stream[kMaxDevices] = {};
static bool g_static_has_call[kMaxDevices] = {};

// Device address of `scratch` on the current device, looked up on that device's first use.
static int static_scratch(char** out, int* dev_out = nullptr) {
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(RELAYGR_EINVAL, "static scratch: device index %d out of range", dev);
  std::lock_guard<std::mutex> lk(g_static_mu);
  if (!g_static_ptr[dev]) {
    void* ptr = nullptr;
    HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return fail(RELAYGR_EHIP, "static scratch: hipGetSymbolAddress returned a null address");
    HIP_TRY(hipEventCreateWithFlags(&g_static_done[dev], hipEventDisableTiming));
    g_static_ptr[dev] = (char*)ptr;
  }
  *out = g_static_ptr[dev];
  if (dev_out) *dev_out = dev;
  return RELAYGR_OK;
}

// ---- context ----------------------------------------------------------------------------------
constexpr int kStagingSlots = 4;
struct StagingSlot {
  void* host = nullptr;
  size_t bytes = 0;
  hipEvent_t done = nullptr;
  bool pending = false;
};

struct ProfRec { int cls; hipEvent_t a, b; };

struct relaygr_ctx {
  uint32_t prof_mask = 0;
  int prof_every = 1;                   // time the launches of every n-th call only
  int64_t prof_calls = 0;
  bool prof_this_call = true;
  std::vector<ProfRec> prof_recs;       // recorded, not yet resolved
  std::vector<hipEvent_t> prof_free;    // events ready for reuse
  double prof_ms[RELAYGR_K_COUNT] = {};
  int64_t prof_n[RELAYGR_K_COUNT] = {};
  relaygr_model_config cfg;
  int attn_form = RELAYGR_ATTN_SILU;
  std::vector<relaygr_layer_weights> layers;
  const void *ln_out_g, *ln_out_b, *w_score;
  float b_score;
  char* scratch;                        // the caller's buffer: [packed weights | call scratch]
  size_t scratch_bytes;
  std::vector<const uint16_t*> w1_packed, w2_packed;   // bf16: panels at the start of scratch
  int n_cus = 256;                      // compute units of the device the context was created on
  StagingSlot staging[kStagingSlots];   // pinned, allocated once at creation
  int next_slot = 0;
  // A context's calls share its scratch, so they must not overlap on the GPU.  On one stream they cannot; a call
  // on another stream than the one before it is made to wait for what that stream holds (order_behind).
  hipEvent_t call_done = nullptr;
  hipStream_t last_stream = nullptr;
  bool has_call = false;
  std::mutex mu;                        // one host thread at a time plans and enqueues a call of this context
};

// Device memory one call lays its buffers out in (the part of a context's buffer behind the packed weights).
struct CallScratch { char* base; size_t bytes; };

extern "C" int relaygr_ctx_create(const relaygr_model_config* cfg, const relaygr_weights* w, void* scratch_dev,
                                  size_t scratch_bytes, relaygr_ctx** out) {
  if (!out) return fail(RELAYGR_EINVAL, "ctx_create: out is null");
  *out = nullptr;
  if (!config_ok(cfg)) return fail(RELAYGR_EINVAL, "ctx_create: unsupported model config");
  if (!w || !w->layers || !w->ln_out_g || !w->ln_out_b || !w->w_score) return fail(RELAYGR_EINVAL, "ctx_create: null weights");
  if (!scratch_dev || ((uintptr_t)scratch_dev & 255)) return fail(RELAYGR_EINVAL, "ctx_create: scratch null or not 256-byte aligned");
  for (int l = 0; l < cfg->n_layers; ++l) {
    const relaygr_layer_weights& lw = w->layers[l];
    if (!lw.ln_in_g || !lw.ln_in_b || !lw.w1 || !lw.b1 || !lw.ln_at_g || !lw.ln_at_b || !lw.w2 || !lw.b2)
      return fail(RELAYGR_EINVAL, "ctx_create: layer %d has a null parameter", l);
  }
  relaygr_ctx* c = new (std::nothrow) relaygr_ctx();
  if (!c) return fail(RELAYGR_EINVAL, "ctx_create: out of host memory");
  c->cfg = *cfg;
  c->layers.assign(w->layers, w->layers + cfg->n_layers);
  c->ln_out_g = w->ln_out_g; c->ln_out_b = w->ln_out_b; c->w_score = w->w_score; c->b_score = w->b_score;
  c->scratch = (char*)scratch_dev;
  c->scratch_bytes = scratch_bytes;
  {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
      c->n_cus = cus;
  }
  if (scratch_bytes < wpack_bytes(*cfg)) { delete c; return fail(RELAYGR_ENOSPC, "ctx_create: scratch smaller than the packed weights"); }
  if (is_half16(*cfg)) {
    // re-pack W1 and W2 of every layer into MFMA panels, once
    const size_t d = cfg->d_model;
    uint16_t* wp = (uint16_t*)scratch_dev;
    for (int l = 0; l < cfg->n_layers; ++l) {
      uint16_t* w1p = wp + (size_t)l * 5 * d * d;
      uint16_t* w2p = w1p + 4 * d * d;
      int c1 = (int)(4 * d * d / 8), c2 = (int)(d * d / 8);
      hipLaunchKernelGGL(pack_weight_kernel, dim3((c1 + 255) / 256), dim3(256), 0, 0, (const uint16_t*)c->layers[l].w1,
                         (uint16_t*)w1p, (int)(4 * d), (int)d);
      hipLaunchKernelGGL(pack_weight_kernel, dim3((c2 + 255) / 256), dim3(256), 0, 0, (const uint16_t*)c->layers[l].w2,
                         (uint16_t*)w2p, (int)d, (int)d);
      c->w1_packed.push_back(w1p);
      c->w2_packed.push_back(w2p);
    }
    hipError_t e = hipDeviceSynchronize();
    if (e != hipSuccess) { delete c; return fail(RELAYGR_EHIP, "ctx_create: packing weights: %s", hipGetErrorString(e)); }
  }
  // Pinned staging for the per-call descriptor blob, sized once from what the scratch buffer can hold: a call
  // has at most one row per d*4 bytes of call scratch (the residual stream alone takes that), one attention
  // work item per 64 rows plus two per user, and a buffer sized by relaygr_scratch_bytes for max_users holds
  // two K/V tiles per user; calls beyond that are refused (RELAYGR_ENOSPC), so no compute call allocates.
  {
    const size_t call_bytes = scratch_bytes - wpack_bytes(*cfg);
    const size_t d = cfg->d_model, e = elem_bytes(*cfg);
    const size_t rows_est = call_bytes / (d * 4) + 1;
    const size_t users_est = std::min<size_t>(call_bytes / (4 * kTile * d * e) + 1, 1 << 16);
    const size_t tiles_est = rows_est / 64 + 2 * users_est;
    const size_t want = align_up(users_est * sizeof(UserDesc)) + 2 * align_up((users_est + 1) * 4) + align_up(tiles_est * sizeof(AttnTile));
    for (auto& sl : c->staging) {
      hipError_t e1 = hipHostMalloc(&sl.host, want, hipHostMallocDefault);
      hipError_t e2 = e1 == hipSuccess ? hipEventCreateWithFlags(&sl.done, hipEventDisableTiming) : e1;
      if (e1 != hipSuccess || e2 != hipSuccess) {
        relaygr_ctx_destroy(c);
        return fail(RELAYGR_EHIP, "ctx_create: pinned staging of %zu bytes: %s", want, hipGetErrorString(e1 != hipSuccess ? e1 : e2));
      }
      sl.bytes = want;
    }
  }
  {
    hipError_t e = hipEventCreateWithFlags(&c->call_done, hipEventDisableTiming);
    if (e != hipSuccess) { relaygr_ctx_destroy(c); return fail(RELAYGR_EHIP, "ctx_create: event: %s", hipGetErrorString(e)); }
  }
  {   // set-up for relaygr_rank_with_cache_static: this device's address of the library's own scratch
    char* unused = nullptr;
    int rc = static_scratch(&unused);
    if (rc != RELAYGR_OK) { relaygr_ctx_destroy(c); return rc; }
  }
  *out = c;
  return RELAYGR_OK;
}

extern "C" int relaygr_ctx_set_attention(relaygr_ctx* c, int32_t form) {
  if (!c) return fail(RELAYGR_EINVAL, "ctx_set_attention: null context");
  if (form != RELAYGR_ATTN_SILU && form != RELAYGR_ATTN_SOFTMAX) return fail(RELAYGR_EINVAL, "ctx_set_attention: unknown form %d", form);
  c->attn_form = form;
  return RELAYGR_OK;
}

extern "C" void relaygr_ctx_destroy(relaygr_ctx* c) {
  if (!c) return;
  for (auto& r : c->prof_recs) { (void)hipEventSynchronize(r.b); (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
  for (auto e : c->prof_free) (void)hipEventDestroy(e);
  for (auto& s : c->staging) {
    if (s.done) { if (s.pending) (void)hipEventSynchronize(s.done); (void)hipEventDestroy(s.done); }
    if (s.host) (void)hipHostFree(s.host);
  }
  if (c->call_done) (void)hipEventDestroy(c->call_done);
  delete c;
}

// Pinned staging for the descriptor blob: a ring of slots allocated at context creation, each guarded by an
// event so that a slot is not rewritten while an earlier call's copy may still read it.  The only host wait of
// a compute call is here: when the upload of the call kStagingSlots calls ago has not completed yet.
static int staging_acquire(relaygr_ctx* c, size_t bytes, StagingSlot** out) {
  StagingSlot& s = c->staging[c->next_slot];
  if (s.bytes < bytes)
    return fail(RELAYGR_ENOSPC, "batch descriptors need %zu bytes of staging, the context holds %zu (sized from its scratch buffer: "
                "too many users or row tiles for one call)", bytes, s.bytes);
  c->next_slot = (c->next_slot + 1) % kStagingSlots;
  if (s.pending) { HIP_TRY(hipEventSynchronize(s.done)); s.pending = false; }
  *out = &s;
  return RELAYGR_OK;
}

// ---- per-kernel timing ------------------------------------------------------------------------
struct ProfScope {
  relaygr_ctx* c; int cls; hipStream_t st; hipEvent_t a = nullptr, b = nullptr;
  ProfScope(relaygr_ctx* c_, int cls_, hipStream_t st_) : c(c_), cls(cls_), st(st_) {
    if (!(c->prof_mask & (1u << cls)) || !c->prof_this_call) return;
    auto get = [&]() -> hipEvent_t {
      hipEvent_t e = nullptr;
      if (!c->prof_free.empty()) { e = c->prof_free.back(); c->prof_free.pop_back(); }
      else if (hipEventCreate(&e) != hipSuccess) e = nullptr;
      return e;
    };
    a = get(); b = get();
    if (a && b) (void)hipEventRecord(a, st);
  }
  ~ProfScope() {
    if (!a || !b) return;
    (void)hipEventRecord(b, st);
    c->prof_recs.push_back({cls, a, b});
  }
};

static int prof_resolve(relaygr_ctx* c) {
  for (auto& r : c->prof_recs) {
    HIP_TRY(hipEventSynchronize(r.b));
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, r.a, r.b));
    c->prof_ms[r.cls] += ms;
    c->prof_n[r.cls] += 1;
    c->prof_free.push_back(r.a);
    c->prof_free.push_back(r.b);
  }
  c->prof_recs.clear();
  return RELAYGR_OK;
}

extern "C" int relaygr_ctx_profile_enable(relaygr_ctx* c, uint32_t class_mask) {
  if (!c) return fail(RELAYGR_EINVAL, "profile_enable: null context");
  int rc = prof_resolve(c);
  if (rc != RELAYGR_OK) return rc;
  c->prof_mask = class_mask & ((1u << RELAYGR_K_COUNT) - 1);
  for (int k = 0; k < RELAYGR_K_COUNT; ++k) { c->prof_ms[k] = 0.0; c->prof_n[k] = 0; }
  return RELAYGR_OK;
}

extern "C" int relaygr_ctx_profile_sample(relaygr_ctx* c, int32_t every_n_calls) {
  if (!c || every_n_calls < 1) return fail(RELAYGR_EINVAL, "profile_sample: null context or every_n_calls < 1");
  c->prof_every = every_n_calls;
  c->prof_calls = 0;
  return RELAYGR_OK;
}

extern "C" int relaygr_ctx_profile_read(relaygr_ctx* c, int32_t cls, double* total_ms, int64_t* launches) {
  if (!c || cls < 0 || cls >= RELAYGR_K_COUNT) return fail(RELAYGR_EINVAL, "profile_read: bad argument");
  int rc = prof_resolve(c);
  if (rc != RELAYGR_OK) return rc;
  if (total_ms) *total_ms = c->prof_ms[cls];
  if (launches) *launches = c->prof_n[cls];
  return RELAYGR_OK;
}

// ---- pool ABI ---------------------------------------------------------------------------------
extern "C" int relaygr_kv_pool_create(const relaygr_model_config* cfg, void* slab_dev, size_t slab_bytes,
                                      int32_t page_tokens, relaygr_kv_pool** out) {
  if (!out) return fail(RELAYGR_EINVAL, "kv_pool_create: out is null");
  *out = nullptr;
  if (!config_ok(cfg)) return fail(RELAYGR_EINVAL, "kv_pool_create: unsupported model config");
  if (!slab_dev || ((uintptr_t)slab_dev & 255)) return fail(RELAYGR_EINVAL, "kv_pool_create: slab null or not 256-byte aligned");
  if (page_tokens < kTile || page_tokens % kTile) return fail(RELAYGR_EINVAL, "kv_pool_create: page_tokens must be a positive multiple of 64");
  size_t page_bytes = (size_t)2 * cfg->n_layers * page_tokens * cfg->d_model * elem_bytes(*cfg);
  int64_t n_pages = (int64_t)(slab_bytes / page_bytes);
  if (n_pages < 1) return fail(RELAYGR_ENOSPC, "kv_pool_create: slab smaller than one page (%zu bytes)", page_bytes);
  if (n_pages * (int64_t)page_tokens >= (1ll << 31)) return fail(RELAYGR_EINVAL, "kv_pool_create: slab holds 2^31 tokens or more");
  KvPool* p = new (std::nothrow) KvPool();
  if (!p) return fail(RELAYGR_EINVAL, "kv_pool_create: out of host memory");
  p->cfg = *cfg;
  p->slab = slab_dev;
  p->slab_bytes = slab_bytes;
  p->page_tokens = page_tokens;
  p->n_pages = n_pages;
  p->layer_stride = (int64_t)2 * kTile * cfg->d_model;
  p->tile_stride = p->layer_stride * cfg->n_layers;
  p->free_extents[0] = n_pages;
  *out = reinterpret_cast<relaygr_kv_pool*>(p);
  return RELAYGR_OK;
}

extern "C" void relaygr_kv_pool_destroy(relaygr_kv_pool* pool) { delete reinterpret_cast<KvPool*>(pool); }

extern "C" int relaygr_kv_pool_alloc(relaygr_kv_pool* pool, uint64_t user_id, int32_t prefix_len, relaygr_kv_handle* out) {
  if (!pool || !out) return fail(RELAYGR_EINVAL, "kv_pool_alloc: null argument");
  int rc = reinterpret_cast<KvPool*>(pool)->alloc(user_id, prefix_len, out);
  if (rc == RELAYGR_ENOSPC) return fail(rc, "kv_pool_alloc: no free extent for %d tokens", prefix_len);
  if (rc != RELAYGR_OK) return fail(rc, "kv_pool_alloc: prefix_len < 1 or user %llu already has a live entry", (unsigned long long)user_id);
  return rc;
}

extern "C" int relaygr_kv_pool_free(relaygr_kv_pool* pool, relaygr_kv_handle h) {
  if (!pool) return fail(RELAYGR_EINVAL, "kv_pool_free: null pool");
  int rc = reinterpret_cast<KvPool*>(pool)->release(h);
  if (rc != RELAYGR_OK) return fail(rc, "kv_pool_free: stale or unknown handle");
  return rc;
}

extern "C" int relaygr_kv_pool_lookup(relaygr_kv_pool* pool, uint64_t user_id, relaygr_kv_handle* out) {
  if (!pool || !out) return fail(RELAYGR_EINVAL, "kv_pool_lookup: null argument");
  int rc = reinterpret_cast<KvPool*>(pool)->lookup(user_id, out);
  if (rc != RELAYGR_OK) return fail(rc, "kv_pool_lookup: user %llu has no live entry", (unsigned long long)user_id);
  return rc;
}

extern "C" int relaygr_kv_pool_entry_len(relaygr_kv_pool* pool, relaygr_kv_handle h, int32_t* prefix_len) {
  if (!pool || !prefix_len) return fail(RELAYGR_EINVAL, "kv_pool_entry_len: null argument");
  PoolEntry e;
  int rc = reinterpret_cast<KvPool*>(pool)->resolve(h, &e);
  if (rc != RELAYGR_OK) return fail(rc, "kv_pool_entry_len: stale or unknown handle");
  *prefix_len = e.prefix_len;
  return RELAYGR_OK;
}

extern "C" int relaygr_kv_pool_stats(relaygr_kv_pool* pool, int64_t* total, int64_t* free_pages, int64_t* live, int64_t* largest) {
  if (!pool) return fail(RELAYGR_EINVAL, "kv_pool_stats: null pool");
  reinterpret_cast<KvPool*>(pool)->stats(total, free_pages, live, largest);
  return RELAYGR_OK;
}

extern "C" int relaygr_kv_pool_locate(relaygr_kv_pool* pool, relaygr_kv_handle h, int32_t layer, int32_t token,
                                      int32_t feature, int64_t* k_index, int64_t* v_index) {
  if (!pool || !k_index || !v_index) return fail(RELAYGR_EINVAL, "kv_pool_locate: null argument");
  KvPool* p = reinterpret_cast<KvPool*>(pool);
  PoolEntry e;
  int rc = p->resolve(h, &e);
  if (rc != RELAYGR_OK) return fail(rc, "kv_pool_locate: stale or unknown handle");
  if (layer < 0 || layer >= p->cfg.n_layers || token < 0 || token >= e.prefix_len || feature < 0 || feature >= p->cfg.d_model)
    return fail(RELAYGR_EINVAL, "kv_pool_locate: index out of range");
  int dh = p->cfg.d_model / p->cfg.n_heads;
  int head = feature / dh, f = feature % dh;
  int64_t tile = e.page0 * (p->page_tokens / kTile) + token / kTile;
  int r = token % kTile;
  int64_t base = tile * p->tile_stride + (int64_t)layer * p->layer_stride + (int64_t)head * 2 * kTile * dh;
  if (p->cfg.dtype == RELAYGR_DTYPE_FP32) {
    *k_index = base + KvLayout<float>::k_off(r, f, dh);
    *v_index = base + KvLayout<float>::v_off(r, f, dh);
  } else {
    *k_index = base + KvLayout16::k_off(r, f, dh);
    *v_index = base + KvLayout16::v_off(r, f, dh);
  }
  return RELAYGR_OK;
}

// ---- the layer sequence -----------------------------------------------------------------------
enum Mode { kPrefill, kRankCached, kRankFull };

template <typename F>
static inline bool dispatch_e(int d, F&& f) {
  switch (d / 64) {
    case 1: f(std::integral_constant<int, 1>()); return true;
    case 2: f(std::integral_constant<int, 2>()); return true;
    case 4: f(std::integral_constant<int, 4>()); return true;
    case 8: f(std::integral_constant<int, 8>()); return true;
    case 16: f(std::integral_constant<int, 16>()); return true;
  }
  return false;
}

template <typename T> struct GemmLaunch;

template <> struct GemmLaunch<float> {
  static constexpr int BM = kSgemmBM;
  template <class Epi>
  static void run(const float* A, const float* W, int K, int r0, int r1, const ColMap& cm, const Epi& epi, hipStream_t st) {
    int mt = (r1 - r0 + BM - 1) / BM;
    int total = mt * cm.nblk * (cm.d / kSgemmBN);
    hipLaunchKernelGGL((gemm_f32_kernel<Epi>), dim3(total), dim3(256), 0, st, A, W, K, r0, r1, cm, mt, epi);
  }
};

// bf16: the MFMA kernels of gemm_bf16.h take parameter blocks instead of functors
template <> struct GemmLaunch<__hip_bfloat16> {
  static constexpr int BM = 64 * kF1TM;
};
template <> struct GemmLaunch<__half> {
  static constexpr int BM = 64 * kF1TM;
};

template <typename T>
static int launch_attention(const relaygr_model_config& cfg, const AttnParams& ap, int n_tiles, int nq, bool softmax, hipStream_t st);   // ap.gs: groups per workgroup

template <bool SM>
static int launch_attention_f32(const relaygr_model_config& cfg, const AttnParams& ap, int n_tiles, hipStream_t st) {
  dim3 grid(n_tiles, cfg.n_heads, ap.nsplit);
  switch (cfg.d_model / cfg.n_heads) {
    case 32: hipLaunchKernelGGL((attn_f32_kernel<32, SM>), grid, dim3(64), 0, st, ap); break;
    case 64: hipLaunchKernelGGL((attn_f32_kernel<64, SM>), grid, dim3(64), 0, st, ap); break;
    case 128: hipLaunchKernelGGL((attn_f32_kernel<128, SM>), grid, dim3(64), 0, st, ap); break;
    default: return fail(RELAYGR_EINVAL, "attention: unsupported d_head");
  }
  LAUNCH_CHECK("attn_f32");
  return RELAYGR_OK;
}
template <>
int launch_attention<float>(const relaygr_model_config& cfg, const AttnParams& ap, int n_tiles, int, bool softmax, hipStream_t st) {
  return softmax ? launch_attention_f32<true>(cfg, ap, n_tiles, st) : launch_attention_f32<false>(cfg, ap, n_tiles, st);
}

template <typename H, bool SM>
static int launch_attention16(const relaygr_model_config& cfg, const AttnParams& ap, int n_tiles, int nq, hipStream_t st) {
  int total = n_tiles * cfg.n_heads * ap.nsplit;
  dim3 grid((total + 7) / 8 * 8);
  switch (cfg.d_model / cfg.n_heads) {
    case 32: hipLaunchKernelGGL((attn_bf16_kernel<H, 32, 1, 4, SM>), grid, dim3(256), 0, st, ap); break;
    case 64:
      if (nq == 2 && ap.gs == 2) hipLaunchKernelGGL((attn_bf16_kernel<H, 64, 2, 4, SM, 2>), grid, dim3(512), 0, st, ap);
      else if (ap.gs == 2) hipLaunchKernelGGL((attn_bf16_kernel<H, 64, 1, 4, SM, 2>), grid, dim3(512), 0, st, ap);
      else if (nq == 2) hipLaunchKernelGGL((attn_bf16_kernel<H, 64, 2, 4, SM>), grid, dim3(256), 0, st, ap);
      else hipLaunchKernelGGL((attn_bf16_kernel<H, 64, 1, 4, SM>), grid, dim3(256), 0, st, ap);
      break;
    case 128:
      if (nq == 2) hipLaunchKernelGGL((attn_bf16_kernel<H, 128, 2, 4, SM>), grid, dim3(256), 0, st, ap);
      else hipLaunchKernelGGL((attn_bf16_kernel<H, 128, 1, 4, SM>), grid, dim3(256), 0, st, ap);
      break;
    default: return fail(RELAYGR_EINVAL, "attention: unsupported d_head");
  }
  LAUNCH_CHECK("attn (16-bit)");
  return RELAYGR_OK;
}
template <>
int launch_attention<__hip_bfloat16>(const relaygr_model_config& cfg, const AttnParams& ap, int n_tiles, int nq, bool softmax, hipStream_t st) {
  return softmax ? launch_attention16<Bf16, true>(cfg, ap, n_tiles, nq, st) : launch_attention16<Bf16, false>(cfg, ap, n_tiles, nq, st);
}
template <>
int launch_attention<__half>(const relaygr_model_config& cfg, const AttnParams& ap, int n_tiles, int nq, bool softmax, hipStream_t st) {
  return softmax ? launch_attention16<F16, true>(cfg, ap, n_tiles, nq, st) : launch_attention16<F16, false>(cfg, ap, n_tiles, nq, st);
}

static int check_offsets(const int32_t* off, int n, const char* what) {
  if (!off) return RELAYGR_OK;
  if (off[0] != 0) return fail(RELAYGR_EINVAL, "%s offsets must start at 0", what);
  for (int i = 0; i < n; ++i)
    if (off[i + 1] < off[i]) return fail(RELAYGR_EINVAL, "%s offsets not monotone at user %d", what, i);
  return RELAYGR_OK;
}

template <typename T>
static int run_typed(relaygr_ctx* c, KvPool* pool, const relaygr_batch* b, Mode mode, float* scores, const CallScratch& cs, hipStream_t st) {
  const relaygr_model_config& cfg = c->cfg;
  const int d = cfg.d_model, H = cfg.n_heads, dh = d / H, NL = cfg.n_layers, n = b->n_users;
  const bool bf16 = is_half16(cfg);   // either 16-bit type: the MFMA path
  using HT = typename HalfOf<T>::type;
  const int palign = prefix_row_align(cfg);

  // -- per-user shapes and K/V sources
  std::vector<UserDesc> users(n);
  std::vector<int32_t> pstart(n + 1, 0), nstart(n + 1, 0);
  Plan p;
  p.n_users = n;
  int64_t prow = 0, nrow = 0, sfx_tiles = 0, kvs_tiles = 0;
  for (int u = 0; u < n; ++u) {
    UserDesc& ud = users[u];
    memset(&ud, 0, sizeof(ud));
    int L = b->prefix_off ? b->prefix_off[u + 1] - b->prefix_off[u] : 0;
    int S = (mode != kPrefill && b->suffix_off) ? b->suffix_off[u + 1] - b->suffix_off[u] : 0;
    int M = (mode != kPrefill && b->cand_off) ? b->cand_off[u + 1] - b->cand_off[u] : 0;
    ud.L = L; ud.S = S; ud.M = M;
    ud.prefix_src0 = b->prefix_off ? b->prefix_off[u] : 0;
    ud.suffix_src0 = b->suffix_off ? b->suffix_off[u] : 0;
    ud.cand_src0 = b->cand_off ? b->cand_off[u] : 0;
    relaygr_kv_handle h = (mode == kRankFull || !b->handles) ? RELAYGR_NO_CACHE : b->handles[u];
    bool compute_prefix;
    if (h != RELAYGR_NO_CACHE) {
      if (!pool) return fail(RELAYGR_EINVAL, "user %d has a handle but no pool was given", u);
      PoolEntry e;
      if (pool->resolve(h, &e) != RELAYGR_OK) return fail(RELAYGR_ENOENT, "user %d: stale or unknown handle", u);
      if (e.prefix_len != L) return fail(RELAYGR_EINVAL, "user %d: prefix length %d differs from the cached entry's %d", u, L, e.prefix_len);
      ud.kv = pool->slab;
      ud.kv_tile0 = e.page0 * (pool->page_tokens / kTile) * pool->tile_stride;
      ud.kv_tile_stride = pool->tile_stride;
      ud.kv_layer_stride = pool->layer_stride;
      compute_prefix = (mode == kPrefill);
    } else {
      if (mode == kPrefill) {
        if (L > 0) return fail(RELAYGR_EINVAL, "prefill: user %d has no handle", u);
        compute_prefix = false;
      } else {
        compute_prefix = L > 0;
        ud.kv_tile0 = kvs_tiles * (int64_t)(2 * kTile * d);   // pointer filled in once scratch is carved
        ud.kv_tile_stride = (int64_t)2 * kTile * d;
        ud.kv_layer_stride = 0;
        kvs_tiles += (L + kTile - 1) / kTile;
      }
    }
    pstart[u] = (int32_t)prow;
    ud.prow0 = compute_prefix ? (int32_t)prow : -1;
    if (compute_prefix) {
      if (!b->prefix_emb) return fail(RELAYGR_EINVAL, "user %d needs prefix_emb", u);
      prow += ((int64_t)L + palign - 1) / palign * palign;   // filler rows up to the next aligned start
    }
    nstart[u] = (int32_t)nrow;
    ud.nrow0 = (mode != kPrefill) ? (int32_t)nrow : -1;
    ud.sfx_tile0 = sfx_tiles * (int64_t)(2 * kTile * d);
    if (mode != kPrefill) { nrow += S + M; sfx_tiles += (S + kTile - 1) / kTile; }
    if (prow + nrow >= (1ll << 31) - 1) return fail(RELAYGR_EINVAL, "batch has 2^31 rows or more");
  }
  if (mode == kPrefill && b->handles) {   // two users writing one pool entry would race
    std::vector<relaygr_kv_handle> hs;
    for (int u = 0; u < n; ++u) if (b->handles[u] != RELAYGR_NO_CACHE) hs.push_back(b->handles[u]);
    std::sort(hs.begin(), hs.end());
    if (std::adjacent_find(hs.begin(), hs.end()) != hs.end()) return fail(RELAYGR_EINVAL, "prefill: two users of the batch carry the same handle");
  }
  pstart[n] = (int32_t)prow;
  p.n_prows = (int)prow; p.n_nrows = (int)nrow; p.n_rows = (int)(prow + nrow);
  p.sfx_tiles = sfx_tiles; p.kvs_tiles = kvs_tiles;
  for (int u = 0; u <= n; ++u) nstart[u] = (u < n ? nstart[u] : (int32_t)nrow) + p.n_prows;
  for (int u = 0; u < n; ++u) if (users[u].nrow0 >= 0) users[u].nrow0 += p.n_prows;
  if (p.n_rows == 0) return RELAYGR_OK;
  if (mode != kPrefill && nrow > 0) {
    if ((sfx_tiles > 0 && !b->suffix_emb)) return fail(RELAYGR_EINVAL, "suffix tokens present but suffix_emb is null");
    if (!b->cand_emb && b->cand_off && b->cand_off[n] > 0) return fail(RELAYGR_EINVAL, "candidates present but cand_emb is null");
    if (!scores && b->cand_off && b->cand_off[n] > 0) return fail(RELAYGR_EINVAL, "scores_dev is null");
  }

  // Rows per attention work item.  The MFMA kernel reads half as much LDS and L2 per score element
  // with 256-row items (two row blocks per wavefront); use them when that still yields at least
  // one workgroup per compute unit.
  int nq = 1;
  if (bf16 && (dh == 64 || dh == 128)) {
    int64_t items256 = 0;
    for (int u = 0; u < n; ++u) {
      if (users[u].nrow0 >= 0) items256 += (users[u].S + users[u].M + 255) / 256;
      if (users[u].prow0 >= 0) items256 += (users[u].L + 255) / 256;
    }
    if (items256 * H >= 256) nq = 2;
  }
  const int rpt = rows_per_attn_tile(cfg, nq);

  // -- attention work items: new-row tiles first (kept when the last layer skips prefix rows),
  //    each group sorted by key-tile count, longest first
  std::vector<AttnTile> tiles_new, tiles_prefix;
  int min_key_tiles = 1 << 30;
  for (int u = 0; u < n; ++u) {
    const UserDesc& ud = users[u];
    int Tn = ud.S + ud.M;
    if (ud.nrow0 >= 0)
      for (int t0 = 0; t0 < Tn; t0 += rpt) {
        AttnTile at = {u, ud.nrow0 + t0, std::min(rpt, Tn - t0), 1, t0, {0, 0, 0}};
        tiles_new.push_back(at);
        min_key_tiles = std::min(min_key_tiles, (ud.L + kTile - 1) / kTile + (ud.S + kTile - 1) / kTile);
      }
    if (ud.prow0 >= 0)
      for (int i0 = 0; i0 < ud.L; i0 += rpt) {
        AttnTile at = {u, ud.prow0 + i0, std::min(rpt, ud.L - i0), 0, i0, {0, 0, 0}};
        tiles_prefix.push_back(at);
      }
  }
  auto key_tiles = [&](const AttnTile& a) {
    const UserDesc& ud = users[a.user];
    return a.kind == 0 ? (a.pos0 + a.nrows + kTile - 1) / kTile : (ud.L + kTile - 1) / kTile + (ud.S + kTile - 1) / kTile;
  };
  auto by_cost = [&](const AttnTile& a, const AttnTile& b2) { return key_tiles(a) > key_tiles(b2); };
  std::stable_sort(tiles_new.begin(), tiles_new.end(), by_cost);
  std::stable_sort(tiles_prefix.begin(), tiles_prefix.end(), by_cost);
  p.n_tiles_new = (int)tiles_new.size();
  p.n_tiles_prefix = (int)tiles_prefix.size();
  const int n_tiles_all = p.n_tiles_new + p.n_tiles_prefix;
  if (tiles_prefix.size()) min_key_tiles = 1;   // the first causal tile has a single key tile
  if (min_key_tiles == (1 << 30)) min_key_tiles = 1;

  // -- scratch
  p.nsplit = wanted_splits(n_tiles_all, H, min_key_tiles);
  // d_head 64: two of the key splits go to the two wavefront groups of one workgroup, which add their
  // sums in LDS -- half the partial sums for the layer tail to read -- where that still gives every compute unit a
  // workgroup (with fewer, e.g. one user with 512 candidates, the attention launch itself gets 25 % slower)
  p.gs = 1;
  if (bf16 && dh == 64 && p.nsplit % 2 == 0 &&
      (int64_t)n_tiles_all * H * (p.nsplit / 2) >= c->n_cus) {
    p.gs = 2;
    p.nsplit /= 2;
  }
  carve(cfg, p);
  while (p.total > cs.bytes && p.nsplit > 1) { p.nsplit -= 1; carve(cfg, p); }
  if (p.total > cs.bytes)
    return fail(RELAYGR_ENOSPC, "scratch too small: call needs %zu bytes, %zu are available", p.total, cs.bytes);
  char* S0 = cs.base;
  float* x = (float*)(S0 + p.off_x);
  T* xh = (T*)(S0 + p.off_xh);
  T* ubuf = (T*)(S0 + p.off_u);
  T* qbuf = (T*)(S0 + p.off_q);
  T* knew = (T*)(S0 + p.off_knew);
  T* vnew = (T*)(S0 + p.off_vnew);
  T* sfx = (T*)(S0 + p.off_sfx);
  T* kvs = (T*)(S0 + p.off_kvs);
  float* part = (float*)(S0 + p.off_part);
  float* ml = (float*)(S0 + p.off_ml);
  const bool softmax = c->attn_form == RELAYGR_ATTN_SOFTMAX;
  RowTables rt;
  {
    size_t rb = align_up((size_t)p.n_rows * 4);
    char* r0 = S0 + p.off_rows;
    rt.user = (int32_t*)r0; rt.kind = (int32_t*)(r0 + rb); rt.idx = (int32_t*)(r0 + 2 * rb);
    rt.lim = (int32_t*)(r0 + 3 * rb); rt.src = (int32_t*)(r0 + 4 * rb);
  }
  for (int u = 0; u < n; ++u)
    if (!users[u].kv) users[u].kv = kvs;

  // -- descriptor blob: users | pstart | nstart | tiles(new, prefix)
  StagingSlot* slot;
  int rc = staging_acquire(c, p.blob_bytes, &slot);
  if (rc != RELAYGR_OK) return rc;
  size_t o_users = 0, o_ps = align_up((size_t)n * sizeof(UserDesc)), o_ns = o_ps + align_up((size_t)(n + 1) * 4),
         o_tiles = o_ns + align_up((size_t)(n + 1) * 4);
  char* hb = (char*)slot->host;
  memcpy(hb + o_users, users.data(), (size_t)n * sizeof(UserDesc));
  memcpy(hb + o_ps, pstart.data(), (size_t)(n + 1) * 4);
  memcpy(hb + o_ns, nstart.data(), (size_t)(n + 1) * 4);
  if (p.n_tiles_new) memcpy(hb + o_tiles, tiles_new.data(), tiles_new.size() * sizeof(AttnTile));
  if (p.n_tiles_prefix) memcpy(hb + o_tiles + tiles_new.size() * sizeof(AttnTile), tiles_prefix.data(), tiles_prefix.size() * sizeof(AttnTile));
  char* db = S0 + p.off_blob;
  HIP_TRY(hipMemcpyAsync(db, hb, p.blob_bytes, hipMemcpyHostToDevice, st));
  HIP_TRY(hipEventRecord(slot->done, st));
  slot->pending = true;
  const UserDesc* d_users = (const UserDesc*)(db + o_users);
  const int32_t* d_ps = (const int32_t*)(db + o_ps);
  const int32_t* d_ns = (const int32_t*)(db + o_ns);
  const AttnTile* d_tiles = (const AttnTile*)(db + o_tiles);

  {
  ProfScope ps(c, RELAYGR_K_SETUP, st);
  // (the row tables are built by the first layer's input LayerNorm kernel, which visits every row anyway)
  if (p.n_prows && std::is_same<T, float>::value) {   // the bf16 f1 epilogue zero-fills the ragged tail itself
    hipLaunchKernelGGL((zero_kv_tail_kernel<T>), dim3(n), dim3(256), 0, st, d_users, n, NL, H, dh);
    LAUNCH_CHECK("zero_kv_tail");
  }
  if (p.sfx_tiles) {
    hipLaunchKernelGGL((zero_suffix_tail_kernel<T>), dim3(n), dim3(256), 0, st, d_users, n, sfx, H, dh);
    LAUNCH_CHECK("zero_suffix_tail");
  }
  }

  const float alpha = 1.0f / sqrtf((float)dh);
  const float kLog2e = 1.4426950408889634f, kLn2 = 0.69314718055994531f;
  const float q_mul = bf16 ? alpha * kLog2e : 1.0f;       // what f1 multiplies q by before storing it
  const float score_mul = bf16 ? 1.0f : alpha;            // what the attention kernel still applies
  const float gate_mul = bf16 ? kLn2 : alpha;             // stored q . k  ->  alpha <q,k> for the self term
  const T* emb_p = (const T*)b->prefix_emb;
  const T* emb_s = (const T*)b->suffix_emb;
  const T* emb_c = (const T*)b->cand_emb;
  const int R = p.n_rows;
  constexpr bool kPanel = !std::is_same<T, float>::value;   // bf16: xh / y are written as MFMA panels

  // 16-bit types: one row-local kernel per layer takes everything between the attention and the next
  // layer's projections (combine, gate, output projection, residual, next input LayerNorm, score head)
  constexpr bool fuse_ln = kPanel;
  for (int l = 0; l < NL; ++l) {
    const relaygr_layer_weights& lw = c->layers[l];
    const bool last = (l == NL - 1);
    // rows whose layer output is still needed: in the last layer prefix rows only supply K and V
    const int a0 = last ? p.n_prows : 0;
    const bool have_active = a0 < R;

    // step 1: input LayerNorm (first layer also gathers the embeddings into the residual stream);
    // later layers of the fused bf16 path got it from the previous layer's output projection
    if (l == 0 || !fuse_ln) {
      ProfScope ps(c, RELAYGR_K_LN, st);
      dim3 grid((R + kRowsPerBlock - 1) / kRowsPerBlock);
      bool ok = dispatch_e(d, [&](auto e) {
        constexpr int E = decltype(e)::value;
        const RowBuild rb = {d_users, d_ps, d_ns, n, p.n_prows};
        if (l == 0)
          hipLaunchKernelGGL((ln_in_kernel<T, E, true, kPanel>), grid, dim3(256), 0, st, x, xh, (const T*)lw.ln_in_g, (const T*)lw.ln_in_b,
                             emb_p, emb_s, emb_c, rt, rb, 0, R, cfg.ln_eps);
        else if constexpr (!fuse_ln)
          hipLaunchKernelGGL((ln_in_kernel<T, E, false, kPanel>), grid, dim3(256), 0, st, x, xh, (const T*)lw.ln_in_g, (const T*)lw.ln_in_b,
                             emb_p, emb_s, emb_c, rt, rb, 0, R, cfg.ln_eps);
      });
      if (!ok) return fail(RELAYGR_EINVAL, "unsupported d_model");
      LAUNCH_CHECK("ln_in");
    }
    // step 2: projections
    ColMap all4 = {4, {0, 1, 2, 3}, d}, kv_only = {2, {1, 3, 0, 0}, d};
    auto run_f1 = [&](int r0, int r1, const ColMap& cm) {
      if constexpr (std::is_same<T, float>::value) {
        F1Epilogue<T> e1;
        e1.bias = (const T*)lw.b1; e1.u = ubuf; e1.q = qbuf; e1.knew = knew; e1.vnew = vnew; e1.sfx = sfx;
        e1.users = d_users; e1.rt = rt; e1.d = d; e1.dh = dh; e1.n_prows = p.n_prows; e1.layer = l; e1.q_mul = q_mul;
        GemmLaunch<T>::run(xh, (const T*)lw.w1, d, r0, r1, cm, e1, st);
      } else {
        F1Params fp;
        fp.A = (const uint16_t*)xh; fp.W = c->w1_packed[l]; fp.bias = (const uint16_t*)lw.b1;
        fp.u = (uint16_t*)ubuf; fp.q = (uint16_t*)qbuf; fp.knew = (uint16_t*)knew; fp.vnew = (uint16_t*)vnew; fp.sfx = (uint16_t*)sfx;
        fp.users = d_users; fp.rt = rt; fp.d = d; fp.dh = dh; fp.n_prows = p.n_prows; fp.layer = l;
        fp.row_begin = r0; fp.row_end = r1; fp.n_mtiles = (r1 - r0 + 64 * kF1TM - 1) / (64 * kF1TM);
        fp.cm = cm; fp.q_mul = q_mul; fp.stream_out = (r1 - r0) >= kF1StreamMinRows ? 1 : 0;
        // launches of a few thousand rows take the weight-stationary kernel: one persistent workgroup per compute unit,
        // (compute units / column slices) row groups, a multiple of 8 so that each XCD takes whole row groups
        const int n_slices = cm.nblk * (d / 128);
        const int n_rg = d <= 512 ? (c->n_cus / n_slices) & ~7 : 0;
        if (r1 - r0 >= kF1WsMinRows && (r0 & 63) == 0 && n_rg >= 8) {
          const dim3 grid(n_slices * n_rg);
          switch (d) {
            case 128: hipLaunchKernelGGL((f1_ws_bf16_kernel<HT, 128>), grid, dim3(512), 0, st, fp); break;
            case 256: hipLaunchKernelGGL((f1_ws_bf16_kernel<HT, 256>), grid, dim3(512), 0, st, fp); break;
            default: hipLaunchKernelGGL((f1_ws_bf16_kernel<HT, 512>), grid, dim3(512), 0, st, fp); break;
          }
          return;
        }
        if (r1 - r0 <= kF1SmallMaxRows) {       // a few hundred rows: small tiles, deep pipeline
          fp.n_mtiles = (r1 - r0 + 64 * kF1SmallTM - 1) / (64 * kF1SmallTM);
          int total = fp.n_mtiles * cm.nblk * (d / (64 * kF1TN));
          hipLaunchKernelGGL((f1_gemm_bf16_kernel<HT, kF1SmallTM, kF1SmallStages>), dim3((total + 7) / 8 * 8), dim3(256), 0, st, fp);
          return;
        }
        int total = fp.n_mtiles * cm.nblk * (d / (64 * kF1TN));
        hipLaunchKernelGGL((f1_gemm_bf16_kernel<HT, kF1TM, kF1Stages>), dim3((total + 7) / 8 * 8), dim3(256), 0, st, fp);
      }
    };
    if (last && p.n_prows) {
      ProfScope ps(c, RELAYGR_K_F1, st);
      run_f1(0, p.n_prows, kv_only);
      LAUNCH_CHECK("f1 (k,v only)");
    }
    if (have_active) {
      ProfScope ps(c, RELAYGR_K_F1, st);
      run_f1(a0, R, all4);
      LAUNCH_CHECK("f1");
    }
    if (!have_active) continue;
    // step 3: attention partial sums
    AttnParams ap;
    ap.tiles = d_tiles; ap.users = d_users; ap.rt = rt; ap.q = qbuf; ap.sfx = sfx; ap.part = part;
    ap.split_stride = (size_t)R * d; ap.nsplit = p.nsplit; ap.d = d; ap.n_heads = H; ap.layer = l; ap.score_mul = score_mul;
    ap.ml = ml; ap.ml_stride = (size_t)R * H * 2; ap.gs = p.gs;
    // 16-bit SiLU form: the attention kernel adds the candidates' own keys, so the layer tail does not read q, k, v again
    const bool self_in_attn = bf16 && !softmax;
    ap.knew = self_in_attn ? (const void*)knew : nullptr; ap.vnew = vnew; ap.n_prows = p.n_prows;
    int nt = last ? p.n_tiles_new : n_tiles_all;
    ap.n_tiles = nt;
    if (nt > 0) {
      ProfScope ps(c, RELAYGR_K_ATTN, st);
      rc = launch_attention<T>(cfg, ap, nt, nq, softmax, st);
      if (rc != RELAYGR_OK) return rc;
    }
    // softmax form: merge the key splits and the candidate's own key into the finished o (in part[0]);
    // the fused 16-bit tail kernel does this merge itself
    if constexpr (!fuse_ln) if (softmax) {
      ProfScope ps(c, RELAYGR_K_GATE, st);
      dim3 grid((R - a0 + kRowsPerBlock - 1) / kRowsPerBlock);
      dispatch_e(d, [&](auto e) {
        constexpr int E = decltype(e)::value;
        hipLaunchKernelGGL((softmax_combine_kernel<T, E>), grid, dim3(256), 0, st, part, ml, p.nsplit, (size_t)R * d, (size_t)R * H * 2,
                           qbuf, knew, vnew, rt, p.n_prows, a0, R, dh, H, bf16 ? 1.0f : alpha, bf16 ? 1.0f : kLog2e);
      });
      LAUNCH_CHECK("softmax_combine");
    }
    // steps 3-4: combine splits, self term, 1/n, LayerNorm, gate by u (part of the fused kernel below otherwise)
    if constexpr (!fuse_ln) {
      ProfScope ps(c, RELAYGR_K_GATE, st);
      dim3 grid((R - a0 + kRowsPerBlock - 1) / kRowsPerBlock);
      dispatch_e(d, [&](auto e) {
        constexpr int E = decltype(e)::value;
        hipLaunchKernelGGL((attn_gate_kernel<T, E, kPanel>), grid, dim3(256), 0, st, part, p.nsplit, (size_t)R * d, ubuf, qbuf, knew, vnew, xh,
                           (const T*)lw.ln_at_g, (const T*)lw.ln_at_b, rt, p.n_prows, a0, R, dh, gate_mul, cfg.ln_eps, softmax ? 1 : 0);
      });
      LAUNCH_CHECK("attn_gate");
    }
    // step 4: output projection and residual
    {
      ProfScope ps(c, RELAYGR_K_F2, st);
      if constexpr (std::is_same<T, float>::value) {
        F2Epilogue<T> e2;
        e2.bias = (const T*)lw.b2; e2.x = x; e2.d = d;
        ColMap one = {1, {0, 0, 0, 0}, d};
        GemmLaunch<T>::run(xh, (const T*)lw.w2, d, a0, R, one, e2, st);
      } else {
        {
          F2LnParams fp;
          fp.W = c->w2_packed[l]; fp.bias = (const uint16_t*)lw.b2; fp.x = x; fp.rt = rt;
          // the last layer of a ranking call ends in the score head instead of the next layer's LayerNorm
          const bool score_here = last && mode != kPrefill && scores != nullptr;
          fp.xh = last ? nullptr : (uint16_t*)xh;
          fp.gain = last ? (const uint16_t*)c->ln_out_g : (const uint16_t*)c->layers[l + 1].ln_in_g;
          fp.offs = last ? (const uint16_t*)c->ln_out_b : (const uint16_t*)c->layers[l + 1].ln_in_b;
          fp.w_score = (const uint16_t*)c->w_score; fp.b_score = c->b_score; fp.scores = score_here ? scores : nullptr;
          fp.row_begin = a0; fp.row_end = R; fp.eps = cfg.ln_eps;
          fp.part = part; fp.nsplit = p.nsplit; fp.split_stride = (size_t)R * d;
          fp.u = (const uint16_t*)ubuf; fp.q = self_in_attn ? nullptr : (const uint16_t*)qbuf; fp.knew = (const uint16_t*)knew; fp.vnew = (const uint16_t*)vnew;
          fp.gate_gain = (const uint16_t*)lw.ln_at_g; fp.gate_offs = (const uint16_t*)lw.ln_at_b;
          fp.n_prows = p.n_prows; fp.dh = dh; fp.qk_mul = gate_mul;
          fp.ml = softmax ? ml : nullptr; fp.ml_stride = (size_t)R * H * 2; fp.n_heads = H;
          // two row blocks per workgroup halve the passes over W2 once that still leaves every
          // compute unit two workgroups
          const int rows = R - a0;
          const bool rb2 = d <= 512 && rows >= 64 * 384;
          // a few hundred rows (one user per call): 8 rows per workgroup, so that four times as many
          // compute units share the split partial sums
          const bool vr8 = (d == 256 || d == 512) && rows <= kTailVr8MaxRows;
          const bool vr16 = (d == 256 || d == 512) && !vr8 && rows <= kTailVr16MaxRows;
          dim3 grid(vr8 ? (rows + 7) / 8 : vr16 ? (rows + 15) / 16 : (rows + (rb2 ? 63 : 31)) / (rb2 ? 64 : 32));
          auto launch_tail = [&](auto sm) {
            constexpr bool SM = decltype(sm)::value;
            switch (d) {
              case 128:
                if (rb2) hipLaunchKernelGGL((f2_ln_bf16_kernel<HT, 128, 4, 2, SM>), grid, dim3(256), 0, st, fp);
                else hipLaunchKernelGGL((f2_ln_bf16_kernel<HT, 128, 4, 1, SM>), grid, dim3(256), 0, st, fp);
                break;
              case 256:
                if (rb2) hipLaunchKernelGGL((f2_ln_bf16_kernel<HT, 256, 8, 2, SM>), grid, dim3(512), 0, st, fp);
                else if (vr8) hipLaunchKernelGGL((f2_ln_bf16_kernel<HT, 256, 8, 1, SM, 1, 8>), grid, dim3(512), 0, st, fp);
                else if (vr16) hipLaunchKernelGGL((f2_ln_bf16_kernel<HT, 256, 8, 1, SM, 1, 16>), grid, dim3(512), 0, st, fp);
                else hipLaunchKernelGGL((f2_ln_bf16_kernel<HT, 256, 8, 1, SM>), grid, dim3(512), 0, st, fp);
                break;
              case 512:
                if (rb2) hipLaunchKernelGGL((f2_ln_bf16_kernel<HT, 512, 8, 2, SM, 2>), grid, dim3(512), 0, st, fp);
                else if (vr8) hipLaunchKernelGGL((f2_ln_bf16_kernel<HT, 512, 8, 1, SM, 1, 8>), grid, dim3(512), 0, st, fp);
                else if (vr16) hipLaunchKernelGGL((f2_ln_bf16_kernel<HT, 512, 8, 1, SM, 1, 16>), grid, dim3(512), 0, st, fp);
                else hipLaunchKernelGGL((f2_ln_bf16_kernel<HT, 512, 8, 1, SM>), grid, dim3(512), 0, st, fp);
                break;
              default: hipLaunchKernelGGL((f2_ln_bf16_kernel<HT, 1024, 8, 1, SM>), grid, dim3(512), 0, st, fp); break;
            }
          };
          if (softmax) launch_tail(std::true_type());
          else launch_tail(std::false_type());
        }
      }
    }
    LAUNCH_CHECK("f2");
  }

  if constexpr (!fuse_ln) if (mode != kPrefill && p.n_nrows) {   // the fused 16-bit tail kernel has written the scores already
    ProfScope ps(c, RELAYGR_K_SCORE, st);
    dim3 grid((p.n_nrows + kRowsPerBlock - 1) / kRowsPerBlock);
    dispatch_e(d, [&](auto e) {
      constexpr int E = decltype(e)::value;
      hipLaunchKernelGGL((score_kernel<T, E>), grid, dim3(256), 0, st, x, (const T*)c->ln_out_g, (const T*)c->ln_out_b,
                         (const T*)c->w_score, c->b_score, rt, p.n_prows, R, cfg.ln_eps, scores);
    });
    LAUNCH_CHECK("score");
  }
  return RELAYGR_OK;
}

static bool stream_is_capturing(hipStream_t st) {
  hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(st, &cap) != hipSuccess) { (void)hipGetLastError(); return false; }
  return cap != hipStreamCaptureStatusNone;
}

// Makes stream `st` wait for everything enqueued so far on `prev` (the stream of the previous call on the same
// scratch): the event is recorded on `prev` only now, when a call arrives on another stream, so that calls that
// stay on one stream pay nothing.  If `prev` can no longer take an event (destroyed by its owner while its work may
// still be running) the device is synchronised instead.
static hipError_t order_behind(hipStream_t st, hipStream_t prev, hipEvent_t ev) {
  hipError_t e = hipEventRecord(ev, prev);
  if (e == hipSuccess) e = hipStreamWaitEvent(st, ev, 0);
  if (e == hipSuccess) return e;
  (void)hipGetLastError();
  return hipDeviceSynchronize();
}

static int run(relaygr_ctx* c, relaygr_kv_pool* pool, const relaygr_batch* b, Mode mode, float* scores, void* stream,
               const CallScratch* other = nullptr) {
  if (!c || !b) return fail(RELAYGR_EINVAL, "null context or batch");
  if (b->n_users < 0) return fail(RELAYGR_EINVAL, "n_users < 0");
  if (b->n_users == 0) return RELAYGR_OK;
  std::lock_guard<std::mutex> call_lock(c->mu);
  c->prof_this_call = (c->prof_calls++ % c->prof_every) == 0;
  int rc;
  if ((rc = check_offsets(b->prefix_off, b->n_users, "prefix")) != RELAYGR_OK) return rc;
  if ((rc = check_offsets(b->suffix_off, b->n_users, "suffix")) != RELAYGR_OK) return rc;
  if ((rc = check_offsets(b->cand_off, b->n_users, "candidate")) != RELAYGR_OK) return rc;
  KvPool* kp = reinterpret_cast<KvPool*>(pool);
  if (kp) {
    const relaygr_model_config &a = kp->cfg, &m = c->cfg;
    if (a.n_layers != m.n_layers || a.d_model != m.d_model || a.n_heads != m.n_heads || a.dtype != m.dtype)
      return fail(RELAYGR_EINVAL, "pool and context were created for different model shapes");
  }
  hipStream_t st = (hipStream_t)stream;
  (void)hipGetLastError();   // a failure the caller's own HIP calls left behind is not this call's: launch checks below start clean
  const size_t wp = wpack_bytes(c->cfg);
  const CallScratch own = {c->scratch + wp, c->scratch_bytes - wp};
  const CallScratch& cs = other ? *other : own;
  // (a stream under graph capture takes neither the wait nor the event: the captured work is ordered by its graph,
  // and against the context's other calls by whoever launches that graph)
  const bool capturing = stream_is_capturing(st);
  if (!capturing && c->has_call && c->last_stream != st) HIP_TRY(order_behind(st, c->last_stream, c->call_done));
  if (c->cfg.dtype == RELAYGR_DTYPE_FP32) rc = run_typed<float>(c, kp, b, mode, scores, cs, st);
  else if (c->cfg.dtype == RELAYGR_DTYPE_FP16) rc = run_typed<__half>(c, kp, b, mode, scores, cs, st);
  else rc = run_typed<__hip_bfloat16>(c, kp, b, mode, scores, cs, st);
  if (!capturing) { c->last_stream = st; c->has_call = true; }
  return rc;
}

extern "C" int relaygr_prefill_prefix(relaygr_ctx* ctx, relaygr_kv_pool* pool, const relaygr_batch* batch, void* hip_stream) {
  if (!pool) return fail(RELAYGR_EINVAL, "prefill_prefix: null pool");
  if (batch && !batch->handles) return fail(RELAYGR_EINVAL, "prefill_prefix: null handles");
  return run(ctx, pool, batch, kPrefill, nullptr, hip_stream);
}

extern "C" int relaygr_rank_with_cache(relaygr_ctx* ctx, relaygr_kv_pool* pool, const relaygr_batch* batch, float* scores_dev,
                                       void* hip_stream) {
  return run(ctx, pool, batch, kRankCached, scores_dev, hip_stream);
}

extern "C" int relaygr_rank_with_cache_static(relaygr_ctx* ctx, relaygr_kv_pool* pool, const relaygr_batch* batch, float* scores_dev,
                                              void* hip_stream) {
  char* base = nullptr;
  int dev = 0;
  int rc = static_scratch(&base, &dev);      // a table lookup after the first call on this device
  if (rc != RELAYGR_OK) return rc;
  const CallScratch cs = {base, kStaticScratchBytes};
  {
    // one caller at a time enqueues on the shared array, behind the call that used it last
    std::lock_guard<std::mutex> lk(g_static_mu);
    hipStream_t st = (hipStream_t)hip_stream;
    const bool capturing = stream_is_capturing(st);
    if (!capturing && g_static_has_call[dev] && g_static_last_stream[dev] != st) HIP_TRY(order_behind(st, g_static_last_stream[dev], g_static_done[dev]));
    rc = run(ctx, pool, batch, kRankCached, scores_dev, hip_stream, &cs);
    if (!capturing) { g_static_last_stream[dev] = st; g_static_has_call[dev] = true; }
  }
  if (rc == RELAYGR_ENOSPC)
    return fail(rc, "rank_with_cache_static: the call does not fit the library's %zu-byte scratch (%s); use relaygr_rank_with_cache",
                kStaticScratchBytes, std::string(relaygr_last_error()).c_str());
  return rc;
}

extern "C" size_t relaygr_static_scratch_bytes(void) { return kStaticScratchBytes; }

extern "C" int relaygr_rank_full_recompute(relaygr_ctx* ctx, const relaygr_batch* batch, float* scores_dev, void* hip_stream) {
  return run(ctx, nullptr, batch, kRankFull, scores_dev, hip_stream);
}
