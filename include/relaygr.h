/*
 * relaygr.h -- C ABI of the relay-race ranking hot path on one MI355X (gfx950).
 *
 * The paper (arXiv 2601.01712) splits ranking-model inference for a user with a
 * long behaviour history in two (Section 2.3, the relay-race identity; Section
 * 3.1, "Cache object"; Section 3.2, "Concurrency inside a special instance"):
 *
 *   pre-infer   run the backbone over the long-term prefix alone and leave psi,
 *               the per-layer K/V of that prefix, in HBM under the user's id;
 *   rank        later, look psi up by user id and run only the incremental
 *               tokens (short-term suffix, candidates) against it; if psi is
 *               absent, fall back to full inference (Section 3.1, invariant I1;
 *               Section 3.3).
 *
 * This library is that instance-side path: an HBM pool of psi objects, prefix
 * pre-inference into the pool, ranking with the cached prefix, and full
 * recompute.  The model is an HSTU-style backbone with a scalar score head; per
 * user the sequence is [prefix p_0..p_{L-1} | suffix s_0..s_{S-1} | candidates
 * c_0..c_{M-1}] and token i may attend to key j iff j <= i and j is not another
 * candidate.  Per layer:
 *
 *     xh = LN(x; g_in, b_in)                      [u|v|q|k] = SiLU(xh W1^T + b1)
 *     o_i^h = (1/n_i) sum_j m_ij SiLU(<q_i^h,k_j^h>/sqrt(d_head)) v_j^h
 *     x  <- x + (LN(o; g_at, b_at) * u) W2^T + b2
 *     score_c = <w_s, LN(x_c; g_out, b_out)> + b_s        (candidate rows, after the last layer)
 *
 * with n_i the number of keys row i may see, LN the LayerNorm with biased
 * variance and SiLU(t) = t / (1 + exp(-t)).
 *
 * Conventions
 *   - Plain C types only.  "device" pointers are HIP device addresses on the
 *     current device; "host" pointers are ordinary process memory.
 *   - The caller owns every device buffer (weights, embeddings, the pool slab,
 *     the scratch buffer, the score output).  The library allocates no device
 *     memory; it owns host-side metadata and, per context, a small pinned staging
 *     area allocated in relaygr_ctx_create (no compute call allocates or frees).
 *   - Compute calls enqueue work on the given HIP stream and return without
 *     synchronising the device or the stream.  One bounded host wait exists: a
 *     call's batch descriptors go through a ring of four pinned staging slots, so
 *     the fifth call in a row waits until the upload of the first has completed
 *     (microseconds once the stream has reached it).  Buffers passed to a call
 *     must stay valid and unmodified until that stream has passed the call's work.  A context is one model slot:
 *     its calls share its scratch buffer and staging area, so they run one after the other on the GPU: a call
 *     given another stream than the context's previous call is made to wait for the work that stream holds at
 *     that moment (an event, no host wait; if that stream has been destroyed meanwhile, the device is
 *     synchronised instead; a stream under graph capture is left alone), and host threads calling
 *     with one context enqueue one at a time (the profiling calls of a context are not synchronised with
 *     them); several contexts may share one pool, whose calls (and the expander's and trigger's) are thread-safe.
 *   - Every function returning int returns RELAYGR_OK or a negative code; the
 *     text of the last failure on the calling thread is relaygr_last_error().
 *   - dtype selects storage AND arithmetic: RELAYGR_DTYPE_FP32 keeps everything
 *     in fp32; RELAYGR_DTYPE_BF16 and RELAYGR_DTYPE_FP16 store weights, embeddings,
 *     activations and cached K/V as bfloat16 / IEEE half and accumulate, normalise and
 *     keep the residual stream in fp32 (fp16 is the half precision the paper mentions,
 *     Section 4.2; values beyond its range of 65504 are the caller's concern).  Scores
 *     are always fp32.
 *   - Constraints checked at context creation: d_model in {64, 128, 256, 512, 1024}
 *     (bf16, fp16: at least 128); d_head = d_model / n_heads in {32, 64, 128} and at least
 *     d_model / 64.
 *   - In the 16-bit modes the first bytes of the scratch buffer hold the weights re-packed
 *     for the matrix cores (done once in relaygr_ctx_create, which synchronises the
 *     device); relaygr_scratch_bytes includes them.
 */
#ifndef RELAYGR_H
#define RELAYGR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define RELAYGR_OK       0
#define RELAYGR_EINVAL  (-1)  /* null pointer, bad shape, offsets not monotone, unsupported config */
#define RELAYGR_ENOSPC  (-2)  /* pool has no free extent of the needed size / scratch too small  */
#define RELAYGR_ENOENT  (-3)  /* unknown user id, or stale / freed handle                        */
#define RELAYGR_EHIP    (-4)  /* a HIP runtime call failed; see relaygr_last_error()             */

#define RELAYGR_DTYPE_FP32 0
#define RELAYGR_DTYPE_BF16 1
#define RELAYGR_DTYPE_FP16 2

#define RELAYGR_TILE_TOKENS 64   /* cached K/V are laid out in tiles of 64 tokens */

typedef struct relaygr_ctx     relaygr_ctx;      /* model view + scratch plan (opaque)         */
typedef struct relaygr_kv_pool relaygr_kv_pool;  /* extent allocator over a caller slab (opaque) */

/* Handle of one user's psi in a pool: (generation << 32) | (slot + 1).  0 means "no cache". */
typedef uint64_t relaygr_kv_handle;
#define RELAYGR_NO_CACHE ((relaygr_kv_handle)0)

typedef struct {
  int32_t n_layers;
  int32_t d_model;
  int32_t n_heads;
  int32_t dtype;     /* RELAYGR_DTYPE_* */
  float   ln_eps;    /* LayerNorm epsilon, e.g. 1e-5 */
} relaygr_model_config;

/* One layer's parameters, all DEVICE pointers in the storage dtype.
 * w1 is [4*d_model, d_model] row-major, output-major (y = x W1^T + b1), its output rows
 * ordered u | v | q | k (four blocks of d_model).  w2 is [d_model, d_model], output-major. */
typedef struct {
  const void *ln_in_g, *ln_in_b;   /* [d_model] */
  const void *w1, *b1;             /* [4d, d], [4d] */
  const void *ln_at_g, *ln_at_b;   /* [d_model] */
  const void *w2, *b2;             /* [d, d], [d] */
} relaygr_layer_weights;

typedef struct {
  const relaygr_layer_weights* layers;  /* HOST array of n_layers entries (copied at create) */
  const void *ln_out_g, *ln_out_b;      /* device [d_model] */
  const void *w_score;                  /* device [d_model] */
  float b_score;
} relaygr_weights;

/* One jagged batch of users.  Offsets are HOST int32 arrays of n_users + 1 monotone entries
 * starting at 0; embeddings are DEVICE arrays [rows, d_model] in the storage dtype, users
 * concatenated in order.  A segment a call does not need may be null with null offsets
 * (treated as all-empty). */
typedef struct {
  int32_t n_users;
  const uint64_t* user_ids;            /* host [n_users]; informational (may be null) */
  const relaygr_kv_handle* handles;    /* host [n_users]; see each call */
  const void* prefix_emb; const int32_t* prefix_off;   /* [sum L, d] */
  const void* suffix_emb; const int32_t* suffix_off;   /* [sum S, d] */
  const void* cand_emb;   const int32_t* cand_off;     /* [sum M, d] */
} relaygr_batch;

/* ---- sizes -------------------------------------------------------------------------- */

/* Exact bytes of psi for one user: 2 (K and V) * n_layers * prefix_len * d_model * element size
 * (Section 4.1 "Cache semantics": 2K tokens, 8 layers, d 256, fp32 -> 32 MB).  0 on bad input. */
size_t relaygr_kv_footprint_bytes(const relaygr_model_config* cfg, int32_t prefix_len);

/* Bytes the same psi occupies in a pool whose pages hold page_tokens tokens (page-rounded). */
size_t relaygr_kv_pool_bytes_for(const relaygr_model_config* cfg, int32_t prefix_len, int32_t page_tokens);

/* Scratch bytes a context needs so that any single call may carry up to max_users users,
 * max_prefix_tokens prefix tokens that must be COMPUTED in that call (prefill, full recompute,
 * uncached users) and max_new_tokens suffix + candidate tokens.  0 on bad input. */
size_t relaygr_scratch_bytes(const relaygr_model_config* cfg, int32_t max_users,
                             int64_t max_prefix_tokens, int64_t max_new_tokens);

/* ---- context ------------------------------------------------------------------------ */

/* Binds a model (config + device weights) to a caller-owned device scratch buffer of
 * scratch_bytes (256-byte aligned).  Weight memory is referenced (biases, LayerNorm and
 * score-head parameters are read from it on every call), so it must outlive the context.
 * The pinned staging for batch descriptors is sized here from scratch_bytes (what a call that fits
 * the buffer can need); a call with more users or row tiles than that is RELAYGR_ENOSPC. */
int  relaygr_ctx_create(const relaygr_model_config* cfg, const relaygr_weights* weights,
                        void* scratch_dev, size_t scratch_bytes, relaygr_ctx** out);
void relaygr_ctx_destroy(relaygr_ctx* ctx);

/* Attention form of a context's backbone.  The paper evaluates a second backbone that differs
 * from the first only in its attention computation (Section 4.4) and gives no formula for it;
 * this library's reading of it is a softmax over the visible keys,
 *   o_i^h = sum_j m_ij exp(alpha <q_i^h, k_j^h>) v_j^h / sum_j m_ij exp(alpha <q_i^h, k_j^h>),
 * in place of sum_j m_ij SiLU(alpha <q_i^h, k_j^h>) v_j^h / n_i; projections, visibility, gate,
 * residual, score head and therefore the cached K/V layout are the same.  A new context uses
 * RELAYGR_ATTN_SILU.  The form holds for every later call on the context; psi written under
 * one form is not meaningful under the other (layers above the first see different inputs).
 * Rows attend in fp32 with a running maximum, so large scores do not overflow.
 * Returns RELAYGR_EINVAL for a null context or an unknown form. */
#define RELAYGR_ATTN_SILU    0
#define RELAYGR_ATTN_SOFTMAX 1
int  relaygr_ctx_set_attention(relaygr_ctx* ctx, int32_t form);

/* ---- HBM pool of psi objects (Section 3.3, "HBM as a lifecycle window") -------------- */

/* Creates an allocator over slab_dev (device, 256-byte aligned, slab_bytes long) for models of
 * shape cfg.  A page holds page_tokens tokens (a multiple of 64) of every layer's K and V:
 * 2 * n_layers * page_tokens * d_model * element size bytes.  A user's psi is one contiguous
 * extent of pages.  The pool never evicts: when no extent fits, alloc says RELAYGR_ENOSPC and the
 * caller frees consumed entries or ranks that user by full recompute (invariant I2). */
int  relaygr_kv_pool_create(const relaygr_model_config* cfg, void* slab_dev, size_t slab_bytes,
                            int32_t page_tokens, relaygr_kv_pool** out);
void relaygr_kv_pool_destroy(relaygr_kv_pool* pool);

/* Reserves space for a prefix of prefix_len >= 1 tokens under user_id and returns its handle.
 * A user id holds at most one live entry: allocating again for a live id is RELAYGR_EINVAL.
 * The entry's contents are undefined until relaygr_prefill_prefix has run for it. */
int  relaygr_kv_pool_alloc(relaygr_kv_pool* pool, uint64_t user_id, int32_t prefix_len,
                           relaygr_kv_handle* out);
/* Releases an entry.  RELAYGR_ENOENT if the handle is stale or was never issued.  The caller
 * must not free an entry that enqueued work still reads. */
int  relaygr_kv_pool_free(relaygr_kv_pool* pool, relaygr_kv_handle handle);
/* Finds the live entry of user_id.  RELAYGR_ENOENT (and *out = RELAYGR_NO_CACHE) if there is none:
 * the caller then ranks that user without a cache. */
int  relaygr_kv_pool_lookup(relaygr_kv_pool* pool, uint64_t user_id, relaygr_kv_handle* out);
/* prefix_len of a live handle into *prefix_len; RELAYGR_ENOENT if stale. */
int  relaygr_kv_pool_entry_len(relaygr_kv_pool* pool, relaygr_kv_handle handle, int32_t* prefix_len);
/* Pool occupancy: total pages, free pages, live entries, largest free extent in pages. */
int  relaygr_kv_pool_stats(relaygr_kv_pool* pool, int64_t* pages_total, int64_t* pages_free,
                           int64_t* live_entries, int64_t* largest_free_extent);
/* Where one cached element lives, in ELEMENTS from the start of the slab: K of (layer, token,
 * feature) at *k_index; V of the same at *v_index.  For inspection and tests. */
int  relaygr_kv_pool_locate(relaygr_kv_pool* pool, relaygr_kv_handle handle, int32_t layer,
                            int32_t token, int32_t feature, int64_t* k_index, int64_t* v_index);

/* ---- compute (Section 3.2: the instance dispatches on the request's stage) ------------ */

/* stage = pre-infer.  For every user of the batch: run the backbone over prefix_emb rows of that
 * user and write every layer's K and V into the pool entry handles[u], whose length must equal
 * the user's prefix length.  Suffix and candidate segments are ignored.  No output besides the
 * pool contents.  RELAYGR_ENOENT if a handle is stale, RELAYGR_ENOSPC if scratch is too small,
 * RELAYGR_EINVAL if two users of the batch carry the same handle (nothing is enqueued). */
int  relaygr_prefill_prefix(relaygr_ctx* ctx, relaygr_kv_pool* pool, const relaygr_batch* batch,
                            void* hip_stream);

/* stage = rank.  Scores every candidate of every user into scores_dev (device float32
 * [sum M], candidate order, users concatenated by cand_off).  A user with a live handle runs only
 * its suffix and candidate tokens against the cached prefix (prefix_emb rows of that user are not
 * read, but prefix_off must still give the prefix length, which must equal the entry's).  A user
 * whose handle is RELAYGR_NO_CACHE is recomputed in the same call from prefix_emb (the paper's
 * miss fallback); pool may be null if every handle is RELAYGR_NO_CACHE.  A stale handle is
 * RELAYGR_ENOENT and nothing is enqueued: the caller retries with RELAYGR_NO_CACHE for that user.
 * A batch of zero users, or one without candidates, is not an error (scores_dev may then be null). */
int  relaygr_rank_with_cache(relaygr_ctx* ctx, relaygr_kv_pool* pool, const relaygr_batch* batch,
                             float* scores_dev, void* hip_stream);

/* relaygr_rank_with_cache for callers that cannot allocate device memory or bring a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and
 * same scores as relaygr_rank_with_cache, but the call's working buffers (residual stream, projections,
 * attention partial sums, row tables, batch descriptors) are laid out in a buffer that lives inside the
 * library -- RELAYGR_STATIC_SCRATCH_BYTES of device memory per GPU, held from the moment the library is
 * loaded until the process ends -- instead of in the context's scratch buffer (of which only the re-packed
 * weights at its head are read).  The call allocates and frees nothing, on the device or pinned on the host.
 * A call whose buffers do not fit (about 2000 suffix + candidate rows at d_model 512 with eight key-range
 * splits; fewer splits are tried first) is RELAYGR_ENOSPC and nothing is enqueued.  Every call on a GPU,
 * from any context, shares that GPU's buffer, which keeps the previous call's contents: work on it that
 * overlaps on one GPU races.  The library keeps its own calls apart (a call on another stream than the
 * previous one on that GPU waits for it with an event; host threads enqueue one at a time), but not what it
 * cannot see: a captured graph holding such a call must not be replayed while another call or replay on that
 * GPU may still be running -- serialise those, or give the other stream relaygr_rank_with_cache.  Nothing in
 * the buffer needs clearing between calls: every kernel writes what a later one reads. */
#define RELAYGR_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
int  relaygr_rank_with_cache_static(relaygr_ctx* ctx, relaygr_kv_pool* pool, const relaygr_batch* batch,
                                    float* scores_dev, void* hip_stream);
/* RELAYGR_STATIC_SCRATCH_BYTES as the loaded library was built. */
size_t relaygr_static_scratch_bytes(void);

/* Baseline: full inference inline for every user (Section 4.1 "Baselines"); handles are ignored
 * and no pool is touched.  Same output as relaygr_rank_with_cache. */
int  relaygr_rank_full_recompute(relaygr_ctx* ctx, const relaygr_batch* batch,
                                 float* scores_dev, void* hip_stream);

/* ---- measurement ---------------------------------------------------------------------- */

/* Kernel classes of the layer sequence, for per-kernel timing. */
#define RELAYGR_K_SETUP 0   /* row tables, tail clearing                       */
#define RELAYGR_K_LN    1   /* input LayerNorm (and first-layer gather)        */
#define RELAYGR_K_F1    2   /* u|v|q|k projection GEMM + SiLU + K/V scatter     */
#define RELAYGR_K_ATTN  3   /* pointwise-SiLU attention over the key sequence   */
#define RELAYGR_K_GATE  4   /* split combine, self term, 1/n, LayerNorm, gate   */
#define RELAYGR_K_F2    5   /* output projection GEMM + residual                */
#define RELAYGR_K_SCORE 6   /* final LayerNorm + score head                     */
#define RELAYGR_K_COUNT 7

/* Turns per-launch timing on for the classes in class_mask (bit k = class k; 0 turns it off) and
 * clears the accumulated figures.  While on, each launch of a selected class is bracketed by a
 * pair of HIP events recorded on the call's stream. */
int  relaygr_ctx_profile_enable(relaygr_ctx* ctx, uint32_t class_mask);
/* Times the launches of every n-th compute call only (default 1: every call), counting from this
 * call on: an event pair costs a few microseconds on the stream, which a throughput measurement
 * running beside the timing should not pay on every call. */
int  relaygr_ctx_profile_sample(relaygr_ctx* ctx, int32_t every_n_calls);
/* Waits for the recorded events and returns the summed kernel time (milliseconds) and the number
 * of launches of one class since the last enable.  Synchronises with the GPU. */
int  relaygr_ctx_profile_read(relaygr_ctx* ctx, int32_t kernel_class, double* total_ms, int64_t* launches);

/* ---- DRAM tier (Section 3.4, memory-aware expander) ------------------------------------ */

/* Bytes of the pool extent holding the entry (page-rounded): the size of its spill image.  0 if stale. */
size_t relaygr_kv_pool_entry_bytes(relaygr_kv_pool* pool, relaygr_kv_handle handle);
/* Enqueues on hip_stream a copy of the entry's extent into host_dst (HOST memory, pinned for an
 * asynchronous copy; host_bytes must equal relaygr_kv_pool_entry_bytes).  The entry stays live.  The
 * image is position independent: it can be reloaded into any pool of the same model shape and page size. */
int  relaygr_kv_pool_spill(relaygr_kv_pool* pool, relaygr_kv_handle handle, void* host_dst, size_t host_bytes,
                           void* hip_stream);
/* Allocates an entry for user_id / prefix_len and enqueues on hip_stream the copy of a spill image
 * into it (the `load` step of the paper's latency breakdown).  RELAYGR_ENOSPC as for alloc. */
int  relaygr_kv_pool_reload(relaygr_kv_pool* pool, uint64_t user_id, int32_t prefix_len, const void* host_src,
                            size_t host_bytes, void* hip_stream, relaygr_kv_handle* out);

/* The expander keeps consumed psi objects in server-local DRAM for short-term reuse across requests
 * of the same user, behind a two-level lookup HBM -> DRAM.  Its DRAM is ONE pinned host arena of
 * dram_budget_bytes (rounded down to whole pool pages; 0 = no DRAM tier) allocated at creation and
 * freed at destruction; images are placed in it like entries in the pool, least recently used
 * dropped first when an image does not fit.  At most max_inflight_reloads reloads are in flight and
 * a user has at most one copy per tier.  Calls are thread-safe; copies run on two streams the expander
 * owns (default priority; one for spills, one for reloads, so that a reload never queues behind other
 * users' spills), ordered against each other and the caller's streams with events, never host waits. */
typedef struct relaygr_expander relaygr_expander;
int  relaygr_expander_create(relaygr_kv_pool* pool, size_t dram_budget_bytes, int32_t max_inflight_reloads,
                             relaygr_expander** out);
/* Waits for the expander's outstanding copies, frees its DRAM.  Pool entries stay as they are. */
void relaygr_expander_destroy(relaygr_expander* ex);
/* After ranking has consumed an entry: once hip_stream has passed this point the entry is copied to
 * DRAM on the expander's own spill stream.  When that copy has completed (observed at a later
 * expander call) the entry becomes RECLAIMABLE: it stays in HBM, still found by
 * relaygr_expander_lookup (which makes it live again), until relaygr_expander_alloc or a reload
 * needs its pages; reclaimable entries leave oldest retirement first.  The caller must not use the
 * handle in work enqueued after this call unless a later relaygr_expander_lookup returns it again.
 * RELAYGR_ENOSPC if the image cannot be placed in DRAM (the entry then becomes reclaimable without
 * an image, once hip_stream has passed this point). */
int  relaygr_expander_retire(relaygr_expander* ex, relaygr_kv_handle handle, void* hip_stream);
/* Allocation for pre-inference under the sliding-window policy (Section 3.3, "HBM as a lifecycle
 * window"): a free extent if there is one; otherwise reclaimable entries are released, oldest
 * retirement first, until the extent fits.  An entry that was never retired is never displaced:
 * RELAYGR_ENOSPC when live entries alone leave no room (Section 3.1, invariant I2).  A reclaimable
 * entry of the same user is replaced; RELAYGR_EINVAL if the user has a live one. */
int  relaygr_expander_alloc(relaygr_expander* ex, uint64_t user_id, int32_t prefix_len, relaygr_kv_handle* out);
/* Rate limit of DRAM -> HBM reloads (Section 3.4: reloads are rate-limited and scheduled with bounded
 * concurrency): a token bucket of burst_bytes refilled at bytes_per_second on the host's monotonic
 * clock.  A lookup that would reload an image is refused with RELAYGR_EBUSY while the bucket holds
 * less than the image (or less than burst_bytes, for an image larger than the bucket); an accepted
 * reload takes its bytes out, so the long-run rate holds.  bytes_per_second = 0 lifts the limit (the
 * state of a new expander).  RELAYGR_EINVAL for negative values or a rate without a burst size. */
int  relaygr_expander_set_reload_rate(relaygr_expander* ex, double bytes_per_second, double burst_bytes);
/* Releases reclaimable entries, oldest retirement first, until at most `keep` remain in HBM. */
int  relaygr_expander_trim(relaygr_expander* ex, int32_t keep);
/* The idempotent probe issued before every rank (pseudo-pre-infer): *source = 0 and the live handle if
 * psi is in HBM (a pending retire of it is cancelled; hip_stream is made to wait only if a reload of
 * this very entry is still in flight, never for other users' copies); *source = 1 if it was found in DRAM, in which
 * case an entry is allocated (as by relaygr_expander_alloc), the reload is enqueued on the expander's reload stream and hip_stream is made to wait
 * for it (no host wait); RELAYGR_ENOENT if neither tier has it (the caller ranks by full recompute
 * or pre-infers); RELAYGR_EBUSY if the limit of reloads in flight or the reload rate limit is reached
 * (the caller falls back, nothing queued). */
int  relaygr_expander_lookup(relaygr_expander* ex, uint64_t user_id, void* hip_stream, relaygr_kv_handle* out,
                             int32_t* source);
/* Counters since creation: [0] HBM hits, [1] DRAM hits (reloads), [2] misses, [3] refusals (busy),
 * [4] spills, [5] DRAM evictions, [6] DRAM bytes in use, [7] DRAM entries, [8] HBM entries released
 * by the window policy, [9] reclaimable HBM entries now. */
int  relaygr_expander_stats(relaygr_expander* ex, int64_t stats[10]);

/* ---- sequence-aware trigger, host side (Section 3.2, Eq. 1-3) --------------------------- */

typedef struct {
  double  q_m;            /* sustainable pre-infer throughput of one model slot, queries/s          */
  int32_t model_slots;    /* M: concurrent model slots of a special instance                        */
  double  kv_p99_bytes;   /* P99 footprint of psi per admitted user                                 */
  double  hbm_bytes;      /* HBM of the instance                                                    */
  double  r1;             /* fraction of HBM reserved for live caches, in (0, 1]                    */
  int32_t n_instances;    /* N: ranking instances in total                                          */
  double  r2;             /* fraction of them designated special, in (0, 1]                         */
  double  t_life_s;       /* lifecycle window: pre-infer issued -> ranking consumes psi, seconds    */
} relaygr_admission_params;

typedef struct {
  double max_live_caches;   /* Eq. 2: floor(r1 * HBM / kv_p99)                                     */
  double q_admit_hbm;       /* Eq. 1 with that bound: max_live_caches / T_life                     */
  double q_admit_compute;   /* Eq. 3, first inequality: Q_m * M                                    */
  double q_admit;           /* min of the two: admitted pre-infer rate per special instance        */
  double q_max;             /* Eq. 3, second inequality: (Q_m * M) * (r2 * N), pool-wide           */
} relaygr_admission_budget;

int    relaygr_admission_budget_compute(const relaygr_admission_params* params, relaygr_admission_budget* out);
/* floor(1000 / pre_infer_ms): queries/s one model slot sustains (the paper's Q_m estimate). */
double relaygr_slot_throughput(double pre_infer_ms);

#define RELAYGR_TRIGGER_ADMIT        1   /* send the pre-infer signal                               */
#define RELAYGR_TRIGGER_NOT_AT_RISK  0   /* short prefix: zero extra work                            */
#define RELAYGR_TRIGGER_REFUSED      2   /* at risk, but over the live-cache or rate budget          */
#define RELAYGR_EBUSY              (-5)  /* a rate / concurrency limit is reached; retry or fall back */

/* Admission gate of one special instance: a request is admitted iff its prefix has at least
 * len_threshold tokens (the metadata risk test), the live-cache count stays within max_live_caches
 * and a token bucket refilled at q_admit per second (one second deep) has a token. */
typedef struct relaygr_trigger relaygr_trigger;
int  relaygr_trigger_create(const relaygr_admission_budget* budget, int32_t len_threshold, relaygr_trigger** out);
void relaygr_trigger_destroy(relaygr_trigger* t);
/* Returns RELAYGR_TRIGGER_* (or a negative code on bad arguments).  now_s: caller's monotonic clock. */
int  relaygr_trigger_admit(relaygr_trigger* t, double now_s, int32_t prefix_len);
/* The admitted request's psi was consumed (or dropped): one live cache fewer. */
int  relaygr_trigger_release(relaygr_trigger* t);
int  relaygr_trigger_stats(relaygr_trigger* t, int64_t* live, int64_t* admitted, int64_t* refused, int64_t* not_at_risk);

/* Text of the calling thread's last failure ("" if none).  Valid until the thread's next call. */
const char* relaygr_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* RELAYGR_H */
