// Row-wise kernels: row-table construction, the three LayerNorm sites, the attention
// combine + gate, and the score head.  One 64-lane wavefront owns one row of d = 64*E features;
// lane l holds features [l*E, l*E + E).
#pragma once

#include "common.h"

namespace relaygr {

constexpr int kRowsPerBlock = 4;  // wavefronts (rows) per 256-thread workgroup

// ---- row tables ------------------------------------------------------------------------------
// pstart / nstart: n_users + 1 row boundaries of the prefix rows and of the new rows.  The entry of row r:
// its user, kind, index inside the user's prefix / suffix / candidates, number of keys it sees in the
// [prefix | suffix] sequence, and its row in the caller's embedding array.
struct RowBuild {
  const UserDesc* users;
  const int32_t* pstart;
  const int32_t* nstart;
  int n_users, n_prows;
};
struct RowEntry { int user, kind, idx, lim, src; };

__device__ __forceinline__ RowEntry row_entry(const RowBuild& rb, int r) {
  const int32_t* start = (r < rb.n_prows) ? rb.pstart : rb.nstart;
  int lo = 0, hi = rb.n_users;  // find u with start[u] <= r < start[u+1]
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (start[mid] <= r) lo = mid; else hi = mid;
  }
  const UserDesc& ud = rb.users[lo];
  RowEntry e;
  e.user = lo;
  if (r < rb.n_prows) {
    e.idx = r - start[lo];
    if (e.idx < ud.L) { e.kind = kRowPrefix; e.lim = e.idx + 1; e.src = ud.prefix_src0 + e.idx; }
    else              { e.kind = kRowPad; e.lim = 0; e.src = 0; }
  } else {
    int t = r - start[lo];
    if (t < ud.S) { e.kind = kRowSuffix; e.idx = t; e.lim = ud.L + t + 1; e.src = ud.suffix_src0 + t; }
    else          { e.kind = kRowCand; e.idx = t - ud.S; e.lim = ud.L + ud.S; e.src = ud.cand_src0 + e.idx; }
  }
  return e;
}

// ---- LayerNorm helpers -----------------------------------------------------------------------
template <int E>
__device__ __forceinline__ void ln_stats(const float (&v)[E], int d, float eps, float& mean, float& rstd) {
  float s = 0.f;
#pragma unroll
  for (int e = 0; e < E; ++e) s += v[e];
  mean = wave_sum(s) / (float)d;
  float q = 0.f;
#pragma unroll
  for (int e = 0; e < E; ++e) { float c = v[e] - mean; q += c * c; }
  rstd = rsqrtf(wave_sum(q) / (float)d + eps);
}

// Writes a lane's E consecutive features [lane*E, lane*E+E) of row r, either row-major or into the
// MFMA-ordered panels the bf16 GEMM reads (E and 8 divide one another, so a lane's run never
// straddles a 16-byte fragment chunk unless it is made of whole chunks).
template <typename T, int E, bool PANEL>
__device__ __forceinline__ void store_row_run(T* __restrict__ out, int r, int lane, int d, const float (&v)[E]) {
  if (PANEL) {
    constexpr int RUN = E < 8 ? E : 8;
#pragma unroll
    for (int c = 0; c < E; c += RUN) {
      T* dst = out + panel_off(r, lane * E + c, d);
#pragma unroll
      for (int i = 0; i < RUN; ++i) Elem<T>::st(dst + i, v[c + i]);
    }
  } else {
#pragma unroll
    for (int i = 0; i < E; ++i) Elem<T>::st(out + (size_t)r * d + lane * E + i, v[i]);
  }
}

// Input LayerNorm of a layer (step 1 of a layer): xh = LN(x; g, b) in the storage type.
// With GATHER (first layer of a call) the wavefront first works out its row's table entry and writes it
// for the kernels that follow (the call's row tables are built here, not by a launch of their own), then
// fetches the row from its embedding array and also writes it to the fp32 residual stream x.
template <typename T, int E, bool GATHER, bool PANEL>
__global__ __launch_bounds__(256) void ln_in_kernel(float* __restrict__ x, T* __restrict__ xh,
                                                    const T* __restrict__ gain, const T* __restrict__ offs,
                                                    const T* __restrict__ emb_prefix, const T* __restrict__ emb_suffix,
                                                    const T* __restrict__ emb_cand, RowTables rt, RowBuild rb,
                                                    int row_begin, int row_end, float eps) {
  const int d = 64 * E;
  int r = row_begin + blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
  if (r >= row_end) return;
  int lane = threadIdx.x & 63;
  float v[E];
  int kind, src = 0;
  if (GATHER) {
    const RowEntry e = row_entry(rb, r);
    if (lane == 0) { rt.user[r] = e.user; rt.kind[r] = e.kind; rt.idx[r] = e.idx; rt.lim[r] = e.lim; rt.src[r] = e.src; }
    kind = e.kind; src = e.src;
  } else {
    kind = rt.kind[r];
  }
  if (kind == kRowPad) {   // keep filler rows finite
#pragma unroll
    for (int i = 0; i < E; ++i) v[i] = 0.f;
    store_row_run<T, E, PANEL>(xh, r, lane, d, v);
    return;
  }
  if (GATHER) {
    const T* e = (kind == kRowPrefix ? emb_prefix : kind == kRowSuffix ? emb_suffix : emb_cand) + (size_t)src * d + lane * E;
#pragma unroll
    for (int i = 0; i < E; ++i) { v[i] = Elem<T>::ld(e + i); x[(size_t)r * d + lane * E + i] = v[i]; }
  } else {
#pragma unroll
    for (int i = 0; i < E; ++i) v[i] = x[(size_t)r * d + lane * E + i];
  }
  float mean, rstd;
  ln_stats<E>(v, d, eps, mean, rstd);
#pragma unroll
  for (int i = 0; i < E; ++i) {
    int f = lane * E + i;
    v[i] = (v[i] - mean) * rstd * Elem<T>::ld(gain + f) + Elem<T>::ld(offs + f);
  }
  store_row_run<T, E, PANEL>(xh, r, lane, d, v);
}

// Attention combine + gate (steps 3-4 of a layer, everything after the key loop):
//   o_i = ( sum over key splits of the partial sums  +  self term for a candidate ) / n_i
//   y_i = LN(o_i; g_at, b_at) * u_i
// part holds nsplit unnormalised partial sums [nsplit][rows][d] of SiLU(alpha q.k) v over the key
// sequence, added here in split order (fixed order => reproducible bits).  A candidate's self
// term SiLU(alpha <q_c^h, k_c^h>) v_c^h is evaluated here from the row's own q, k, v.
// qk_mul turns the stored q into alpha*q (q may be stored pre-scaled).
// With plain_o set, part[0] already holds the finished o_i (softmax form, after
// softmax_combine_kernel): no split sum, no self term, no 1/n.
template <typename T, int E, bool PANEL>
__global__ __launch_bounds__(256) void attn_gate_kernel(const float* __restrict__ part, int nsplit, size_t split_stride,
                                                        const T* __restrict__ u, const T* __restrict__ q,
                                                        const T* __restrict__ knew, const T* __restrict__ vnew,
                                                        T* __restrict__ y, const T* __restrict__ gain,
                                                        const T* __restrict__ offs, RowTables rt, int n_prows,
                                                        int row_begin, int row_end, int dh, float qk_mul, float eps,
                                                        int plain_o) {
  const int d = 64 * E;
  int r = row_begin + blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
  if (r >= row_end) return;
  int lane = threadIdx.x & 63;
  size_t base = (size_t)r * d + lane * E;
  float o[E];
  if (plain_o) nsplit = 1;
  if (rt.kind[r] == kRowPad) {
#pragma unroll
    for (int i = 0; i < E; ++i) o[i] = 0.f;
    store_row_run<T, E, PANEL>(y, r, lane, d, o);
    return;
  }
#pragma unroll
  for (int i = 0; i < E; ++i) o[i] = 0.f;
  for (int s = 0; s < nsplit; ++s) {
#pragma unroll
    for (int i = 0; i < E; ++i) o[i] += part[s * split_stride + base + i];
  }
  int n = plain_o ? 1 : rt.lim[r];
  if (rt.kind[r] == kRowCand && !plain_o) {
    size_t nb = (size_t)(r - n_prows) * d + lane * E;
    float dot = 0.f;
#pragma unroll
    for (int i = 0; i < E; ++i) dot += Elem<T>::ld(q + base + i) * Elem<T>::ld(knew + nb + i);
    // lanes of one head are dh/E consecutive lanes (a power of two): segmented butterfly
    for (int m = (dh / E) >> 1; m > 0; m >>= 1) dot += __shfl_xor(dot, m, 64);
    float p = silu_f32(dot * qk_mul);
#pragma unroll
    for (int i = 0; i < E; ++i) o[i] += p * Elem<T>::ld(vnew + nb + i);
    n += 1;
  }
  float inv_n = 1.0f / (float)n;
#pragma unroll
  for (int i = 0; i < E; ++i) o[i] *= inv_n;
  float mean, rstd;
  ln_stats<E>(o, d, eps, mean, rstd);
#pragma unroll
  for (int i = 0; i < E; ++i) {
    int f = lane * E + i;
    float z = (o[i] - mean) * rstd * Elem<T>::ld(gain + f) + Elem<T>::ld(offs + f);
    o[i] = z * Elem<T>::ld(u + base + i);
  }
  store_row_run<T, E, PANEL>(y, r, lane, d, o);
}

// Second attention form (softmax over the visible keys): merges a row's key splits and, for a
// candidate, its own key into the finished attention output
//   o_i^h = ( sum_s w_s part_s  +  w_self v_c^h ) / ( sum_s w_s l_s + w_self ),
//   w_s = exp(m_s - M),  w_self = exp(t_self - M),  M = max(m_s, t_self),
// where split s delivered part_s = sum_j exp(t_j - m_s) v_j, l_s = sum_j exp(t_j - m_s) and m_s
// (ml holds m and l as [split][row][head][2]; m_s = -inf and l_s = 0 for a split in which the row
// sees no key).  Scores are stored scaled by 1/to_log2 relative to base-2 exponents: the fp32 path
// keeps natural-log scores (to_log2 = log2 e), the 16-bit path stores q pre-multiplied by
// alpha * log2(e) (to_log2 = 1, qk_mul = 1).  Splits are merged in fixed order.  The result
// overwrites split 0's partial sums, which the gate then reads with its plain_o flag set.
template <typename T, int E>
__global__ __launch_bounds__(256) void softmax_combine_kernel(float* __restrict__ part, const float* __restrict__ ml, int nsplit,
                                                              size_t split_stride, size_t ml_stride, const T* __restrict__ q,
                                                              const T* __restrict__ knew, const T* __restrict__ vnew, RowTables rt,
                                                              int n_prows, int row_begin, int row_end, int dh, int n_heads,
                                                              float qk_mul, float to_log2) {
  const int d = 64 * E;
  int r = row_begin + blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
  if (r >= row_end) return;
  const int kind = rt.kind[r];
  if (kind == kRowPad) return;
  int lane = threadIdx.x & 63;
  const int head = lane * E / dh;
  size_t base = (size_t)r * d + lane * E;
  const float* mlr = ml + ((size_t)r * n_heads + head) * 2;
  float M = -INFINITY;
  for (int s = 0; s < nsplit; ++s) M = fmaxf(M, mlr[s * ml_stride]);
  float tself = 0.f;
  size_t nb = 0;
  if (kind == kRowCand) {
    nb = (size_t)(r - n_prows) * d + lane * E;
    float dot = 0.f;
#pragma unroll
    for (int i = 0; i < E; ++i) dot += Elem<T>::ld(q + base + i) * Elem<T>::ld(knew + nb + i);
    for (int m = (dh / E) >> 1; m > 0; m >>= 1) dot += __shfl_xor(dot, m, 64);
    tself = dot * qk_mul;
    M = fmaxf(M, tself);
  }
  float o[E], L = 0.f;
#pragma unroll
  for (int i = 0; i < E; ++i) o[i] = 0.f;
  for (int s = 0; s < nsplit; ++s) {
    const float ms = mlr[s * ml_stride], ls = mlr[s * ml_stride + 1];
    const float w = (ms == -INFINITY) ? 0.f : exp2f((ms - M) * to_log2);
    L += w * ls;
#pragma unroll
    for (int i = 0; i < E; ++i) o[i] += w * part[s * split_stride + base + i];
  }
  if (kind == kRowCand) {
    const float w = exp2f((tself - M) * to_log2);
    L += w;
#pragma unroll
    for (int i = 0; i < E; ++i) o[i] += w * Elem<T>::ld(vnew + nb + i);
  }
  const float inv = 1.0f / L;
#pragma unroll
  for (int i = 0; i < E; ++i) part[base + i] = o[i] * inv;
}

// Score head: score_c = <w_s, LN(x_c; g_out, b_out)> + b_s for candidate rows, written at the
// candidate's position in the caller's candidate order.
template <typename T, int E>
__global__ __launch_bounds__(256) void score_kernel(const float* __restrict__ x, const T* __restrict__ gain,
                                                    const T* __restrict__ offs, const T* __restrict__ w_score,
                                                    float b_score, RowTables rt, int row_begin, int row_end,
                                                    float eps, float* __restrict__ scores) {
  const int d = 64 * E;
  int r = row_begin + blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
  if (r >= row_end) return;
  if (rt.kind[r] != kRowCand) return;
  int lane = threadIdx.x & 63;
  float v[E];
#pragma unroll
  for (int i = 0; i < E; ++i) v[i] = x[(size_t)r * d + lane * E + i];
  float mean, rstd;
  ln_stats<E>(v, d, eps, mean, rstd);
  float acc = 0.f;
#pragma unroll
  for (int i = 0; i < E; ++i) {
    int f = lane * E + i;
    acc += ((v[i] - mean) * rstd * Elem<T>::ld(gain + f) + Elem<T>::ld(offs + f)) * Elem<T>::ld(w_score + f);
  }
  acc = wave_sum(acc);
  if (lane == 0) scores[rt.src[r]] = acc + b_score;
}

// Zero the unused token slots of each computed prefix's last K/V tile (all layers this call
// writes), so that a ragged tile never holds stale non-finite bits: 0 * NaN would otherwise
// reach the accumulators through the masked-out keys.
template <typename T>
__global__ void zero_kv_tail_kernel(const UserDesc* __restrict__ users, int n_users, int n_layers, int n_heads, int dh) {
  int u = blockIdx.x;
  if (u >= n_users) return;
  const UserDesc ud = users[u];
  if (ud.prow0 < 0) return;
  int tail0 = ud.L % kTile;
  if (tail0 == 0) return;
  int64_t tile = ud.L / kTile;
  int layers = ud.kv_layer_stride ? n_layers : 1;
  int per_head = (kTile - tail0) * dh;  // elements of K (and of V) to clear per layer and head
  T* base = const_cast<T*>(reinterpret_cast<const T*>(ud.kv)) + ud.kv_tile0 + tile * ud.kv_tile_stride;
  int total = layers * n_heads * per_head;
  for (int i = threadIdx.x; i < total; i += blockDim.x) {
    int lh = i / per_head, w = i % per_head;
    int layer = lh / n_heads, head = lh % n_heads;
    T* kt = base + (int64_t)layer * ud.kv_layer_stride + (int64_t)head * 2 * kTile * dh;
    int rr = tail0 + w / dh, f = w % dh;
    Elem<T>::st(kt + KvLayout<T>::k_off(rr, f, dh), 0.f);
    Elem<T>::st(kt + KvLayout<T>::v_off(rr, f, dh), 0.f);
  }
}

// Same for the suffix tiles of every user with a suffix (single-layer scratch space).
template <typename T>
__global__ void zero_suffix_tail_kernel(const UserDesc* __restrict__ users, int n_users, T* __restrict__ sfx,
                                        int n_heads, int dh) {
  int u = blockIdx.x;
  if (u >= n_users) return;
  const UserDesc ud = users[u];
  int tail0 = ud.S % kTile;
  if (ud.nrow0 < 0 || tail0 == 0) return;
  int64_t tile = ud.S / kTile;
  int per_head = (kTile - tail0) * dh;
  T* base = sfx + ud.sfx_tile0 + tile * (int64_t)(2 * kTile * dh * n_heads);
  int total = n_heads * per_head;
  for (int i = threadIdx.x; i < total; i += blockDim.x) {
    int head = i / per_head, w = i % per_head;
    T* kt = base + (int64_t)head * 2 * kTile * dh;
    int rr = tail0 + w / dh, f = w % dh;
    Elem<T>::st(kt + KvLayout<T>::k_off(rr, f, dh), 0.f);
    Elem<T>::st(kt + KvLayout<T>::v_off(rr, f, dh), 0.f);
  }
}

}  // namespace relaygr
