// bf16 projection GEMMs on the 32x32x16 MFMA: C[tokens, features] = A[tokens, K] * W[features, K]^T
// with the layer's pointwise work fused in (steps 2 and 4 of a layer):
//   f1: SiLU(xh W1^T + b1) split into u | v | q | k and written where the next kernel wants it:
//       u, q (and k, v of candidate rows) row-major; k, v of prefix / suffix rows straight into the
//       K/V tile layout of the pool or of scratch;
//   f2: x <- x + y W2^T + b2 on the fp32 residual stream.
//
// Operand layout.  Both operands live in global memory already in MFMA fragment order ("panels"):
// a panel is 128 rows x K, stored as 1 KiB fragments [k-step ks = k/16][row block rb = (row%128)/32]
// [lane][8], lane (g, l32) holding row rb*32 + l32, k = ks*16 + 8g .. +7.  The LayerNorm kernels
// write activations that way and the weights are re-packed once per context.  A k-tile of a panel
// is therefore one contiguous run of bytes that is copied HBM -> LDS with direct 16-byte-per-lane
// loads (fully coalesced, no registers), lands as the exact LDS image the MFMA reads, and every
// operand fetch is one linear ds_read_b128 with no bank conflicts.  Because token and feature
// fragments have the same shape, either can be the MFMA's row operand: "feature-major" products
// leave each lane with 4 consecutive features of one token (what row-major outputs and K tiles
// want), "token-major" products leave 4 consecutive tokens of one feature (exactly a V-tile
// fragment, and what the fp32 residual update wants).
#pragma once

#include "common.h"
#include "gemm.h"

namespace relaygr {

constexpr int kPanelRows = 128;
constexpr int kGemmKTile = 32;          // k per main-loop step (2 MFMA k-steps)
constexpr int kPrefixRowAlign = 256;    // prefix rows of a user start at a multiple of this in the row space

// Re-packs a row-major [N, K] weight into panels.
__global__ void pack_weight_kernel(const uint16_t* __restrict__ w, uint16_t* __restrict__ packed, int N, int K) {
  int idx = blockIdx.x * blockDim.x + threadIdx.x;   // one 8-element chunk per thread
  int chunks_per_row = K >> 3;
  if (idx >= N * chunks_per_row) return;
  int n = idx / chunks_per_row, kc = idx - n * chunks_per_row;
  uint4 v = *reinterpret_cast<const uint4*>(w + (size_t)n * K + kc * 8);
  *reinterpret_cast<uint4*>(packed + panel_off(n, kc * 8, K)) = v;
}

// ---- main loop ----------------------------------------------------------------------------------
// Workgroup tile: 64*TM tokens x 64*TN features, 4 wavefronts as 2 x 2, each owning TM x TN blocks of
// 32 x 32.  LDS holds a ring of NSTAGE stages of [token pieces | feature pieces], a piece being one
// 1 KiB fragment; NSTAGE-1 stages are in flight while one is consumed, because with K of a few
// hundred a tile is short and the ramp of its operand stream would otherwise dominate it.
template <int TM, int TN, int NSTAGE>
struct GemmTile {
  static constexpr int BMt = 64 * TM, BNf = 64 * TN;
  static constexpr int TOK_PIECES = (BMt / 32) * 2, FEAT_PIECES = (BNf / 32) * 2;   // per stage (2 k-steps)
  static constexpr int PIECES = TOK_PIECES + FEAT_PIECES;
  static constexpr int STAGE = PIECES * 512;   // elements
  static constexpr int LDS_ELEMS = NSTAGE * STAGE;
  static constexpr int LOADS_PER_WAVE = PIECES / 4;
  static_assert(PIECES % 4 == 0, "pieces are dealt evenly to the 4 wavefronts");
  static_assert(TM == 1 || TM % 2 == 0, "a tile is half a 128-row panel or whole panels");
};

// FEATURE_MAJOR: features are the MFMA row operand (lane = token column, 4-feature runs per lane).
template <typename H, int TM, int TN, int NSTAGE, bool FEATURE_MAJOR>
__device__ __forceinline__ void gemm_mainloop(const uint16_t* __restrict__ A, const uint16_t* __restrict__ W, int K, int m0, int n0,
                                              uint16_t* lds, f32x16_t (&acc)[TM][TN]) {
  using G = GemmTile<TM, TN, NSTAGE>;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int KS = K >> 4;
  // piece p of a stage: token pieces first, ordered [panel][ksl][rb]; then feature pieces [npanel][ksl][nb]
  auto issue = [&](int kt, int slot) {
    uint16_t* dst = lds + slot * G::STAGE;
#pragma unroll
    for (int p = wave; p < G::PIECES; p += 4) {
      const uint16_t* src;
      if (p < G::TOK_PIECES) {
        if constexpr (TM >= 2) {     // whole 128-row panels: pieces ordered [panel][k-step][row block]
          int panel = p >> 3, ksl = (p >> 2) & 1, rb = p & 3;
          src = A + ((size_t)((m0 >> 7) + panel) * KS + (kt * 2 + ksl)) * 2048 + rb * 512;
        } else {                     // a 64-row tile is half a panel (m0 is a multiple of 64): [k-step][row block]
          int ksl = p >> 1, rb = ((m0 >> 5) & 3) + (p & 1);
          src = A + ((size_t)(m0 >> 7) * KS + (kt * 2 + ksl)) * 2048 + rb * 512;
        }
      } else {
        int q = p - G::TOK_PIECES;
        int panel = q >> 3, ksl = (q >> 2) & 1, nb = q & 3;
        src = W + ((size_t)((n0 >> 7) + panel) * KS + (kt * 2 + ksl)) * 2048 + nb * 512;
      }
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + lane * 8),
                                       (__attribute__((address_space(3))) void*)(dst + p * 512), 16, 0, 0);
    }
  };
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int n_kt = K / kGemmKTile;
#pragma unroll
  for (int s = 0; s < NSTAGE - 1; ++s)
    if (s < n_kt) issue(s, s);
  int slot = 0;
  for (int kt = 0; kt < n_kt; ++kt) {
    // stage kt must have landed; the NSTAGE-2 younger stages may stay in flight (near the end fewer
    // are outstanding, so wait for all of them there)
    // (a bare s_barrier: __syncthreads() would also make the compiler wait for every outstanding load,
    // i.e. for the stages that are meant to stay in flight)
    if (kt + NSTAGE - 2 < n_kt) asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NSTAGE - 2) * G::LOADS_PER_WAVE) : "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();   // also: every wavefront is past stage kt-1, whose slot is refilled next
    asm volatile("" ::: "memory");
    if (kt + NSTAGE - 1 < n_kt) issue(kt + NSTAGE - 1, slot == 0 ? NSTAGE - 1 : slot - 1);
    const uint16_t* tokp = lds + slot * G::STAGE + lane * 8;
    const uint16_t* featp = tokp + G::TOK_PIECES * 512;
    // fetch the fragments of both k-steps first, so that the second set's LDS latency hides under
    // the first set's MFMAs
    uint4 tf[2][TM], ff[2][TN];
#pragma unroll
    for (int ksl = 0; ksl < 2; ++ksl) {
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        int rbAll = wm * TM + i;   // 32-row block inside the workgroup tile
        if constexpr (TM >= 2) tf[ksl][i] = *reinterpret_cast<const uint4*>(tokp + (((rbAll >> 2) * 2 + ksl) * 4 + (rbAll & 3)) * 512);
        else tf[ksl][i] = *reinterpret_cast<const uint4*>(tokp + (ksl * 2 + rbAll) * 512);
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        int nbAll = wn * TN + j;
        ff[ksl][j] = *reinterpret_cast<const uint4*>(featp + (((nbAll >> 2) * 2 + ksl) * 4 + (nbAll & 3)) * 512);
      }
    }
    __builtin_amdgcn_sched_barrier(0);   // keep all twelve reads ahead of the MFMAs
#pragma unroll
    for (int ksl = 0; ksl < 2; ++ksl)
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = FEATURE_MAJOR ? H::mfma(ff[ksl][j], tf[ksl][i], acc[i][j]) : H::mfma(tf[ksl][i], ff[ksl][j], acc[i][j]);
    slot = (slot == NSTAGE - 1) ? 0 : slot + 1;
  }
  __syncthreads();   // every wavefront is done reading LDS: the epilogue may reuse it
}

// ---- f1 -------------------------------------------------------------------------------------------
struct F1Params {
  const uint16_t* A;        // xh panels
  const uint16_t* W;        // packed W1 [4d, d]
  const uint16_t* bias;     // [4d]
  uint16_t* u; uint16_t* q; uint16_t* knew; uint16_t* vnew; uint16_t* sfx;
  const UserDesc* users;
  RowTables rt;
  int d, dh, n_prows, layer, row_begin, row_end, n_mtiles;
  ColMap cm;
  float q_mul;
  int stream_out;           // weight-stationary kernel: outputs leave with streaming stores (launches that write far more than L2 holds)
};


constexpr int kF1TM = 4, kF1TN = 2, kF1Stages = 3;   // 256 tokens x 128 features per workgroup
constexpr int kStageLd = 64 * kF1TN + 8;          // epilogue staging row stride (elements)
// Launches of a few hundred rows (one user's candidates): the big tile gives the chip a few dozen workgroups, each
// waiting a memory round trip per k-step with two stages in flight.  The small tile (64 tokens) with six stages has
// more than a third of K = 512 in flight per workgroup and four times the workgroups; six stages are 72 KiB of LDS, so
// that a compute unit holds two such workgroups and a launch of up to 512 of them (2048 rows at d = 512) runs in one
// round (with eight stages, one workgroup per unit: 2048 rows 30 % slower, 512 rows the same).
constexpr int kF1SmallTM = 1, kF1SmallStages = 6, kF1SmallMaxRows = 4095;

template <typename H, int TM, int NSTAGE>
__global__ __launch_bounds__(256, TM == 4 ? 2 : 1) void f1_gemm_bf16_kernel(F1Params p) {
  constexpr int TN = kF1TN;
  constexpr int ROWS = 64 * TM;                  // tokens per workgroup tile
  using G = GemmTile<TM, TN, NSTAGE>;
  constexpr int LDS_ELEMS = (G::LDS_ELEMS > ROWS * kStageLd) ? G::LDS_ELEMS : ROWS * kStageLd;
  __shared__ __attribute__((aligned(16))) uint16_t lds[LDS_ELEMS];

  const int ntiles_per_blk = p.cm.d / G::BNf;
  const int n_ntiles = p.cm.nblk * ntiles_per_blk;
  const int total = p.n_mtiles * n_ntiles;
  const int logical = xcd_remap(blockIdx.x, total);
  if (logical >= total) return;
  const int mt = logical / n_ntiles, nt = logical - mt * n_ntiles;
  const int m0 = p.row_begin + mt * G::BMt;
  const int blk = p.cm.blk[nt / ntiles_per_blk];           // 0 u, 1 v, 2 q, 3 k
  const int c0 = (nt % ntiles_per_blk) * G::BNf;            // first feature inside the block
  const int n0 = blk * p.cm.d + c0;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1, l32 = lane & 31, g = lane >> 5;
  const int d = p.d, dh = p.dh;

  // A tile of prefix rows is one user's consecutive prefix positions starting at a multiple of 256
  // (row-space alignment), possibly followed by padding rows.
  const bool prefix_tile = m0 < p.n_prows;
  f32x16_t acc[TM][TN];

  if (blk == 1 && prefix_tile) {
    // ---- V of prefix rows: token-major product; the accumulator of a 32-token x 32-feature block
    // is, lane for lane, two V-tile fragments (m = 0, 1), stored as 1 KiB contiguous runs.
    gemm_mainloop<H, TM, TN, NSTAGE, false>(p.A, p.W, d, m0, n0, lds, acc);
    const int user = p.rt.user[m0];
    const UserDesc ud = p.users[user];
    const int pos0 = p.rt.idx[m0];
    const int L = ud.L, Lceil = (L + kTile - 1) / kTile * kTile;
    uint16_t* kvb = reinterpret_cast<uint16_t*>(const_cast<void*>(ud.kv)) + ud.kv_tile0 + (int64_t)p.layer * ud.kv_layer_stride;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int c = c0 + wn * 64 + j * 32;                  // first feature of this 32-feature block
      const int head = c / dh, db = (c - head * dh) >> 5;
      const float bias = H::to_f32(p.bias[n0 + wn * 64 + j * 32 + l32]);
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int tok0 = pos0 + wm * (32 * TM) + i * 32;    // first token of this 32-token block
        if (tok0 >= Lceil) continue;
        const int kb = (tok0 >> 5) & 1;
        uint16_t* frag = kvb + (int64_t)(tok0 >> 6) * ud.kv_tile_stride + (int64_t)head * 2 * kTile * dh + kTile * dh;
#pragma unroll
        for (int m = 0; m < 2; ++m) {
          uint32_t w[4];
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            const int e4 = 2 * m + h;
            float v[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const int tok = tok0 + 8 * e4 + 4 * g + r;
              float val = silu_fast(acc[i][j][4 * e4 + r] + bias);
              v[r] = tok < L ? val : 0.f;                    // the ragged tail of the last tile holds zeros
            }
            w[2 * h] = H::pack2(v[0], v[1]);
            w[2 * h + 1] = H::pack2(v[2], v[3]);
          }
          *reinterpret_cast<uint4*>(frag + (((db * 2 + kb) * 2 + m) * 64 + lane) * 8) = make_uint4(w[0], w[1], w[2], w[3]);
        }
      }
    }
    return;
  }

  // ---- everything else: feature-major product, staged through LDS as [token][feature] so that
  // every global store is a 16-byte chunk of 8 consecutive features of one token.
  // In the store phase a thread owns 16-byte chunk (tid & 15) of rows (tid >> 4) + 16*it of the
  // tile; fetch those rows' kinds now, so that the lookups complete under the main loop.
  constexpr int ITS = ROWS / 16;                 // 16 rows per pass of the store phase
  int kinds[ITS];
#pragma unroll
  for (int it = 0; it < ITS; ++it) {
    const int row = m0 + (tid >> 4) + 16 * it;
    kinds[it] = row < p.row_end ? p.rt.kind[row] : kRowPad;
  }
  // a prefix tile belongs to one user and holds consecutive prefix positions from pos0 on
  const int tile_user = prefix_tile ? p.rt.user[m0] : 0;
  const int pos0 = prefix_tile ? p.rt.idx[m0] : 0;
  gemm_mainloop<H, TM, TN, NSTAGE, true>(p.A, p.W, d, m0, n0, lds, acc);
  const float mul = (blk == 2) ? p.q_mul : 1.0f;
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int e4 = 0; e4 < 4; ++e4) {
      const int f = wn * 64 + j * 32 + 8 * e4 + 4 * g;  // 4 consecutive features held by this lane
      const uint2 bb = *reinterpret_cast<const uint2*>(p.bias + n0 + f);
      const float b0 = H::to_f32(bb.x & 0xFFFF), b1 = H::to_f32(bb.x >> 16);
      const float b2 = H::to_f32(bb.y & 0xFFFF), b3 = H::to_f32(bb.y >> 16);
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int t = wm * (32 * TM) + i * 32 + l32;
        uint2 w;
        w.x = H::pack2(silu_fast(acc[i][j][4 * e4] + b0) * mul, silu_fast(acc[i][j][4 * e4 + 1] + b1) * mul);
        w.y = H::pack2(silu_fast(acc[i][j][4 * e4 + 2] + b2) * mul, silu_fast(acc[i][j][4 * e4 + 3] + b3) * mul);
        *reinterpret_cast<uint2*>(&lds[t * kStageLd + f]) = w;
      }
    }
  __syncthreads();
  const UserDesc tud = p.users[tile_user];
  // ROWS tokens x 16 chunks of 8 features
#pragma unroll
  for (int it = 0; it < ITS; ++it) {
    const int t = (tid >> 4) + 16 * it, fc = tid & 15;
    const int row = m0 + t;
    if (row >= p.row_end) continue;
    const int kind = kinds[it];
    if (kind == kRowPad && (blk == 0 || blk == 2)) continue;
    uint4 val = *reinterpret_cast<const uint4*>(&lds[t * kStageLd + fc * 8]);
    const int c = c0 + fc * 8;                             // feature inside the block
    if (blk == 0) { *reinterpret_cast<uint4*>(p.u + (size_t)row * d + c) = val; continue; }
    if (blk == 2) { *reinterpret_cast<uint4*>(p.q + (size_t)row * d + c) = val; continue; }
    if (kind == kRowCand) {
      *reinterpret_cast<uint4*>((blk == 3 ? p.knew : p.vnew) + (size_t)(row - p.n_prows) * d + c) = val;
      continue;
    }
    const int head = c / dh, f = c - head * dh;
    uint16_t* base;
    int idx;
    if (kind == kRowSuffix) {
      const UserDesc& ud = p.users[p.rt.user[row]];
      idx = p.rt.idx[row];
      base = p.sfx + ud.sfx_tile0 + (int64_t)(idx >> 6) * (2 * kTile * d) + (int64_t)head * 2 * kTile * dh;
    } else {   // prefix row or filler of a prefix tile (blk == 3 here: V of prefix tiles took the other path)
      idx = pos0 + t;
      if (idx >= (tud.L + kTile - 1) / kTile * kTile) continue;   // filler beyond the user's last tile
      if (kind == kRowPad) val = make_uint4(0, 0, 0, 0);          // ragged tail of the last tile: zeros
      base = reinterpret_cast<uint16_t*>(const_cast<void*>(tud.kv)) + tud.kv_tile0 + (int64_t)(idx >> 6) * tud.kv_tile_stride +
             (int64_t)p.layer * tud.kv_layer_stride + (int64_t)head * 2 * kTile * dh;
    }
    const int rr = idx & 63;
    if (blk == 3) {
      *reinterpret_cast<uint4*>(base + KvLayout16::k_off(rr, f, dh)) = val;
    } else {   // V of a suffix row: its 8 features go to 8 different fragments
      const uint16_t* e = reinterpret_cast<const uint16_t*>(&val);
#pragma unroll
      for (int x = 0; x < 8; ++x) base[KvLayout16::v_off(rr, f + x, dh)] = e[x];
    }
  }
}

// ---- f1, weight-stationary form ----------------------------------------------------------------
// For launches of a few thousand rows and more.  One persistent workgroup of 8 wavefronts per compute unit
// keeps a 128-feature slice of W1 (128 x D, up to 128 KiB) in LDS for its whole life and walks 64-row units
// of its share of the rows; the workgroups of one XCD take the same row groups, so that a token panel comes
// from memory once per XCD.  Each wavefront owns whole units (64 rows x 128 features, 2 x 4 MFMA blocks):
// its token fragments go from global memory straight into registers, PF k-steps ahead (a token fragment is
// 1 KiB of contiguous panel bytes, one 16-byte load per lane), the weight fragments are linear LDS reads one
// k-step ahead, and nothing in the main loop waits for another wavefront: no barrier after the slice has
// landed, so the two wavefronts of a SIMD drift apart and one's epilogue (vector ALU, stores) runs beside
// the other's main loop (matrix cores).  The accumulators start from the bias.  Results are staged through
// 4 KiB of wavefront-private LDS (32 tokens x 64 features, 16-byte chunks swizzled by token so that neither
// the 8-byte writes nor the 16-byte reads pile up on a bank) and leave as 128-byte row segments; V of prefix
// rows takes the token-major product, whose accumulators are V-tile fragments as they stand.  Launches that
// write far more than the L2s hold use streaming stores (see st_stream): with plain stores the output lines
// evict the token panels the workgroups of an XCD share and the kernel runs at the speed of the re-fetches
// (65 536 x 2048 x 512 stand-alone: 225 us plain, 152 us streaming, 205 us for the tiled kernel above); small
// launches keep plain stores, because what they write fits the L2s and the attention and layer-tail kernels
// read it straight back (8192 rows: the layer tail is 2 us slower behind streaming stores).
constexpr int kF1WsPF = 4;          // k-steps of token fragments in flight per wavefront
constexpr int kF1WsMinRows = 4096;  // below this the tiled kernel's many small workgroups fill the chip better
constexpr int kF1StreamMinRows = 16384;   // from here on a launch writes 64 MiB and more (at d = 512): streaming stores
constexpr int kTailVr8MaxRows = 1024;   // layer tail: launches of at most this many rows use 8-row workgroups (d = 256, 512),
constexpr int kTailVr16MaxRows = 4096;  // of at most this many 16-row workgroups: still at most one workgroup per compute unit

template <typename H, int D, bool FEATURE_MAJOR>
__device__ __forceinline__ void f1_ws_mainloop(const uint16_t* __restrict__ tp0, const uint16_t* __restrict__ tp1,
                                               const uint16_t* wlane, f32x16_t (&acc)[2][4]) {
  constexpr int KS = D / 16, PF = kF1WsPF;
  uint4 t[PF][2], ff[2][4];
#pragma unroll
  for (int pf = 0; pf < PF; ++pf) {
    t[pf][0] = *reinterpret_cast<const uint4*>(tp0 + (size_t)pf * 2048);
    t[pf][1] = *reinterpret_cast<const uint4*>(tp1 + (size_t)pf * 2048);
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) ff[0][j] = *reinterpret_cast<const uint4*>(wlane + j * 512);
#pragma unroll 1
  for (int ks0 = 0; ks0 < KS; ks0 += PF) {
#pragma unroll
    for (int pf = 0; pf < PF; ++pf) {
      const int ks = ks0 + pf, cur = pf & 1, nxt = cur ^ 1;
      if (ks + 1 < KS) {
#pragma unroll
        for (int j = 0; j < 4; ++j) ff[nxt][j] = *reinterpret_cast<const uint4*>(wlane + ((ks + 1) * 4 + j) * 512);
      }
      __builtin_amdgcn_sched_barrier(0);   // the next k-step's LDS reads stay ahead of this k-step's MFMAs
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = FEATURE_MAJOR ? H::mfma(ff[cur][j], t[pf][i], acc[i][j]) : H::mfma(t[pf][i], ff[cur][j], acc[i][j]);
      if (ks + PF < KS) {
        t[pf][0] = *reinterpret_cast<const uint4*>(tp0 + (size_t)(ks + PF) * 2048);
        t[pf][1] = *reinterpret_cast<const uint4*>(tp1 + (size_t)(ks + PF) * 2048);
      }
    }
  }
}

__device__ __forceinline__ void st_out(uint4* dst, uint4 v, int stream) {
  if (stream) st_stream(dst, v);
  else *dst = v;
}

template <typename H, int D>
__global__ __launch_bounds__(512, 1) void f1_ws_bf16_kernel(F1Params p) {
  constexpr int KS = D / 16;
  static_assert(KS % kF1WsPF == 0 && (KS * 4) % 8 == 0, "shape");
  __shared__ __attribute__((aligned(16))) uint16_t wl[KS * 2048];       // 128 features x D, fragment order
  __shared__ __attribute__((aligned(16))) uint16_t stage[8 * 32 * 64];   // per wavefront: 32 tokens x 64 features
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, g = lane >> 5;
  const int d = p.d, dh = p.dh;
  const int slices_per_blk = d >> 7;
  const int n_slices = p.cm.nblk * slices_per_blk;
  const int n_rg = (int)gridDim.x / n_slices;                 // row groups: a multiple of 8 (host)
  const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3;
  const int slice = idx % n_slices;
  const int rg = xcd * (n_rg >> 3) + idx / n_slices;
  const int blk = p.cm.blk[slice / slices_per_blk];            // 0 u, 1 v, 2 q, 3 k
  const int c0 = (slice % slices_per_blk) * 128;               // first feature inside the block
  const int n0 = blk * d + c0;
  {
    const uint16_t* src = p.W + (size_t)(n0 >> 7) * KS * 2048;
#pragma unroll
    for (int it = 0; it < KS * 4 / 8; ++it) {
      const int piece = it * 8 + wave;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + piece * 512 + lane * 8),
                                       (__attribute__((address_space(3))) void*)(wl + piece * 512), 16, 0, 0);
    }
  }
  const int n_units = (p.row_end - p.row_begin + 63) >> 6;
  const int upr = (n_units + n_rg - 1) / n_rg;
  const int u_begin = rg * upr, u_end = min(n_units, u_begin + upr);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  const uint16_t* wlane = wl + lane * 8;
  uint16_t* st = stage + wave * (32 * 64);
  const float mul = (blk == 2) ? p.q_mul : 1.0f;

  for (int unit = u_begin + wave; unit < u_end; unit += 8) {
    const int m0 = p.row_begin + unit * 64;                    // row_begin is a multiple of 64 (host)
    const int B = m0 >> 5;
    const uint16_t* tp0 = p.A + ((size_t)(B >> 2) * KS) * 2048 + (B & 3) * 512 + lane * 8;
    const uint16_t* tp1 = p.A + ((size_t)((B + 1) >> 2) * KS) * 2048 + ((B + 1) & 3) * 512 + lane * 8;
    // a unit of prefix rows lies inside one user's (256-aligned) prefix region: consecutive positions from pos0
    const bool prefix_unit = m0 < p.n_prows;
    const int tile_user = prefix_unit ? p.rt.user[m0] : 0;
    const int pos0 = prefix_unit ? p.rt.idx[m0] : 0;
    f32x16_t acc[2][4];

    if (blk == 1 && prefix_unit) {
      // ---- V of prefix rows: token-major product, accumulators are V-tile fragments
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float b = H::to_f32(p.bias[n0 + j * 32 + l32]);
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int e = 0; e < 16; ++e) acc[i][j][e] = b;
      }
      f1_ws_mainloop<H, D, false>(tp0, tp1, wlane, acc);
      const UserDesc ud = p.users[tile_user];
      const int L = ud.L, Lceil = (L + kTile - 1) / kTile * kTile;
      uint16_t* kvb = reinterpret_cast<uint16_t*>(const_cast<void*>(ud.kv)) + ud.kv_tile0 + (int64_t)p.layer * ud.kv_layer_stride;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int c = c0 + j * 32;
        const int head = c / dh, db = (c - head * dh) >> 5;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          const int tok0 = pos0 + i * 32;
          if (tok0 >= Lceil) continue;
          const int kb = (tok0 >> 5) & 1;
          uint16_t* frag = kvb + (int64_t)(tok0 >> 6) * ud.kv_tile_stride + (int64_t)head * 2 * kTile * dh + kTile * dh;
#pragma unroll
          for (int m = 0; m < 2; ++m) {
            uint32_t w[4];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
              const int e4 = 2 * m + h;
              float v[4];
#pragma unroll
              for (int r = 0; r < 4; ++r) {
                const int tok = tok0 + 8 * e4 + 4 * g + r;
                const float val = silu_fast(acc[i][j][4 * e4 + r]);
                v[r] = tok < L ? val : 0.f;                  // the ragged tail of the last tile holds zeros
              }
              w[2 * h] = H::pack2(v[0], v[1]);
              w[2 * h + 1] = H::pack2(v[2], v[3]);
            }
            st_out(reinterpret_cast<uint4*>(frag + (((db * 2 + kb) * 2 + m) * 64 + lane) * 8), make_uint4(w[0], w[1], w[2], w[3]), p.stream_out);
          }
        }
      }
      continue;
    }

    // ---- everything else: feature-major product (a lane ends up with 4-feature runs of one token)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4) {
        const uint2 bb = *reinterpret_cast<const uint2*>(p.bias + n0 + j * 32 + 8 * e4 + 4 * g);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          acc[i][j][4 * e4] = H::to_f32(bb.x & 0xFFFF);
          acc[i][j][4 * e4 + 1] = H::to_f32(bb.x >> 16);
          acc[i][j][4 * e4 + 2] = H::to_f32(bb.y & 0xFFFF);
          acc[i][j][4 * e4 + 3] = H::to_f32(bb.y >> 16);
        }
      }
    f1_ws_mainloop<H, D, true>(tp0, tp1, wlane, acc);
    const UserDesc tud = p.users[tile_user];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      // this lane stores 16-byte chunk lane & 7 of rows (lane >> 3) + 8 n of the 32-row block, n = 0..3
      int kinds[4];
#pragma unroll
      for (int n = 0; n < 4; ++n) {
        const int row = m0 + i * 32 + (lane >> 3) + 8 * n;
        kinds[n] = row < p.row_end ? p.rt.kind[row] : -1;
      }
#pragma unroll
      for (int jh = 0; jh < 2; ++jh) {
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
          const int j = jh * 2 + jj;
#pragma unroll
          for (int e4 = 0; e4 < 4; ++e4) {
            const int fl = jj * 32 + 8 * e4 + 4 * g;
            uint2 w;
            w.x = H::pack2(silu_fast(acc[i][j][4 * e4]) * mul, silu_fast(acc[i][j][4 * e4 + 1]) * mul);
            w.y = H::pack2(silu_fast(acc[i][j][4 * e4 + 2]) * mul, silu_fast(acc[i][j][4 * e4 + 3]) * mul);
            *reinterpret_cast<uint2*>(st + l32 * 64 + (((fl >> 3) ^ (l32 & 7)) << 3) + (fl & 7)) = w;
          }
        }
        __builtin_amdgcn_wave_barrier();   // LDS serves a wavefront's accesses in order: the reads below see the writes above
#pragma unroll
        for (int n = 0; n < 4; ++n) {
          const int tk = (lane >> 3) + 8 * n;
          int fc = lane & 7;
          // (opaque to the compiler: otherwise it hoists the index arithmetic of the rare suffix-V scatter below out of
          // the unit loop, 32 values per lane that it then has to spill -- 16 MiB of scratch writes per launch)
          asm volatile("" : "+v"(fc));
          uint4 val = *reinterpret_cast<const uint4*>(st + tk * 64 + ((fc ^ (tk & 7)) << 3));
          const int row = m0 + i * 32 + tk;
          const int kind = kinds[n];
          if (kind < 0) continue;                                // beyond the launch's last row
          if (kind == kRowPad && (blk == 0 || blk == 2)) continue;
          const int c = c0 + jh * 64 + fc * 8;                   // feature inside the block
          if (blk == 0) { st_out(reinterpret_cast<uint4*>(p.u + (size_t)row * d + c), val, p.stream_out); continue; }
          if (blk == 2) { st_out(reinterpret_cast<uint4*>(p.q + (size_t)row * d + c), val, p.stream_out); continue; }
          if (kind == kRowCand) {
            st_out(reinterpret_cast<uint4*>((blk == 3 ? p.knew : p.vnew) + (size_t)(row - p.n_prows) * d + c), val, p.stream_out);
            continue;
          }
          const int head = c / dh, f = c - head * dh;
          uint16_t* base;
          int pos;
          if (kind == kRowSuffix) {
            const UserDesc& ud = p.users[p.rt.user[row]];
            pos = p.rt.idx[row];
            base = p.sfx + ud.sfx_tile0 + (int64_t)(pos >> 6) * (2 * kTile * d) + (int64_t)head * 2 * kTile * dh;
          } else {   // prefix row or filler of a prefix unit (blk == 3 here: V of prefix units took the other path)
            pos = pos0 + i * 32 + tk;
            if (pos >= (tud.L + kTile - 1) / kTile * kTile) continue;   // filler beyond the user's last tile
            if (kind == kRowPad) val = make_uint4(0, 0, 0, 0);          // ragged tail of the last tile: zeros
            base = reinterpret_cast<uint16_t*>(const_cast<void*>(tud.kv)) + tud.kv_tile0 + (int64_t)(pos >> 6) * tud.kv_tile_stride +
                   (int64_t)p.layer * tud.kv_layer_stride + (int64_t)head * 2 * kTile * dh;
          }
          const int rr = pos & 63;
          if (blk == 3) {
            st_out(reinterpret_cast<uint4*>(base + KvLayout16::k_off(rr, f, dh)), val, p.stream_out);
          } else {   // V of a suffix row: its 8 features go to 8 different fragments
            const uint16_t* e = reinterpret_cast<const uint16_t*>(&val);
#pragma unroll
            for (int x = 0; x < 8; ++x) base[KvLayout16::v_off(rr, f + x, dh)] = e[x];
          }
        }
        __builtin_amdgcn_wave_barrier();   // the next pass overwrites the staging area
      }
    }
  }
}

// ---- gate + f2 + next layer's input LayerNorm in one kernel ------------------------------------
// Everything between the attention of one layer and the projections of the next is local to a row:
//   y  = LN((sum of key-split partial sums + a candidate's self term) / n; g_at, b_at) * u
//   x <- x + y W2^T + b2
//   xh = LN(x; next layer's g_in, b_in)
// so one workgroup takes 32*RB rows over the full width D and does all three: y never goes to HBM,
// the residual row is read and written once, and two row-wise passes disappear.  Each wavefront
// gates ROWS/NW rows (lane = D/64 consecutive features, DPP reductions) and writes them into LDS as
// MFMA token fragments shared by all wavefronts; it owns D/32/NW feature blocks of the product and
// streams its own slice of the packed W2 from L2 straight into registers (no wavefront shares
// weights with another, so LDS would add nothing), PF k-steps ahead.  Feature-major product: a lane
// ends up with one token and runs of 4 features, so the row statistics of the second LayerNorm are
// a lane-local sum, one cross-half shuffle and one exchange between wavefronts through LDS.  Global
// loads that depend on no result go out as early as the registers allow: the rows' split sums, u and
// the residual rows before the first wait, the weight fragments once the split buffers are free, the
// second LayerNorm's gain and offset before the product.
struct F2LnParams {
  // gate inputs
  const float* part;        // [nsplit][rows][D] unnormalised attention sums
  int nsplit;
  size_t split_stride;
  const uint16_t* u;        // [rows, D]
  const uint16_t* q;        // [rows, D] (pre-scaled); null: the attention kernel has added the candidates' own keys already
  const uint16_t* knew;     // [new rows, D] row-major k and v of suffix and candidate rows
  const uint16_t* vnew;
  const uint16_t* gate_gain;
  const uint16_t* gate_offs;
  int n_prows, dh;
  float qk_mul;             // stored q . k -> alpha <q, k>
  // softmax form (kernels instantiated with SM): part holds sums of exp2(t - m) v, ml the (m, l) of every row, head and
  // split as [split][row][head][2]; the splits and the candidate's own key are merged here
  const float* ml;
  size_t ml_stride;
  int n_heads;
  const uint16_t* W;        // packed W2 [D, D]
  const uint16_t* bias;     // b2 [D]
  float* x;                 // residual stream [rows, D], updated in place
  uint16_t* xh;             // LN(x) panels for the next layer; nullptr: none wanted (last layer)
  const uint16_t* gain;     // next layer's input LayerNorm
  const uint16_t* offs;
  RowTables rt;
  int row_begin, row_end;   // row_begin is a multiple of 32
  float eps;
  // last layer of a ranking call: instead of xh, score_c = <w_score, LN(x; gain, offs)> + b_score for
  // candidate rows, written at the candidate's position in the caller's order (scores != nullptr)
  const uint16_t* w_score;
  float b_score;
  float* scores;
};


// E consecutive bf16 values (E = 2, 4, 8 or 16; address aligned to 2*E bytes, at most 16) as packed words.
template <int E>
__device__ __forceinline__ void ld_bf16_run(const uint16_t* src, uint32_t (&w)[E / 2]) {
  if constexpr (E == 2) {
    w[0] = *reinterpret_cast<const uint32_t*>(src);
  } else if constexpr (E == 4) {
    const uint2 v = *reinterpret_cast<const uint2*>(src);
    w[0] = v.x; w[1] = v.y;
  } else {
#pragma unroll
    for (int c = 0; c < E / 8; ++c) {
      const uint4 v = *reinterpret_cast<const uint4*>(src + 8 * c);
      w[4 * c] = v.x; w[4 * c + 1] = v.y; w[4 * c + 2] = v.z; w[4 * c + 3] = v.w;
    }
  }
}

// One row of the attention combine + gate, by one wavefront, lane owning features [lane*E, lane*E+E).
// SELF: the row's own q, k, v are wanted (softmax form: the candidate's own key is merged here; in the
// SiLU form the attention kernel has it in its sums already).
template <int E, bool SELF>
struct GateRow {
  float o[E];
  uint32_t ub[E / 2], qb[SELF ? E / 2 : 1], kb[SELF ? E / 2 : 1], vb[SELF ? E / 2 : 1];
  int n, kind;
  float mpart, lpart;   // softmax form: reference score of o and the matching sum of weights
};

template <int E>
__device__ __forceinline__ void ld_f32_run(const float* src, float (&v)[E]) {
  if constexpr (E == 2) {
    const float2 t = *reinterpret_cast<const float2*>(src);
    v[0] = t.x; v[1] = t.y;
  } else {
#pragma unroll
    for (int c = 0; c < E / 4; ++c) {
      const float4 t = *reinterpret_cast<const float4*>(src + 4 * c);
      v[4 * c] = t.x; v[4 * c + 1] = t.y; v[4 * c + 2] = t.z; v[4 * c + 3] = t.w;
    }
  }
}

// The key-split partial sums of G rows, summed in split order, NB splits (all G rows each) in flight at a
// time: a call with 8 key splits waits for 8 / NB round trips to memory per group of rows, not for one per
// row and split.  begin() issues the rows' other inputs and the first NB splits; the caller may issue further
// loads before finish() adds them up and walks the remaining splits.
// Rows beyond the launch read the workgroup's first row instead and are marked as filler.
template <int D, bool SM, int G, int NB>
struct GateLoad {
  static constexpr int E = D / 64;
  size_t base[G];
  const float* mlr[G];
  float M[G];
  float buf[NB][G][E];
  float2 mlb[NB][G];

  __device__ __forceinline__ void issue(const F2LnParams& p, int sp0) {
#pragma unroll
    for (int k = 0; k < NB; ++k) {
      if (sp0 + k >= p.nsplit) break;      // uniform
#pragma unroll
      for (int r = 0; r < G; ++r) {
        ld_f32_run<E>(p.part + (sp0 + k) * p.split_stride + base[r], buf[k][r]);
        if constexpr (SM) mlb[k][r] = *reinterpret_cast<const float2*>(mlr[r] + (sp0 + k) * p.ml_stride);
      }
    }
  }
  __device__ __forceinline__ void add(const F2LnParams& p, int sp0, GateRow<E, SM> (&gr)[G]) {
#pragma unroll
    for (int k = 0; k < NB; ++k) {
      if (sp0 + k >= p.nsplit) break;
#pragma unroll
      for (int r = 0; r < G; ++r) {
        float w = 1.0f;
        if constexpr (SM) {
          w = (mlb[k][r].x == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mlb[k][r].x - M[r]);
          gr[r].lpart += w * mlb[k][r].y;
        }
#pragma unroll
        for (int i = 0; i < E; ++i) gr[r].o[i] += w * buf[k][r][i];
      }
    }
  }
  __device__ __forceinline__ void begin(const F2LnParams& p, int row_first, int row_safe, int lane, GateRow<E, SM> (&gr)[G]) {
#pragma unroll
    for (int r = 0; r < G; ++r) {
      const bool ok = row_first + r < p.row_end;
      const int row = ok ? row_first + r : row_safe;
      const int kind = p.rt.kind[row];
      gr[r].kind = ok ? kind : kRowPad;
      gr[r].n = p.rt.lim[row];
      base[r] = (size_t)row * D + lane * E;
      ld_bf16_run<E>(p.u + base[r], gr[r].ub);
      mlr[r] = nullptr;
      M[r] = 0.f;
      if constexpr (SM) {
#pragma unroll
        for (int i = 0; i < E / 2; ++i) gr[r].qb[i] = gr[r].kb[i] = gr[r].vb[i] = 0u;
        if (row >= p.n_prows) {   // suffix and candidate rows have row-major q, k, v (only candidates use them)
          const size_t nb = (size_t)(row - p.n_prows) * D + lane * E;
          ld_bf16_run<E>(p.q + base[r], gr[r].qb);
          ld_bf16_run<E>(p.knew + nb, gr[r].kb);
          ld_bf16_run<E>(p.vnew + nb, gr[r].vb);
        }
        // split s counts with weight 2^(m_s - M), M the largest m_s of this lane's head
        mlr[r] = p.ml + ((size_t)row * p.n_heads + lane * E / p.dh) * 2;
        float m = -INFINITY;
#pragma unroll
        for (int sp = 0; sp < 8; ++sp) m = fmaxf(m, mlr[r][(size_t)min(sp, p.nsplit - 1) * p.ml_stride]);   // at most 8 key splits
        M[r] = m;
      }
      gr[r].mpart = M[r];
      gr[r].lpart = SM ? 0.f : 1.f;
#pragma unroll
      for (int i = 0; i < E; ++i) gr[r].o[i] = 0.f;
    }
    issue(p, 0);
  }
  __device__ __forceinline__ void finish(const F2LnParams& p, GateRow<E, SM> (&gr)[G]) {
    add(p, 0, gr);
    for (int sp0 = NB; sp0 < p.nsplit; sp0 += NB) {
      issue(p, sp0);
      add(p, sp0, gr);
    }
  }
};

// Finishes G rows at once (their reductions interleave) and writes y (bf16) into the token
// fragments: local row lr0 + i of the workgroup goes to row block (lr0+i)/32, row (lr0+i)%32.
template <typename H, int D, int G, bool SM, int FRAG>
__device__ __forceinline__ void finish_gate_rows(const F2LnParams& p, GateRow<D / 64, SM> (&gr)[G], int lane, uint16_t* tok, int lr0,
                                                 const uint32_t (&gw)[D / 128], const uint32_t (&ow)[D / 128]) {
  constexpr int E = D / 64, KS = D / 16;
  float s[G], inv_n[G];
#pragma unroll
  for (int r = 0; r < G; ++r) {
    int n = gr[r].n;
    float lsum = gr[r].lpart;
    if constexpr (!SM) {
      if (gr[r].kind == kRowCand) n += 1;   // the own key is in the attention kernel's sums already; it counts as a visible key
    } else if (gr[r].kind == kRowCand) {      // the candidate's own key, per head
      float dot = 0.f;
#pragma unroll
      for (int i = 0; i < E; ++i) dot += H::of_word(gr[r].qb[i >> 1], i) * H::of_word(gr[r].kb[i >> 1], i);
      // the lanes of one head are dh/E consecutive lanes
      const int hl = p.dh / E;
      if (hl == 2) dot = lanes2_sum(dot);
      else if (hl == 4) dot = lanes4_sum(dot);
      else if (hl == 8) dot = lanes8_sum(dot);
      else if (hl == 16) dot = lanes16_sum(dot);
      else if (hl == 32) dot = lanes32_sum(dot);
      else if (hl == 64) dot = wave_sum_dpp(dot);
      // the stored q carries alpha * log2(e), so dot is the own key's score in the units of m; bring the
      // merged splits and the own key to their common maximum
      const float Mn = fmaxf(gr[r].mpart, dot);
      const float c = (gr[r].mpart == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(gr[r].mpart - Mn);
      const float ws = __builtin_amdgcn_exp2f(dot - Mn);
#pragma unroll
      for (int i = 0; i < E; ++i) gr[r].o[i] = gr[r].o[i] * c + ws * H::of_word(gr[r].vb[i >> 1], i);
      lsum = lsum * c + ws;
    }
    inv_n[r] = SM ? 1.0f / (lsum > 0.f ? lsum : 1.0f) : 1.0f / (float)(n > 0 ? n : 1);
    s[r] = 0.f;
#pragma unroll
    for (int i = 0; i < E; ++i) { gr[r].o[i] *= inv_n[r]; s[r] += gr[r].o[i]; }
  }
  float mean[G], qv[G];
#pragma unroll
  for (int r = 0; r < G; ++r) mean[r] = wave_sum_dpp(s[r]) * (1.0f / (float)D);
#pragma unroll
  for (int r = 0; r < G; ++r) {
    qv[r] = 0.f;
#pragma unroll
    for (int i = 0; i < E; ++i) { const float c = gr[r].o[i] - mean[r]; qv[r] += c * c; }
  }
#pragma unroll
  for (int r = 0; r < G; ++r) {
    const float rstd = rsqrtf(wave_sum_dpp(qv[r]) * (1.0f / (float)D) + p.eps);
    uint32_t yw[E / 2];
#pragma unroll
    for (int i = 0; i < E / 2; ++i) {
      float z0 = (gr[r].o[2 * i] - mean[r]) * rstd * H::of_word(gw[i], 0) + H::of_word(ow[i], 0);
      float z1 = (gr[r].o[2 * i + 1] - mean[r]) * rstd * H::of_word(gw[i], 1) + H::of_word(ow[i], 1);
      f32x2_t two = {z0 * H::of_word(gr[r].ub[i], 0), z1 * H::of_word(gr[r].ub[i], 1)};
      if (gr[r].kind == kRowPad) { two[0] = 0.f; two[1] = 0.f; }
      yw[i] = H::pack2(two[0], two[1]);
    }
    // feature f of a row block's local row rr sits at fragment f/16, lane (f/8 % 2)*32 + rr, element f%8
    const int lr = lr0 + r;
    uint16_t* tokb = tok + (lr >> 5) * KS * FRAG;
    const int rr = lr & 31;
    constexpr int RUN = E < 8 ? E : 8;
#pragma unroll
    for (int c = 0; c < E; c += RUN) {
      const int f = lane * E + c;
      uint16_t* dst = tokb + (f >> 4) * FRAG + (((f >> 3) & 1) * 32 + rr) * 8 + (f & 7);
      if constexpr (RUN == 2) *reinterpret_cast<uint32_t*>(dst) = yw[c / 2];
      else if constexpr (RUN == 4) *reinterpret_cast<uint2*>(dst) = make_uint2(yw[c / 2], yw[c / 2 + 1]);
      else *reinterpret_cast<uint4*>(dst) = make_uint4(yw[c / 2], yw[c / 2 + 1], yw[c / 2 + 2], yw[c / 2 + 3]);
    }
  }
}

// ---- L2 warm-up -----------------------------------------------------------------------------------
// Workgroups that stream the same operand run in step, so without help every slice of it is a first
// touch for the whole XCD and costs a full trip to HBM or the memory-side cache, with only the few
// k-steps in flight to cover it.  Instead, each workgroup asks for one 4-byte word of every 128-byte
// line of ITS share of the operand when it starts: together the sharers pull the whole operand into
// their XCD's L2 in one round trip, and the later loads hit L2.  (Measured: 9 % off the layer-tail
// kernel, whose W2 stream waits on latency; the same warm-up made the f1 GEMM 9 % slower -- its
// operand stream is bound by L2 -> LDS bandwidth, not latency -- and is not used there.)
// Touches lines [share * per, share * per + per) of `lines` lines, per = lines / n_shares, at most
// MAXLD loads per thread, all issued at once (a thread with fewer lines to touch repeats its last one);
// v receives the words (to be consumed by a never-taken branch once the loads are known to have landed).
template <int MAXLD>
__device__ __forceinline__ void l2_touch(const void* base, int lines, int share, int n_shares, int tid, int n_threads, int (&v)[MAXLD]) {
  const int per = lines / n_shares;
  const char* b = reinterpret_cast<const char*>(base) + (size_t)share * per * 128;
#pragma unroll
  for (int u = 0; u < MAXLD; ++u) {
    const int i = min(tid + u * n_threads, per - 1);
    v[u] = (u == 0 || (u * n_threads < per)) ? *reinterpret_cast<const int*>(b + (size_t)i * 128) : 0;
  }
}

// OCC = 2: built to fit two workgroups on a compute unit (128 registers per lane), so that one's gate
// phase (memory) overlaps the other's product phase (L2 and matrix cores) when a launch has several
// workgroups per unit: fewer k-steps and gate rows in flight, and the weight fragments and the
// residual rows are requested after the gate instead of before it.
// VR < 32: a workgroup takes only VR rows (a partly filled row block).  For launches of a few hundred to a
// few thousand rows (one user per call): with 32 rows each they would occupy a few dozen compute units, each
// pulling 16 KiB of split partial sums per row through its own memory path; with VR = 8 or 16 four times or
// twice as many units share that.
template <typename H, int D, int NW, int RB, bool SM, int OCC = 1, int VR = 32>
__global__ __launch_bounds__(NW * 64, OCC) void f2_ln_bf16_kernel(F2LnParams p) {
  constexpr int KS = D / 16;            // k-steps
  constexpr int FB = D / 32 / NW;       // 32-feature blocks per wavefront
  constexpr int PF = FB >= 4 ? 2 : (OCC == 2 ? 4 : 8);   // k-steps of weight fragments in flight per wavefront (16 spills: 38 % slower)
  constexpr int ROWS = 32 * RB;         // rows per workgroup: RB blocks of 32 share one pass over W2
  static_assert(FB >= 1 && FB * NW * 32 == D && KS % PF == 0, "shape");
  static_assert(RB * KS * 1024 <= 65536, "token fragments fit static LDS");
  // A row's 16-byte chunks go to the same place of consecutive fragments: with fragments exactly 1 KiB apart all
  // 64 lanes of such a write would hit one bank, so fragments sit 16 bytes further apart where static LDS allows it
  constexpr int FRAG = 512 + (RB == 1 ? 8 : 0);   // elements between token fragments
  __shared__ __attribute__((aligned(16))) uint16_t tok[RB * KS * FRAG];   // ROWS tokens x D, fragment order
  float* red = reinterpret_cast<float*>(tok);                             // reused after the product: [2][NW][ROWS]
  static_assert(VR == 32 || (RB == 1 && OCC == 1 && VR % NW == 0 && VR < 32), "partly filled row blocks: one or two rows per wavefront");
  constexpr int VROWS = VR < 32 ? VR : ROWS;   // rows this workgroup really has
  const int row0 = p.row_begin + blockIdx.x * VROWS;
  if (row0 >= p.row_end) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l32 = lane & 31, g = lane >> 5;

  // The gate makes the tokens: each wavefront takes ROWS/NW rows, a few at a time
  // so that their loads are in flight together.  The first group's loads go out before anything
  // else, since they are what the workgroup needs first.
  constexpr int RPW = VROWS / NW, GMAX = OCC == 2 ? 2 : (RB * FB >= 4 ? (D >= 1024 ? 1 : 2) : (SM ? 2 : 4)), GROUP = RPW < GMAX ? RPW : GMAX;
  static_assert(RPW >= 1 && RPW % GROUP == 0, "rows per wavefront");
  // splits in flight per group of rows: what the registers allow (all 8 when a wavefront has one row)
  constexpr int NB = VR < 32 ? (64 / (GROUP * (D / 64)) > 8 ? 8 : 64 / (GROUP * (D / 64))) : (D >= 1024 ? 1 : 2);
  GateRow<D / 64, SM> gr[GROUP];
  uint32_t gw[D / 128], ow[D / 128];
  GateLoad<D, SM, GROUP, NB> gl;
  gl.begin(p, row0 + wave * RPW, row0, lane, gr);
  ld_bf16_run<D / 64>(p.gate_gain + lane * (D / 64), gw);
  ld_bf16_run<D / 64>(p.gate_offs + lane * (D / 64), ow);

  // L2 warm-up of W2 (every workgroup streams all of it, in step): the workgroups of an XCD (every
  // eighth one) each ask for a slice now, so that the product phase below finds W2 in L2
  const int wgs_per_xcd = (int)gridDim.x >> 3;
  const int n_slices = wgs_per_xcd < 1 ? 1 : (wgs_per_xcd < 16 ? wgs_per_xcd : 16);
  int touched[4];
  l2_touch<4>(p.W, D * D / 64, ((int)blockIdx.x >> 3) % n_slices, n_slices, (int)threadIdx.x, NW * 64, touched);

  // this wavefront's weight fragments: feature block fb lives in panel fb/4, row block fb%4
  const uint16_t* wbase[FB];
#pragma unroll
  for (int j = 0; j < FB; ++j) {
    const int fb = wave * FB + j;
    wbase[j] = p.W + (size_t)(fb >> 2) * KS * 2048 + (fb & 3) * 512 + lane * 8;
  }
  // the workgroups of an XCD walk the k-steps from different starting points, so that at any moment
  // they ask the XCD's L2 for different slices of W2 instead of all for the same one
  // (the sum over k then runs in a different order per block; for prefix rows the starting point is
  // taken from the block's position inside its user's prefix, not from the block index, so that the
  // K/V a pre-inference leaves in the pool do not depend on which other users shared its batch)
  static_assert((KS & (KS - 1)) == 0, "k-steps: a power of two");
  const int blk_id = row0 < p.n_prows ? p.rt.idx[row0] / ROWS : (int)blockIdx.x;
  const int rot = ((blk_id >> 3) * PF) & (KS - 1);
  uint4 wf[PF][FB];
  auto prefetch_w = [&]() {
#pragma unroll
    for (int i = 0; i < PF; ++i)
#pragma unroll
      for (int j = 0; j < FB; ++j) wf[i][j] = *reinterpret_cast<const uint4*>(wbase[j] + (size_t)((i + rot) & (KS - 1)) * 2048);
  };
  // The accumulators start from the residual row plus the bias, fetched now so that the gate and
  // the product hide the latency (the row's kind is only needed when results are stored): element
  // e of acc[b][j] is feature (wave*FB + j)*32 + 8*(e/4) + 4*g + e%4 of token row0 + 32*b + l32.
  bool in_range[RB], live[RB];
  float* xrow[RB];
  int kind_ep[RB];
  f32x16_t acc[RB][FB];
  auto init_acc = [&]() {
#pragma unroll
    for (int b = 0; b < RB; ++b) {
      const int row = row0 + 32 * b + l32;
      in_range[b] = row < p.row_end && 32 * b + l32 < VROWS;
      kind_ep[b] = p.rt.kind[in_range[b] ? row : row0];
      xrow[b] = p.x + (size_t)(in_range[b] ? row : row0) * D;
#pragma unroll
      for (int j = 0; j < FB; ++j)
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
          const int c = (wave * FB + j) * 32 + 8 * e4 + 4 * g;
          const uint2 bb = *reinterpret_cast<const uint2*>(p.bias + c);
          const float4 v = *reinterpret_cast<const float4*>(xrow[b] + c);
          acc[b][j][4 * e4] = v.x + H::to_f32(bb.x & 0xFFFF);
          acc[b][j][4 * e4 + 1] = v.y + H::to_f32(bb.x >> 16);
          acc[b][j][4 * e4 + 2] = v.z + H::to_f32(bb.y & 0xFFFF);
          acc[b][j][4 * e4 + 3] = v.w + H::to_f32(bb.y >> 16);
        }
    }
  };

  // The residual rows are requested now, behind the rows' first loads; the weight fragments once the
  // split buffers are free; then the first rows are reduced and written as token fragments, and
  // further groups of rows follow.
  constexpr bool EARLY_W = OCC == 1 && !SM && D < 1024;      // elsewhere the registers do not allow it
  if constexpr (EARLY_W) init_acc();
  gl.finish(p, gr);
  if constexpr (EARLY_W) prefetch_w();                       // in flight while the rows are normalised and written to LDS
  finish_gate_rows<H, D, GROUP, SM, FRAG>(p, gr, lane, tok, wave * RPW, gw, ow);
#pragma unroll
  for (int r0 = GROUP; r0 < RPW; r0 += GROUP) {
    gl.begin(p, row0 + wave * RPW + r0, row0, lane, gr);
    gl.finish(p, gr);
    finish_gate_rows<H, D, GROUP, SM, FRAG>(p, gr, lane, tok, wave * RPW + r0, gw, ow);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if ((touched[0] ^ touched[1] ^ touched[2] ^ touched[3]) == 0x5a17c0de && p.eps < 0.f) red[0] = 0.f;   // never taken: keeps the warm-up loads
  if constexpr (!EARLY_W) { prefetch_w(); init_acc(); }

  // gain and offset of the LayerNorm that follows the product: requested now where the registers allow it,
  // so that the output pass does not wait for them
  constexpr bool EARLY_LN = OCC == 1 && FB <= 2;
  uint2 lng[FB][4], lno[FB][4];
  if constexpr (EARLY_LN) {
#pragma unroll
    for (int j = 0; j < FB; ++j)
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4) {
        const int c = (wave * FB + j) * 32 + 8 * e4 + 4 * g;
        lng[j][e4] = *reinterpret_cast<const uint2*>(p.gain + c);
        lno[j][e4] = *reinterpret_cast<const uint2*>(p.offs + c);
      }
  }
  for (int ks0 = 0; ks0 < KS; ks0 += PF) {
#pragma unroll
    for (int i = 0; i < PF; ++i) {
      const int ks = (ks0 + i + rot) & (KS - 1);
      uint4 tf[RB];
#pragma unroll
      for (int b = 0; b < RB; ++b) tf[b] = *reinterpret_cast<const uint4*>(&tok[(b * KS + ks) * FRAG + lane * 8]);
#pragma unroll
      for (int j = 0; j < FB; ++j)
#pragma unroll
        for (int b = 0; b < RB; ++b) acc[b][j] = H::mfma(wf[i][j], tf[b], acc[b][j]);
      if (ks0 + i + PF < KS) {
#pragma unroll
        for (int j = 0; j < FB; ++j) wf[i][j] = *reinterpret_cast<const uint4*>(wbase[j] + (size_t)((ks + PF) & (KS - 1)) * 2048);
      }
    }
  }

  // the new residual rows go back; their sums start the LayerNorm statistics
  const bool want_score = p.scores != nullptr;
  float s1[RB];
#pragma unroll
  for (int b = 0; b < RB; ++b) {
    live[b] = in_range[b] && kind_ep[b] != kRowPad;
    s1[b] = 0.f;
#pragma unroll
    for (int j = 0; j < FB; ++j)
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4) {
        const int c = (wave * FB + j) * 32 + 8 * e4 + 4 * g;
        const float4 v = make_float4(acc[b][j][4 * e4], acc[b][j][4 * e4 + 1], acc[b][j][4 * e4 + 2], acc[b][j][4 * e4 + 3]);
        if (live[b] && !want_score) *reinterpret_cast<float4*>(xrow[b] + c) = v;   // nothing reads x after the score head
        s1[b] += (v.x + v.y) + (v.z + v.w);
      }
  }
  if (p.xh == nullptr && !want_score) return;          // uniform over the grid

  // LayerNorm of the new residual rows: two passes over the registers, sums exchanged through LDS
  __syncthreads();                      // every wavefront is done reading tok
#pragma unroll
  for (int b = 0; b < RB; ++b) {
    s1[b] += __shfl_xor(s1[b], 32, 64);
    if (g == 0) red[wave * ROWS + 32 * b + l32] = s1[b];
  }
  __syncthreads();
  float mean[RB], s2[RB];
#pragma unroll
  for (int b = 0; b < RB; ++b) {
    mean[b] = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) mean[b] += red[w * ROWS + 32 * b + l32];
    mean[b] *= 1.0f / (float)D;
    s2[b] = 0.f;
#pragma unroll
    for (int j = 0; j < FB; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) { const float c = acc[b][j][e] - mean[b]; s2[b] += c * c; }
    s2[b] += __shfl_xor(s2[b], 32, 64);
    if (g == 0) red[(NW + wave) * ROWS + 32 * b + l32] = s2[b];
  }
  __syncthreads();
  float score_part[RB];
#pragma unroll
  for (int b = 0; b < RB; ++b) {
    float var = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) var += red[(NW + w) * ROWS + 32 * b + l32];
    const float rstd = rsqrtf(var * (1.0f / (float)D) + p.eps);
    if (want_score) {       // uniform over the grid: the score head's dot product, reduced like the statistics below
      float sc = 0.f;
#pragma unroll
      for (int j = 0; j < FB; ++j)
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
          const int c = (wave * FB + j) * 32 + 8 * e4 + 4 * g;
          const uint2 gg = EARLY_LN ? lng[j][e4] : *reinterpret_cast<const uint2*>(p.gain + c);
          const uint2 oo = EARLY_LN ? lno[j][e4] : *reinterpret_cast<const uint2*>(p.offs + c);
          const uint2 ww = *reinterpret_cast<const uint2*>(p.w_score + c);
          sc += ((acc[b][j][4 * e4] - mean[b]) * rstd * H::to_f32(gg.x & 0xFFFF) + H::to_f32(oo.x & 0xFFFF)) * H::to_f32(ww.x & 0xFFFF);
          sc += ((acc[b][j][4 * e4 + 1] - mean[b]) * rstd * H::to_f32(gg.x >> 16) + H::to_f32(oo.x >> 16)) * H::to_f32(ww.x >> 16);
          sc += ((acc[b][j][4 * e4 + 2] - mean[b]) * rstd * H::to_f32(gg.y & 0xFFFF) + H::to_f32(oo.y & 0xFFFF)) * H::to_f32(ww.y & 0xFFFF);
          sc += ((acc[b][j][4 * e4 + 3] - mean[b]) * rstd * H::to_f32(gg.y >> 16) + H::to_f32(oo.y >> 16)) * H::to_f32(ww.y >> 16);
        }
      score_part[b] = sc + __shfl_xor(sc, 32, 64);
      continue;
    }
    if (!in_range[b]) continue;
    const int row = row0 + 32 * b + l32;
#pragma unroll
    for (int j = 0; j < FB; ++j)
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4) {
        const int c = (wave * FB + j) * 32 + 8 * e4 + 4 * g;
        const uint2 gg = EARLY_LN ? lng[j][e4] : *reinterpret_cast<const uint2*>(p.gain + c);
        const uint2 oo = EARLY_LN ? lno[j][e4] : *reinterpret_cast<const uint2*>(p.offs + c);
        float z0 = (acc[b][j][4 * e4] - mean[b]) * rstd * H::to_f32(gg.x & 0xFFFF) + H::to_f32(oo.x & 0xFFFF);
        float z1 = (acc[b][j][4 * e4 + 1] - mean[b]) * rstd * H::to_f32(gg.x >> 16) + H::to_f32(oo.x >> 16);
        float z2 = (acc[b][j][4 * e4 + 2] - mean[b]) * rstd * H::to_f32(gg.y & 0xFFFF) + H::to_f32(oo.y & 0xFFFF);
        float z3 = (acc[b][j][4 * e4 + 3] - mean[b]) * rstd * H::to_f32(gg.y >> 16) + H::to_f32(oo.y >> 16);
        if (!live[b]) z0 = z1 = z2 = z3 = 0.f;     // filler rows stay finite
        f32x2_t lo = {z0, z1}, hi = {z2, z3};
        uint2 out;
        out.x = H::pack2(lo[0], lo[1]);
        out.y = H::pack2(hi[0], hi[1]);
        *reinterpret_cast<uint2*>(p.xh + panel_off(row, c, D)) = out;
      }
  }
  if (want_score) {
    __syncthreads();                    // the variance sums have been read
#pragma unroll
    for (int b = 0; b < RB; ++b)
      if (g == 0) red[wave * ROWS + 32 * b + l32] = score_part[b];
    __syncthreads();
    if (wave == 0 && g == 0) {
#pragma unroll
      for (int b = 0; b < RB; ++b) {
        float total = p.b_score;
#pragma unroll
        for (int w = 0; w < NW; ++w) total += red[w * ROWS + 32 * b + l32];
        const int row = row0 + 32 * b + l32;
        if (in_range[b] && kind_ep[b] == kRowCand) p.scores[p.rt.src[row]] = total;
      }
    }
  }
}

}  // namespace relaygr
