// Pointwise-SiLU attention over a user's ordered key sequence [prefix | suffix] (step 3 of a
// layer).  For row i of head h the kernels produce the UNNORMALISED partial sum
//     part_i^h = sum over the keys j of this split with j < lim_i of  SiLU(alpha <q_i^h, k_j^h>) v_j^h
// There is no softmax: terms of different keys simply add, so a split of the key range over
// workgroups needs no renormalisation -- partial sums are added later in fixed split order, the
// candidate's self term and the 1/n_i are applied there too.
//
// Second form (SOFTMAX template flag; the backbone variant of Section 4.4 read as a softmax over
// the visible keys): the kernels produce, per row, head and key split, a reference score m, the
// sum l of exp(s_j - m) over the split's visible keys and the sum of exp(s_j - m) v_j; m is a
// running maximum, so nothing overflows, and the splits and the candidate's own key are merged
// afterwards by softmax_combine_kernel (rowwise.h).
//
// Keys come in tiles of 64 tokens (layout in common.h): a K tile [64][dh] followed by a V tile
// stored transposed [dh][64].  Prefix tiles come from the user's K/V space (pool or scratch),
// suffix tiles from the suffix scratch space.  Only three kinds of tile need a per-element
// visibility test: the ragged last prefix tile, suffix tiles (causal for suffix rows), and the
// diagonal tiles of the causal prefix pass.
#pragma once

#include "common.h"
#include "gemm.h"

namespace relaygr {

struct AttnParams {
  const AttnTile* tiles;
  const UserDesc* users;
  RowTables rt;
  const void* q;      // [rows][d]
  const void* sfx;    // suffix K/V space (single layer)
  float* part;        // [nsplit][rows][d]
  size_t split_stride;
  float* ml;          // softmax form: [nsplit][rows][n_heads][2] = (m, l) of each row, head and split
  size_t ml_stride;   // floats between the (m, l) tables of consecutive splits
  int nsplit;
  int n_tiles;        // work items in this launch
  int d, n_heads, layer;
  float score_mul;    // multiplies <q,k> before SiLU (alpha, or 1 if q is stored pre-scaled)
  // MFMA kernel, SiLU form: a candidate's own key (the diagonal of the candidate block: a per-row dot product, never an
  // M x M tile) is where the sums of one of the row's key splits start (row block qb: split qb mod nsplit), from the
  // row-major k and v of the new rows; null: left to the layer-tail kernel
  const void* knew;   // [new rows][d]
  const void* vnew;
  int n_prows;        // rows before the first new row
  int gs;             // MFMA kernel: key splits taken by the wavefront groups of one workgroup and added in LDS (1 or 2)
};

// Key-tile schedule of one work item, shared by both kernels.
struct TileRange {
  int nkp;       // prefix tiles this item needs
  int nfull;     // leading prefix tiles every row of the item sees completely
  int nks;       // suffix tiles
  int t0, t1;    // this split's range in the concatenated list [prefix tiles | suffix tiles]
};

__device__ __forceinline__ TileRange tile_range(const AttnTile& at, const UserDesc& ud, int split, int nsplit) {
  TileRange tr;
  if (at.kind == 0) {  // prefix rows: causal, keys 0 .. pos0 + nrows - 1
    tr.nkp = (at.pos0 + at.nrows + kTile - 1) / kTile;
    tr.nfull = (at.pos0 + 1) / kTile;
    tr.nks = 0;
  } else {             // new rows: the whole prefix, then the suffix
    tr.nkp = (ud.L + kTile - 1) / kTile;
    tr.nfull = ud.L / kTile;
    tr.nks = (ud.S + kTile - 1) / kTile;
  }
  int total = tr.nkp + tr.nks;
  int per = (total + nsplit - 1) / nsplit;
  tr.t0 = min(split * per, total);
  tr.t1 = min(tr.t0 + per, total);
  return tr;
}

// ---- fp32 kernel: one thread per row, keys broadcast from LDS -----------------------------------
template <int DH, bool SOFTMAX>
__global__ __launch_bounds__(64) void attn_f32_kernel(AttnParams p) {
  __shared__ float Ks[kTile * DH];
  __shared__ float Vs[DH * kTile];
  const AttnTile at = p.tiles[blockIdx.x];
  const int head = blockIdx.y, split = blockIdx.z;
  const UserDesc ud = p.users[at.user];
  const TileRange tr = tile_range(at, ud, split, p.nsplit);
  const int t = threadIdx.x;
  const bool active = t < at.nrows;
  const int row = at.row0 + (active ? t : 0);
  const int lim = active ? p.rt.lim[row] : 0;

  float qv[DH], o[DH];
  const float* qrow = reinterpret_cast<const float*>(p.q) + (size_t)row * p.d + head * DH;
#pragma unroll
  for (int f = 0; f < DH; ++f) { qv[f] = qrow[f] * p.score_mul; o[f] = 0.f; }
  float m = -INFINITY, l = 0.f;   // softmax form: running maximum and sum of exp(s - m)

  for (int tt = tr.t0; tt < tr.t1; ++tt) {
    const bool is_sfx = tt >= tr.nkp;
    const float* src;
    int key0, seg_end;
    if (!is_sfx) {
      src = reinterpret_cast<const float*>(ud.kv) + ud.kv_tile0 + (int64_t)tt * ud.kv_tile_stride +
            (int64_t)p.layer * ud.kv_layer_stride + (int64_t)head * 2 * kTile * DH;
      key0 = tt * kTile; seg_end = ud.L;
    } else {
      int st = tt - tr.nkp;
      src = reinterpret_cast<const float*>(p.sfx) + ud.sfx_tile0 + (int64_t)st * (2 * kTile * p.d) +
            (int64_t)head * 2 * kTile * DH;
      key0 = ud.L + st * kTile; seg_end = ud.L + ud.S;
    }
    __syncthreads();
    for (int i = t; i < kTile * DH; i += 64) { Ks[i] = src[i]; Vs[i] = src[kTile * DH + i]; }
    __syncthreads();
    const int vis = min(lim, seg_end) - key0;  // keys [0, vis) of this tile are visible to this row
    for (int j = 0; j < kTile; ++j) {
      float s = 0.f;
#pragma unroll
      for (int f = 0; f < DH; ++f) s = fmaf(qv[f], Ks[j * DH + f], s);
      float pj;
      if constexpr (SOFTMAX) {
        if (j < vis && s > m) {        // new maximum: bring what was summed so far to the new reference
          const float c = __expf(m - s);
          l *= c;
#pragma unroll
          for (int f = 0; f < DH; ++f) o[f] *= c;
          m = s;
        }
        pj = (j < vis) ? __expf(s - m) : 0.f;
        l += pj;
      } else {
        pj = (j < vis) ? silu_f32(s) : 0.f;
      }
#pragma unroll
      for (int f = 0; f < DH; ++f) o[f] = fmaf(pj, Vs[f * kTile + j], o[f]);
    }
  }
  if (active) {
    float* dst = p.part + split * p.split_stride + (size_t)row * p.d + head * DH;
#pragma unroll
    for (int f = 0; f < DH; ++f) dst[f] = o[f];
    if constexpr (SOFTMAX) {
      float* mlp = p.ml + split * p.ml_stride + ((size_t)row * p.n_heads + head) * 2;
      mlp[0] = m; mlp[1] = l;
    }
  }
}

// ---- bf16 MFMA kernel ---------------------------------------------------------------------------
// A workgroup of NW wavefronts owns up to NW*32*NQ rows (each wavefront NQ blocks of 32 rows) of one
// user and one head and walks the key tiles of its split.  Per 32-key half tile and wavefront:
//   S^T[32 keys][32 rows]  = K half (A operand, rows = keys)  x  Q^T (B operand, held in registers)
//   P^T = SiLU'(S^T) rounded to bf16 -- the accumulator layout of S^T (lane = row, 4-key runs) is
//         exactly the B-operand layout of the next product once the V fragment holds the same key
//         permutation (it does, see the layout note in common.h), so P never leaves registers
//   O^T[dh][32 rows]      += V^T half (A operand, rows = features) x P^T
// q is stored pre-multiplied by alpha*log2(e); SiLU'(t) = t / (1 + 2^-t) = SiLU(s)/ln 2 with
// s = t ln 2, and the ln 2 is applied once to the output.
//
// A K/V tile in HBM is already the LDS image (fragment order), so tiles stream HBM -> LDS with
// direct 16-byte-per-lane loads into a ring of three buffers, one barrier per tile, and every MFMA
// operand is one linear ds_read_b128.  The loop is software-pipelined by half tiles: while the
// vector ALU evaluates the SiLU of half h, the matrix pipe runs the first product of half h+1 and
// the second product of half h-1, none of which depend on that SiLU.  What bounds the kernel is the SiLU itself: one v_exp_f32 and one v_rcp_f32
// (quarter-rate) plus add, multiply and half a packed bf16 convert per score element, against
// 2*DH/32 MFMA passes per 32 x 32 block.

template <typename H, int DH, int NQ>
__device__ __forceinline__ void attn_s_half(const uint16_t* __restrict__ khalf, const uint4 (&qf)[NQ][DH / 16],
                                            f32x16_t (&s)[NQ]) {
  constexpr int KS = DH / 16;
#pragma unroll
  for (int qb = 0; qb < NQ; ++qb)
#pragma unroll
    for (int e = 0; e < 16; ++e) s[qb][e] = 0.f;
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    const uint4 kf = *reinterpret_cast<const uint4*>(khalf + ks * 512);
#pragma unroll
    for (int qb = 0; qb < NQ; ++qb) s[qb] = H::mfma(kf, qf[qb][ks], s[qb]);
  }
}

template <typename H, int DH, int NQ>
__device__ __forceinline__ void attn_pv_half(const uint16_t* __restrict__ vhalf, const uint32_t (&pk)[NQ][8],
                                             f32x16_t (&oacc)[DH / 32][NQ]) {
  constexpr int DB = DH / 32;
#pragma unroll
  for (int m = 0; m < 2; ++m) {
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      const uint4 vf = *reinterpret_cast<const uint4*>(vhalf + (db * 4 + m) * 512);
#pragma unroll
      for (int qb = 0; qb < NQ; ++qb) {
        uint4 pp = make_uint4(pk[qb][4 * m], pk[qb][4 * m + 1], pk[qb][4 * m + 2], pk[qb][4 * m + 3]);
        oacc[db][qb] = H::mfma(vf, pp, oacc[db][qb]);
      }
    }
  }
}

// One pipeline step of a wavefront: the SiLU of the half tile whose first product is in s_in runs
// on the vector ALU while the matrix pipe computes the first product of the following half
// (khalf -> s_out) and the second product owed from the preceding half (vhalf, pk_in -> oacc).
// A wavefront issues in order and an MFMA cannot issue while the matrix pipe still works on the
// previous one, so MFMAs placed back to back would leave the vector ALU idle behind them.  The
// step is therefore cut into slots -- the SiLU of 128/DH score elements per row block, then NQ
// MFMAs that take about as long -- and the scheduler is fenced between slots.
template <typename H, int DH, int NQ, bool MASKED, bool SOFTMAX>
__device__ __forceinline__ void attn_step(const uint16_t* __restrict__ khalf, const uint16_t* __restrict__ vhalf,
                                          const uint4 (&qf)[NQ][DH / 16], const f32x16_t (&s_in)[NQ], f32x16_t (&s_out)[NQ],
                                          const uint32_t (&pk_in)[NQ][8], uint32_t (&pk_out)[NQ][8],
                                          f32x16_t (&oacc)[DH / 32][NQ], const int (&vis)[NQ],
                                          const float (&mref)[NQ], float (&lsum)[NQ]) {
  constexpr int KS = DH / 16, DB = DH / 32;
  constexpr int SLOTS = KS + 2 * DB;      // = DH / 8
  constexpr int EPS = 16 / SLOTS > 0 ? 16 / SLOTS : 1;   // score elements per row block and slot
  static_assert(SLOTS * EPS == 16 || (SLOTS == 16 && EPS == 1), "slot split");
  uint4 kf[KS], vf[2][DB];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) kf[ks] = *reinterpret_cast<const uint4*>(khalf + ks * 512);
#pragma unroll
  for (int m = 0; m < 2; ++m)
#pragma unroll
    for (int db = 0; db < DB; ++db) vf[m][db] = *reinterpret_cast<const uint4*>(vhalf + (db * 4 + m) * 512);
  float pv[NQ][16];
  const f32x16_t zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int slot = 0; slot < SLOTS; ++slot) {
    // vector ALU first (the fragment reads above are still in flight during slot 0): SiLU' of this
    // slot's score elements; element e is key 8*(e/4) + 4*g + e%4 of the half
#pragma unroll
    for (int qb = 0; qb < NQ; ++qb) {
#pragma unroll
      for (int e = slot * EPS; e < (slot + 1) * EPS; ++e) {
        const float t = s_in[qb][e];
        float pe;
        if constexpr (SOFTMAX) pe = __builtin_amdgcn_exp2f(t - mref[qb]);
        else pe = t * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-t));
        if (MASKED) pe = (8 * (e >> 2) + (e & 3) < vis[qb]) ? pe : 0.f;
        if constexpr (SOFTMAX) lsum[qb] += pe;
        pv[qb][e] = pe;
        if (e & 1) {
          f32x2_t two = {pv[qb][e - 1], pv[qb][e]};
          pk_out[qb][e >> 1] = H::pack2(two[0], two[1]);   // one packed convert
        }
      }
    }
    // matrix pipe: even slots feed the first product, odd slots the second (KS == 2*DB), so that
    // dependent MFMAs are two slots apart
    const int si = slot / 2;
    if (slot % 2 == 0) {
#pragma unroll
      for (int qb = 0; qb < NQ; ++qb)
        s_out[qb] = H::mfma(kf[si], qf[qb][si], si == 0 ? zero : s_out[qb]);
    } else {
      const int m = si / DB, db = si % DB;
#pragma unroll
      for (int qb = 0; qb < NQ; ++qb) {
        uint4 pp = make_uint4(pk_in[qb][4 * m], pk_in[qb][4 * m + 1], pk_in[qb][4 * m + 2], pk_in[qb][4 * m + 3]);
        oacc[db][qb] = H::mfma(vf[m][db], pp, oacc[db][qb]);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  }
}

// Softmax form: keeps each row's reference score m (in log2 units, like the stored q) within
// kSoftmaxSlack of the largest visible score seen so far, so that exp2(t - m) <= 2^kSoftmaxSlack fits
// either 16-bit type.  Called before the step that exponentiates the half tile s: when no lane
// holds a score above m + slack (the common case after the first half tile) nothing happens.
// Otherwise, for the whole wavefront: the second product still owed from the preceding half
// (computed against the old references) is issued now and its P cleared, then m rises to the
// running maximum -- the two lanes of a row (l32, g = 0 and 1) exchange theirs, a row has one m --
// and the sums gathered so far are scaled by 2^(m_old - m_new).
constexpr float kSoftmaxSlack = 8.0f;

template <typename H, int DH, int NQ, bool MASKED>
__device__ __forceinline__ void softmax_track(const f32x16_t (&s)[NQ], const int (&vis)[NQ], float (&mref)[NQ], float (&lsum)[NQ],
                                              f32x16_t (&oacc)[DH / 32][NQ], uint32_t (&pk_owed)[NQ][8],
                                              const uint16_t* __restrict__ v_owed) {
  float mx[NQ];
  bool need = false;
#pragma unroll
  for (int qb = 0; qb < NQ; ++qb) {
    mx[qb] = -INFINITY;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      float t = s[qb][e];
      if (MASKED) t = (8 * (e >> 2) + (e & 3) < vis[qb]) ? t : -INFINITY;
      mx[qb] = fmaxf(mx[qb], t);
    }
    need |= mx[qb] > mref[qb] + kSoftmaxSlack;
  }
  if (__builtin_amdgcn_ballot_w64(need) == 0) return;
  attn_pv_half<H, DH, NQ>(v_owed, pk_owed, oacc);
#pragma unroll
  for (int qb = 0; qb < NQ; ++qb) {
#pragma unroll
    for (int e = 0; e < 8; ++e) pk_owed[qb][e] = 0u;
    const float both = fmaxf(mx[qb], __shfl_xor(mx[qb], 32, 64));
    const float mn = fmaxf(mref[qb], both);
    const float c = (mn == mref[qb]) ? 1.0f : __builtin_amdgcn_exp2f(mref[qb] - mn);   // from -inf: 0
    mref[qb] = mn;
    lsum[qb] *= c;
#pragma unroll
    for (int db = 0; db < DH / 32; ++db)
#pragma unroll
      for (int e = 0; e < 16; ++e) oacc[db][qb][e] *= c;
  }
}

// GS = 2: the workgroup is two groups of NW wavefronts over the SAME rows; each group takes one of two
// consecutive key splits with a tile ring of its own, and at the end the second group's sums go through LDS to the
// first, which adds them (first + second, a fixed order; in the softmax form after bringing both to the larger of their
// reference scores) and writes one partial sum: two key splits cost the layer tail the HBM traffic of one.  Both
// groups pass the same barriers; a group with fewer tiles pads with empty ones.
template <typename H, int DH, int NQ, int NW, bool SOFTMAX, int GS = 1>
__global__ __launch_bounds__(NW * GS * 64, (DH >= 128 || GS > 1) ? 1 : 512 / (NW * 64)) void attn_bf16_kernel(AttnParams p) {   // DH = 128: the 96 KiB tile ring admits one workgroup per compute unit
  constexpr int KS = DH / 16;              // k-steps of the first product
  constexpr int DB = DH / 32;              // 32-feature blocks of the output
  constexpr int TILE = 2 * kTile * DH;     // elements of one K tile + one V tile
  constexpr int CHUNKS = TILE / 8 / (NW * 64);   // 16-byte chunks each thread moves per tile
  static_assert(CHUNKS >= 1, "a tile is at least one 16-byte chunk per thread");
  static_assert(GS == 1 || GS == 2, "groups: one or two");
  static_assert(GS * 3 * TILE * 2 >= (GS - 1) * NW * 64 * (DB * NQ * 16 + 2 * NQ) * 4, "the second group's sums fit the rings' LDS");
  __shared__ __attribute__((aligned(16))) uint16_t bufs_all[GS][3][TILE];

  // Work items that stream the same K/V (row tiles of one user, same head and split) get
  // consecutive logical ids, and each of the 8 XCDs (own L2 each; workgroups are dealt to them
  // round-robin) takes a contiguous run of logical ids: the K/V tiles are then fetched from HBM
  // once per XCD and found in its L2 by the neighbouring row tiles.
  const int total = p.n_tiles * p.n_heads * p.nsplit;
  const int logical = xcd_remap(blockIdx.x, total);
  if (logical >= total) return;
  const int tile_i = logical % p.n_tiles, hs = logical / p.n_tiles;
  const int head = hs % p.n_heads, split_ext = hs / p.n_heads;
  const AttnTile at = p.tiles[tile_i];
  const UserDesc ud = p.users[at.user];
  const int tid = threadIdx.x, lane = tid & 63;
  const int grp = GS == 1 ? 0 : __builtin_amdgcn_readfirstlane((tid >> 6) / NW);    // wavefront group (a scalar: loop counts below depend on it)
  const int wave = (tid >> 6) - grp * NW;           // wavefront inside its group: its rows, its share of a tile
  const int split = split_ext * GS + grp, nsplit = p.nsplit * GS;   // this group's key split of all
  const TileRange tr = tile_range(at, ud, split, nsplit);
  uint16_t (*bufs)[TILE] = bufs_all[grp];
  const int l32 = lane & 31, g = lane >> 5;

  // this lane's rows: block qb covers rows wave*32*NQ + qb*32 + l32 of the work item
  int lim[NQ];
  uint4 qf[NQ][KS];
  const uint16_t* qbase = reinterpret_cast<const uint16_t*>(p.q);
#pragma unroll
  for (int qb = 0; qb < NQ; ++qb) {
    int lr = wave * 32 * NQ + qb * 32 + l32;
    bool ok = lr < at.nrows;
    int row = at.row0 + (ok ? lr : 0);
    lim[qb] = ok ? p.rt.lim[row] : 0;
    const uint16_t* qr = qbase + (size_t)row * p.d + head * DH + g * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[qb][ks] = *reinterpret_cast<const uint4*>(qr + ks * 16);
  }

  f32x16_t oacc[DB][NQ];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int qb = 0; qb < NQ; ++qb)
#pragma unroll
      for (int e = 0; e < 16; ++e) oacc[db][qb][e] = 0.f;
  float mref[NQ], lsum[NQ];   // softmax form: reference score of the row, this lane's sum of exp2(t - m)
#pragma unroll
  for (int qb = 0; qb < NQ; ++qb) { mref[qb] = -INFINITY; lsum[qb] = 0.f; }

  // The candidate's own key (SiLU form): the sums of key split 0 start from it instead of from zero.  Its k and v rows
  // are requested here, ahead of the first key tiles, and used once those are on their way.  q and k carry the same
  // scaling as in the key tiles (t in log2 units), the term takes the common ln 2 at the end; fp32 throughout.  A
  // row's q fragments are split over its two lanes (g = 0, 1).
  // With several key splits the row blocks' own keys are dealt over the splits' work items (block qb to split qb mod nsplit),
  // so that no work item carries all of them.
  const bool own_key = !SOFTMAX && p.knew != nullptr && at.kind == 1 && split < NQ;
  uint4 kself[NQ][KS];
  uint2 vself[NQ][DB][4];
  bool cand[NQ];
#pragma unroll
  for (int qb = 0; qb < NQ; ++qb) {
    const int lr = wave * 32 * NQ + qb * 32 + l32;
    cand[qb] = own_key && (qb % nsplit) == split && lr < at.nrows && at.pos0 + lr >= ud.S;   // new rows: suffix rows, then candidates
    if (cand[qb]) {
      const size_t nb = (size_t)(at.row0 + lr - p.n_prows) * p.d + head * DH;
      const uint16_t* kn = reinterpret_cast<const uint16_t*>(p.knew) + nb;
      const uint16_t* vn = reinterpret_cast<const uint16_t*>(p.vnew) + nb;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) kself[qb][ks] = *reinterpret_cast<const uint4*>(kn + ks * 16 + g * 8);
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) vself[qb][db][e4] = *reinterpret_cast<const uint2*>(vn + db * 32 + 8 * e4 + 4 * g);
    }
  }
  auto start_from_own_key = [&]() {
    if (!own_key) return;                       // uniform over the workgroup
#pragma unroll
    for (int qb = 0; qb < NQ; ++qb) {
      float dot = 0.f;
      if (cand[qb]) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          const uint32_t qw[4] = {qf[qb][ks].x, qf[qb][ks].y, qf[qb][ks].z, qf[qb][ks].w};
          const uint32_t kw[4] = {kself[qb][ks].x, kself[qb][ks].y, kself[qb][ks].z, kself[qb][ks].w};
#pragma unroll
          for (int i = 0; i < 4; ++i) dot = H::dot2(qw[i], kw[i], dot);
        }
      }
      dot += __shfl_xor(dot, 32, 64);
      const float pe = cand[qb] ? dot / (1.0f + __builtin_amdgcn_exp2f(-dot)) : 0.f;
      if (cand[qb]) {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int e4 = 0; e4 < 4; ++e4) {
            oacc[db][qb][4 * e4] = pe * H::of_word(vself[qb][db][e4].x, 0);
            oacc[db][qb][4 * e4 + 1] = pe * H::of_word(vself[qb][db][e4].x, 1);
            oacc[db][qb][4 * e4 + 2] = pe * H::of_word(vself[qb][db][e4].y, 0);
            oacc[db][qb][4 * e4 + 3] = pe * H::of_word(vself[qb][db][e4].y, 1);
          }
      }
    }
  };

  const uint16_t* kv_base = reinterpret_cast<const uint16_t*>(ud.kv) + ud.kv_tile0 + (int64_t)p.layer * ud.kv_layer_stride +
                            (int64_t)head * TILE;
  const uint16_t* sfx_base = reinterpret_cast<const uint16_t*>(p.sfx) + ud.sfx_tile0 + (int64_t)head * TILE;
  const int64_t sfx_stride = (int64_t)2 * kTile * p.d;

  // HBM -> LDS, no registers in between: wavefront w moves the 1 KiB pieces w, w+NW, ... of the tile
  auto issue_tile = [&](int tt, int b) {
    const uint16_t* src = (tt < tr.nkp) ? kv_base + (int64_t)tt * ud.kv_tile_stride : sfx_base + (int64_t)(tt - tr.nkp) * sfx_stride;
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) {
      const int piece = i * NW + wave;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + piece * 512 + lane * 8),
                                       (__attribute__((address_space(3))) void*)(&bufs[b][piece * 512]), 16, 0, 0);
    }
  };

  // a wavefront whose rows all lie beyond the work item's last row only helps move tiles
  const bool wave_active = wave * 32 * NQ < at.nrows;
  const int nt = tr.t1 - tr.t0;
  int nt_all = nt;                    // barriers every wavefront of the workgroup passes in the tile loop
  if constexpr (GS == 2) {
    const TileRange tro = tile_range(at, ud, split ^ 1, nsplit);
    nt_all = max(nt, tro.t1 - tro.t0);
  }
  if (nt == 0) start_from_own_key();
  if (nt > 0) {
    issue_tile(tr.t0, 0);
    if (nt > 1) issue_tile(tr.t0 + 1, 1);
    start_from_own_key();             // its loads are older than the tiles'
    if (nt > 1) {
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(CHUNKS) : "memory");   // tile 0 landed, tile 1 may still fly
    } else {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    __syncthreads();

    // Pipeline state.  s_cur: first product of the half about to get its SiLU.  pk_prev: P of the
    // half before it, whose second product is still owed, with vprev pointing at its V half.
    f32x16_t s_cur[NQ], s_nxt[NQ];
    uint32_t pk_a[NQ][8], pk_b[NQ][8];
#pragma unroll
    for (int qb = 0; qb < NQ; ++qb)
#pragma unroll
      for (int e = 0; e < 8; ++e) pk_b[qb][e] = 0u;          // nothing owed yet: P = 0 adds nothing
    const uint16_t* vprev = &bufs[0][lane * 8] + kTile * DH;  // any finite V will do with P = 0
    attn_s_half<H, DH, NQ>(&bufs[0][lane * 8], qf, s_cur);
    int b = 0;                                                 // ring slot of tile i

    // one tile = two pipeline steps; MASKED tiles apply the per-element visibility test
    auto tile_iter = [&](auto masked_tag, int i) {
      constexpr bool MASKED = decltype(masked_tag)::value;
      int vis[NQ] = {};
      if (MASKED) {
        const int tt = tr.t0 + i;
        const bool is_sfx = tt >= tr.nkp;
        const int key0 = is_sfx ? ud.L + (tt - tr.nkp) * kTile : tt * kTile;
        const int seg_end = is_sfx ? ud.L + ud.S : ud.L;
#pragma unroll
        for (int qb = 0; qb < NQ; ++qb) vis[qb] = min(lim[qb], seg_end) - key0 - 4 * g;
      }
      const uint16_t* kt = &bufs[b][lane * 8];
      const uint16_t* vt = kt + kTile * DH;
      // step 1: SiLU of the first half | first product of the second half, second product owed from before
      if (wave_active) {
        if constexpr (SOFTMAX) softmax_track<H, DH, NQ, MASKED>(s_cur, vis, mref, lsum, oacc, pk_b, vprev);
        attn_step<H, DH, NQ, MASKED, SOFTMAX>(kt + KS * 512, vprev, qf, s_cur, s_nxt, pk_b, pk_a, oacc, vis, mref, lsum);
      }
      // the next tile must have landed before its first product; every wavefront is now past tile i-1
      const int bn = (b == 2) ? 0 : b + 1;
      const bool more = i + 1 < nt;
      if (more) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (i + 2 < nt) issue_tile(tr.t0 + i + 2, (bn == 2) ? 0 : bn + 1);
      }
      // step 2: SiLU of the second half | first product of the next tile's first half (a repeat of
      // this tile's when there is none: its result is dropped), second product of the first half
      if (MASKED) {
#pragma unroll
        for (int qb = 0; qb < NQ; ++qb) vis[qb] -= 32;
      }
      if (wave_active) {
        if constexpr (SOFTMAX) softmax_track<H, DH, NQ, MASKED>(s_nxt, vis, mref, lsum, oacc, pk_a, vt);
        attn_step<H, DH, NQ, MASKED, SOFTMAX>(more ? &bufs[bn][lane * 8] : kt, vt, qf, s_nxt, s_cur, pk_a, pk_b, oacc, vis, mref, lsum);
      }
      vprev = vt + 2 * 512;
      b = bn;
    };

    // tiles of this split in order: [fully visible prefix tiles][tiles needing the visibility test]
    const int n_plain = max(0, min(tr.t1, tr.nfull) - tr.t0);
    int i = 0;
    for (; i < n_plain; ++i) tile_iter(std::false_type(), i);
    for (; i < nt; ++i) tile_iter(std::true_type(), i);
    attn_pv_half<H, DH, NQ>(vprev, pk_b, oacc);                   // the last half's second product
  }

  if constexpr (GS == 2) {
    // A group passed nt barriers above (none if it had no tiles); both groups pass nt_all, then two more around the
    // hand-over of the second group's sums.  Nothing below returns before the last of them.
    for (int e = nt; e < nt_all; ++e) __syncthreads();
    __syncthreads();                                  // both groups are done with their tile rings
    float* xch = reinterpret_cast<float*>(&bufs_all[0][0][0]);
    const int slot = wave * 64 + lane;                // lane of the first group that holds the same rows and features
    if (grp == 1) {
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int qb = 0; qb < NQ; ++qb)
#pragma unroll
          for (int e = 0; e < 16; ++e) xch[((db * NQ + qb) * 16 + e) * (NW * 64) + slot] = oacc[db][qb][e];
      if constexpr (SOFTMAX) {
#pragma unroll
        for (int qb = 0; qb < NQ; ++qb) {
          xch[(DB * NQ * 16 + 2 * qb) * (NW * 64) + slot] = mref[qb];
          xch[(DB * NQ * 16 + 2 * qb + 1) * (NW * 64) + slot] = lsum[qb];
        }
      }
    }
    __syncthreads();
    if (grp == 1) return;
    // softmax form: both groups' sums are brought to the larger of their two reference scores first
    float c0[NQ], c1[NQ];
#pragma unroll
    for (int qb = 0; qb < NQ; ++qb) {
      c0[qb] = 1.0f; c1[qb] = 1.0f;
      if constexpr (SOFTMAX) {
        const float m1 = xch[(DB * NQ * 16 + 2 * qb) * (NW * 64) + slot], l1 = xch[(DB * NQ * 16 + 2 * qb + 1) * (NW * 64) + slot];
        const float M = fmaxf(mref[qb], m1);
        c0[qb] = (mref[qb] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mref[qb] - M);
        c1[qb] = (m1 == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m1 - M);
        lsum[qb] = lsum[qb] * c0[qb] + l1 * c1[qb];
        mref[qb] = M;
      }
    }
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int qb = 0; qb < NQ; ++qb)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const float x = xch[((db * NQ + qb) * 16 + e) * (NW * 64) + slot];
          if constexpr (SOFTMAX) oacc[db][qb][e] = oacc[db][qb][e] * c0[qb] + x * c1[qb];
          else oacc[db][qb][e] += x;
        }
  }

  // element e of oacc[db][qb]: feature db*32 + 8*(e/4) + 4*g + e%4, row l32 of block qb
  const float kLn2 = SOFTMAX ? 1.0f : 0.69314718055994531f;
  if constexpr (SOFTMAX) {   // a row's sum is spread over its two lanes
#pragma unroll
    for (int qb = 0; qb < NQ; ++qb) lsum[qb] += __shfl_xor(lsum[qb], 32, 64);
  }
#pragma unroll
  for (int qb = 0; qb < NQ; ++qb) {
    int lr = wave * 32 * NQ + qb * 32 + l32;
    if (lr >= at.nrows) continue;
    if constexpr (SOFTMAX) {
      if (g == 0) {
        float* mlp = p.ml + split_ext * p.ml_stride + ((size_t)(at.row0 + lr) * p.n_heads + head) * 2;
        *reinterpret_cast<float2*>(mlp) = make_float2(mref[qb], lsum[qb]);
      }
    }
    float* dst = p.part + split_ext * p.split_stride + (size_t)(at.row0 + lr) * p.d + head * DH;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4) {
        float4 v = make_float4(oacc[db][qb][4 * e4] * kLn2, oacc[db][qb][4 * e4 + 1] * kLn2,
                               oacc[db][qb][4 * e4 + 2] * kLn2, oacc[db][qb][4 * e4 + 3] * kLn2);
        *reinterpret_cast<float4*>(dst + db * 32 + 8 * e4 + 4 * g) = v;
      }
  }
}

}  // namespace relaygr
