// Shared device/host declarations of the relay-race kernels (gfx950 only).
//
// Row space of one call.  Every token processed in a call is a "row":
//   [ prefix rows of the users whose prefix is computed in this call, user by user |
//     new rows of every user: that user's suffix tokens, then its candidates ]
// (sequence order of Section 2.3: long-term prefix, short-term / cross tokens, candidates).
// Each row carries its user, its kind, its index inside that segment, the number of keys of
// the user's ordered key sequence [prefix | suffix] it may see (lim), and where its embedding
// comes from.  A candidate additionally sees itself; that term never enters the key sequence.
//
// Cached K/V layout.  Keys are stored in tiles of 64 tokens.  One tile block holds, for every
// layer and head, a K tile (64 tokens x d_head) followed by a V tile (d_head x 64 tokens):
//     base(tile, layer, head) = tile*tile_stride + layer*layer_stride + head*128*dh
//     K element (token r, feature f) at base + KvLayout::k_off(r, f, dh)
//     V element (token r, feature f) at base + KvLayout::v_off(r, f, dh)      (includes the 64*dh K part)
// with tile_stride = n_layers*2*64*d and layer_stride = 2*64*d in the pool, and a single-layer
// form (tile_stride = 2*64*d, layer_stride = 0) in scratch for suffix tokens and for prefixes
// recomputed inside a ranking call.
//   fp32: K row-major [r][f]; V transposed [f][r].
//   bf16: both tiles are stored in the order the 32x32x16 MFMA consumes them, as 1 KiB fragments
//         of 64 lanes x 8 elements, so that a tile in HBM is byte-for-byte the LDS image and every
//         operand fetch is one linear, conflict-free 16-byte read per lane:
//         K fragment (kb, ks): lane (g, l32) holds token kb*32+l32, features ks*16+8g .. +7
//         V fragment (db, kb, m): lane (g, l32) holds feature db*32+l32 and the 8 tokens
//                    kb*32+16m+4g+{0..3}, kb*32+16m+8+4g+{0..3} -- the key order in which the
//                    first product's accumulator hands P to the second product.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

namespace relaygr {

constexpr int kTile = 64;   // tokens per K/V tile

// kRowPad: filler between users in the prefix region of the row space (prefix rows of a user start
// at an aligned row so that GEMM tiles never straddle users); it carries the user and a position >= L.
enum RowKind : int32_t { kRowPrefix = 0, kRowSuffix = 1, kRowCand = 2, kRowPad = 3 };

struct UserDesc {
  const void* kv;          // space holding this user's prefix K/V (pool slab or scratch)
  int64_t kv_tile0;        // element offset of the user's tile 0, layer 0, head 0
  int64_t kv_tile_stride;  // elements between consecutive tiles
  int64_t kv_layer_stride; // elements between layers (0 in single-layer scratch)
  int64_t sfx_tile0;       // element offset of the user's suffix tile 0 in the suffix scratch space
  int32_t L, S, M;
  int32_t prow0;           // first prefix row of this user in the call's row space, -1 if not computed
  int32_t nrow0;           // first new row (suffix rows, then candidates), -1 if the call has none
  int32_t prefix_src0, suffix_src0, cand_src0;  // first row in each embedding array
  int32_t pad0, pad1;
};
static_assert(sizeof(UserDesc) == 80, "UserDesc layout");

// One attention work item: nrows (<= rows per workgroup) consecutive rows of one user.
struct AttnTile {
  int32_t user;
  int32_t row0;     // first row in the call's row space
  int32_t nrows;
  int32_t kind;     // 0: prefix rows (causal over the prefix); 1: new rows
  int32_t pos0;     // prefix rows: position of row0 in the prefix; new rows: index among new rows
  int32_t pad[3];
};
static_assert(sizeof(AttnTile) == 32, "AttnTile layout");

struct RowTables {
  int32_t* user;
  int32_t* kind;
  int32_t* idx;    // index inside the user's segment of that kind
  int32_t* lim;    // keys of [prefix | suffix] visible to this row
  int32_t* src;    // row in the embedding array of its kind
};

template <typename T> struct KvLayout;
template <> struct KvLayout<float> {
  static __host__ __device__ __forceinline__ int k_off(int r, int f, int dh) { return r * dh + f; }
  static __host__ __device__ __forceinline__ int v_off(int r, int f, int dh) { return kTile * dh + f * kTile + r; }
};
// both 16-bit storage types: MFMA fragment order
struct KvLayout16 {
  static __host__ __device__ __forceinline__ int k_off(int r, int f, int dh) {
    int kb = r >> 5, l32 = r & 31, ks = f >> 4, g = (f >> 3) & 1, j = f & 7;
    return ((kb * (dh >> 4) + ks) * 64 + g * 32 + l32) * 8 + j;
  }
  static __host__ __device__ __forceinline__ int v_off(int r, int f, int dh) {
    int db = f >> 5, l32 = f & 31, kb = r >> 5, m = (r >> 4) & 1, w = r & 15;
    int g = (w >> 2) & 1, j = ((w >> 3) << 2) | (w & 3);
    return kTile * dh + (((db * 2 + kb) * 2 + m) * 64 + g * 32 + l32) * 8 + j;
  }
};
template <> struct KvLayout<__hip_bfloat16> : KvLayout16 {};
template <> struct KvLayout<__half> : KvLayout16 {};

// ---- element access in the two storage types ------------------------------------------------
template <typename T> struct Elem;
template <> struct Elem<float> {
  static __device__ __forceinline__ float ld(const float* p) { return *p; }
  static __device__ __forceinline__ void st(float* p, float v) { *p = v; }
};
template <> struct Elem<__hip_bfloat16> {
  static __device__ __forceinline__ float ld(const __hip_bfloat16* p) {
    return __uint_as_float(((uint32_t)(*reinterpret_cast<const uint16_t*>(p))) << 16);
  }
  static __device__ __forceinline__ void st(__hip_bfloat16* p, float v) { *p = __float2bfloat16(v); }
};

template <> struct Elem<__half> {
  static __device__ __forceinline__ float ld(const __half* p) { return __half2float(*p); }
  static __device__ __forceinline__ void st(__half* p, float v) { *p = __float2half(v); }
};

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ uint16_t float_to_bf16_bits(float v) {
  __hip_bfloat16 h = __float2bfloat16(v);
  return *reinterpret_cast<uint16_t*>(&h);
}

// SiLU(t) = t / (1 + exp(-t)), fp32, accurate form (fp32 path and row-wise kernels).
__device__ __forceinline__ float silu_f32(float t) { return t / (1.0f + __expf(-t)); }
// The same through the hardware exp2 and reciprocal approximations (about 1 ulp each): bf16 path.
__device__ __forceinline__ float silu_fast(float t) {
  return t * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(t * -1.4426950408889634f));
}

// element offset of (row, k) in an array of MFMA-ordered panels of row length K: a panel is 128
// rows, stored as 1 KiB fragments [k/16][(row%128)/32][lane][8], lane = ((k/8)%2)*32 + row%32
__host__ __device__ __forceinline__ size_t panel_off(int row, int k, int K) {
  int panel = row >> 7, rb = (row >> 5) & 3, l32 = row & 31, ks = k >> 4, g = (k >> 3) & 1, j = k & 7;
  return ((size_t)panel * (K >> 4) + ks) * 2048 + (size_t)rb * 512 + (g * 32 + l32) * 8 + j;
}

// Streaming stores (the `nt` hint): for kernel outputs that nothing in the same launch reads back.  A plain store
// allocates its line in the XCD's L2, and a launch that writes tens of megabytes pushes out the operand lines the
// workgroups of that XCD share (token panels, weight slices, K/V tiles), which are then fetched again and again
// from the memory side; marked non-temporal, the output lines leave L2 first.  Measured on the projection GEMM
// at 65 536 rows: 225 us with plain stores, 152 us with these (150 us with no stores at all).  Not a general win:
// a workgroup ends only when its stores are acknowledged, which a streaming store is later than a cached one --
// the attention kernel's partial sums and the layer tail's outputs, written once at the end of short-lived
// workgroups, got 13 % and 5-17 % slower with it and keep plain stores.
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void st_stream(uint4* p, uint4 v) { __builtin_nontemporal_store(u32x4_t{v.x, v.y, v.z, v.w}, reinterpret_cast<u32x4_t*>(p)); }
__device__ __forceinline__ void st_stream(uint2* p, uint2 v) { __builtin_nontemporal_store(u32x2_t{v.x, v.y}, reinterpret_cast<u32x2_t*>(p)); }
__device__ __forceinline__ void st_stream(float4* p, float4 v) { __builtin_nontemporal_store(f32x4_t{v.x, v.y, v.z, v.w}, reinterpret_cast<f32x4_t*>(p)); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// v + (v of the lane the DPP control selects), on the vector ALU (no LDS crossbar round trip).
template <int CTRL>
__device__ __forceinline__ float dpp_add(float v) {
  return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
// Sum over each group of 2, 4, 8, 16 consecutive lanes, left in every lane of the group:
// quad_perm [1,0,3,2], quad_perm [2,3,0,1], row_half_mirror, row_mirror.
__device__ __forceinline__ float lanes2_sum(float v) { return dpp_add<0xB1>(v); }
__device__ __forceinline__ float lanes4_sum(float v) { return dpp_add<0x4E>(lanes2_sum(v)); }
__device__ __forceinline__ float lanes8_sum(float v) { return dpp_add<0x141>(lanes4_sum(v)); }
__device__ __forceinline__ float lanes16_sum(float v) { return dpp_add<0x140>(lanes8_sum(v)); }
// Sum over each half of the wavefront, in every lane of the half.
__device__ __forceinline__ float lanes32_sum(float v) {
  v = lanes16_sum(v);
  const int b = __float_as_int(v);
  const float lo = __int_as_float(__builtin_amdgcn_readlane(b, 0)) + __int_as_float(__builtin_amdgcn_readlane(b, 16));
  const float hi = __int_as_float(__builtin_amdgcn_readlane(b, 32)) + __int_as_float(__builtin_amdgcn_readlane(b, 48));
  return (threadIdx.x & 32) ? hi : lo;
}
// Sum over the wavefront, in every lane: 16-lane sums by DPP, the four of them through scalar registers.
__device__ __forceinline__ float wave_sum_dpp(float v) {
  v = lanes16_sum(v);
  const int b = __float_as_int(v);
  return (__int_as_float(__builtin_amdgcn_readlane(b, 0)) + __int_as_float(__builtin_amdgcn_readlane(b, 16))) +
         (__int_as_float(__builtin_amdgcn_readlane(b, 32)) + __int_as_float(__builtin_amdgcn_readlane(b, 48)));
}

}  // namespace relaygr
