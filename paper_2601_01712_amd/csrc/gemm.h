// Projection GEMMs of a layer (steps 2 and 4): C[rows, N] = A[rows, K] * W[N, K]^T, with the
// layer's pointwise work fused into the epilogue.
//   f1: SiLU(xh W1^T + b1), split into u | v | q | k; u and q go to row-major scratch, k and v of
//       prefix / suffix rows are scattered straight into K/V tile layout (pool or scratch), k and
//       v of candidate rows go to row-major scratch for the self term.
//   f2: x <- x + y W2^T + b2 on the fp32 residual stream.
// This file holds what the fp32 path uses (per-element epilogue functors, a plain LDS-tiled FMA
// GEMM) and small pieces shared with the bf16 MFMA GEMMs of gemm_bf16.h.
#pragma once

#include "common.h"

namespace relaygr {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));

// The two 16-bit storage types of the MFMA path (bf16: the benchmark's; fp16: the half precision the
// paper mentions as lowering the rank stage, Section 4.2).  Kernels are written against this
// interface: bit patterns in, fp32 out; pack2 rounds to nearest even; mfma is the 32x32x16 product
// of two 8-element fragments.
struct Bf16 {
  using elem = __hip_bfloat16;
  static __device__ __forceinline__ float to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
  static __device__ __forceinline__ float of_word(uint32_t w, int i) { return __uint_as_float((i & 1) ? (w & 0xFFFF0000u) : (w << 16)); }
  static __device__ __forceinline__ uint32_t pack2(float a, float b) {
    f32x2_t v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));     // one v_cvt_pk_bf16_f32
  }
  // c + a.lo * b.lo + a.hi * b.hi on two packed pairs, fp32 accumulate (v_dot2c_f32_bf16)
  static __device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), c, false);
  }
  static __device__ __forceinline__ f32x16_t mfma(uint4 a, uint4 b, f32x16_t c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
  }
};
struct F16 {
  using elem = __half;
  static __device__ __forceinline__ float to_f32(uint16_t b) { return (float)__builtin_bit_cast(_Float16, b); }
  static __device__ __forceinline__ float of_word(uint32_t w, int i) { return (float)__builtin_bit_cast(f16x2_t, w)[i & 1]; }
  static __device__ __forceinline__ uint32_t pack2(float a, float b) {
    f32x2_t v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2_t));      // one v_cvt_pk_f16_f32
  }
  static __device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c) {
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2_t, a), __builtin_bit_cast(f16x2_t, b), c, false);
  }
  static __device__ __forceinline__ f32x16_t mfma(uint4 a, uint4 b, f32x16_t c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
  }
};
template <typename T> struct HalfOf { using type = Bf16; };
template <> struct HalfOf<__half> { using type = F16; };

// Which output column blocks (of width d) a launch produces: block j of the launch is block
// blk[j] of the weight (f1 on last-layer prefix rows needs only v and k).
struct ColMap {
  int nblk;
  int blk[4];
  int d;   // block width
};

// ---- epilogues -------------------------------------------------------------------------------
template <typename T>
struct F1Epilogue {
  const T* bias;
  T* u; T* q; T* knew; T* vnew; T* sfx;
  const UserDesc* users;
  RowTables rt;
  int d, dh, n_prows, layer;
  float q_mul;  // q is stored as q_mul * SiLU(.)

  __device__ __forceinline__ void operator()(int r, int col, float acc) const {
    float val = silu_f32(acc + Elem<T>::ld(bias + col));
    int blk = col / d, c = col - blk * d;
    if (blk == 0) { Elem<T>::st(u + (size_t)r * d + c, val); return; }
    if (blk == 2) { Elem<T>::st(q + (size_t)r * d + c, val * q_mul); return; }
    bool is_k = (blk == 3);
    int kind = rt.kind[r];
    if (kind == kRowCand) {
      Elem<T>::st((is_k ? knew : vnew) + (size_t)(r - n_prows) * d + c, val);
      return;
    }
    const UserDesc& ud = users[rt.user[r]];
    int idx = rt.idx[r];
    int h = c / dh, f = c - h * dh;
    int64_t tile = idx / kTile;
    int rr = idx % kTile;
    T* base;
    if (kind == kRowPrefix)
      base = const_cast<T*>(reinterpret_cast<const T*>(ud.kv)) + ud.kv_tile0 + tile * ud.kv_tile_stride +
             (int64_t)layer * ud.kv_layer_stride + (int64_t)h * 2 * kTile * dh;
    else
      base = sfx + ud.sfx_tile0 + tile * (int64_t)(2 * kTile * d) + (int64_t)h * 2 * kTile * dh;
    Elem<T>::st(base + (is_k ? KvLayout<T>::k_off(rr, f, dh) : KvLayout<T>::v_off(rr, f, dh)), val);
  }
};

template <typename T>
struct F2Epilogue {
  const T* bias;
  float* x;
  int d;
  __device__ __forceinline__ void operator()(int r, int col, float acc) const {
    size_t i = (size_t)r * d + col;
    x[i] = x[i] + acc + Elem<T>::ld(bias + col);
  }
};

// Workgroups are dispatched round-robin over the 8 XCDs, each with its own L2.  Give each XCD a
// contiguous run of logical tiles (n fastest) so that the N-tiles sharing one A row-panel run on
// the same XCD close together in time.
__device__ __forceinline__ int xcd_remap(int id, int total) {
  int chunk = (total + 7) >> 3;
  return (id & 7) * chunk + (id >> 3);
}

// ---- fp32 GEMM: 64x64 tile, BK = 16, 4x4 outputs per thread ---------------------------------------
constexpr int kSgemmBM = 64, kSgemmBN = 64, kSgemmBK = 16;

template <class Epi>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ A, const float* __restrict__ W, int K,
                                                       int row_begin, int row_end, ColMap cm, int n_mtiles, Epi epi) {
  __shared__ float As[kSgemmBK][kSgemmBM + 4];
  __shared__ float Bs[kSgemmBK][kSgemmBN + 4];
  const int ntiles_per_blk = cm.d / kSgemmBN;
  const int n_ntiles = cm.nblk * ntiles_per_blk;
  const int total = n_mtiles * n_ntiles;
  int logical = blockIdx.x;
  if (logical >= total) return;
  const int mt = logical / n_ntiles, nt = logical - mt * n_ntiles;
  const int m0 = row_begin + mt * kSgemmBM;
  const int n0 = cm.blk[nt / ntiles_per_blk] * cm.d + (nt % ntiles_per_blk) * kSgemmBN;
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += kSgemmBK) {
    // 64 rows x 16 k per operand = 1024 elements, 4 per thread (one float4 along k)
    {
      int row = tid >> 2, kc = (tid & 3) * 4;
      int ar = min(m0 + row, row_end - 1);
      float4 a = *reinterpret_cast<const float4*>(A + (size_t)ar * K + k0 + kc);
      float4 b = *reinterpret_cast<const float4*>(W + (size_t)(n0 + row) * K + k0 + kc);
      As[kc + 0][row] = a.x; As[kc + 1][row] = a.y; As[kc + 2][row] = a.z; As[kc + 3][row] = a.w;
      Bs[kc + 0][row] = b.x; Bs[kc + 1][row] = b.y; Bs[kc + 2][row] = b.z; Bs[kc + 3][row] = b.w;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < kSgemmBK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[kk][ty * 4 + i]; b[i] = Bs[kk][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int r = m0 + ty * 4 + i, c = n0 + tx * 4 + j;
      if (r < row_end) epi(r, c, acc[i][j]);
    }
}

}  // namespace relaygr
