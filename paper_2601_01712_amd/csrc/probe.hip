// Diagnostic probe: what the chip sustains on the MFMA the hot path uses (v_mfma_f32_32x32x16_bf16)
// in a pure MFMA loop, with constant or pseudo-random operands.  The published peak assumes the
// nominal clock; under its power limit the chip clocks lower the more the operand bits toggle, so
// this is the practical ceiling a roofline fraction should be read against.
#include <hip/hip_runtime.h>

#include "../../include/relaygr.h"
#include "errors.h"
#include "gemm.h"

using namespace relaygr;

namespace {
__device__ __forceinline__ unsigned mix32(unsigned x) {
  x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
  return x;
}

// out[0], out[1]: shader-clock cycles and 100 MHz wall ticks of workgroup 0's loop; out[2 + thread]: a checksum
__global__ __launch_bounds__(256) void mfma_probe_kernel(float* out, int iters, int random_data) {
  bf16x8_t av[4], bv[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float fa = 1.0f, fb = 1.0f;
      if (random_data) {
        const unsigned h = mix32(threadIdx.x * 64 + blockIdx.x * 7919 + j * 8 + i);
        fa = ((int)(h & 0xffff) - 32768) / 32768.f;
        fb = ((int)(h >> 16) - 32768) / 32768.f;
      }
      av[j][i] = (__bf16)fa;
      bv[j][i] = (__bf16)fb;
    }
  f32x16_t acc[4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[a][e] = 0.f;
  const long long t0 = clock64(), w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 8; ++j)
      acc[j & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[j & 3], bv[(j + (j >> 2)) & 3], acc[j & 3], 0, 0, 0);
  }
  const long long t1 = clock64(), w1 = wall_clock64();
  float s = 0.f;
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int e = 0; e < 16; ++e) s += acc[a][e];
  out[2 + blockIdx.x * blockDim.x + threadIdx.x] = s;
  if (threadIdx.x == 0 && blockIdx.x == 0) { out[0] = (float)(t1 - t0); out[1] = (float)(w1 - w0); }
}
}  // namespace

extern "C" size_t relaygr_probe_bytes(void) { return (size_t)(2 + 512 * 256) * sizeof(float); }

extern "C" int relaygr_probe_mfma(void* work_dev, size_t work_bytes, int32_t random_data, int32_t iters, void* stream,
                                  double* tflops, double* shader_ghz) {
  if (!work_dev || work_bytes < relaygr_probe_bytes() || iters < 1 || iters > (1 << 22) || !tflops || !shader_ghz)
    return fail(RELAYGR_EINVAL, "probe_mfma: null argument, work buffer below relaygr_probe_bytes() or iters out of range");
  hipStream_t st = (hipStream_t)stream;
  hipEvent_t a, b;
  if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return fail(RELAYGR_EHIP, "probe_mfma: cannot create events");
  float* out = (float*)work_dev;
  const int blocks = 512;    // two workgroups of four wavefronts per compute unit
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(blocks), dim3(256), 0, st, out, 16, random_data);   // warm-up
  hipError_t e = hipEventRecord(a, st);
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(blocks), dim3(256), 0, st, out, iters, random_data);
  if (e == hipSuccess) e = hipEventRecord(b, st);
  if (e == hipSuccess) e = hipEventSynchronize(b);
  float ms = 0.f, t[2] = {0.f, 0.f};
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, a, b);
  if (e == hipSuccess) e = hipMemcpy(t, out, sizeof(t), hipMemcpyDeviceToHost);
  (void)hipEventDestroy(a);
  (void)hipEventDestroy(b);
  if (e != hipSuccess) return fail(RELAYGR_EHIP, "probe_mfma: %s", hipGetErrorString(e));
  const double flop = (double)blocks * 4 * (double)iters * 8 * 32768.0;   // 2*32*32*16 per MFMA and wavefront
  *tflops = flop / (ms * 1e-3) / 1e12;
  *shader_ghz = t[1] > 0 ? (double)t[0] / ((double)t[1] / 100e6) / 1e9 : 0.0;
  return RELAYGR_OK;
}
