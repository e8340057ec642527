// Measurement aids, not part of the method: the two yardstick kernels that bench.py times on
// the box to report achievable ceilings beside the published peaks: a plain streaming copy
// (16-byte loads and stores, grid-stride) and an MFMA-only loop (four independent
// v_mfma_f32_32x32x16_bf16 accumulation chains per wave, no memory traffic).
#include "spa_common.h"

namespace spa {

__global__ void __launch_bounds__(256)
ceiling_copy_kernel(const uintx4* __restrict__ src, uintx4* __restrict__ dst, long n) {
  const long stride = (long)gridDim.x * blockDim.x;
  for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

__global__ void __launch_bounds__(256)
ceiling_mfma_kernel(float* __restrict__ sink, int iters) {
  bf16x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    a[e] = static_cast<__bf16>(threadIdx.x * 0.001f + e);
    b[e] = static_cast<__bf16>(e * 0.5f);
  }
  floatx16 c0, c1, c2, c3;
#pragma unroll
  for (int r = 0; r < 16; ++r) { c0[r] = 0.f; c1[r] = 0.f; c2[r] = 0.f; c3[r] = 0.f; }
  for (int i = 0; i < iters; ++i) {
    c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
    c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
    c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
    c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int r = 0; r < 16; ++r) s += c0[r] + c1[r] + c2[r] + c3[r];
  if (s == 12345.678f) sink[0] = s;   // keeps the loop alive, never true
}

}  // namespace spa

using namespace spa;

extern "C" int spa_ceiling_copy(const void* src, void* dst, size_t bytes, void* stream) {
  SPA_REQUIRE(src && dst && bytes >= 16 && bytes % 16 == 0, SPA_ERR_INVALID_ARG,
              "spa_ceiling_copy: null pointer or size not a positive multiple of 16");
  SPA_REQUIRE(aligned16(src) && aligned16(dst), SPA_ERR_INVALID_ARG, "spa_ceiling_copy: buffers not 16-byte aligned");
  const long n = (long)(bytes / 16);
  long wgs = (n + 255) / 256;
  if (wgs > 256 * 16) wgs = 256 * 16;
  hipLaunchKernelGGL(ceiling_copy_kernel, dim3((unsigned)wgs), dim3(256), 0, as_stream(stream),
                     static_cast<const uintx4*>(src), static_cast<uintx4*>(dst), n);
  return check_launch("spa_ceiling_copy");
}

extern "C" double spa_ceiling_mfma(float* sink, int waves_per_simd, int iters, void* stream) {
  if (sink == nullptr || waves_per_simd < 1 || waves_per_simd > 8 || iters < 1) {
    fail(SPA_ERR_INVALID_ARG, "spa_ceiling_mfma: bad argument");
    return -1.0;
  }
  const int blocks = 256 * waves_per_simd;   // 256 CUs x 4 SIMDs x waves_per_simd waves of 64 lanes
  hipLaunchKernelGGL(ceiling_mfma_kernel, dim3(blocks), dim3(256), 0, as_stream(stream), sink, iters);
  if (check_launch("spa_ceiling_mfma") != SPA_OK) return -1.0;
  return (double)blocks * 4.0 * iters * 4.0 * 32768.0;   // flops issued by the launch
}
