// Gate scoring + hard selection (Section 3.2, equations for s and r_p), the 2x2 max-pool
// that resizes up-scale scores, and the gate backward with the selection loss
// (Section 3.3).  All kernels are bandwidth-bound: every feature row is read once with
// 16-byte loads, a group of G lanes per token, fp32 accumulation.
#include <cmath>

#include "spa_common.h"

namespace spa {

constexpr int kGateThreads = 256;
constexpr int kMaxGateC = 8192;   // gate weight is staged in LDS as fp32

template <typename T> struct Vec16;
template <> struct Vec16<float> {
  static constexpr int kElems = 4;
  __device__ static __forceinline__ void load(const float* p, float (&f)[4]) {
    floatx4 v = *reinterpret_cast<const floatx4*>(p);
    f[0] = v[0]; f[1] = v[1]; f[2] = v[2]; f[3] = v[3];
  }
  __device__ static __forceinline__ void store(float* p, const float (&f)[4]) {
    floatx4 v = {f[0], f[1], f[2], f[3]};
    *reinterpret_cast<floatx4*>(p) = v;
  }
};
template <> struct Vec16<__bf16> {
  static constexpr int kElems = 8;
  __device__ static __forceinline__ void load(const __bf16* p, float (&f)[8]) {
    floatx8 v = bf16x8_to_float(*reinterpret_cast<const bf16x8*>(p));
#pragma unroll
    for (int i = 0; i < 8; ++i) f[i] = v[i];
  }
  __device__ static __forceinline__ void store(__bf16* p, const float (&f)[8]) {
    floatx8 v;
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = f[i];
    *reinterpret_cast<bf16x8*>(p) = float_to_bf16x8(v);
  }
};

template <int G>
__device__ __forceinline__ float group_sum(float v) {
#pragma unroll
  for (int o = G / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

// One group of G lanes per token; the group strides over the row's 16-byte chunks.
template <typename T, int G>
__global__ void __launch_bounds__(kGateThreads)
gate_select_kernel(const T* __restrict__ x, const T* __restrict__ w, float bias,
                   const float* __restrict__ s_up, float theta, int ntok, int N, int C,
                   float* __restrict__ scores, uint8_t* __restrict__ mask,
                   int32_t* __restrict__ counts) {
  constexpr int VE = Vec16<T>::kElems;
  extern __shared__ float w_lds[];
  for (int c = threadIdx.x; c < C; c += kGateThreads) w_lds[c] = static_cast<float>(w[c]);
  __syncthreads();

  constexpr int kGroups = kGateThreads / G;
  const int grp = threadIdx.x / G;
  const int gl = threadIdx.x % G;
  const int chunks = C / VE;
  for (long tok = (long)blockIdx.x * kGroups + grp; tok < ntok; tok += (long)gridDim.x * kGroups) {
    const T* row = x + tok * (long)C;
    float acc = 0.f;
#pragma unroll 4
    for (int ch = gl; ch < chunks; ch += G) {
      float f[VE];
      Vec16<T>::load(row + ch * VE, f);
      const float* wp = w_lds + ch * VE;
#pragma unroll
      for (int i = 0; i < VE; ++i) acc = fmaf(f[i], wp[i], acc);
    }
    acc = group_sum<G>(acc);
    if (gl == 0) {
      float s = acc + bias;
      if (s_up != nullptr) s = fmaxf(s, s_up[tok]);
      const bool sel = s > theta;
      scores[tok] = s;
      mask[tok] = sel ? 1 : 0;
      if (counts != nullptr && sel) atomicAdd(&counts[tok / N], 1);
    }
  }
}

__global__ void zero_i32_kernel(int32_t* p, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

__global__ void maxpool2x2_kernel(const float* __restrict__ s, int B, int h, int w,
                                  float* __restrict__ out) {
  const int ho = h / 2, wo = w / 2;
  const long n = (long)B * ho * wo;
  for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (long)gridDim.x * blockDim.x) {
    const int b = i / (ho * wo);
    const int r = i % (ho * wo);
    const int oy = r / wo, ox = r % wo;
    const float* p = s + (long)b * h * w + (long)(2 * oy) * w + 2 * ox;
    out[i] = fmaxf(fmaxf(p[0], p[1]), fmaxf(p[w], p[w + 1]));
  }
}

template <typename T>
static int launch_gate(const void* x, const void* w, float bias, const float* s_up, float theta,
                       int B, int N, int C, float* scores, uint8_t* mask, int32_t* counts,
                       hipStream_t st) {
  constexpr int VE = Vec16<T>::kElems;
  const int chunks = C / VE;
  const long ntok = (long)B * N;
  const size_t lds = (size_t)C * sizeof(float);
  if (counts != nullptr) {
    hipLaunchKernelGGL(zero_i32_kernel, dim3((B + 255) / 256), dim3(256), 0, st, counts, B);
  }
  auto go = [&](auto gtag) {
    constexpr int G = decltype(gtag)::value;
    const long per_wg = kGateThreads / G;
    long wgs = (ntok + per_wg - 1) / per_wg;
    if (wgs > 4096) wgs = 4096;
    hipLaunchKernelGGL((gate_select_kernel<T, G>), dim3((unsigned)wgs), dim3(kGateThreads), lds, st,
                       static_cast<const T*>(x), static_cast<const T*>(w), bias, s_up, theta,
                       (int)ntok, N, C, scores, mask, counts);
  };
  if (chunks <= 8) go(std::integral_constant<int, 8>{});
  else if (chunks <= 64) go(std::integral_constant<int, 16>{});
  else if (chunks <= 256) go(std::integral_constant<int, 32>{});
  else go(std::integral_constant<int, 64>{});
  return check_launch("spa_gate_select");
}

}  // namespace spa

using namespace spa;

extern "C" int spa_gate_select(const void* x, const void* w, float bias, const float* s_up,
                               float tau, int B, int N, int C, int dtype, float* scores,
                               uint8_t* mask, int32_t* counts, void* stream) {
  SPA_REQUIRE(x && w && scores && mask, SPA_ERR_INVALID_ARG, "spa_gate_select: null pointer");
  SPA_REQUIRE(B >= 1 && N >= 1 && C >= 1, SPA_ERR_INVALID_ARG, "spa_gate_select: B, N, C must be >= 1");
  SPA_REQUIRE((long)B * N < 2147483647L, SPA_ERR_INVALID_ARG, "spa_gate_select: B*N must be < 2^31");
  SPA_REQUIRE(tau > 0.f && tau < 1.f, SPA_ERR_INVALID_ARG, "spa_gate_select: tau must lie in (0,1), got %g", (double)tau);
  SPA_REQUIRE(dtype == SPA_F32 || dtype == SPA_BF16, SPA_ERR_UNSUPPORTED, "spa_gate_select: unknown dtype %d", dtype);
  SPA_REQUIRE(((long)C * elem_size(dtype)) % 16 == 0, SPA_ERR_INVALID_ARG,
              "spa_gate_select: row length C*elem = %ld bytes is not a multiple of 16", (long)C * elem_size(dtype));
  SPA_REQUIRE(aligned16(x), SPA_ERR_INVALID_ARG, "spa_gate_select: x is not 16-byte aligned");
  SPA_REQUIRE(C <= kMaxGateC, SPA_ERR_UNSUPPORTED, "spa_gate_select: C = %d exceeds %d", C, kMaxGateC);
  const float theta = (float)std::log((double)tau / (1.0 - (double)tau));
  hipStream_t st = as_stream(stream);
  if (dtype == SPA_F32) return launch_gate<float>(x, w, bias, s_up, theta, B, N, C, scores, mask, counts, st);
  return launch_gate<__bf16>(x, w, bias, s_up, theta, B, N, C, scores, mask, counts, st);
}

extern "C" int spa_maxpool2x2(const float* s, int B, int h, int w, float* pooled, void* stream) {
  SPA_REQUIRE(s && pooled, SPA_ERR_INVALID_ARG, "spa_maxpool2x2: null pointer");
  SPA_REQUIRE(B >= 1 && h >= 2 && w >= 2 && h % 2 == 0 && w % 2 == 0, SPA_ERR_INVALID_ARG,
              "spa_maxpool2x2: need B >= 1 and even h, w >= 2 (got %d, %d, %d)", B, h, w);
  const long n = (long)B * (h / 2) * (w / 2);
  long wgs = (n + 255) / 256;
  if (wgs > 2048) wgs = 2048;
  hipLaunchKernelGGL(maxpool2x2_kernel, dim3((unsigned)wgs), dim3(256), 0, as_stream(stream), s, B, h, w, pooled);
  return check_launch("spa_maxpool2x2");
}
