// Internal helpers shared by the libspa translation units (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "spa.h"

namespace spa {

// ---- host side -------------------------------------------------------------------
int fail(int code, const char* fmt, ...);          // records the message, returns code
int check_launch(const char* what);                // hipGetLastError -> SPA_ERR_HIP

// Launch options (tuning aids and kernel selection for tests), see spa_set_option in spa.h.
struct Options {
  bool fwd_whole, fwd_step64, fwd_plain;   // attn_fwd_short
  bool fwd_long_two;                       // attn_fwd_long = two (two query chains per wave)
  int fwd_nw, fwd_bn;                      // attn_fwd_cfg (0 = automatic)
  int fwd_wave_max;                        // attn_fwd_wave_max
  int bwd_short;                           // attn_bwd_short: 0 one kernel, 1 split, 2 tiled
  bool bwd_long_two;                       // attn_bwd_long = two
  int gemm_tm, gemm_splits, pack_tile;     // 0 = automatic
};
const Options& options();

inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int elem_size(int dtype) { return dtype == SPA_BF16 ? 2 : 4; }

#define SPA_REQUIRE(cond, code, ...)                 \
  do {                                               \
    if (!(cond)) return ::spa::fail(code, __VA_ARGS__); \
  } while (0)

// ---- device side -----------------------------------------------------------------
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));
typedef uint32_t uintx2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

// Number of set bits of a wave-wide ballot below this lane.
__device__ __forceinline__ int rank_in_ballot(uint64_t ballot) {
  return __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(ballot >> 32),
                                   __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(ballot), 0));
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

// 8 bf16 (one 16-byte chunk) <-> 8 floats
__device__ __forceinline__ floatx8 bf16x8_to_float(bf16x8 v) { return __builtin_convertvector(v, floatx8); }
__device__ __forceinline__ bf16x8 float_to_bf16x8(floatx8 v) { return __builtin_convertvector(v, bf16x8); }

__device__ __forceinline__ float sigmoidf_dev(float s) {
  float e = __expf(-fabsf(s));
  float r = 1.0f / (1.0f + e);
  return s >= 0.f ? r : e * r;
}

}  // namespace spa
