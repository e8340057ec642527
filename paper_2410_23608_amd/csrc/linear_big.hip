// Large-tile variant of the packed projection (see linear.hip for what is computed):
// workgroup tile 256 x 256 x 64, four waves as 2 x 2, each wave a 128 x 128 block held as
// 4 x 4 v_mfma_f32_32x32x16_bf16 accumulator tiles (256 accumulator registers, one wave per
// SIMD).  Per flop it moves half the operand bytes of the 128 x 128 tile from L2 to LDS and
// reads half the bytes back from LDS, which is what bounds the small-tile kernel.
// This file is compiled WITHOUT the "MFMA results in ordinary VGPRs" option of the other
// files: the accumulators live in the accumulation half of the register file.
#include <type_traits>

#include "attn_tiles.h"
#include "spa_common.h"

namespace spa {

constexpr int kBigM = 256, kBigN = 256, kBigK = 64, kBigThreads = 256;
constexpr int kBigRS = kBigK + 8;   // LDS row stride (elements): conflict-free 16-byte fragment reads
constexpr size_t kBigOperandBytes = (size_t)2 * (kBigM + kBigN) * kBigRS * sizeof(__bf16);   // two stages

template <bool kGather, bool kScale>
__global__ void __launch_bounds__(kBigThreads) __attribute__((amdgpu_waves_per_eu(1, 1)))
linear_bf16_big_kernel(const __bf16* __restrict__ x, const int32_t* __restrict__ gather_idx,
                       const float* __restrict__ gate_scores, const int32_t* __restrict__ total,
                       const __bf16* __restrict__ W, const __bf16* __restrict__ bias, int m_cap, int K, int n_out,
                       __bf16* __restrict__ out, long out_stride, int m_tiles, int n_tiles) {
  constexpr int BM = kBigM, BN = kBigN, BK = kBigK, RS = kBigRS;
  extern __shared__ __attribute__((aligned(16))) unsigned char big_smem[];
  __bf16(*As)[BM * RS] = reinterpret_cast<__bf16(*)[BM * RS]>(big_smem);
  __bf16(*Bs)[BN * RS] = reinterpret_cast<__bf16(*)[BN * RS]>(big_smem + 2 * BM * RS * sizeof(__bf16));
  __shared__ long a_row[BM];
  __shared__ float a_scale[BM];
  __shared__ float bias_s[BN];

  // Tile order.  Workgroup ids go to the 8 XCDs round-robin (id % 8) and each XCD has its own
  // L2.  The LIVE tiles (the row count is only known here, on the device) are numbered m-major
  // and cut into 8 equal contiguous ranges, one per XCD: the workgroups that share a block of A
  // rows run on one XCD, and every XCD gets the same number of tiles.
  const int M = total != nullptr ? min(total[0], m_cap) : m_cap;
  const int live_tiles = ((M + BM - 1) / BM) * n_tiles, per_xcd = (live_tiles + 7) >> 3;
  const int xcd = blockIdx.x & 7, jx = blockIdx.x >> 3, tile_id = xcd * per_xcd + jx;
  if (jx >= per_xcd || tile_id >= live_tiles) return;
  const int mt = tile_id / n_tiles, nt = tile_id - mt * n_tiles;
  const int m0 = mt * BM, n0 = nt * BN;

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, l32 = lane & 31, hh = lane >> 5;
  const int wm = (wv >> 1) * 128, wn = (wv & 1) * 128;

  {
    const int r = m0 + tid;
    long src = -1;
    float sc = 1.f;
    if (r < M) {
      src = kGather ? (long)gather_idx[r] : (long)r;
      if (kScale) sc = sigmoidf_dev(gate_scores[src]);
    }
    a_row[tid] = src;
    a_scale[tid] = sc;
    bias_s[tid] = bias != nullptr && n0 + tid < n_out ? static_cast<float>(bias[n0 + tid]) : 0.f;
  }
  __syncthreads();

  // staging: 8 chunks of 16 bytes per row and k-tile; thread -> chunk tid % 8 of rows
  // tid / 8 + 32 u, u = 0..7, of both operands.  Rows past the valid range load a valid row
  // (their outputs are never stored).
  constexpr int NU = 8, RSTEP = kBigThreads / 8;
  const int st_r = tid >> 3, st_c = tid & 7;
  const int lds_off = st_r * RS + st_c * 8;
  const __bf16* ap[NU];
  const __bf16* bp[NU];
#pragma unroll
  for (int u = 0; u < NU; ++u) {
    const long src = a_row[st_r + u * RSTEP];
    ap[u] = x + (src >= 0 ? src : 0) * K + st_c * 8;
    bp[u] = W + (long)min(n0 + st_r + u * RSTEP, n_out - 1) * K + st_c * 8;
  }
  // When K is not a multiple of BK the partial k-tile comes first, so the main loop only sees
  // whole tiles: tile t >= 1 starts at k = k_first + t * BK.
  const int k_tail = K % BK, nk = (K + BK - 1) / BK, k_first = k_tail ? k_tail - BK : 0;
  bf16x8 areg[NU], breg[NU];
  auto gload = [&](int t) {
    const int k0 = k_first + t * BK;
#pragma unroll
    for (int u = 0; u < NU; ++u) {
      areg[u] = *reinterpret_cast<const bf16x8*>(ap[u] + k0);
      breg[u] = *reinterpret_cast<const bf16x8*>(bp[u] + k0);
    }
  };
  auto gload_first = [&]() {
    if (k_tail == 0) { gload(0); return; }
    const bool in_k = st_c * 8 < k_tail;
#pragma unroll
    for (int u = 0; u < NU; ++u) {
      areg[u] = in_k ? *reinterpret_cast<const bf16x8*>(ap[u]) : zero_bf16x8();
      breg[u] = in_k ? *reinterpret_cast<const bf16x8*>(bp[u]) : zero_bf16x8();
    }
  };
  auto lstore = [&](int buf) {
#pragma unroll
    for (int u = 0; u < NU; ++u) {
      *reinterpret_cast<bf16x8*>(&As[buf][lds_off + u * RSTEP * RS]) = areg[u];
      *reinterpret_cast<bf16x8*>(&Bs[buf][lds_off + u * RSTEP * RS]) = breg[u];
    }
  };

  floatx16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int jn = 0; jn < 4; ++jn)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][jn][r] = 0.f;

  // One k-tile = 4 sub-steps of 16 columns, 16 MFMAs each.  Everything else a step has to do is
  // cut into quarters and issued between the MFMA groups, so that the matrix pipe never waits
  // for a whole phase of memory instructions: in sub-step kk the wave
  //   (1) stores quarter kk of tile t+1 (registers, loaded during the previous step) into the
  //       other LDS buffer,
  //   (2) reloads those registers with quarter kk of tile t+2,
  //   (3) reads the fragments of sub-step kk+1 from LDS,
  //   (4) issues the 16 MFMAs of sub-step kk.
  // kMove = false: the last tile, nothing left to move.
  auto step = [&](auto move_tag, int buf, int t_load) {
    constexpr bool kMove = decltype(move_tag)::value;
    const int k0 = k_first + t_load * BK;
    const __bf16* a_base = &As[buf][(wm + l32) * RS + hh * 8];
    const __bf16* b_base = &Bs[buf][(wn + l32) * RS + hh * 8];
    bf16x8 af[2][4], bfr[2][4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      af[0][i] = *reinterpret_cast<const bf16x8*>(a_base + i * 32 * RS);
      bfr[0][i] = *reinterpret_cast<const bf16x8*>(b_base + i * 32 * RS);
    }
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      const int cur = kk & 1, nxt = cur ^ 1;
      if (kMove) {
#pragma unroll
        for (int u = 2 * kk; u < 2 * kk + 2; ++u) {
          *reinterpret_cast<bf16x8*>(&As[buf ^ 1][lds_off + u * RSTEP * RS]) = areg[u];
          *reinterpret_cast<bf16x8*>(&Bs[buf ^ 1][lds_off + u * RSTEP * RS]) = breg[u];
        }
#pragma unroll
        for (int u = 2 * kk; u < 2 * kk + 2; ++u) {
          areg[u] = *reinterpret_cast<const bf16x8*>(ap[u] + k0);
          breg[u] = *reinterpret_cast<const bf16x8*>(bp[u] + k0);
        }
      }
      if (kk + 1 < BK / 16) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          af[nxt][i] = *reinterpret_cast<const bf16x8*>(a_base + i * 32 * RS + (kk + 1) * 16);
          bfr[nxt][i] = *reinterpret_cast<const bf16x8*>(b_base + i * 32 * RS + (kk + 1) * 16);
        }
      }
      // C^T tiles: rows = output columns n, cols = tokens m (a lane's 4 consecutive accumulator
      // registers are 4 consecutive n of one token)
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int jn = 0; jn < 4; ++jn)
          acc[i][jn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[cur][jn], af[cur][i], acc[i][jn], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);   // keep the quarters where they are
    }
  };

  // pipeline: at the start of step t LDS buffer t & 1 holds tile t and the registers hold tile
  // t + 1.  Loads past the last tile repeat it; what they bring is stored but never multiplied.
  const int last = nk - 1;
  gload_first();
  lstore(0);
  if (nk > 1) gload(1);
  __syncthreads();
  for (int kt = 0; kt + 1 < nk; kt += 2) {
    step(std::true_type{}, 0, min(kt + 2, last));
    __syncthreads();
    step(std::true_type{}, 1, min(kt + 3, last));
    __syncthreads();
  }
  if (nk & 1) {
    step(std::false_type{}, 0, last);
    __syncthreads();                 // the epilogue reuses the operand buffers
  }

  // epilogue: scale, bias, bf16; 32 tokens x 128 columns of the wave at a time are parked in
  // LDS and leave as whole 16-byte pieces of 256-byte row segments
  constexpr int ORS = 128 + 8;
  static_assert((size_t)4 * 32 * ORS * sizeof(__bf16) <= kBigOperandBytes, "output staging fits in the operand buffers");
  __bf16* tile = reinterpret_cast<__bf16*>(big_smem) + wv * 32 * ORS;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float rs = a_scale[wm + i * 32 + l32];
#pragma unroll
    for (int jn = 0; jn < 4; ++jn)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int nloc = jn * 32 + 8 * g + 4 * hh;        // 4 consecutive output columns
        floatx4 f = {acc[i][jn][4 * g], acc[i][jn][4 * g + 1], acc[i][jn][4 * g + 2], acc[i][jn][4 * g + 3]};
        if (kScale) f *= rs;
        f += *reinterpret_cast<const floatx4*>(&bias_s[wn + nloc]);
        *reinterpret_cast<bf16x4*>(&tile[l32 * ORS + nloc]) = __builtin_convertvector(f, bf16x4);
      }
    __syncthreads();
    // 32 rows x 16 chunks per wave
    for (int c = lane; c < 32 * 16; c += 64) {
      const int r = c >> 4, ch = c & 15;
      const int m = m0 + wm + i * 32 + r, n = n0 + wn + ch * 8;
      if (m < M && n < n_out)
        *reinterpret_cast<bf16x8*>(out + (long)m * out_stride + n) = *reinterpret_cast<const bf16x8*>(&tile[r * ORS + ch * 8]);
    }
    __syncthreads();
  }
}

// Launch helper used by spa_linear_packed.  Returns hipSuccess or the error of the attribute call.
hipError_t launch_linear_bf16_big(bool gather, bool scale, const void* x, const int32_t* gather_idx,
                                  const float* gate_scores, const int32_t* total, const void* W, const void* bias,
                                  int M_cap, int K, int N_out, void* out, long out_row_stride, hipStream_t st) {
  const int m_tiles = (M_cap + kBigM - 1) / kBigM, n_tiles = (N_out + kBigN - 1) / kBigN;
  const unsigned grid = (unsigned)((long)((m_tiles + 7) / 8) * 8 * n_tiles);
#define SPA_BIG(G_, S_)                                                                                       \
  do {                                                                                                        \
    const hipError_t attr = hipFuncSetAttribute((const void*)linear_bf16_big_kernel<G_, S_>,                  \
                                                hipFuncAttributeMaxDynamicSharedMemorySize,                   \
                                                (int)kBigOperandBytes);                                       \
    if (attr != hipSuccess) return attr;                                                                      \
    hipLaunchKernelGGL((linear_bf16_big_kernel<G_, S_>), dim3(grid), dim3(kBigThreads), kBigOperandBytes, st, \
                       (const __bf16*)x, gather_idx, gate_scores, total, (const __bf16*)W, (const __bf16*)bias, \
                       M_cap, K, N_out, (__bf16*)out, out_row_stride, m_tiles, n_tiles);                      \
  } while (0)
  if (gather && scale) SPA_BIG(true, true); else if (gather) SPA_BIG(true, false); else SPA_BIG(false, false);
#undef SPA_BIG
  return hipSuccess;
}

}  // namespace spa
