// Linear projection of packed tokens (the 3 L C^2 and N C^2 terms of the SPA complexity
// formula, Section 3.2): out[j,:] = (s_j * x[row(j),:]) W^T + bias, where row(j) is either j
// or gather_idx[j] (the token gather of the packing step folded into the A-operand load) and
// s_j is 1 or sigmoid(score) of the token (the gated representation r_g = Sigmoid(s) . r).
// The row scale s_j is applied to the fp32 accumulator in the epilogue: (s a) W^T = s (a W^T),
// one rounding fewer than multiplying a materialised bf16 r_g.
//
// bf16 path: MFMA GEMM, C[M,N] = A[M,K] B[N,K]^T with both operands K-contiguous ("NT").
// Workgroup tile 128 x 128 x 64, four waves in a 2 x 2 grid, each wave a 64 x 64 block
// (2 x 2 v_mfma_f32_32x32x16_bf16 tiles), A and B tiles double-buffered in LDS with two
// k-tiles of rows in flight in registers.  Row stride 72 elements keeps the 16-byte
// fragment reads bank-conflict free.  The output tile leaves through LDS as whole rows.
// The live tiles (the row count is only known on the device) are numbered m-major and cut
// into 8 equal contiguous ranges, one per XCD (workgroup id % 8): the workgroups that share a
// block of A rows run on one XCD's L2 and every XCD gets the same number of tiles.
// Large problems with long k-loops take the 256 x 256 x 64 kernel of linear_big.hip.
// fp32 path (tiny workload): one thread per output element.
#include "attn_tiles.h"
#include "spa_common.h"

namespace spa {

constexpr int kGemmBN = 128, kGemmThreads = 256;

// 256 x 256 x 64 tiles (linear_big.hip)
hipError_t launch_linear_bf16_big(bool gather, bool scale, const void* x, const int32_t* gather_idx,
                                  const float* gate_scores, const int32_t* total, const void* W, const void* bias,
                                  int M_cap, int K, int N_out, void* out, long out_row_stride, hipStream_t st);

// Workgroup tile (64 TM) x 128, four waves as 2 x 2, each wave (32 TM) x 64 of the output held
// as TM x 2 MFMA tiles.  TM = 2: 128 x 128 tiles (more workgroups for small problems);
// TM = 4: 256 x 128 tiles (a third less operand traffic per flop).
template <bool kGather, bool kScale, int BK, int TM>
__global__ void __launch_bounds__(kGemmThreads)
linear_bf16_kernel(const __bf16* __restrict__ x, const int32_t* __restrict__ gather_idx,
                   const float* __restrict__ gate_scores, const int32_t* __restrict__ total,
                   const __bf16* __restrict__ W, const __bf16* __restrict__ bias, int m_cap, int K, int n_out,
                   __bf16* out, long out_stride, int m_tiles, int n_tiles,
                   const int32_t* __restrict__ scatter_idx, const __bf16* residual) {
  constexpr int BM = 64 * TM, BN = kGemmBN, RS = BK + 8;   // RS = LDS row stride (elements)
  extern __shared__ __attribute__((aligned(16))) unsigned char gemm_smem[];   // 2 x (A tile, B tile)
  __bf16(*As)[BM * RS] = reinterpret_cast<__bf16(*)[BM * RS]>(gemm_smem);
  __bf16(*Bs)[BN * RS] = reinterpret_cast<__bf16(*)[BN * RS]>(gemm_smem + 2 * BM * RS * sizeof(__bf16));
  __shared__ long a_row[BM];       // source row of every tile row (-1 = past the end)
  __shared__ float a_scale[BM];
  __shared__ float bias_s[BN];     // bias of the tile's output columns (0 past n_out or without bias)
  __shared__ int o_row[BM];        // output row of every tile row when the result is scattered

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
  const int wm = (wv >> 1) * 32 * TM, wn = (wv & 1) * 64;

  for (int t = tid; t < BM; t += kGemmThreads) {
    const int r = m0 + t;
    long src = -1;
    float sc = 1.f;
    if (r < M) {
      src = kGather ? (long)gather_idx[r] : (long)r;
      if (kScale) sc = sigmoidf_dev(gate_scores[src]);
    }
    a_row[t] = src;
    a_scale[t] = sc;
    o_row[t] = scatter_idx != nullptr && r < M ? scatter_idx[r] : r;
  }
  if (tid < BN) bias_s[tid] = bias != nullptr && n0 + tid < n_out ? static_cast<float>(bias[n0 + tid]) : 0.f;
  __syncthreads();

  // staging: a tile is rows x BK/8 chunks of 16 bytes.  The rows and chunk columns a thread
  // stages never change, so their addresses are computed once.
  // Rows past the end of the tile's valid range load a valid row instead of zeros: a row of A
  // only reaches its own output row and a row of W its own output column, and the epilogue
  // stores neither.
  constexpr int CPRW = BK / 8, CA = BM * CPRW / kGemmThreads, CB = BN * CPRW / kGemmThreads;
  const __bf16* ap[CA];
  const __bf16* bp[CB];
  const int st_r = tid / CPRW, st_c = tid % CPRW;           // chunk u of a thread: row st_r + u * (256 / CPRW)
  constexpr int RSTEP = kGemmThreads / CPRW;
  const int lds_off = st_r * RS + st_c * 8;
#pragma unroll
  for (int u = 0; u < CA; ++u) {
    const long src = a_row[st_r + u * RSTEP];
    ap[u] = x + (src >= 0 ? src : 0) * K + st_c * 8;
  }
#pragma unroll
  for (int u = 0; u < CB; ++u) bp[u] = W + (long)min(n0 + st_r + u * RSTEP, n_out - 1) * K + st_c * 8;

  // Two k-tiles in flight in registers.  When K is not a multiple of BK the PARTIAL k-tile comes
  // first (k in [0, K % BK)), so that only the prologue needs masked loads and every tile the
  // main loop touches is whole: tile t >= 1 starts at k = k_first + t * BK.
  constexpr int PF = 2;
  bf16x8 areg[PF][CA], breg[PF][CB];
  const int k_tail = K % BK, nk = (K + BK - 1) / BK, k_first = k_tail ? k_tail - BK : 0;
  auto gload = [&](int slot, int t) {   // whole tile t (t >= 1 when K % BK != 0)
    const int k0 = k_first + t * BK;
#pragma unroll
    for (int u = 0; u < CA; ++u) areg[slot][u] = *reinterpret_cast<const bf16x8*>(ap[u] + k0);
#pragma unroll
    for (int u = 0; u < CB; ++u) breg[slot][u] = *reinterpret_cast<const bf16x8*>(bp[u] + k0);
  };
  auto gload_first = [&](int slot) {
    if (k_tail == 0) { gload(slot, 0); return; }
    const bool in_k = st_c * 8 < k_tail;   // columns past the partial tile are zero in both operands
#pragma unroll
    for (int u = 0; u < CA; ++u) areg[slot][u] = in_k ? *reinterpret_cast<const bf16x8*>(ap[u]) : zero_bf16x8();
#pragma unroll
    for (int u = 0; u < CB; ++u) breg[slot][u] = in_k ? *reinterpret_cast<const bf16x8*>(bp[u]) : zero_bf16x8();
  };
  auto lstore = [&](int slot, int buf) {
#pragma unroll
    for (int u = 0; u < CA; ++u) *reinterpret_cast<bf16x8*>(&As[buf][lds_off + u * RSTEP * RS]) = areg[slot][u];
#pragma unroll
    for (int u = 0; u < CB; ++u) *reinterpret_cast<bf16x8*>(&Bs[buf][lds_off + u * RSTEP * RS]) = breg[slot][u];
  };
  auto compute = [&](int buf, floatx16 (&acc)[TM][2]) {
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8 af[TM], bfr[2];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        af[i] = *reinterpret_cast<const bf16x8*>(&As[buf][(wm + i * 32 + l32) * RS + kk * 16 + hh * 8]);
#pragma unroll
      for (int jn = 0; jn < 2; ++jn)
        bfr[jn] = *reinterpret_cast<const bf16x8*>(&Bs[buf][(wn + jn * 32 + l32) * RS + kk * 16 + hh * 8]);
      // C^T tile: rows = output columns n, cols = tokens m, so that a lane's 4 consecutive
      // accumulator registers are 4 consecutive n of one token (8-byte output pieces)
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int jn = 0; jn < 2; ++jn)
          acc[i][jn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[jn], af[i], acc[i][jn], 0, 0, 0);
    }
  };

  floatx16 acc[TM][2];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int jn = 0; jn < 2; ++jn)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][jn][r] = 0.f;

  // Software pipeline over k-tiles, two per trip so that register slots and LDS buffers are
  // static.  Entering a trip: LDS buffer 0 holds tile kt, slot 1 holds tile kt+1, slot 0 is free.
  // Loads past the last tile repeat the last tile and what they bring is never multiplied, which
  // keeps the loop body free of branches (the compiler then counts outstanding loads exactly).
  const int last = nk - 1;
  gload_first(0);
  if (nk > 1) gload(1, 1);
  lstore(0, 0);
  __syncthreads();
  for (int kt = 0; kt + 1 < nk; kt += 2) {
    gload(0, min(kt + 2, last));
    compute(0, acc);
    lstore(1, 1);        // tile kt+1
    __syncthreads();
    gload(1, min(kt + 3, last));
    compute(1, acc);
    lstore(0, 0);        // tile kt+2, or a repeat of the last tile
    __syncthreads();
  }
  if (nk & 1) {
    compute(0, acc);
    __syncthreads();     // the epilogue reuses the operand buffers
  }

  // epilogue: scale, bias, bf16; 64 rows x 64 columns of the wave at a time are parked in LDS
  // (the operand buffers are free after the last barrier) and leave as whole 16-byte pieces
  constexpr int ORS = 64 + 8;
  static_assert(4 * 64 * ORS <= 2 * (BM + BN) * RS, "output staging fits in the operand buffers");
  __bf16* tile = reinterpret_cast<__bf16*>(gemm_smem) + wv * 64 * ORS;   // 64 rows x 72 per wave
  float row_scale[TM];
#pragma unroll
  for (int i = 0; i < TM; ++i) row_scale[i] = a_scale[wm + i * 32 + l32];
#pragma unroll
  for (int half = 0; half < TM / 2; ++half) {
#pragma unroll
    for (int ii = 0; ii < 2; ++ii)
#pragma unroll
      for (int jn = 0; jn < 2; ++jn)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int i = half * 2 + ii;
          const int nloc = jn * 32 + 8 * g + 4 * hh;        // 4 consecutive output columns
          floatx4 f = {acc[i][jn][4 * g], acc[i][jn][4 * g + 1], acc[i][jn][4 * g + 2], acc[i][jn][4 * g + 3]};
          if (kScale) f *= row_scale[i];
          f += *reinterpret_cast<const floatx4*>(&bias_s[wn + nloc]);
          *reinterpret_cast<bf16x4*>(&tile[(ii * 32 + l32) * ORS + nloc]) = __builtin_convertvector(f, bf16x4);
        }
    __syncthreads();
    // 64 rows x 8 chunks per wave
    for (int i = lane; i < 64 * 8; i += 64) {
      const int r = i >> 3, c = i & 7;
      const int m = m0 + wm + half * 64 + r, n = n0 + wn + c * 8;
      if (m < M && n < n_out) {
        const long off = (long)o_row[wm + half * 64 + r] * out_stride + n;
        bf16x8 val = *reinterpret_cast<const bf16x8*>(&tile[r * ORS + c * 8]);
        if (residual != nullptr)
          val = float_to_bf16x8(bf16x8_to_float(val) + bf16x8_to_float(*reinterpret_cast<const bf16x8*>(residual + off)));
        *reinterpret_cast<bf16x8*>(out + off) = val;
      }
    }
    __syncthreads();
  }
}

template <bool kGather, bool kScale>
__global__ void __launch_bounds__(256)
linear_f32_kernel(const float* __restrict__ x, const int32_t* __restrict__ gather_idx,
                  const float* __restrict__ gate_scores, const int32_t* __restrict__ total,
                  const float* __restrict__ W, const float* __restrict__ bias, int m_cap, int K, int n_out,
                  float* out, long out_stride, const int32_t* __restrict__ scatter_idx, const float* residual) {
  const int M = total != nullptr ? min(total[0], m_cap) : m_cap;
  const long work = (long)M * n_out;
  for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < work; i += (long)gridDim.x * blockDim.x) {
    const int m = (int)(i / n_out), n = (int)(i - (long)m * n_out);
    const long src = kGather ? (long)gather_idx[m] : (long)m;
    const float sc = kScale ? sigmoidf_dev(gate_scores[src]) : 1.f;
    const float* xr = x + src * K;
    const float* wr = W + (long)n * K;
    float a = 0.f;
    for (int kq = 0; kq < K; ++kq) a = fmaf(sc * xr[kq], wr[kq], a);
    const long off = (long)(scatter_idx != nullptr ? scatter_idx[m] : m) * out_stride + n;
    out[off] = a + (bias != nullptr ? bias[n] : 0.f) + (residual != nullptr ? residual[off] : 0.f);
  }
}

}  // namespace spa

using namespace spa;

static int linear_common(const char* fn, const void* x, const int32_t* gather_idx, const float* gate_scores,
                         const int32_t* total, const void* W, const void* bias, int M_cap, int K, int N_out,
                         int dtype, void* out, int64_t out_row_stride, const int32_t* scatter_idx,
                         const void* residual, void* stream) {
  SPA_REQUIRE(x && W && out, SPA_ERR_INVALID_ARG, "%s: null pointer", fn);
  SPA_REQUIRE(M_cap >= 1 && K >= 1 && N_out >= 1, SPA_ERR_INVALID_ARG, "%s: M_cap, K, N_out must be >= 1", fn);
  SPA_REQUIRE(dtype == SPA_F32 || dtype == SPA_BF16, SPA_ERR_UNSUPPORTED, "%s: unknown dtype %d", fn, dtype);
  SPA_REQUIRE(!(gate_scores != nullptr && gather_idx == nullptr), SPA_ERR_INVALID_ARG,
              "%s: gate_scores are indexed by token and need gather_idx", fn);
  SPA_REQUIRE(out_row_stride >= N_out, SPA_ERR_INVALID_ARG, "%s: out_row_stride < N_out", fn);
  hipStream_t st = as_stream(stream);
  const bool g = gather_idx != nullptr, sc = gate_scores != nullptr;
  if (dtype == SPA_F32) {
    long wgs = ((long)M_cap * N_out + 255) / 256;
    if (wgs > 8192) wgs = 8192;
#define SPA_LIN_F32(G_, S_)                                                                                   \
  hipLaunchKernelGGL((linear_f32_kernel<G_, S_>), dim3((unsigned)wgs), dim3(256), 0, st, (const float*)x,    \
                     gather_idx, gate_scores, total, (const float*)W, (const float*)bias, M_cap, K, N_out,   \
                     (float*)out, (long)out_row_stride, scatter_idx, (const float*)residual)
    if (g && sc) SPA_LIN_F32(true, true); else if (g) SPA_LIN_F32(true, false); else SPA_LIN_F32(false, false);
#undef SPA_LIN_F32
    return check_launch(fn);
  }
  SPA_REQUIRE(K % 8 == 0, SPA_ERR_UNSUPPORTED, "%s: K = %d must be a multiple of 8 for bf16", fn, K);
  SPA_REQUIRE(N_out % 8 == 0 && out_row_stride % 8 == 0, SPA_ERR_INVALID_ARG,
              "%s: N_out and out_row_stride must be multiples of 8 for bf16", fn);
  SPA_REQUIRE(aligned16(x) && aligned16(W) && aligned16(out), SPA_ERR_INVALID_ARG, "%s: x / W / out not 16-byte aligned", fn);
  // tile shape: 256 x 256 x 64 only where it measured faster than 128 x 128 x 64: long k-loops
  // and enough tiles that the live ones (about half of the capacity for a packed stream) still
  // cover most CUs.  option gemm_tm = 2 | 4 | 8 forces 128 x 128, 256 x 128 or 256 x 256 (tuning aid).
  const int cfg_env = options().gemm_tm;
  const long tiles_big = (long)((M_cap + 255) / 256) * ((N_out + 255) / 256);
  const bool plain_out = scatter_idx == nullptr && residual == nullptr;
  const bool big = plain_out && (cfg_env == 8 || (cfg_env == 0 && tiles_big >= 384 && K >= 512));
  if (big) {
    const hipError_t e = launch_linear_bf16_big(g, sc, x, gather_idx, gate_scores, total, W, bias, M_cap, K, N_out,
                                                out, (long)out_row_stride, st);
    SPA_REQUIRE(e == hipSuccess, SPA_ERR_HIP, "%s: cannot reserve LDS for the 256 x 256 tile: %s", fn,
                hipGetErrorString(e));
    return check_launch(fn);
  }
  const int tm = cfg_env == 4 ? 4 : 2;
  const int bm = 64 * tm;
  const int m_tiles = (M_cap + bm - 1) / bm, n_tiles = (N_out + kGemmBN - 1) / kGemmBN;
  SPA_REQUIRE((long)m_tiles * n_tiles + 8 < 2147483647L / 2, SPA_ERR_INVALID_ARG, "%s: too many tiles", fn);
  const unsigned grid = (unsigned)((long)((m_tiles + 7) / 8) * 8 * n_tiles);
#define SPA_LIN_BF16(G_, S_, BK_, TM_)                                                                        \
  do {                                                                                                        \
    constexpr size_t smem = (size_t)2 * (64 * TM_ + kGemmBN) * (BK_ + 8) * sizeof(__bf16);                     \
    const hipError_t attr = hipFuncSetAttribute((const void*)linear_bf16_kernel<G_, S_, BK_, TM_>,            \
                                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);       \
    SPA_REQUIRE(attr == hipSuccess, SPA_ERR_HIP, "%s: cannot reserve %zu bytes of LDS", fn, smem);            \
    hipLaunchKernelGGL((linear_bf16_kernel<G_, S_, BK_, TM_>), dim3(grid), dim3(kGemmThreads), smem, st,      \
                       (const __bf16*)x, gather_idx, gate_scores, total, (const __bf16*)W, (const __bf16*)bias, \
                       M_cap, K, N_out, (__bf16*)out, (long)out_row_stride, m_tiles, n_tiles, scatter_idx,     \
                       (const __bf16*)residual);                                                              \
  } while (0)
#define SPA_LIN_BF16_CFG(BK_, TM_)                                                                            \
  do {                                                                                                        \
    if (g && sc) SPA_LIN_BF16(true, true, BK_, TM_); else if (g) SPA_LIN_BF16(true, false, BK_, TM_);         \
    else SPA_LIN_BF16(false, false, BK_, TM_);                                                                \
  } while (0)
  if (tm == 4) SPA_LIN_BF16_CFG(32, 4); else SPA_LIN_BF16_CFG(64, 2);
#undef SPA_LIN_BF16_CFG
#undef SPA_LIN_BF16
  return check_launch(fn);
}

extern "C" int spa_linear_packed(const void* x, const int32_t* gather_idx, const float* gate_scores,
                                 const int32_t* total, const void* W, const void* bias, int M_cap, int K,
                                 int N_out, int dtype, void* out, int64_t out_row_stride, void* stream) {
  return linear_common("spa_linear_packed", x, gather_idx, gate_scores, total, W, bias, M_cap, K, N_out, dtype, out,
                       out_row_stride, nullptr, nullptr, stream);
}

extern "C" int spa_linear_packed_scatter(const void* x, const int32_t* total, const void* W, const void* bias,
                                         int M_cap, int K, int N_out, int dtype, const int32_t* scatter_idx,
                                         const void* residual, void* y, int64_t y_row_stride, void* stream) {
  const char* fn = "spa_linear_packed_scatter";
  SPA_REQUIRE(scatter_idx != nullptr, SPA_ERR_INVALID_ARG, "%s: scatter_idx is null", fn);
  SPA_REQUIRE(aligned16(residual), SPA_ERR_INVALID_ARG, "%s: residual not 16-byte aligned", fn);
  return linear_common(fn, x, nullptr, nullptr, total, W, bias, M_cap, K, N_out, dtype, y, y_row_stride, scatter_idx,
                       residual, stream);
}
