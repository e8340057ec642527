// Linear projection of packed tokens (the 3 L C^2 and N C^2 terms of the SPA complexity
// formula, Section 3.2): out[j,:] = (s_j * x[row(j),:]) W^T + bias, where row(j) is either j
// or gather_idx[j] (the token gather of the packing step folded into the A-operand load) and
// s_j is 1 or sigmoid(score) of the token (the gated representation r_g = Sigmoid(s) . r).
// The row scale s_j is applied to the fp32 accumulator in the epilogue: (s a) W^T = s (a W^T),
// one rounding fewer than multiplying a materialised bf16 r_g.
//
// bf16 path: MFMA GEMM, C[M,N] = A[M,K] B[N,K]^T with both operands K-contiguous ("NT").
// Workgroup tile 128 x 128 x 32, four waves in a 2 x 2 grid, each wave a 64 x 64 block
// (2 x 2 v_mfma_f32_32x32x16_bf16 tiles), A and B tiles double-buffered in LDS with the
// next tile's rows in flight in registers.  Row stride 40 elements keeps the 16-byte
// fragment reads bank-conflict free.  The output tile leaves through LDS as whole rows.
// Tiles are numbered so that XCD x (= id % 8) owns the M-tiles x, x+8, x+16, ... and walks
// the N-tiles of one M-tile consecutively: an A tile is fetched into that XCD's L2 once and
// reused by all its N-tiles, the weights fit in every L2, and the live M-tiles (the row count
// is only known on the device) spread evenly over the XCDs.
// fp32 path (tiny workload): one thread per output element.
#include "attn_tiles.h"
#include "spa_common.h"

namespace spa {

constexpr int kGemmBM = 128, kGemmBN = 128, kGemmBK = 32, kGemmThreads = 256;
constexpr int kGemmRS = kGemmBK + 8;   // LDS row stride (elements)

template <bool kGather, bool kScale>
__global__ void __launch_bounds__(kGemmThreads)
linear_bf16_kernel(const __bf16* __restrict__ x, const int32_t* __restrict__ gather_idx,
                   const float* __restrict__ gate_scores, const int32_t* __restrict__ total,
                   const __bf16* __restrict__ W, const __bf16* __restrict__ bias, int m_cap, int K, int n_out,
                   __bf16* __restrict__ out, long out_stride, int m_tiles, int n_tiles) {
  constexpr int BM = kGemmBM, BN = kGemmBN, BK = kGemmBK, RS = kGemmRS;
  __shared__ __attribute__((aligned(16))) __bf16 As[2][BM * RS];
  __shared__ __attribute__((aligned(16))) __bf16 Bs[2][BN * RS];
  __shared__ long a_row[BM];       // source row of every tile row (-1 = past the end)
  __shared__ float a_scale[BM];

  const int id = blockIdx.x, xcd = id & 7, j = id >> 3;
  const int mg = j / n_tiles, nt = j - mg * n_tiles;
  const int mt = mg * 8 + xcd;
  if (mt >= m_tiles) return;
  const int M = total != nullptr ? min(total[0], m_cap) : m_cap;
  const int m0 = mt * BM, n0 = nt * BN;
  if (m0 >= M) return;

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, l32 = lane & 31, hh = lane >> 5;
  const int wm = (wv >> 1) * 64, wn = (wv & 1) * 64;

  if (tid < BM) {
    const int r = m0 + tid;
    long src = -1;
    float sc = 1.f;
    if (r < M) {
      src = kGather ? (long)gather_idx[r] : (long)r;
      if (kScale) sc = sigmoidf_dev(gate_scores[src]);
    }
    a_row[tid] = src;
    a_scale[tid] = sc;
  }
  __syncthreads();

  // staging: a tile is 128 rows x BK/8 chunks of 16 bytes, CPT chunks per thread.  The rows
  // and chunk columns a thread stages never change, so their addresses are computed once.
  constexpr int CPRW = BK / 8, CPT = BM * CPRW / kGemmThreads;
  const __bf16* ap[CPT];
  const __bf16* bp[CPT];
  int lds_off[CPT];
#pragma unroll
  for (int t = 0; t < CPT; ++t) {
    const int i = tid + t * kGemmThreads, r = i / CPRW, c = i % CPRW;
    const long src = a_row[r];
    ap[t] = src >= 0 ? x + src * K + c * 8 : nullptr;
    bp[t] = n0 + r < n_out ? W + (long)(n0 + r) * K + c * 8 : nullptr;
    lds_off[t] = r * RS + c * 8;
  }
  // two tiles in flight in registers (PF = prefetch distance in k-tiles)
  constexpr int PF = 2;
  bf16x8 areg[PF][CPT], breg[PF][CPT];
  auto gload = [&](int slot, int k0) {
#pragma unroll
    for (int t = 0; t < CPT; ++t) {
      areg[slot][t] = ap[t] != nullptr ? *reinterpret_cast<const bf16x8*>(ap[t] + k0) : zero_bf16x8();
      breg[slot][t] = bp[t] != nullptr ? *reinterpret_cast<const bf16x8*>(bp[t] + k0) : zero_bf16x8();
    }
  };
  auto lstore = [&](int slot, int buf) {
#pragma unroll
    for (int t = 0; t < CPT; ++t) {
      *reinterpret_cast<bf16x8*>(&As[buf][lds_off[t]]) = areg[slot][t];
      *reinterpret_cast<bf16x8*>(&Bs[buf][lds_off[t]]) = breg[slot][t];
    }
  };
  auto compute = [&](int buf, floatx16 (&acc)[2][2]) {
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8 af[2], bfr[2];
#pragma unroll
      for (int i = 0; i < 2; ++i)
        af[i] = *reinterpret_cast<const bf16x8*>(&As[buf][(wm + i * 32 + l32) * RS + kk * 16 + hh * 8]);
#pragma unroll
      for (int jn = 0; jn < 2; ++jn)
        bfr[jn] = *reinterpret_cast<const bf16x8*>(&Bs[buf][(wn + jn * 32 + l32) * RS + kk * 16 + hh * 8]);
      // C^T tile: rows = output columns n, cols = tokens m, so that a lane's 4 consecutive
      // accumulator registers are 4 consecutive n of one token (8-byte output pieces)
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int jn = 0; jn < 2; ++jn)
          acc[i][jn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[jn], af[i], acc[i][jn], 0, 0, 0);
    }
  };

  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int jn = 0; jn < 2; ++jn)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][jn][r] = 0.f;

  // software pipeline over k-tiles, unrolled by 2 so that the register slots are static:
  // tile t is in LDS buffer t&1, tile t+1 in register slot (t+1)&1, tile t+2 being loaded
  const int nk = K / BK;
  gload(0, 0);
  if (nk > 1) gload(1, BK);
  lstore(0, 0);
  __syncthreads();
  for (int kt = 0; kt < nk; kt += 2) {
    // even step: LDS buffer 0 holds tile kt; slot 1 holds kt+1; slot 0 is free -> load kt+2
    if (kt + 2 < nk) gload(0, (kt + 2) * BK);
    compute(0, acc);
    if (kt + 1 < nk) lstore(1, 1);
    __syncthreads();
    if (kt + 1 >= nk) break;
    // odd step: buffer 1 holds kt+1; slot 0 holds kt+2; slot 1 is free -> load kt+3
    if (kt + 3 < nk) gload(1, (kt + 3) * BK);
    compute(1, acc);
    if (kt + 2 < nk) lstore(0, 0);
    __syncthreads();
  }

  // epilogue: bias, bf16, park the 64 x 64 block of this wave in LDS (its quarter of As/Bs is
  // free after the last barrier), then whole-row stores
  constexpr int ORS = 64 + 8;
  float row_scale[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) row_scale[i] = a_scale[wm + i * 32 + l32];   // read before the tiles are reused
  __bf16* tile = (wv < 2 ? &As[0][0] : &Bs[0][0]) + (wv & 1) * 64 * ORS;   // 64 rows x 72 per wave
  static_assert(2 * 64 * ORS <= 2 * BM * RS, "output staging fits in the operand buffers");
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int jn = 0; jn < 2; ++jn)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int nloc = jn * 32 + 8 * g + 4 * hh;        // 4 consecutive output columns
        floatx4 f = {acc[i][jn][4 * g], acc[i][jn][4 * g + 1], acc[i][jn][4 * g + 2], acc[i][jn][4 * g + 3]};
        if (kScale) f *= row_scale[i];
        if (bias != nullptr) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int n = n0 + wn + nloc + e;
            if (n < n_out) f[e] += static_cast<float>(bias[n]);
          }
        }
        *reinterpret_cast<bf16x4*>(&tile[(i * 32 + l32) * ORS + nloc]) = __builtin_convertvector(f, bf16x4);
      }
  __syncthreads();
  // 64 rows x 8 chunks per wave
  for (int i = lane; i < 64 * 8; i += 64) {
    const int r = i >> 3, c = i & 7;
    const int m = m0 + wm + r, n = n0 + wn + c * 8;
    if (m < M && n < n_out)
      *reinterpret_cast<bf16x8*>(out + (long)m * out_stride + n) = *reinterpret_cast<const bf16x8*>(&tile[r * ORS + c * 8]);
  }
}

template <bool kGather, bool kScale>
__global__ void __launch_bounds__(256)
linear_f32_kernel(const float* __restrict__ x, const int32_t* __restrict__ gather_idx,
                  const float* __restrict__ gate_scores, const int32_t* __restrict__ total,
                  const float* __restrict__ W, const float* __restrict__ bias, int m_cap, int K, int n_out,
                  float* __restrict__ out, long out_stride) {
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
    out[(long)m * out_stride + n] = a + (bias != nullptr ? bias[n] : 0.f);
  }
}

}  // namespace spa

using namespace spa;

extern "C" int spa_linear_packed(const void* x, const int32_t* gather_idx, const float* gate_scores,
                                 const int32_t* total, const void* W, const void* bias, int M_cap, int K,
                                 int N_out, int dtype, void* out, int64_t out_row_stride, void* stream) {
  const char* fn = "spa_linear_packed";
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
                     (float*)out, (long)out_row_stride)
    if (g && sc) SPA_LIN_F32(true, true); else if (g) SPA_LIN_F32(true, false); else SPA_LIN_F32(false, false);
#undef SPA_LIN_F32
    return check_launch(fn);
  }
  SPA_REQUIRE(K % kGemmBK == 0, SPA_ERR_UNSUPPORTED, "%s: K = %d must be a multiple of %d for bf16", fn, K, kGemmBK);
  SPA_REQUIRE(N_out % 8 == 0 && out_row_stride % 8 == 0, SPA_ERR_INVALID_ARG,
              "%s: N_out and out_row_stride must be multiples of 8 for bf16", fn);
  SPA_REQUIRE(aligned16(x) && aligned16(W) && aligned16(out), SPA_ERR_INVALID_ARG, "%s: x / W / out not 16-byte aligned", fn);
  const int m_tiles = (M_cap + kGemmBM - 1) / kGemmBM, n_tiles = (N_out + kGemmBN - 1) / kGemmBN;
  SPA_REQUIRE((long)m_tiles * n_tiles + 8 < 2147483647L / 2, SPA_ERR_INVALID_ARG, "%s: too many tiles", fn);
  const unsigned grid = (unsigned)((long)((m_tiles + 7) / 8) * 8 * n_tiles);
#define SPA_LIN_BF16(G_, S_)                                                                                  \
  hipLaunchKernelGGL((linear_bf16_kernel<G_, S_>), dim3(grid), dim3(kGemmThreads), 0, st, (const __bf16*)x,  \
                     gather_idx, gate_scores, total, (const __bf16*)W, (const __bf16*)bias, M_cap, K, N_out, \
                     (__bf16*)out, (long)out_row_stride, m_tiles, n_tiles)
  if (g && sc) SPA_LIN_BF16(true, true); else if (g) SPA_LIN_BF16(true, false); else SPA_LIN_BF16(false, false);
#undef SPA_LIN_BF16
  return check_launch(fn);
}
