// Backward of the projections of the packed tokens (the 3 L C^2 and N C^2 terms of the SPA
// complexity formula, Section 3.2).  For out_j = r_j W^T + bias, with r_j the (gathered,
// optionally gate-scaled) row j and g_j the upstream gradient of out_j:
//   input side    d_rows[j,:] = g_j W                       [M, N_out] x [N_out, K]
//   weight side   dW = sum_j g_j^T r_j, dbias = sum_j g_j   [N_out, M] x [M, K]
// Both are MFMA GEMMs whose contraction index is the slow index of at least one operand in
// memory (W is [N_out][K] and the input side contracts over N_out; the weight side contracts
// over the tokens).  Those operands are staged in LDS exactly as they lie in memory, rows =
// contraction index, with whole 16-byte pieces, and the MFMA fragments are taken with the
// transposing LDS read (ds_read_b64_tr_b16), so nothing is transposed in memory or staged twice.
//
// Input side: 128 x 128 x 64 tiles, four waves 2 x 2, the live tiles cut into 8 contiguous
// ranges, one per XCD (as in the forward kernel).  The gather of the upstream rows
// (dout_idx), the scatter of the result rows (dx_idx) and the zero fill of the rows no
// packed row maps to are folded in.
// Weight side: the output is only N_out x K (a few dozen 128 x 128 tiles), so the tokens are
// cut into `splits` chunks (chunk length fixed on the device from the live row count, so all
// chunks carry work) and every (chunk, tile) is a workgroup; the partial tiles go to a
// workspace in fp32 and a second kernel adds them in chunk order: deterministic, no atomics.
// Items are numbered chunk-major and cut into 8 contiguous ranges, one per XCD, so the tiles
// that read the same rows share an L2.  dbias comes from the same fragments: one more MFMA
// per step against a vector of ones in the workgroups of the first column tile.
// fp32 (tiny workload): one thread per output element.
#include <stdlib.h>

#include "attn_tiles.h"
#include "spa_common.h"

namespace spa {

constexpr int kLbThreads = 256;
constexpr int kLbT = 128;          // output tile edge
constexpr int kLbK = 64;           // contraction step
constexpr int kLbRS = kLbT + 16;   // row stride (elements) of a [contraction][128] tile: 72 dwords = 8 mod 64,
                                   // the 4 rows x 32 bytes a 16-lane block reads fall on distinct banks
constexpr int kLbRSA = kLbK + 8;   // row stride of a [128][contraction] tile (16-byte fragment reads)
constexpr size_t kLbInputLds = (size_t)2 * (kLbT * kLbRSA + kLbK * kLbRS) * sizeof(__bf16);
constexpr int kLbRows = 512;       // rows of a chunk whose sources are tabled in LDS at a time (6 KB: with the
                                   // operand stages 78 KB per workgroup, two workgroups per compute unit)
constexpr size_t kLbWeightLds = (size_t)2 * 2 * kLbK * kLbRS * sizeof(__bf16);

// MFMA operand fragment taken DOWN the columns of a row-major tile whose rows are the
// contraction index: lane (l32, hh) receives tile[k0 + 8 hh + e][c0 + l32], e = 0..7, the same
// contraction order as a 16-byte read along a row of a [column][contraction] tile.  Within each
// block of 16 lanes the transposing read hands lane i, element e, the value that lane
// (4 e + i / 4) of the block addressed at its own element i % 4: lane s of a block points at
// row k0 + s / 4, columns 4 (s % 4) .. + 3, and lane i receives rows k0 .. k0 + 3 of column i.
template <int RS>
__device__ __forceinline__ bf16x8 frag_down_columns(const __bf16* tile, int k0, int c0, int lane) {
  const int blk = lane >> 4, s = lane & 15;
  const __bf16* p = tile + (k0 + 8 * (blk >> 1) + (s >> 2)) * RS + c0 + 16 * (blk & 1) + 4 * (s & 3);
  typedef shortx4_lds __attribute__((address_space(3))) * lds_ptr;
  const shortx4_lds lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p));
  const shortx4_lds hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p + 4 * RS));
  const bf16x4 l4 = __builtin_bit_cast(bf16x4, lo), h4 = __builtin_bit_cast(bf16x4, hi);
  return __builtin_shufflevector(l4, h4, 0, 1, 2, 3, 4, 5, 6, 7);
}

// ------------------------------------------------------------------------------ input side
// dx[o(j), :] = dout[a(j), :] W for j < M, W [kc][ncols] row-major (kc = N_out of the forward,
// the contraction; ncols = K of the forward).
__global__ void __launch_bounds__(kLbThreads)
linear_bwd_input_bf16_kernel(const __bf16* __restrict__ dout, const int32_t* __restrict__ dout_idx, long ldd,
                             const int32_t* __restrict__ total, const __bf16* __restrict__ W, int m_cap, int kc,
                             int ncols, __bf16* __restrict__ dx, long ldx, const int32_t* __restrict__ dx_idx,
                             const int32_t* __restrict__ inv_pos, long rows, int n_tiles) {
  constexpr int BM = kLbT, BN = kLbT, BK = kLbK, RSA = kLbRSA, RSB = kLbRS;
  extern __shared__ __attribute__((aligned(16))) unsigned char lb_smem[];
  __bf16(*As)[BM * RSA] = reinterpret_cast<__bf16(*)[BM * RSA]>(lb_smem);
  __bf16(*Bs)[BK * RSB] = reinterpret_cast<__bf16(*)[BK * RSB]>(lb_smem + 2 * BM * RSA * sizeof(__bf16));
  __shared__ long a_row[BM];   // source row of every tile row (-1 = past the end)
  __shared__ int o_row[BM];    // destination row

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, l32 = lane & 31, hh = lane >> 5;

  // every wave of the grid clears its share of the rows no packed row maps to
  if (inv_pos != nullptr) {
    const long units = (long)gridDim.x * 4, u = (long)blockIdx.x * 4 + wv;
    const long per = (rows + units - 1) / units, r0 = min(rows, u * per), r1 = min(rows, r0 + per);
    zero_unselected_rows(dx, ldx, ncols, inv_pos, r0, r1, lane);
  }

  const int M = total != nullptr ? min(total[0], m_cap) : m_cap;
  const int live_tiles = ((M + BM - 1) / BM) * n_tiles, per_xcd = (live_tiles + 7) >> 3;
  const int xcd = blockIdx.x & 7, jx = blockIdx.x >> 3, tile_id = xcd * per_xcd + jx;
  if (jx >= per_xcd || tile_id >= live_tiles) return;
  const int mt = tile_id / n_tiles, nt = tile_id - mt * n_tiles;
  const int m0 = mt * BM, n0 = nt * BN;
  const int wm = (wv >> 1) * 64, wn = (wv & 1) * 64;

  if (tid < BM) {
    const int r = m0 + tid;
    a_row[tid] = r < M ? (dout_idx != nullptr ? (long)dout_idx[r] : (long)r) : -1;
    o_row[tid] = r < M && dx_idx != nullptr ? dx_idx[r] : r;
  }
  __syncthreads();

  // staging.  A: 128 rows x 8 chunks of 16 bytes, thread -> chunk tid % 8 of rows tid / 8 + 32 u.
  // B: 64 contraction rows x 16 chunks, thread -> chunk tid % 16 of rows tid / 16 + 16 u.
  // Rows of A past the valid range load a valid row and columns of B past ncols load a valid
  // column: such a row or column only reaches outputs that are never stored.
  constexpr int NU = 4;
  const int sa_r = tid >> 3, sa_c = tid & 7, sb_r = tid >> 4, sb_c = tid & 15;
  const int lds_a = sa_r * RSA + sa_c * 8, lds_b = sb_r * RSB + sb_c * 8;
  const __bf16* ap[NU];
#pragma unroll
  for (int u = 0; u < NU; ++u) {
    const long src = a_row[sa_r + u * 32];
    ap[u] = dout + (src >= 0 ? src : 0) * ldd + sa_c * 8;
  }
  const __bf16* bcol = W + (n0 + sb_c * 8 < ncols ? n0 + sb_c * 8 : n0);

  // When kc is not a multiple of BK the PARTIAL contraction tile comes first (its data at the
  // front of the tile, zeros behind), so only the prologue needs masked loads: tile t >= 1
  // starts at contraction index k_first + t * BK.
  constexpr int PF = 2;
  bf16x8 areg[PF][NU], breg[PF][NU];
  const int k_tail = kc % BK, nk = (kc + BK - 1) / BK, k_first = k_tail ? k_tail - BK : 0;
  auto gload = [&](int slot, int t) {
    const int k0 = k_first + t * BK;
#pragma unroll
    for (int u = 0; u < NU; ++u) areg[slot][u] = *reinterpret_cast<const bf16x8*>(ap[u] + k0);
#pragma unroll
    for (int u = 0; u < NU; ++u)
      breg[slot][u] = *reinterpret_cast<const bf16x8*>(bcol + (long)(k0 + sb_r + u * 16) * ncols);
  };
  auto gload_first = [&](int slot) {
    if (k_tail == 0) { gload(slot, 0); return; }
#pragma unroll
    for (int u = 0; u < NU; ++u)
      areg[slot][u] = sa_c * 8 < k_tail ? *reinterpret_cast<const bf16x8*>(ap[u]) : zero_bf16x8();
#pragma unroll
    for (int u = 0; u < NU; ++u)
      breg[slot][u] = sb_r + u * 16 < k_tail ? *reinterpret_cast<const bf16x8*>(bcol + (long)(sb_r + u * 16) * ncols)
                                             : zero_bf16x8();
  };
  auto lstore = [&](int slot, int buf) {
#pragma unroll
    for (int u = 0; u < NU; ++u) *reinterpret_cast<bf16x8*>(&As[buf][lds_a + u * 32 * RSA]) = areg[slot][u];
#pragma unroll
    for (int u = 0; u < NU; ++u) *reinterpret_cast<bf16x8*>(&Bs[buf][lds_b + u * 16 * RSB]) = breg[slot][u];
  };

  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int jn = 0; jn < 2; ++jn)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][jn][r] = 0.f;

  auto compute = [&](int buf) {
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8 af[2], bfr[2];
#pragma unroll
      for (int i = 0; i < 2; ++i)
        af[i] = *reinterpret_cast<const bf16x8*>(&As[buf][(wm + i * 32 + l32) * RSA + kk * 16 + hh * 8]);
#pragma unroll
      for (int jn = 0; jn < 2; ++jn) bfr[jn] = frag_down_columns<RSB>(Bs[buf], kk * 16, wn + jn * 32, lane);
      // C^T tiles: rows = output columns, cols = packed rows (a lane's 4 consecutive accumulator
      // registers are 4 consecutive columns of one row)
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int jn = 0; jn < 2; ++jn)
          acc[i][jn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[jn], af[i], acc[i][jn], 0, 0, 0);
    }
  };

  // Entering a trip: LDS buffer 0 holds tile kt, slot 1 holds tile kt + 1, slot 0 is free.
  // Loads past the last tile repeat it; what they bring is stored but never multiplied.
  const int last = nk - 1;
  gload_first(0);
  if (nk > 1) gload(1, 1);
  lstore(0, 0);
  __syncthreads();
  for (int kt = 0; kt + 1 < nk; kt += 2) {
    gload(0, min(kt + 2, last));
    compute(0);
    lstore(1, 1);
    __syncthreads();
    gload(1, min(kt + 3, last));
    compute(1);
    lstore(0, 0);
    __syncthreads();
  }
  if (nk & 1) {
    compute(0);
    __syncthreads();     // the epilogue reuses the operand buffers
  }

  // epilogue: the wave's 64 x 64 block is parked in LDS as bf16 and leaves as 16-byte pieces
  constexpr int ORS = 64 + 8;
  static_assert((size_t)4 * 64 * ORS * sizeof(__bf16) <= kLbInputLds, "output staging fits in the operand buffers");
  __bf16* tile = reinterpret_cast<__bf16*>(lb_smem) + wv * 64 * ORS;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int jn = 0; jn < 2; ++jn)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const floatx4 f = {acc[i][jn][4 * g], acc[i][jn][4 * g + 1], acc[i][jn][4 * g + 2], acc[i][jn][4 * g + 3]};
        *reinterpret_cast<bf16x4*>(&tile[(i * 32 + l32) * ORS + jn * 32 + 8 * g + 4 * hh]) =
            __builtin_convertvector(f, bf16x4);
      }
  __syncthreads();
  for (int c = lane; c < 64 * 8; c += 64) {
    const int r = c >> 3, ch = c & 7;
    const int m = m0 + wm + r, n = n0 + wn + ch * 8;
    if (m < M && n < ncols)
      *reinterpret_cast<bf16x8*>(dx + (long)o_row[wm + r] * ldx + n) = *reinterpret_cast<const bf16x8*>(&tile[r * ORS + ch * 8]);
  }
}

__global__ void __launch_bounds__(256)
linear_bwd_input_f32_kernel(const float* __restrict__ dout, const int32_t* __restrict__ dout_idx, long ldd,
                            const int32_t* __restrict__ total, const float* __restrict__ W, int m_cap, int kc, int ncols,
                            float* __restrict__ dx, long ldx, const int32_t* __restrict__ dx_idx,
                            const int32_t* __restrict__ inv_pos, long rows) {
  const long stride = (long)gridDim.x * blockDim.x, first = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (inv_pos != nullptr)
    for (long i = first; i < rows * ncols; i += stride) {
      const long r = i / ncols;
      if (inv_pos[r] < 0) dx[r * ldx + (i - r * ncols)] = 0.f;
    }
  const int M = total != nullptr ? min(total[0], m_cap) : m_cap;
  for (long i = first; i < (long)M * ncols; i += stride) {
    const int m = (int)(i / ncols), c = (int)(i - (long)m * ncols);
    const float* g = dout + (dout_idx != nullptr ? (long)dout_idx[m] : (long)m) * ldd;
    float a = 0.f;
    for (int n = 0; n < kc; ++n) a = fmaf(g[n], W[(long)n * ncols + c], a);
    dx[(dx_idx != nullptr ? (long)dx_idx[m] : (long)m) * ldx + c] = a;
  }
}

// ----------------------------------------------------------------------------- weight side
// Chunk length and number of chunks that carry rows, from the live row count.
struct TokenSplit {
  int chunk, live;
};
__device__ __forceinline__ TokenSplit token_split(int M, int splits) {
  TokenSplit s;
  s.chunk = (((M + splits - 1) / splits) + kLbK - 1) & ~(kLbK - 1);
  s.live = s.chunk > 0 ? (M + s.chunk - 1) / s.chunk : 0;
  return s;
}

// part_w[split][n][k] = sum over the chunk's rows j of g_j[n] r_j[k]; part_b[split][n] = sum g_j[n]
template <bool kScale>
__global__ void __launch_bounds__(kLbThreads)
linear_bwd_weight_bf16_kernel(const __bf16* __restrict__ dout, const int32_t* __restrict__ dout_idx, long ldd,
                              const __bf16* __restrict__ x, const int32_t* __restrict__ x_idx,
                              const float* __restrict__ gate_scores, const int32_t* __restrict__ total, int m_cap, int K,
                              int n_out, int splits, int n_tiles, int k_tiles, float* __restrict__ part_w,
                              float* __restrict__ part_b) {
  constexpr int BT = kLbT, BK = kLbK, RS = kLbRS;
  extern __shared__ __attribute__((aligned(16))) unsigned char lb_smem[];
  __bf16(*Gs)[BK * RS] = reinterpret_cast<__bf16(*)[BK * RS]>(lb_smem);
  __bf16(*Xs)[BK * RS] = reinterpret_cast<__bf16(*)[BK * RS]>(lb_smem + 2 * BK * RS * sizeof(__bf16));
  __shared__ int g_src[kLbRows];       // row of dout (-1: past the end of the chunk), of x, and the
  __shared__ int x_src[kLbRows];       // gate scale of every row of the current block
  __shared__ float x_scale[kLbRows];

  const int M = total != nullptr ? min(total[0], m_cap) : m_cap;
  const TokenSplit ts = token_split(M, splits);
  const int tiles = n_tiles * k_tiles, items = ts.live * tiles, per_xcd = (items + 7) >> 3;
  const int xcd = blockIdx.x & 7, jx = blockIdx.x >> 3, item = xcd * per_xcd + jx;
  if (jx >= per_xcd || item >= items) return;
  const int split = item / tiles, tile_id = item - split * tiles;
  const int nt = tile_id / k_tiles, kt_ = tile_id - nt * k_tiles;
  const int n0 = nt * BT, k0 = kt_ * BT;
  const int m_begin = split * ts.chunk, m_end = min(M, m_begin + ts.chunk);

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, l32 = lane & 31, hh = lane >> 5;
  const int wn = (wv >> 1) * 64, wk = (wv & 1) * 64;
  const bool do_bias = kt_ == 0 && wk == 0;

  // staging: both tiles are 64 token rows x 16 chunks of 16 bytes; thread -> chunk tid % 16 of
  // rows tid / 16 + 16 u.  Columns past the matrix edge load a valid column (never stored).
  constexpr int NU = 4;
  const int s_r = tid >> 4, s_c = tid & 15, lds_off = s_r * RS + s_c * 8;
  const __bf16* gcol = dout + (n0 + s_c * 8 < n_out ? n0 + s_c * 8 : n0);
  const __bf16* xcol = x + (k0 + s_c * 8 < K ? k0 + s_c * 8 : k0);

  struct Data {
    bf16x8 g[NU], x[NU];
    float sc[NU];
    bool ok[NU];
  };
  // rows of step t of the current block of tabled rows
  auto gload = [&](Data& d, int t) {
#pragma unroll
    for (int u = 0; u < NU; ++u) {
      const int r = t * BK + s_r + u * 16;
      const int gi = g_src[r];
      d.ok[u] = gi >= 0;
      d.sc[u] = x_scale[r];
      d.g[u] = *reinterpret_cast<const bf16x8*>(gcol + (long)max(gi, 0) * ldd);
      d.x[u] = *reinterpret_cast<const bf16x8*>(xcol + (long)x_src[r] * K);
    }
  };
  auto lstore = [&](const Data& d, int buf) {
#pragma unroll
    for (int u = 0; u < NU; ++u) {
      bf16x8 xv = d.x[u];
      if (kScale) xv = float_to_bf16x8(bf16x8_to_float(xv) * d.sc[u]);   // the gated row, rounded to bf16
      *reinterpret_cast<bf16x8*>(&Gs[buf][lds_off + u * 16 * RS]) = d.ok[u] ? d.g[u] : zero_bf16x8();
      *reinterpret_cast<bf16x8*>(&Xs[buf][lds_off + u * 16 * RS]) = d.ok[u] ? xv : zero_bf16x8();
    }
  };

  floatx16 acc[2][2], accb[2];
#pragma unroll
  for (int jn = 0; jn < 2; ++jn) {
#pragma unroll
    for (int r = 0; r < 16; ++r) accb[jn][r] = 0.f;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][jn][r] = 0.f;
  }
  const __bf16 one = static_cast<__bf16>(1.0f);
  const bf16x8 ones = {one, one, one, one, one, one, one, one};

  auto compute = [&](int buf) {
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8 xf[2], gf[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) xf[i] = frag_down_columns<RS>(Xs[buf], kk * 16, wk + i * 32, lane);
#pragma unroll
      for (int jn = 0; jn < 2; ++jn) gf[jn] = frag_down_columns<RS>(Gs[buf], kk * 16, wn + jn * 32, lane);
      // tiles with rows = k (input feature), cols = n (output feature): a lane's 4 consecutive
      // accumulator registers are 4 consecutive k of one n, 16 bytes of a row of dW
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int jn = 0; jn < 2; ++jn)
          acc[i][jn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf[i], gf[jn], acc[i][jn], 0, 0, 0);
      if (do_bias) {
#pragma unroll
        for (int jn = 0; jn < 2; ++jn)
          accb[jn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ones, gf[jn], accb[jn], 0, 0, 0);
      }
    }
  };

  // The chunk is walked in blocks of kLbRows rows.  Where a block's rows lie (index arrays) and
  // their gate scale are tabled in LDS first, so the row loads of the pipelined loop depend on
  // LDS reads only, not on other loads still in flight (index -> score -> row would be three
  // dependent trips to memory per step).
  for (int blk0 = m_begin; blk0 < m_end; blk0 += kLbRows) {
    const int blk_rows = min(kLbRows, m_end - blk0), steps = (blk_rows + BK - 1) / BK;
    // all index loads first, then all score loads: two trips to memory for the whole table
    constexpr int NF = kLbRows / kLbThreads;
    int gi[NF], xi[NF];
    float sv[NF];
#pragma unroll
    for (int u = 0; u < NF; ++u) {
      const int m = min(blk0 + tid + u * kLbThreads, m_end - 1);
      gi[u] = dout_idx != nullptr ? dout_idx[m] : m;
      xi[u] = x_idx != nullptr ? x_idx[m] : m;
    }
#pragma unroll
    for (int u = 0; u < NF; ++u) sv[u] = kScale ? gate_scores[xi[u]] : 0.f;
#pragma unroll
    for (int u = 0; u < NF; ++u) {
      const int r = tid + u * kLbThreads;
      const bool valid = r < blk_rows;
      if (r < steps * BK) {
        g_src[r] = valid ? gi[u] : -1;
        x_src[r] = valid ? xi[u] : 0;
        x_scale[r] = valid ? (kScale ? sigmoidf_dev(sv[u]) : 1.f) : 0.f;
      }
    }
    __syncthreads();
    // Entering a trip: LDS buffer 0 holds step kt, d1 holds step kt + 1, d0 is free.  Loads
    // past the last step repeat it; what they bring is stored but never multiplied.
    const int last = steps - 1;
    Data d0, d1;
    gload(d0, 0);
    if (steps > 1) gload(d1, 1);
    lstore(d0, 0);
    __syncthreads();
    for (int kt = 0; kt + 1 < steps; kt += 2) {
      gload(d0, min(kt + 2, last));
      compute(0);
      lstore(d1, 1);
      __syncthreads();
      gload(d1, min(kt + 3, last));
      compute(1);
      lstore(d0, 0);
      __syncthreads();
    }
    if (steps & 1) {
      compute(0);
      __syncthreads();     // the next block's tables and the epilogue reuse LDS
    }
  }

  // epilogue: the wave's 64 (n) x 64 (k) block is parked in LDS as fp32 and leaves as 16-byte
  // pieces of 256-byte row segments
  constexpr int ORS = 64 + 4;
  static_assert((size_t)4 * 64 * ORS * sizeof(float) <= kLbWeightLds, "output staging fits in the operand buffers");
  float* tile = reinterpret_cast<float*>(lb_smem) + wv * 64 * ORS;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int jn = 0; jn < 2; ++jn)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const floatx4 f = {acc[i][jn][4 * g], acc[i][jn][4 * g + 1], acc[i][jn][4 * g + 2], acc[i][jn][4 * g + 3]};
        *reinterpret_cast<floatx4*>(&tile[(jn * 32 + l32) * ORS + i * 32 + 8 * g + 4 * hh]) = f;
      }
  __syncthreads();
  float* pw = part_w + (long)split * n_out * K;
  for (int c = lane; c < 64 * 16; c += 64) {
    const int r = c >> 4, ch = c & 15;
    const int n = n0 + wn + r, k = k0 + wk + ch * 4;
    if (n < n_out && k < K)
      *reinterpret_cast<floatx4*>(pw + (long)n * K + k) = *reinterpret_cast<const floatx4*>(&tile[r * ORS + ch * 4]);
  }
  if (do_bias && hh == 0) {
#pragma unroll
    for (int jn = 0; jn < 2; ++jn) {
      const int n = n0 + wn + jn * 32 + l32;
      if (n < n_out) part_b[(long)split * n_out + n] = accb[jn][0];   // every row of the tile holds the column sums
    }
  }
}

// dW = sum of the partial tiles in chunk order; dbias likewise
__global__ void __launch_bounds__(256)
linear_bwd_weight_reduce_kernel(const float* __restrict__ part_w, const float* __restrict__ part_b,
                                const int32_t* __restrict__ total, int m_cap, int splits, long nk, int n_out,
                                float* __restrict__ dW, float* __restrict__ dbias) {
  const int M = total != nullptr ? min(total[0], m_cap) : m_cap;
  const int live = token_split(M, splits).live;
  const long quads = nk >> 2, work = quads + (dbias != nullptr ? n_out : 0);
  for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < work; i += (long)gridDim.x * blockDim.x) {
    if (i < quads) {
      floatx4 a = {0.f, 0.f, 0.f, 0.f};
      for (int s = 0; s < live; ++s) a += *reinterpret_cast<const floatx4*>(part_w + (long)s * nk + 4 * i);
      *reinterpret_cast<floatx4*>(dW + 4 * i) = a;
    } else {
      const long n = i - quads;
      float a = 0.f;
      for (int s = 0; s < live; ++s) a += part_b[(long)s * n_out + n];
      dbias[n] = a;
    }
  }
}

__global__ void __launch_bounds__(256)
linear_bwd_weight_f32_kernel(const float* __restrict__ dout, const int32_t* __restrict__ dout_idx, long ldd,
                             const float* __restrict__ x, const int32_t* __restrict__ x_idx,
                             const float* __restrict__ gate_scores, const int32_t* __restrict__ total, int m_cap, int K,
                             int n_out, float* __restrict__ dW, float* __restrict__ dbias) {
  const int M = total != nullptr ? min(total[0], m_cap) : m_cap;
  const long nk = (long)n_out * K, work = nk + (dbias != nullptr ? n_out : 0);
  for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < work; i += (long)gridDim.x * blockDim.x) {
    const bool is_w = i < nk;
    const int n = is_w ? (int)(i / K) : (int)(i - nk), k = is_w ? (int)(i - (long)n * K) : 0;
    float a = 0.f;
    for (int m = 0; m < M; ++m) {
      const float g = dout[(dout_idx != nullptr ? (long)dout_idx[m] : (long)m) * ldd + n];
      if (is_w) {
        const long xr = x_idx != nullptr ? (long)x_idx[m] : (long)m;
        const float sc = gate_scores != nullptr ? sigmoidf_dev(gate_scores[xr]) : 1.f;
        a = fmaf(g, sc * x[xr * K + k], a);
      } else {
        a += g;
      }
    }
    if (is_w) dW[i] = a; else dbias[n] = a;
  }
}

// Number of token chunks of the weight-side kernel: (chunk, tile) workgroups for about three per
// compute unit (two are resident at a time), at most 16 chunks (the partial tiles are written
// and read once per chunk), chunks of at least 256 rows at full capacity.  The option gemm_splits
// overrides it (tuning aid).
static int weight_splits(int M_cap, int K, int N_out) {
  const int env = options().gemm_splits;
  if (env > 0) return env;
  const long tiles = (long)((N_out + kLbT - 1) / kLbT) * ((K + kLbT - 1) / kLbT);
  long s = (768 + tiles - 1) / tiles;
  const long by_rows = M_cap / 256 > 0 ? M_cap / 256 : 1;
  if (s > by_rows) s = by_rows;
  if (s > 16) s = 16;
  return (int)(s < 1 ? 1 : s);
}

}  // namespace spa

using namespace spa;

extern "C" int spa_linear_packed_bwd_input(const void* dout, const int32_t* dout_idx, int64_t dout_row_stride,
                                           const int32_t* total, const void* W, int M_cap, int K, int N_out, int dtype,
                                           const int32_t* dx_idx, const int32_t* inv_pos, int64_t rows, void* dx,
                                           int64_t dx_row_stride, void* stream) {
  const char* fn = "spa_linear_packed_bwd_input";
  SPA_REQUIRE(dout && W && dx, SPA_ERR_INVALID_ARG, "%s: null pointer", fn);
  SPA_REQUIRE(M_cap >= 1 && K >= 1 && N_out >= 1, SPA_ERR_INVALID_ARG, "%s: M_cap, K, N_out must be >= 1", fn);
  SPA_REQUIRE(dtype == SPA_F32 || dtype == SPA_BF16, SPA_ERR_UNSUPPORTED, "%s: unknown dtype %d", fn, dtype);
  SPA_REQUIRE(dout_row_stride >= N_out && dx_row_stride >= K, SPA_ERR_INVALID_ARG,
              "%s: dout_row_stride < N_out or dx_row_stride < K", fn);
  SPA_REQUIRE(inv_pos == nullptr || (dx_idx != nullptr && rows >= 0), SPA_ERR_INVALID_ARG,
              "%s: inv_pos (zero fill of the rows no packed row maps to) needs dx_idx and rows >= 0", fn);
  hipStream_t st = as_stream(stream);
  if (dtype == SPA_F32) {
    long work = (long)M_cap * K;
    if (inv_pos != nullptr && rows * K > work) work = rows * K;
    long wgs = (work + 255) / 256;
    if (wgs > 8192) wgs = 8192;
    hipLaunchKernelGGL(linear_bwd_input_f32_kernel, dim3((unsigned)wgs), dim3(256), 0, st, (const float*)dout, dout_idx,
                       (long)dout_row_stride, total, (const float*)W, M_cap, N_out, K, (float*)dx, (long)dx_row_stride,
                       dx_idx, inv_pos, (long)rows);
    return check_launch(fn);
  }
  SPA_REQUIRE(K % 8 == 0 && N_out % 8 == 0 && dout_row_stride % 8 == 0 && dx_row_stride % 8 == 0, SPA_ERR_UNSUPPORTED,
              "%s: K, N_out and the row strides must be multiples of 8 for bf16", fn);
  SPA_REQUIRE(aligned16(dout) && aligned16(W) && aligned16(dx), SPA_ERR_INVALID_ARG,
              "%s: dout / W / dx not 16-byte aligned", fn);
  const int m_tiles = (M_cap + kLbT - 1) / kLbT, n_tiles = (K + kLbT - 1) / kLbT;
  SPA_REQUIRE((long)m_tiles * n_tiles + 8 < 2147483647L / 2, SPA_ERR_INVALID_ARG, "%s: too many tiles", fn);
  const unsigned grid = (unsigned)((long)((m_tiles + 7) / 8) * 8 * n_tiles);
  const hipError_t attr = hipFuncSetAttribute((const void*)linear_bwd_input_bf16_kernel,
                                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLbInputLds);
  SPA_REQUIRE(attr == hipSuccess, SPA_ERR_HIP, "%s: cannot reserve %zu bytes of LDS", fn, kLbInputLds);
  hipLaunchKernelGGL(linear_bwd_input_bf16_kernel, dim3(grid), dim3(kLbThreads), kLbInputLds, st, (const __bf16*)dout,
                     dout_idx, (long)dout_row_stride, total, (const __bf16*)W, M_cap, N_out, K, (__bf16*)dx,
                     (long)dx_row_stride, dx_idx, inv_pos, (long)rows, n_tiles);
  return check_launch(fn);
}

extern "C" size_t spa_linear_bwd_weight_workspace_bytes(int M_cap, int K, int N_out, int dtype) {
  if (dtype != SPA_BF16 || M_cap < 1 || K < 1 || N_out < 1) return 0;
  const size_t per_split = ((size_t)N_out * K + N_out) * sizeof(float);
  return ((size_t)weight_splits(M_cap, K, N_out) * per_split + 255) & ~(size_t)255;
}

extern "C" int spa_linear_packed_bwd_weight(const void* dout, const int32_t* dout_idx, int64_t dout_row_stride,
                                            const void* x, const int32_t* x_idx, const float* gate_scores,
                                            const int32_t* total, int M_cap, int K, int N_out, int dtype, float* dW,
                                            float* dbias, void* workspace, size_t workspace_bytes, void* stream) {
  const char* fn = "spa_linear_packed_bwd_weight";
  SPA_REQUIRE(dout && x && dW, SPA_ERR_INVALID_ARG, "%s: null pointer", fn);
  SPA_REQUIRE(M_cap >= 1 && K >= 1 && N_out >= 1, SPA_ERR_INVALID_ARG, "%s: M_cap, K, N_out must be >= 1", fn);
  SPA_REQUIRE(dtype == SPA_F32 || dtype == SPA_BF16, SPA_ERR_UNSUPPORTED, "%s: unknown dtype %d", fn, dtype);
  SPA_REQUIRE(dout_row_stride >= N_out, SPA_ERR_INVALID_ARG, "%s: dout_row_stride < N_out", fn);
  SPA_REQUIRE(!(gate_scores != nullptr && x_idx == nullptr), SPA_ERR_INVALID_ARG,
              "%s: gate_scores are indexed by token and need x_idx", fn);
  hipStream_t st = as_stream(stream);
  if (dtype == SPA_F32) {
    long wgs = ((long)N_out * K + N_out + 255) / 256;
    if (wgs > 8192) wgs = 8192;
    hipLaunchKernelGGL(linear_bwd_weight_f32_kernel, dim3((unsigned)wgs), dim3(256), 0, st, (const float*)dout, dout_idx,
                       (long)dout_row_stride, (const float*)x, x_idx, gate_scores, total, M_cap, K, N_out, dW, dbias);
    return check_launch(fn);
  }
  SPA_REQUIRE(K % 8 == 0 && N_out % 8 == 0 && dout_row_stride % 8 == 0, SPA_ERR_UNSUPPORTED,
              "%s: K, N_out and dout_row_stride must be multiples of 8 for bf16", fn);
  SPA_REQUIRE(aligned16(dout) && aligned16(x) && aligned16(dW), SPA_ERR_INVALID_ARG,
              "%s: dout / x / dW not 16-byte aligned", fn);
  const size_t need = spa_linear_bwd_weight_workspace_bytes(M_cap, K, N_out, dtype);
  SPA_REQUIRE(workspace != nullptr && workspace_bytes >= need, SPA_ERR_WORKSPACE,
              "%s: workspace of %zu bytes needed, %zu given", fn, need, workspace_bytes);
  SPA_REQUIRE((reinterpret_cast<uintptr_t>(workspace) & 255u) == 0, SPA_ERR_INVALID_ARG,
              "%s: workspace not 256-byte aligned", fn);
  const int splits = weight_splits(M_cap, K, N_out);
  const int n_tiles = (N_out + kLbT - 1) / kLbT, k_tiles = (K + kLbT - 1) / kLbT;
  const long items = (long)splits * n_tiles * k_tiles;
  SPA_REQUIRE(items + 8 < 2147483647L / 2, SPA_ERR_INVALID_ARG, "%s: too many tiles", fn);
  const unsigned grid = (unsigned)(((items + 7) / 8) * 8);
  float* part_w = static_cast<float*>(workspace);
  float* part_b = part_w + (size_t)splits * N_out * K;
#define SPA_LBW(S_)                                                                                              \
  do {                                                                                                           \
    const hipError_t attr = hipFuncSetAttribute((const void*)linear_bwd_weight_bf16_kernel<S_>,                  \
                                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLbWeightLds);  \
    SPA_REQUIRE(attr == hipSuccess, SPA_ERR_HIP, "%s: cannot reserve %zu bytes of LDS", fn, kLbWeightLds);       \
    hipLaunchKernelGGL((linear_bwd_weight_bf16_kernel<S_>), dim3(grid), dim3(kLbThreads), kLbWeightLds, st,      \
                       (const __bf16*)dout, dout_idx, (long)dout_row_stride, (const __bf16*)x, x_idx, gate_scores, \
                       total, M_cap, K, N_out, splits, n_tiles, k_tiles, part_w, part_b);                        \
  } while (0)
  if (gate_scores != nullptr) SPA_LBW(true); else SPA_LBW(false);
#undef SPA_LBW
  const int rc = check_launch(fn);
  if (rc != SPA_OK) return rc;
  const long nk = (long)N_out * K;
  long wgs = (nk / 4 + N_out + 255) / 256;
  if (wgs > 4096) wgs = 4096;
  hipLaunchKernelGGL(linear_bwd_weight_reduce_kernel, dim3((unsigned)wgs), dim3(256), 0, st, part_w, part_b, total, M_cap,
                     splits, nk, N_out, dW, dbias);
  return check_launch(fn);
}

