// Backward of the packed, per-image attention: for every (image, head) segment
//   P = exp(S - lse), dV = P^T dO, dP = dO V^T, D_i = sum_d dO_id O_id,
//   dS = P * (dP - D), dQ = dS K * scale, dK = dS^T Q * scale.
// No atomics anywhere; results are run-to-run bit-stable.
// Segments of up to 256 tokens (bf16): ONE kernel, a workgroup per (image, head), S and dP
// computed once (5 GEMM shapes); see attn_bwd_fused_bf16_kernel.
// Longer segments (bf16): two roles in one launch, after a small kernel that writes D_i:
//   dq role   : a wave owns 32 queries and walks the segment's keys.  Like the forward it
//               works on transposed tiles (S^T = K Q^T, dP^T = V dO^T) so lse_i and D_i are
//               one scalar per lane and dS^T is already the B operand of dQ^T += K^T dS^T.
//   dkdv role : a wave owns 32 keys and walks the segment's queries with S = Q K^T and
//               dP = dO V^T un-transposed (lane = key), so P and dS are the B operands of
//               dV^T += dO^T P and dK^T += Q^T dS.
//   S and dP are recomputed in both roles (7 GEMM shapes instead of 5) in exchange for
//   determinism.
// fp32: a thread per row (query side, then key side), the other side streaming through LDS.
// Every form can read the upstream gradient and write dq, dk, dv at token positions (TokenIO).
#include <algorithm>
#include <cmath>
#include <cstdlib>

#include "attn_tiles.h"
#include "spa_common.h"

namespace spa {

constexpr float kLog2e = 1.4426950408889634f;

struct Seg {
  long row0;
  int n;
};
__device__ __forceinline__ Seg seg_of(int b, const int32_t* cu) {
  Seg s;
  const int a = cu[b];
  s.row0 = a;
  s.n = cu[b + 1] - a;
  return s;
}


// Token-position I/O folded into the kernel (gather_idx == nullptr: packed I/O): the upstream
// gradient row of packed token j is dy[gather_idx[j]], the gradients of packed token j go to
// row gather_idx[j] of dq / dk / dv, and the rows of unselected tokens (inv_pos < 0) are zeroed,
// every workgroup of the launch clearing an even share (one-kernel form: its head's columns).
struct TokenIO {
  const int32_t* gather_idx;
  const int32_t* inv_pos;
  long rows;               // B * N
};

template <int DH, int RS>
__device__ __forceinline__ void flush_tile_rows(const __bf16* tile, __bf16* dst, long row_stride, int nrows, int lane,
                                                const int32_t* row_index) {
  constexpr int CPR = DH / 8;
#pragma unroll
  for (int i = lane; i < 32 * CPR; i += 64) {
    const int r = i / CPR, c = i % CPR;
    if (r < nrows)
      *reinterpret_cast<bf16x8*>(dst + (long)row_index[r] * row_stride + c * 8) =
          *reinterpret_cast<const bf16x8*>(&tile[r * RS + c * 8]);
  }
}

// Both bf16 kernels use the forward's launch scheme: 1-D XCD-aware grid (the blocks that
// share one (image, head)'s rows sit on one L2), longest image first, 4 waves x 32 rows per
// workgroup, the other side of the product streaming through double-buffered row-major LDS
// tiles of BT tokens with the next tile's rows in flight in registers.  Short segments
// (<= 256 tokens) use the same kernels with ONE wave per workgroup and 32-token tiles: small
// independent work units that spread over all SIMDs, no longest-first ranking.  Operands whose
// k-dimension is the token index are read with the transposing LDS read from the same
// row-major tiles, so nothing is staged twice.

// --------------------------------------------------------------------------- dQ (bf16)
// LDS of the two long-segment kernels: two row-major operand tiles (double-buffered unless the
// workgroup is one wave, which stores the next tile only after its own reads of the current
// one), the per-query statistics of the dkdv side, and the longest-first ranking.
template <int DH, int NW, int BT, bool LPT>
struct BwdLds {
  static constexpr int RS = DH + 8, NBUF = NW == 1 ? 1 : 2;
  __attribute__((aligned(16))) __bf16 A[NBUF][BT * RS];     // K (dq) | Q (dkdv)
  __attribute__((aligned(16))) __bf16 Bm[NBUF][BT * RS];    // V (dq) | dO (dkdv)
  __attribute__((aligned(16))) float lse2s[NBUF][BT];
  __attribute__((aligned(16))) float Ds[NBUF][BT];
  int s_cu[LPT ? 2 * kLptMaxB + 1 : 1];
  int s_pick;
};

// kHaveD: D_i = <dO_i, O_i> was computed by an earlier launch and is read from dvec; else this
// kernel computes it and writes dvec for the dkdv kernel that follows.
template <int DH, int NW, int BT, bool LPT, bool kHaveD>
__device__ __forceinline__ void
attn_bwd_dq_body(BwdLds<DH, NW, BT, LPT>& lds, const TileId tile_id, const __bf16* __restrict__ q,
                 const __bf16* __restrict__ k, const __bf16* __restrict__ v, long qs, long ks, long vs,
                 const __bf16* __restrict__ out, const __bf16* __restrict__ dout,
                 const float* __restrict__ lse, long lse_stride, const int32_t* __restrict__ cu, int H,
                 float scale, __bf16* __restrict__ dq, long gstride, float* __restrict__ dvec, int B,
                 const TokenIO tok = TokenIO{nullptr, nullptr, 0}, const bool have_live = false,
                 const Segment live = Segment{0, 0, 0}) {
  constexpr int RS = DH + 8, KK = DH / 16, DB = DH / 32, THREADS = 64 * NW, NBUF = NW == 1 ? 1 : 2;
  const bool at_tokens = tok.gather_idx != nullptr;
  auto& Ks = lds.A;
  auto& Vs = lds.Bm;
  int* s_cu = lds.s_cu;
  int& s_pick = lds.s_pick;
  static_assert(NBUF * BT >= 32 * NW, "the K buffers double as the output staging tile");

  if (!tile_id.valid) return;
  const int h = tile_id.h;
  // (live: the caller numbered the live blocks itself and hands over the block's segment)
  const Segment seg = have_live ? live
                      : LPT           ? lpt_segment<THREADS>(tile_id.rank, B, cu, nullptr, 0, s_cu, &s_pick)
                                      : segment_of(tile_id.rank, cu, nullptr, 0);
  const int q0 = tile_id.qb * (32 * NW);
  if (q0 >= seg.nq) return;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, l32 = lane & 31, hh = lane >> 5;
  const int qi = q0 + wv * 32 + l32;
  const bool wave_live = q0 + wv * 32 < seg.nq;
  const bool q_ok = qi < seg.nq;
  const long C = (long)H * DH;
  const float scale_log2 = scale * kLog2e;
  const __bf16* kh = k + h * DH;
  const __bf16* vh = v + h * DH;

  RowStage<DH, THREADS, BT> kst, vst;
  kst.load(kh, seg.row0, seg.nk, ks);
  vst.load(vh, seg.row0, seg.nk, vs);

  bf16x8 qf[KK], dof[KK];
  float dpart = 0.f;
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) {
    qf[kk] = zero_bf16x8();
    dof[kk] = zero_bf16x8();
    if (q_ok) {
      const int col = h * DH + kk * 16 + hh * 8;
      const long grow = at_tokens ? (long)tok.gather_idx[seg.row0 + qi] : seg.row0 + qi;
      qf[kk] = *reinterpret_cast<const bf16x8*>(q + (seg.row0 + qi) * qs + col);
      dof[kk] = *reinterpret_cast<const bf16x8*>(dout + grow * C + col);
      if (!kHaveD) {
        const floatx8 of = bf16x8_to_float(*reinterpret_cast<const bf16x8*>(out + (seg.row0 + qi) * C + col));
        const floatx8 gf = bf16x8_to_float(dof[kk]);
#pragma unroll
        for (int e = 0; e < 8; ++e) dpart = fmaf(of[e], gf[e], dpart);
      }
    }
  }
  float D;
  if (kHaveD) {
    D = q_ok ? dvec[h * lse_stride + seg.row0 + qi] : 0.f;
  } else {
    D = sum_across_halves(dpart);
    if (q_ok && hh == 0) dvec[h * lse_stride + seg.row0 + qi] = D;
  }
  // invalid queries: lse = +inf makes every probability 0
  const float lse2 = q_ok ? lse[h * lse_stride + seg.row0 + qi] * kLog2e : INFINITY;

  floatx16 acc[DB];
#pragma unroll
  for (int d = 0; d < DB; ++d)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[d][r] = 0.f;

  kst.store(Ks[0]);
  vst.store(Vs[0]);
  __syncthreads();
  const int nt = (seg.nk + BT - 1) / BT;
  for (int t = 0; t < nt; ++t) {
    const int buf = t & (NBUF - 1), nbuf = (t + 1) & (NBUF - 1), kt = t * BT;
    if (t + 1 < nt) {
      kst.load(kh, seg.row0 + kt + BT, seg.nk - kt - BT, ks);
      vst.load(vh, seg.row0 + kt + BT, seg.nk - kt - BT, vs);
    }
    if (wave_live) {
#pragma unroll
      for (int sb = 0; sb < BT / 32; ++sb) {
        const int key0 = kt + sb * 32;
        if (key0 >= seg.nk) break;
        floatx16 s, dp;
#pragma unroll
        for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
          const bf16x8 ka = *reinterpret_cast<const bf16x8*>(&Ks[buf][(sb * 32 + l32) * RS + kk * 16 + hh * 8]);
          s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qf[kk], s, 0, 0, 0);
          const bf16x8 va = *reinterpret_cast<const bf16x8*>(&Vs[buf][(sb * 32 + l32) * RS + kk * 16 + hh * 8]);
          dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, dof[kk], dp, 0, 0, 0);
        }
        float ds[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float p = __builtin_amdgcn_exp2f(fmaf(s[r], scale_log2, -lse2));
          if (key0 + acc_row(r, hh) >= seg.nk) p = 0.f;
          ds[r] = p * (dp[r] - D);
        }
#pragma unroll
        for (int mf = 0; mf < 2; ++mf) {
          floatx8 f;
#pragma unroll
          for (int j = 0; j < 8; ++j) f[j] = ds[8 * mf + j];
          const bf16x8 dsb = float_to_bf16x8(f);
#pragma unroll
          for (int d = 0; d < DB; ++d) {
            const bf16x8 a = transposed_frag_rowmajor<RS>(Ks[buf], d, sb * 32, mf, lane);   // K^T
            acc[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, dsb, acc[d], 0, 0, 0);
          }
        }
      }
    }
    if (t + 1 < nt) {
      kst.store(Ks[nbuf]);
      vst.store(Vs[nbuf]);
    }
    __syncthreads();
  }
  __bf16* tile = &Ks[0][0] + wv * 32 * RS;
  if (wave_live) park_tile<DH, RS>(acc, scale, tile, l32, hh);
  __syncthreads();
  if (wave_live) {
    const int nrows = min(32, seg.nq - q0 - wv * 32);
    if (at_tokens)
      flush_tile_rows<DH, RS>(tile, dq + h * DH, gstride, nrows, lane, tok.gather_idx + seg.row0 + q0 + wv * 32);
    else
      flush_tile<DH, RS>(tile, dq + (seg.row0 + q0 + wv * 32) * gstride + h * DH, gstride, nrows, lane);
  }
}

template <int DH, int NW, int BT, bool LPT>
__global__ void __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(NW == 1 ? 3 : 2)))
attn_bwd_dq_bf16_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k,
                        const __bf16* __restrict__ v, long qs, long ks, long vs,
                        const __bf16* __restrict__ out, const __bf16* __restrict__ dout,
                        const float* __restrict__ lse, long lse_stride, const int32_t* __restrict__ cu, int H,
                        float scale, __bf16* __restrict__ dq, long gstride, float* __restrict__ dvec, int B,
                        int nqb) {
  __shared__ BwdLds<DH, NW, BT, LPT> lds;
  attn_bwd_dq_body<DH, NW, BT, LPT, false>(lds, xcd_tile(nqb, H, B), q, k, v, qs, ks, vs, out, dout, lse, lse_stride,
                                           cu, H, scale, dq, gstride, dvec, B);
}

// ------------------------------------------------------------------------ dK, dV (bf16)
template <int DH, int NW, int BT, bool LPT>
__device__ __forceinline__ void
attn_bwd_dkdv_body(BwdLds<DH, NW, BT, LPT>& lds, const TileId tile_id, const __bf16* __restrict__ q,
                   const __bf16* __restrict__ k, const __bf16* __restrict__ v, long qs, long ks, long vs,
                   const __bf16* __restrict__ dout, const float* __restrict__ lse,
                   const float* __restrict__ dvec, long lse_stride, const int32_t* __restrict__ cu, int H,
                   float scale, __bf16* __restrict__ dk, long dks, __bf16* __restrict__ dv, long dvs, int B,
                   const TokenIO tok = TokenIO{nullptr, nullptr, 0}, const bool have_live = false,
                 const Segment live = Segment{0, 0, 0}) {
  constexpr int RS = DH + 8, KK = DH / 16, DB = DH / 32, THREADS = 64 * NW, NBUF = NW == 1 ? 1 : 2;
  const bool at_tokens = tok.gather_idx != nullptr;
  auto& Qs = lds.A;
  auto& Gs = lds.Bm;                  // dO rows
  auto& lse2s = lds.lse2s;
  auto& Ds = lds.Ds;
  int* s_cu = lds.s_cu;
  int& s_pick = lds.s_pick;
  static_assert(NBUF * BT >= 32 * NW, "the Q / dO buffers double as the output staging tiles");

  if (!tile_id.valid) return;
  const int h = tile_id.h;
  const Segment seg = have_live ? live
                      : LPT           ? lpt_segment<THREADS>(tile_id.rank, B, cu, nullptr, 0, s_cu, &s_pick)
                                      : segment_of(tile_id.rank, cu, nullptr, 0);
  const int k0 = tile_id.qb * (32 * NW);
  if (k0 >= seg.nk) return;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, l32 = lane & 31, hh = lane >> 5;
  const int ki = k0 + wv * 32 + l32;
  const bool wave_live = k0 + wv * 32 < seg.nk;
  const bool k_ok = ki < seg.nk;
  const long C = (long)H * DH;
  const float scale_log2 = scale * kLog2e;
  const __bf16* qh = q + h * DH;
  const __bf16* gh = dout + h * DH;
  const float* lse_h = lse + h * lse_stride + seg.row0;
  const float* dvec_h = dvec + h * lse_stride + seg.row0;

  RowStage<DH, THREADS, BT> qst, gst;
  float lreg = 0.f, dreg = 0.f;            // lse / D of query row `tid` of the tile (tid < 64)
  auto load_stats = [&](int qt) {
    if (tid < BT) {
      const bool ok = qt + tid < seg.nq;
      lreg = ok ? lse_h[qt + tid] * kLog2e : INFINITY;   // invalid rows: probability 0
      dreg = ok ? dvec_h[qt + tid] : 0.f;
    }
  };
  auto store_stats = [&](int buf) {
    if (tid < BT) {
      lse2s[buf][tid] = lreg;
      Ds[buf][tid] = dreg;
    }
  };
  qst.load(qh, seg.row0, seg.nq, qs);
  if (at_tokens) gst.load_rows(gh, tok.gather_idx + seg.row0, seg.nq, C);
  else gst.load(gh, seg.row0, seg.nq, C);
  load_stats(0);

  bf16x8 kf[KK], vf[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) {
    kf[kk] = zero_bf16x8();
    vf[kk] = zero_bf16x8();
    if (k_ok) {
      const int col = h * DH + kk * 16 + hh * 8;
      kf[kk] = *reinterpret_cast<const bf16x8*>(k + (seg.row0 + ki) * ks + col);
      vf[kk] = *reinterpret_cast<const bf16x8*>(v + (seg.row0 + ki) * vs + col);
    }
  }
  floatx16 dka[DB], dva[DB];
#pragma unroll
  for (int d = 0; d < DB; ++d)
#pragma unroll
    for (int r = 0; r < 16; ++r) { dka[d][r] = 0.f; dva[d][r] = 0.f; }

  qst.store(Qs[0]);
  gst.store(Gs[0]);
  store_stats(0);
  __syncthreads();
  const int nt = (seg.nq + BT - 1) / BT;
  for (int t = 0; t < nt; ++t) {
    const int buf = t & (NBUF - 1), nbuf = (t + 1) & (NBUF - 1), qt = t * BT;
    if (t + 1 < nt) {
      qst.load(qh, seg.row0 + qt + BT, seg.nq - qt - BT, qs);
      if (at_tokens) gst.load_rows(gh, tok.gather_idx + seg.row0 + qt + BT, seg.nq - qt - BT, C);
      else gst.load(gh, seg.row0 + qt + BT, seg.nq - qt - BT, C);
      load_stats(qt + BT);
    }
    if (wave_live) {
#pragma unroll
      for (int sb = 0; sb < BT / 32; ++sb) {
        if (qt + sb * 32 >= seg.nq) break;
        // S tile: rows = 32 queries, cols = this wave's 32 keys
        floatx16 s, dp;
#pragma unroll
        for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
          const bf16x8 qa = *reinterpret_cast<const bf16x8*>(&Qs[buf][(sb * 32 + l32) * RS + kk * 16 + hh * 8]);
          s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa, kf[kk], s, 0, 0, 0);
          const bf16x8 ga = *reinterpret_cast<const bf16x8*>(&Gs[buf][(sb * 32 + l32) * RS + kk * 16 + hh * 8]);
          dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ga, vf[kk], dp, 0, 0, 0);
        }
        float p[16], ds[16];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const floatx4 l4 = *reinterpret_cast<const floatx4*>(&lse2s[buf][sb * 32 + 8 * g + 4 * hh]);
          const floatx4 d4 = *reinterpret_cast<const floatx4*>(&Ds[buf][sb * 32 + 8 * g + 4 * hh]);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int r = 4 * g + e;
            p[r] = __builtin_amdgcn_exp2f(fmaf(s[r], scale_log2, -l4[e]));
            ds[r] = p[r] * (dp[r] - d4[e]);
          }
        }
#pragma unroll
        for (int mf = 0; mf < 2; ++mf) {
          floatx8 fp, fd;
#pragma unroll
          for (int j = 0; j < 8; ++j) { fp[j] = p[8 * mf + j]; fd[j] = ds[8 * mf + j]; }
          const bf16x8 pb = float_to_bf16x8(fp), dsb = float_to_bf16x8(fd);
#pragma unroll
          for (int d = 0; d < DB; ++d) {
            const bf16x8 ga = transposed_frag_rowmajor<RS>(Gs[buf], d, sb * 32, mf, lane);   // dO^T
            dva[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ga, pb, dva[d], 0, 0, 0);
            const bf16x8 qa = transposed_frag_rowmajor<RS>(Qs[buf], d, sb * 32, mf, lane);   // Q^T
            dka[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa, dsb, dka[d], 0, 0, 0);
          }
        }
      }
    }
    if (t + 1 < nt) {
      qst.store(Qs[nbuf]);
      gst.store(Gs[nbuf]);
      store_stats(nbuf);
    }
    __syncthreads();
  }
  __bf16* ktile = &Qs[0][0] + wv * 32 * RS;
  __bf16* vtile = &Gs[0][0] + wv * 32 * RS;
  if (wave_live) {
    park_tile<DH, RS>(dka, scale, ktile, l32, hh);
    park_tile<DH, RS>(dva, 1.0f, vtile, l32, hh);
  }
  __syncthreads();
  if (wave_live) {
    const int nrows = min(32, seg.nk - k0 - wv * 32);
    if (at_tokens) {
      const int32_t* ri = tok.gather_idx + seg.row0 + k0 + wv * 32;
      flush_tile_rows<DH, RS>(ktile, dk + h * DH, dks, nrows, lane, ri);
      flush_tile_rows<DH, RS>(vtile, dv + h * DH, dvs, nrows, lane, ri);
    } else {
      flush_tile<DH, RS>(ktile, dk + (seg.row0 + k0 + wv * 32) * dks + h * DH, dks, nrows, lane);
      flush_tile<DH, RS>(vtile, dv + (seg.row0 + k0 + wv * 32) * dvs + h * DH, dvs, nrows, lane);
    }
  }
}

template <int DH, int NW, int BT, bool LPT>
__global__ void __launch_bounds__(64 * NW)
attn_bwd_dkdv_bf16_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k,
                          const __bf16* __restrict__ v, long qs, long ks, long vs,
                          const __bf16* __restrict__ dout, const float* __restrict__ lse,
                          const float* __restrict__ dvec, long lse_stride, const int32_t* __restrict__ cu, int H,
                          float scale, __bf16* __restrict__ dk, long dks, __bf16* __restrict__ dv, long dvs,
                          int B, int nkb) {
  __shared__ BwdLds<DH, NW, BT, LPT> lds;
  attn_bwd_dkdv_body<DH, NW, BT, LPT>(lds, xcd_tile(nkb, H, B), q, k, v, qs, ks, vs, dout, lse, dvec, lse_stride, cu,
                                      H, scale, dk, dks, dv, dvs, B);
}

// Long segments, one launch for both sides.  Each of the two kernels above is bound by the
// chain of its longest workgroup (a wave walks all tokens of its image) with one to two
// workgroups per compute unit; launched together, the two chains run side by side.  Workgroup
// -> (xcd = id % 8, role = (id / 8) % 2, j = id / 16): the dq block and the dkdv block of a
// tile number sit on the same XCD (they read the same rows).  D_i = <dO_i, O_i> comes from
// the small kernel below, launched first.
template <int DH, int NW, int BT>
__global__ void __launch_bounds__(64 * NW)
attn_bwd_both_bf16_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k,
                          const __bf16* __restrict__ v, long qs, long ks, long vs,
                          const __bf16* __restrict__ out, const __bf16* __restrict__ dout,
                          const float* __restrict__ lse, float* __restrict__ dvec, long lse_stride,
                          const int32_t* __restrict__ cu, int H, float scale, __bf16* __restrict__ dq, long dqs,
                          __bf16* __restrict__ dk, long dks, __bf16* __restrict__ dv, long dvs, int B, int nblk,
                          TokenIO tok) {
  __shared__ BwdLds<DH, NW, BT, true> lds;
  __shared__ LiveTile s_live;
  const int xcd = blockIdx.x & 7, jj = blockIdx.x >> 3;
  TileId tile_id;
  Segment seg_live = {0, 0, 0};
  const bool live = live_tiles_apply(H, B);     // live blocks first in launch order (see live_tile_wave)
  if (live) {
    const LiveTile lt = live_tile_block(xcd, jj >> 1, H, B, cu, 32 * NW, nblk, &s_live);
    tile_id = {lt.qb, lt.h, lt.img, lt.valid};
    seg_live = {lt.row0, lt.len, lt.len};
  } else {
    tile_id = xcd_tile_at(xcd, jj >> 1, nblk, H, B);
  }
  if (jj & 1)
    attn_bwd_dkdv_body<DH, NW, BT, true>(lds, tile_id, q, k, v, qs, ks, vs, dout, lse, dvec, lse_stride, cu, H, scale,
                                         dk, dks, dv, dvs, B, tok, live, seg_live);
  else
    attn_bwd_dq_body<DH, NW, BT, true, true>(lds, tile_id, q, k, v, qs, ks, vs, out, dout, lse, lse_stride, cu, H,
                                             scale, dq, dqs, dvec, B, tok, live, seg_live);
  if (tok.gather_idx != nullptr) {
    // gradients of the unselected tokens: every workgroup of a role (with or without a tile) zeroes an
    // even share of the rows, a quarter per wave: the dq role in dq, the dkdv role in dk and dv
    const long units = (long)(gridDim.x >> 1) * NW, u = ((long)xcd + 8 * (jj >> 1)) * NW + (threadIdx.x >> 6);
    const long per = (tok.rows + units - 1) / units, r0 = min(tok.rows, u * per), r1 = min(tok.rows, r0 + per);
    const int lane = threadIdx.x & 63;
    if (jj & 1) {
      zero_unselected_rows(dk, dks, H * DH, tok.inv_pos, r0, r1, lane);
      zero_unselected_rows(dv, dvs, H * DH, tok.inv_pos, r0, r1, lane);
    } else {
      zero_unselected_rows(dq, dqs, H * DH, tok.inv_pos, r0, r1, lane);
    }
  }
}

// D[h][j] = <dO_j, O_j> over head h's columns, for the packed rows j < cu[B]: DH / 8 adjacent
// lanes share a (row, head).
template <int DH>
__global__ void __launch_bounds__(256)
attn_bwd_dvec_kernel(const __bf16* __restrict__ out, const __bf16* __restrict__ dout, const int32_t* __restrict__ cu,
                     int B, int H, long lse_stride, float* __restrict__ dvec, const int32_t* __restrict__ gather_idx) {
  constexpr int CPR = DH / 8;
  const long C = (long)H * DH, total = (long)cu[B] * H * CPR;
  for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < ((total + 63) & ~63L); i += (long)gridDim.x * 256) {
    const long rh = i / CPR;
    const int c = (int)(i % CPR);
    const long row = rh / H;
    const int h = (int)(rh % H);
    float d = 0.f;
    if (i < total) {
      const floatx8 of = bf16x8_to_float(*reinterpret_cast<const bf16x8*>(out + row * C + h * DH + c * 8));
      const long grow = gather_idx != nullptr ? (long)gather_idx[row] : row;
      const floatx8 gf = bf16x8_to_float(*reinterpret_cast<const bf16x8*>(dout + grow * C + h * DH + c * 8));
#pragma unroll
      for (int e = 0; e < 8; ++e) d = fmaf(of[e], gf[e], d);
    }
#pragma unroll
    for (int o = 1; o < CPR; o <<= 1) d += __shfl_xor(d, o, kWave);
    if (i < total && c == 0) dvec[h * lse_stride + row] = d;
  }
}

// ------------------------------------------------- dQ, dK, dV in one kernel (short segments)
// One workgroup per (image, head); wave j owns the segment's keys 32j .. 32j+31 (K_j, V_j as
// register operands, dK_j / dV_j in its accumulators).  Q and dO of the whole segment sit in
// LDS, so every operand is read from memory once and S, dP are computed once (5 GEMM shapes).
// In round r wave j works on query tile t = (j + r) mod nw: S = Q_t K_j^T, dP = dO_t V_j^T,
// P, dS; dV_j^T += dO_t^T P, dK_j^T += Q_t^T dS; dS goes through a wave-private LDS tile to
// come back transposed as the B operand of dQ_t^T += K_j^T dS^T, whose fp32 accumulator tile
// lives in LDS and is read-modify-written by exactly one wave per round (a barrier between
// rounds).  Tile t therefore receives its nw contributions in the fixed order j = t, t-1, ...:
// no atomics, run-to-run bit-stable.
// Dynamic LDS, rows = 32 * nw:  Q [rows][DH+8] | dO [rows][DH+8] | dQ accumulators [nw] tiles
// of DH*32 fp32 in register layout | dS tiles [nw][32][40] bf16 | lse*log2(e) [rows] | D [rows].
template <int DH>
__host__ __device__ constexpr size_t bwd_fused_lds_bytes(int nw) {
  return (size_t)nw * (2 * 32 * (DH + 8) * 2 + DH * 32 * 4 + 32 * 40 * 2 + 2 * 32 * 4);
}

template <int DH>
__global__ void __launch_bounds__(512)
attn_bwd_fused_bf16_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k,
                           const __bf16* __restrict__ v, long qs, long ks, long vs,
                           const __bf16* __restrict__ out, const __bf16* __restrict__ dout,
                           const float* __restrict__ lse, long lse_stride, const int32_t* __restrict__ cu, int H,
                           float scale, __bf16* __restrict__ dq, long dqs, __bf16* __restrict__ dk, long dks,
                           __bf16* __restrict__ dv, long dvs, int B, TokenIO tok) {
  constexpr int RS = DH + 8, KK = DH / 16, DB = DH / 32, CPR = DH / 8, SS = 40, PER = CPR / 2;
  constexpr int ACC = DH * 32;                       // floats of one dQ accumulator tile
  extern __shared__ __attribute__((aligned(16))) unsigned char bwd_smem[];
  __shared__ int s_pick;
  const int threads = blockDim.x, nw = threads >> 6, rows_cap = 32 * nw;
  __bf16* Qs = reinterpret_cast<__bf16*>(bwd_smem);
  __bf16* Gs = Qs + rows_cap * RS;
  float* dqacc = reinterpret_cast<float*>(Gs + rows_cap * RS);
  __bf16* scr = reinterpret_cast<__bf16*>(dqacc + nw * ACC);
  float* lse2s = reinterpret_cast<float*>(scr + nw * 32 * SS);
  float* Ds = lse2s + rows_cap;

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, l32 = lane & 31, hh = lane >> 5;
  const int h = blockIdx.x % H, rank = blockIdx.x / H;
  const bool at_tokens = tok.gather_idx != nullptr;
  // zero this head's columns of the unselected rows of this workgroup's share; every thread
  // runs it as its last step, so nothing it computes with waits behind these stores
  auto zero_unselected = [&]() {
    if (!at_tokens) return;
    const long per = (tok.rows + B - 1) / B, i0 = rank * per, i1 = min(tok.rows, i0 + per);
    const bf16x8 z = zero_bf16x8();
    for (long i = i0 * CPR + tid; i < i1 * CPR; i += threads) {
      const long row = i / CPR;
      const int c = (int)(i % CPR);
      if (tok.inv_pos[row] < 0) {
        *reinterpret_cast<bf16x8*>(dq + row * dqs + h * DH + c * 8) = z;
        *reinterpret_cast<bf16x8*>(dk + row * dks + h * DH + c * 8) = z;
        *reinterpret_cast<bf16x8*>(dv + row * dvs + h * DH + c * 8) = z;
      }
    }
  };
  // heaviest image first (work per segment grows like n^2)
  int img = rank, start = 0, len = 0;
  if (B > 1 && B <= kWave) {                         // every wave ranks on its own: no LDS, no barrier
    const RankedSegment rs = ranked_segment_wave(rank, B, cu, nw);
    img = rs.img;
    start = rs.row0;
    len = rs.len;
  } else {
    if (B > 1 && B <= 512 && B * (int)sizeof(int) <= nw * 32 * SS * 2) {     // the ranking borrows the dS tiles
      int* s_len = reinterpret_cast<int*>(scr);
      for (int b = tid; b < B; b += threads) s_len[b] = cu[b + 1] - cu[b];
      __syncthreads();
      for (int b = tid; b < B; b += threads) {
        const int nb = s_len[b];
        int r = 0;
#pragma unroll 8
        for (int j = 0; j < B; ++j) {
          const int nj = s_len[j];
          r += (nj > nb) | ((nj == nb) & (j < b));
        }
        if (r == rank) s_pick = b;
      }
      __syncthreads();
      img = s_pick;
    }
    start = cu[img];
    len = cu[img + 1] - start;
  }
  const long row0 = start;
  const int n = min(len, rows_cap);
  if (n <= 0) {
    zero_unselected();
    return;
  }
  const int nws = (n + 31) >> 5;                     // waves with keys = query tiles = rounds
  const long C = (long)H * DH;
  const float scale_log2 = scale * kLog2e;

  // ---- stage Q, dO (every thread PER chunks of each), D_i = <dO_i, O_i>, lse_i; wave j: K_j, V_j
  bf16x8 qreg[PER], greg[PER], oreg[PER], kreg[PER], vf[KK];
  float lreg[PER];
#pragma unroll
  for (int t = 0; t < PER; ++t) {
    const int i = tid + t * threads, r = i / CPR, c = i % CPR;
    qreg[t] = zero_bf16x8(); greg[t] = zero_bf16x8(); oreg[t] = zero_bf16x8();
    lreg[t] = INFINITY;                              // rows past the segment: probability 0
    if (r < n) {
      const long grow = at_tokens ? (long)tok.gather_idx[row0 + r] : row0 + r;
      qreg[t] = *reinterpret_cast<const bf16x8*>(q + (row0 + r) * qs + h * DH + c * 8);
      greg[t] = *reinterpret_cast<const bf16x8*>(dout + grow * C + h * DH + c * 8);
      oreg[t] = *reinterpret_cast<const bf16x8*>(out + (row0 + r) * C + h * DH + c * 8);
      if (c == 0) lreg[t] = lse[h * lse_stride + row0 + r] * kLog2e;
    }
  }
  const int ki = wv * 32 + l32;
  const bool k_ok = ki < n;
#pragma unroll
  for (int t = 0; t < PER; ++t) {
    const int i = lane + t * 64, r = i / CPR, c = i % CPR;
    kreg[t] = zero_bf16x8();
    if (wv * 32 + r < n) kreg[t] = *reinterpret_cast<const bf16x8*>(k + (row0 + wv * 32 + r) * ks + h * DH + c * 8);
  }
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) {
    vf[kk] = zero_bf16x8();
    if (k_ok) vf[kk] = *reinterpret_cast<const bf16x8*>(v + (row0 + ki) * vs + h * DH + kk * 16 + hh * 8);
  }
#pragma unroll
  for (int t = 0; t < PER; ++t) {
    const int i = tid + t * threads, r = i / CPR, c = i % CPR;
    *reinterpret_cast<bf16x8*>(&Qs[r * RS + c * 8]) = qreg[t];
    *reinterpret_cast<bf16x8*>(&Gs[r * RS + c * 8]) = greg[t];
    const floatx8 gf = bf16x8_to_float(greg[t]), of = bf16x8_to_float(oreg[t]);
    float d = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) d = fmaf(of[e], gf[e], d);
#pragma unroll
    for (int o = 1; o < CPR; o <<= 1) d += __shfl_xor(d, o, kWave);     // the CPR chunks of a row: adjacent lanes
    if (c == 0) {
      Ds[r] = d;
      lse2s[r] = lreg[t];
    }
  }
  // K_j: through this wave's (still unused) dQ accumulator tile to get both operand forms
  bf16x8 kf[KK], ktf[DB][2];
  {
    __bf16* kt = reinterpret_cast<__bf16*>(dqacc + wv * ACC);
#pragma unroll
    for (int t = 0; t < PER; ++t) {
      const int i = lane + t * 64, r = i / CPR, c = i % CPR;
      *reinterpret_cast<bf16x8*>(&kt[r * RS + c * 8]) = kreg[t];
    }
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) kf[kk] = *reinterpret_cast<const bf16x8*>(&kt[l32 * RS + kk * 16 + hh * 8]);
#pragma unroll
    for (int d = 0; d < DB; ++d)
#pragma unroll
      for (int mf = 0; mf < 2; ++mf) ktf[d][mf] = transposed_frag_rowmajor<RS>(kt, d, 0, mf, lane);   // K_j^T
  }
  floatx16 dka[DB], dva[DB];
#pragma unroll
  for (int d = 0; d < DB; ++d)
#pragma unroll
    for (int r = 0; r < 16; ++r) { dka[d][r] = 0.f; dva[d][r] = 0.f; }
  __syncthreads();

  const bool live = wv < nws;
  const bool ragged = live && wv == nws - 1 && (n & 31) != 0;      // this wave's key block has empty lanes
  __bf16* sc = scr + wv * 32 * SS;
  for (int r = 0; r < nws; ++r) {
    if (live) {
      int t = wv + r;
      if (t >= nws) t -= nws;
      const __bf16* Qt = Qs + t * 32 * RS;
      const __bf16* Gt = Gs + t * 32 * RS;
      floatx16 s, dp;
#pragma unroll
      for (int e = 0; e < 16; ++e) { s[e] = 0.f; dp[e] = 0.f; }
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        const bf16x8 qa = *reinterpret_cast<const bf16x8*>(&Qt[l32 * RS + kk * 16 + hh * 8]);
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa, kf[kk], s, 0, 0, 0);
        const bf16x8 ga = *reinterpret_cast<const bf16x8*>(&Gt[l32 * RS + kk * 16 + hh * 8]);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ga, vf[kk], dp, 0, 0, 0);
      }
      float p[16], ds[16];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const floatx4 l4 = *reinterpret_cast<const floatx4*>(&lse2s[t * 32 + 8 * g + 4 * hh]);
        const floatx4 d4 = *reinterpret_cast<const floatx4*>(&Ds[t * 32 + 8 * g + 4 * hh]);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int i = 4 * g + e;
          p[i] = __builtin_amdgcn_exp2f(fmaf(s[i], scale_log2, -l4[e]));
          ds[i] = p[i] * (dp[i] - d4[e]);
        }
      }
      if (ragged) {                                  // keys past the segment must not reach dQ
#pragma unroll
        for (int i = 0; i < 16; ++i) ds[i] = k_ok ? ds[i] : 0.f;
      }
#pragma unroll
      for (int mf = 0; mf < 2; ++mf) {
        floatx8 fp, fd;
#pragma unroll
        for (int j = 0; j < 8; ++j) { fp[j] = p[8 * mf + j]; fd[j] = ds[8 * mf + j]; }
        const bf16x8 pb = float_to_bf16x8(fp), dsb = float_to_bf16x8(fd);
#pragma unroll
        for (int d = 0; d < DB; ++d) {
          const bf16x8 ga = transposed_frag_rowmajor<RS>(Gt, d, 0, mf, lane);   // dO_t^T
          dva[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ga, pb, dva[d], 0, 0, 0);
          const bf16x8 qa = transposed_frag_rowmajor<RS>(Qt, d, 0, mf, lane);   // Q_t^T
          dka[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa, dsb, dka[d], 0, 0, 0);
        }
        // dS tile, [key][query]: registers 8mf .. 8mf+7 are queries 16mf + 4hh + {0..3, 8..11}
        *reinterpret_cast<bf16x4*>(&sc[l32 * SS + 16 * mf + 4 * hh]) = __builtin_shufflevector(dsb, dsb, 0, 1, 2, 3);
        *reinterpret_cast<bf16x4*>(&sc[l32 * SS + 16 * mf + 8 + 4 * hh]) = __builtin_shufflevector(dsb, dsb, 4, 5, 6, 7);
      }
      // dQ_t^T += K_j^T dS^T on the tile's fp32 accumulators in LDS
      floatx4* at = reinterpret_cast<floatx4*>(dqacc + t * ACC);
      floatx16 acc[DB];
#pragma unroll
      for (int d = 0; d < DB; ++d)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          floatx4 a4 = {0.f, 0.f, 0.f, 0.f};
          if (r > 0) a4 = at[(d * 4 + g) * 64 + lane];
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[d][4 * g + e] = a4[e];
        }
#pragma unroll
      for (int mf = 0; mf < 2; ++mf) {
        const bf16x8 dst = transposed_frag_rowmajor<SS>(sc, 0, 0, mf, lane);     // dS^T: lane = query
#pragma unroll
        for (int d = 0; d < DB; ++d) acc[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ktf[d][mf], dst, acc[d], 0, 0, 0);
      }
#pragma unroll
      for (int d = 0; d < DB; ++d)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const floatx4 a4 = {acc[d][4 * g], acc[d][4 * g + 1], acc[d][4 * g + 2], acc[d][4 * g + 3]};
          at[(d * 4 + g) * 64 + lane] = a4;
        }
    }
    __syncthreads();
  }
  if (!live) {
    zero_unselected();
    return;
  }
  // gradients: dK_j, dV_j from the registers, dQ tile j from LDS; parked as bf16 rows, written whole
  __bf16* ktile = Qs + wv * 32 * RS;
  __bf16* vtile = Gs + wv * 32 * RS;
  park_tile<DH, RS>(dka, scale, ktile, l32, hh);
  park_tile<DH, RS>(dva, 1.0f, vtile, l32, hh);
  floatx16 acc[DB];
  const floatx4* at = reinterpret_cast<const floatx4*>(dqacc + wv * ACC);
#pragma unroll
  for (int d = 0; d < DB; ++d)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const floatx4 a4 = at[(d * 4 + g) * 64 + lane];
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[d][4 * g + e] = a4[e];
    }
  __bf16* qtile = reinterpret_cast<__bf16*>(dqacc + wv * ACC);
  // (LDS operations of one wave complete in order: the reads above precede the stores below)
  park_tile<DH, RS>(acc, scale, qtile, l32, hh);
  const int nrows = min(32, n - wv * 32);
  if (at_tokens) {
    const int32_t* ri = tok.gather_idx + row0 + wv * 32;
    flush_tile_rows<DH, RS>(qtile, dq + h * DH, dqs, nrows, lane, ri);
    flush_tile_rows<DH, RS>(ktile, dk + h * DH, dks, nrows, lane, ri);
    flush_tile_rows<DH, RS>(vtile, dv + h * DH, dvs, nrows, lane, ri);
  } else {
    flush_tile<DH, RS>(qtile, dq + (row0 + wv * 32) * dqs + h * DH, dqs, nrows, lane);
    flush_tile<DH, RS>(ktile, dk + (row0 + wv * 32) * dks + h * DH, dks, nrows, lane);
    flush_tile<DH, RS>(vtile, dv + (row0 + wv * 32) * dvs + h * DH, dvs, nrows, lane);
  }
  zero_unselected();
}

// ------------------------------------------------------------------------------- fp32
// One thread per row (a query for dQ, a key for dK/dV); the other side streams through LDS.
// kKeySide = false: rows are queries, outputs dq (and D_i).  true: rows are keys, outputs dk, dv.
template <int DH, bool kKeySide>
__global__ void __launch_bounds__(128)
attn_bwd_f32_kernel(const float* __restrict__ q, const float* __restrict__ k, const float* __restrict__ v,
                    long qs, long ks, long vs, const float* __restrict__ out, const float* __restrict__ dout,
                    const float* __restrict__ lse, float* __restrict__ dvec, long lse_stride,
                    const int32_t* __restrict__ cu, int H, float scale, float* __restrict__ g0, long g0s,
                    float* __restrict__ g1, long g1s, TokenIO tok) {
  constexpr int BM = 128, BN = 32;
  __shared__ __attribute__((aligned(16))) float As[BN * DH];   // K (query side) or Q (key side)
  __shared__ __attribute__((aligned(16))) float Bs[BN * DH];   // V (query side) or dO (key side)
  __shared__ float lses[BN], Dss[BN];

  const int h = blockIdx.y;
  const Seg seg = seg_of(blockIdx.z, cu);
  const int r0 = blockIdx.x * BM;
  const int tid = threadIdx.x;
  const bool at_tokens = tok.gather_idx != nullptr;
  if (at_tokens) {   // gradients of the unselected tokens: this head's columns of an even share of the rows
    const long units = (long)gridDim.x * gridDim.z, u = (long)blockIdx.z * gridDim.x + blockIdx.x;
    const long per = (tok.rows + units - 1) / units, i0 = min(tok.rows, u * per), i1 = min(tok.rows, i0 + per);
    const floatx4 z = {0.f, 0.f, 0.f, 0.f};
    for (long i = i0 * (DH / 4) + tid; i < i1 * (DH / 4); i += BM) {
      const long row = i / (DH / 4);
      const int c = (int)(i % (DH / 4));
      if (tok.inv_pos[row] < 0) {
        *reinterpret_cast<floatx4*>(g0 + row * g0s + h * DH + c * 4) = z;
        if (kKeySide) *reinterpret_cast<floatx4*>(g1 + row * g1s + h * DH + c * 4) = z;
      }
    }
  }
  if (r0 >= seg.n) return;
  const int ri = r0 + tid;
  const bool ok = ri < seg.n;
  const long C = (long)H * DH;
  const long grow = seg.row0 + ri;
  const long trow = ok && at_tokens ? (long)tok.gather_idx[grow] : grow;   // where this row's gradients live

  float a[DH], b[DH], acc0[DH], acc1[DH];
#pragma unroll
  for (int d = 0; d < DH; ++d) { a[d] = 0.f; b[d] = 0.f; acc0[d] = 0.f; acc1[d] = 0.f; }
  float my_lse = 0.f, my_D = 0.f;
  if (ok) {
    if (!kKeySide) {
      float dsum = 0.f;
#pragma unroll
      for (int d = 0; d < DH; ++d) {
        a[d] = q[grow * qs + h * DH + d];
        b[d] = dout[trow * C + h * DH + d];
        dsum = fmaf(b[d], out[grow * C + h * DH + d], dsum);
      }
      my_D = dsum;
      my_lse = lse[h * lse_stride + grow];
      dvec[h * lse_stride + grow] = dsum;
    } else {
#pragma unroll
      for (int d = 0; d < DH; ++d) {
        a[d] = k[grow * ks + h * DH + d];
        b[d] = v[grow * vs + h * DH + d];
      }
    }
  }
  const float* sa = kKeySide ? q : k;
  const float* sb = kKeySide ? dout : v;
  const long sa_stride = kKeySide ? qs : ks;
  const long sb_stride = kKeySide ? C : vs;

  for (int t = 0; t < seg.n; t += BN) {
    __syncthreads();
    for (int i = tid; i < BN * DH / 4; i += BM) {
      const int r = i / (DH / 4), c = i % (DH / 4);
      floatx4 x = {0.f, 0.f, 0.f, 0.f}, y = x;
      if (t + r < seg.n) {
        const long prow = seg.row0 + t + r;
        const long brow = kKeySide && at_tokens ? (long)tok.gather_idx[prow] : prow;   // dO rows sit at the tokens
        x = *reinterpret_cast<const floatx4*>(sa + prow * sa_stride + h * DH + c * 4);
        y = *reinterpret_cast<const floatx4*>(sb + brow * sb_stride + h * DH + c * 4);
      }
      *reinterpret_cast<floatx4*>(&As[r * DH + c * 4]) = x;
      *reinterpret_cast<floatx4*>(&Bs[r * DH + c * 4]) = y;
    }
    if (kKeySide && tid < BN) {
      const bool in = t + tid < seg.n;
      lses[tid] = in ? lse[h * lse_stride + seg.row0 + t + tid] : INFINITY;
      Dss[tid] = in ? dvec[h * lse_stride + seg.row0 + t + tid] : 0.f;
    }
    __syncthreads();
    const int tn = min(BN, seg.n - t);
    for (int j = 0; j < tn; ++j) {
      float s = 0.f, dp = 0.f;
#pragma unroll
      for (int d = 0; d < DH; ++d) {
        s = fmaf(a[d], As[j * DH + d], s);     // q.k
        dp = fmaf(b[d], Bs[j * DH + d], dp);   // dO.v
      }
      const float l = kKeySide ? lses[j] : my_lse;
      const float D = kKeySide ? Dss[j] : my_D;
      const float p = expf(s * scale - l);
      const float ds = p * (dp - D) * scale;
#pragma unroll
      for (int d = 0; d < DH; ++d) {
        acc0[d] = fmaf(ds, As[j * DH + d], acc0[d]);              // dq += ds k   | dk += ds q
        if (kKeySide) acc1[d] = fmaf(p, Bs[j * DH + d], acc1[d]);  //              | dv += p dO
      }
    }
  }
  if (!ok) return;
#pragma unroll
  for (int d = 0; d < DH; ++d) {
    g0[trow * g0s + h * DH + d] = acc0[d];
    if (kKeySide) g1[trow * g1s + h * DH + d] = acc1[d];
  }
}

}  // namespace spa

using namespace spa;

extern "C" size_t spa_attention_bwd_workspace_bytes(int B, int max_seqlen, int H, int Dh, int dtype) {
  (void)Dh; (void)dtype;
  if (B < 1 || max_seqlen < 1 || H < 1) return 0;
  return (size_t)H * (size_t)B * (size_t)max_seqlen * sizeof(float);   // D_i for every (head, row)
}

// tok.gather_idx != nullptr: gradients in and out at token positions (one-kernel form only).
static int attention_bwd_common(const char* fn, const void* q, const void* k, const void* v, int64_t q_row_stride,
                                int64_t k_row_stride, int64_t v_row_stride, const void* out, const void* dout,
                                const float* lse, const int32_t* cu_seqlens, int B, int max_seqlen, int H, int Dh,
                                int dtype, float softmax_scale, void* dq, void* dk, void* dv,
                                int64_t dq_row_stride, int64_t dk_row_stride, int64_t dv_row_stride,
                                void* workspace, size_t workspace_bytes, TokenIO tok, void* stream) {
  const bool at_tokens = tok.gather_idx != nullptr;
  SPA_REQUIRE(q && k && v && out && dout && lse && cu_seqlens && dq && dk && dv, SPA_ERR_INVALID_ARG,
              "%s: null pointer", fn);
  SPA_REQUIRE(B >= 1 && max_seqlen >= 1 && H >= 1, SPA_ERR_INVALID_ARG, "%s: B, max_seqlen, H must be >= 1", fn);
  SPA_REQUIRE((long)B * max_seqlen < 2147483647L, SPA_ERR_INVALID_ARG, "%s: B*max_seqlen must be < 2^31", fn);
  SPA_REQUIRE(B <= 65535 && H <= 65535, SPA_ERR_INVALID_ARG, "%s: B and H must be <= 65535", fn);
  SPA_REQUIRE(dtype == SPA_F32 || dtype == SPA_BF16, SPA_ERR_UNSUPPORTED, "%s: unknown dtype %d", fn, dtype);
  SPA_REQUIRE(Dh == 32 || Dh == 64, SPA_ERR_UNSUPPORTED, "%s: head dim %d not supported (32 or 64)", fn, Dh);
  const int64_t strides[6] = {q_row_stride, k_row_stride, v_row_stride, dq_row_stride, dk_row_stride, dv_row_stride};
  for (int64_t rs : strides) {
    SPA_REQUIRE(rs >= (int64_t)H * Dh, SPA_ERR_INVALID_ARG, "%s: row stride %ld < H*Dh", fn, (long)rs);
    SPA_REQUIRE((rs * elem_size(dtype)) % 16 == 0, SPA_ERR_INVALID_ARG, "%s: row strides must be multiples of 16 bytes", fn);
  }
  SPA_REQUIRE(aligned16(q) && aligned16(k) && aligned16(v) && aligned16(out) && aligned16(dout) &&
                  aligned16(dq) && aligned16(dk) && aligned16(dv),
              SPA_ERR_INVALID_ARG, "%s: tensors not 16-byte aligned", fn);
  SPA_REQUIRE(softmax_scale >= 0.f && std::isfinite(softmax_scale), SPA_ERR_INVALID_ARG,
              "%s: softmax_scale must be finite and >= 0", fn);
  // short segments: the one-kernel form.  Option attn_bwd_short = "split" keeps the two one-wave
  // kernels, "tiled" forces the long-segment kernels.
  const Options& opt = options();
  const bool short_seg = max_seqlen <= 256 && opt.bwd_short != 2;
  const bool one_kernel = dtype == SPA_BF16 && short_seg && (at_tokens || opt.bwd_short != 1);
  const size_t need = one_kernel ? 0 : spa_attention_bwd_workspace_bytes(B, max_seqlen, H, Dh, dtype);
  SPA_REQUIRE(need == 0 || (workspace != nullptr && workspace_bytes >= need), SPA_ERR_WORKSPACE,
              "%s: workspace of %zu bytes needed, %zu given", fn, need, workspace_bytes);
  const float scale = softmax_scale > 0.f ? softmax_scale : 1.0f / std::sqrt((float)Dh);
  const long ls = (long)B * max_seqlen;
  float* dvec = static_cast<float*>(workspace);
  hipStream_t st = as_stream(stream);
  if (dtype == SPA_F32) {
    const dim3 grid((max_seqlen + 127) / 128, H, B), block(128);
#define SPA_BWD_F32(D)                                                                                        \
  hipLaunchKernelGGL((attn_bwd_f32_kernel<D, false>), grid, block, 0, st, (const float*)q, (const float*)k,   \
                     (const float*)v, (long)q_row_stride, (long)k_row_stride, (long)v_row_stride,             \
                     (const float*)out, (const float*)dout, lse, dvec, ls, cu_seqlens, H, scale, (float*)dq,  \
                     (long)dq_row_stride, (float*)nullptr, 0L, tok);                                          \
  hipLaunchKernelGGL((attn_bwd_f32_kernel<D, true>), grid, block, 0, st, (const float*)q, (const float*)k,    \
                     (const float*)v, (long)q_row_stride, (long)k_row_stride, (long)v_row_stride,             \
                     (const float*)out, (const float*)dout, lse, dvec, ls, cu_seqlens, H, scale, (float*)dk,  \
                     (long)dk_row_stride, (float*)dv, (long)dv_row_stride, tok)
    if (Dh == 32) { SPA_BWD_F32(32); } else { SPA_BWD_F32(64); }
#undef SPA_BWD_F32
  } else {
#define SPA_BWD_ARGS_DQ                                                                                       \
  (const __bf16*)q, (const __bf16*)k, (const __bf16*)v, (long)q_row_stride, (long)k_row_stride,               \
      (long)v_row_stride, (const __bf16*)out, (const __bf16*)dout, lse, ls, cu_seqlens, H, scale, (__bf16*)dq, \
      (long)dq_row_stride, dvec, B, nblk
#define SPA_BWD_ARGS_DKDV                                                                                     \
  (const __bf16*)q, (const __bf16*)k, (const __bf16*)v, (long)q_row_stride, (long)k_row_stride,               \
      (long)v_row_stride, (const __bf16*)dout, lse, dvec, ls, cu_seqlens, H, scale, (__bf16*)dk,              \
      (long)dk_row_stride, (__bf16*)dv, (long)dv_row_stride, B, nblk
    if (one_kernel) {
      const int nw = (max_seqlen + 31) / 32;
      SPA_REQUIRE((long)B * H < 2147483647L, SPA_ERR_INVALID_ARG, "%s: B*H must be < 2^31", fn);
#define SPA_BWD_FUSED(D)                                                                                        \
  do {                                                                                                          \
    const size_t smem = bwd_fused_lds_bytes<D>(nw);                                                             \
    const hipError_t attr = hipFuncSetAttribute((const void*)attn_bwd_fused_bf16_kernel<D>,                     \
                                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);         \
    SPA_REQUIRE(attr == hipSuccess, SPA_ERR_HIP, "%s: cannot reserve %zu bytes of LDS", fn, smem);              \
    hipLaunchKernelGGL((attn_bwd_fused_bf16_kernel<D>), dim3((unsigned)(B * H)), dim3(64 * nw), smem, st,       \
                       (const __bf16*)q, (const __bf16*)k, (const __bf16*)v, (long)q_row_stride,                \
                       (long)k_row_stride, (long)v_row_stride, (const __bf16*)out, (const __bf16*)dout, lse, ls, \
                       cu_seqlens, H, scale, (__bf16*)dq, (long)dq_row_stride, (__bf16*)dk, (long)dk_row_stride, \
                       (__bf16*)dv, (long)dv_row_stride, B, tok);                                               \
  } while (0)
      if (Dh == 32) SPA_BWD_FUSED(32); else SPA_BWD_FUSED(64);
#undef SPA_BWD_FUSED
      return check_launch(fn);
    }
    const int rows_per_block = short_seg ? 32 : 128;
    const int nblk = (max_seqlen + rows_per_block - 1) / rows_per_block;
    SPA_REQUIRE(((long)H * B + 8) * nblk < 2147483647L, SPA_ERR_INVALID_ARG, "%s: B*H*blocks must be < 2^31", fn);
    const dim3 grid(xcd_grid(nblk, H, B));
#define SPA_BWD_BF16(D)                                                                                          \
  do {                                                                                                           \
    if (short_seg) {                                                                                             \
      hipLaunchKernelGGL((attn_bwd_dq_bf16_kernel<D, 1, 32, false>), grid, dim3(64), 0, st, SPA_BWD_ARGS_DQ);     \
      hipLaunchKernelGGL((attn_bwd_dkdv_bf16_kernel<D, 1, 32, false>), grid, dim3(64), 0, st, SPA_BWD_ARGS_DKDV); \
    } else {                                                                                                     \
      hipLaunchKernelGGL((attn_bwd_dq_bf16_kernel<D, 4, 64, true>), grid, dim3(256), 0, st, SPA_BWD_ARGS_DQ);     \
      hipLaunchKernelGGL((attn_bwd_dkdv_bf16_kernel<D, 4, 64, true>), grid, dim3(256), 0, st, SPA_BWD_ARGS_DKDV); \
    }                                                                                                            \
  } while (0)
    // long segments: D first, then both sides in one launch (option attn_bwd_long = "two" keeps two launches)
    if (!short_seg && (at_tokens || !opt.bwd_long_two)) {
      SPA_REQUIRE(2L * grid.x < 2147483647L, SPA_ERR_INVALID_ARG, "%s: B*H*blocks must be < 2^30", fn);
      const long rows_cap = (long)B * max_seqlen;
      const unsigned dgrid = (unsigned)std::min<long>((rows_cap * H * (Dh / 8) + 255) / 256, 4096L);
#define SPA_BWD_BOTH(D)                                                                                          \
  do {                                                                                                           \
    hipLaunchKernelGGL((attn_bwd_dvec_kernel<D>), dim3(dgrid), dim3(256), 0, st, (const __bf16*)out,             \
                       (const __bf16*)dout, cu_seqlens, B, H, ls, dvec, tok.gather_idx);                         \
    hipLaunchKernelGGL((attn_bwd_both_bf16_kernel<D, 4, 64>), dim3(2 * grid.x), dim3(256), 0, st,                \
                       (const __bf16*)q, (const __bf16*)k, (const __bf16*)v, (long)q_row_stride,                 \
                       (long)k_row_stride, (long)v_row_stride, (const __bf16*)out, (const __bf16*)dout, lse,     \
                       dvec, ls, cu_seqlens, H, scale, (__bf16*)dq, (long)dq_row_stride, (__bf16*)dk,            \
                       (long)dk_row_stride, (__bf16*)dv, (long)dv_row_stride, B, nblk, tok);                     \
  } while (0)
      if (Dh == 32) SPA_BWD_BOTH(32); else SPA_BWD_BOTH(64);
#undef SPA_BWD_BOTH
    } else {
      if (Dh == 32) SPA_BWD_BF16(32); else SPA_BWD_BF16(64);
    }
#undef SPA_BWD_BF16
#undef SPA_BWD_ARGS_DQ
#undef SPA_BWD_ARGS_DKDV
  }
  return check_launch(fn);
}

extern "C" int spa_packed_attention_bwd(const void* q, const void* k, const void* v, int64_t q_row_stride,
                                        int64_t k_row_stride, int64_t v_row_stride, const void* out,
                                        const void* dout, const float* lse, const int32_t* cu_seqlens, int B,
                                        int max_seqlen, int H, int Dh, int dtype, float softmax_scale,
                                        void* dq, void* dk, void* dv, int64_t dq_row_stride,
                                        int64_t dk_row_stride, int64_t dv_row_stride, void* workspace,
                                        size_t workspace_bytes, void* stream) {
  return attention_bwd_common("spa_packed_attention_bwd", q, k, v, q_row_stride, k_row_stride, v_row_stride, out,
                              dout, lse, cu_seqlens, B, max_seqlen, H, Dh, dtype, softmax_scale, dq, dk, dv,
                              dq_row_stride, dk_row_stride, dv_row_stride, workspace, workspace_bytes,
                              TokenIO{nullptr, nullptr, 0}, stream);
}

extern "C" int spa_packed_attention_bwd_tokens(const void* q, const void* k, const void* v, int64_t q_row_stride,
                                               int64_t k_row_stride, int64_t v_row_stride, const void* out,
                                               const void* dy, const float* lse, const int32_t* cu_seqlens, int B,
                                               int max_seqlen, int H, int Dh, int dtype, float softmax_scale,
                                               const int32_t* gather_idx, const int32_t* inv_pos, int64_t rows,
                                               void* dq, void* dk, void* dv, int64_t dq_row_stride,
                                               int64_t dk_row_stride, int64_t dv_row_stride, void* workspace,
                                               size_t workspace_bytes, void* stream) {
  const char* fn = "spa_packed_attention_bwd_tokens";
  SPA_REQUIRE(gather_idx && inv_pos, SPA_ERR_INVALID_ARG, "%s: null pointer", fn);
  SPA_REQUIRE(rows >= 1 && rows < 2147483647L, SPA_ERR_INVALID_ARG, "%s: rows must be in [1, 2^31)", fn);
  return attention_bwd_common(fn, q, k, v, q_row_stride, k_row_stride, v_row_stride, out, dy, lse, cu_seqlens, B,
                              max_seqlen, H, Dh, dtype, softmax_scale, dq, dk, dv, dq_row_stride, dk_row_stride,
                              dv_row_stride, workspace, workspace_bytes, TokenIO{gather_idx, inv_pos, (long)rows},
                              stream);
}
