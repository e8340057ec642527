// Backward of the packed, per-image attention: for every (image, head) segment
//   P = exp(S - lse), dV = P^T dO, dP = dO V^T, D_i = sum_d dO_id O_id,
//   dS = P * (dP - D), dQ = dS K * scale, dK = dS^T Q * scale.
// Two kernels, no atomics, run-to-run bit-stable:
//   dq kernel   : a wave owns 32 queries and walks the segment's keys.  Like the forward it
//                 works on transposed tiles (S^T = K Q^T, dP^T = V dO^T) so lse_i and D_i are
//                 one scalar per lane and dS^T is already the B operand of
//                 dQ^T += K^T dS^T.  It also writes D_i for the second kernel.
//   dkdv kernel : a wave owns 32 keys and walks the segment's queries with S = Q K^T and
//                 dP = dO V^T un-transposed (lane = key), so P and dS are the B operands of
//                 dV^T += dO^T P and dK^T += Q^T dS.
// S and dP are recomputed in both (7 GEMM shapes instead of 5) in exchange for determinism.
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


// Both bf16 kernels use the forward's launch scheme: 1-D XCD-aware grid (the blocks that
// share one (image, head)'s rows sit on one L2), longest image first, 4 waves x 32 rows per
// workgroup, the other side of the product streaming through double-buffered row-major LDS
// tiles of BT tokens with the next tile's rows in flight in registers.  Short segments
// (<= 256 tokens) use the same kernels with ONE wave per workgroup and 32-token tiles: small
// independent work units that spread over all SIMDs, no longest-first ranking.  Operands whose
// k-dimension is the token index are read with the transposing LDS read from the same
// row-major tiles, so nothing is staged twice.

// --------------------------------------------------------------------------- dQ (bf16)
template <int DH, int NW, int BT, bool LPT>
__global__ void __launch_bounds__(64 * NW)
attn_bwd_dq_bf16_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k,
                        const __bf16* __restrict__ v, long qs, long ks, long vs,
                        const __bf16* __restrict__ out, const __bf16* __restrict__ dout,
                        const float* __restrict__ lse, long lse_stride, const int32_t* __restrict__ cu, int H,
                        float scale, __bf16* __restrict__ dq, long gstride, float* __restrict__ dvec, int B,
                        int nqb) {
  constexpr int RS = DH + 8, KK = DH / 16, DB = DH / 32, THREADS = 64 * NW;
  __shared__ __attribute__((aligned(16))) __bf16 Ks[2][BT * RS];
  __shared__ __attribute__((aligned(16))) __bf16 Vs[2][BT * RS];
  __shared__ int s_cu[LPT ? 2 * kLptMaxB + 1 : 1];
  __shared__ int s_pick;
  static_assert(2 * BT >= 32 * NW, "the K buffers double as the output staging tile");

  const TileId tile_id = xcd_tile(nqb, H, B);
  if (!tile_id.valid) return;
  const int h = tile_id.h;
  const Segment seg = LPT ? lpt_segment<THREADS>(tile_id.rank, B, cu, nullptr, 0, s_cu, &s_pick)
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
      qf[kk] = *reinterpret_cast<const bf16x8*>(q + (seg.row0 + qi) * qs + col);
      dof[kk] = *reinterpret_cast<const bf16x8*>(dout + (seg.row0 + qi) * C + col);
      const floatx8 of = bf16x8_to_float(*reinterpret_cast<const bf16x8*>(out + (seg.row0 + qi) * C + col));
      const floatx8 gf = bf16x8_to_float(dof[kk]);
#pragma unroll
      for (int e = 0; e < 8; ++e) dpart = fmaf(of[e], gf[e], dpart);
    }
  }
  const float D = sum_across_halves(dpart);
  // invalid queries: lse = +inf makes every probability 0
  const float lse2 = q_ok ? lse[h * lse_stride + seg.row0 + qi] * kLog2e : INFINITY;
  if (q_ok && hh == 0) dvec[h * lse_stride + seg.row0 + qi] = D;

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
    const int buf = t & 1, kt = t * BT;
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
      kst.store(Ks[buf ^ 1]);
      vst.store(Vs[buf ^ 1]);
    }
    __syncthreads();
  }
  __bf16* tile = &Ks[0][0] + wv * 32 * RS;
  if (wave_live) park_tile<DH, RS>(acc, scale, tile, l32, hh);
  __syncthreads();
  if (wave_live)
    flush_tile<DH, RS>(tile, dq + (seg.row0 + q0 + wv * 32) * gstride + h * DH, gstride,
                       min(32, seg.nq - q0 - wv * 32), lane);
}

// ------------------------------------------------------------------------ dK, dV (bf16)
template <int DH, int NW, int BT, bool LPT>
__global__ void __launch_bounds__(64 * NW)
attn_bwd_dkdv_bf16_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k,
                          const __bf16* __restrict__ v, long qs, long ks, long vs,
                          const __bf16* __restrict__ dout, const float* __restrict__ lse,
                          const float* __restrict__ dvec, long lse_stride, const int32_t* __restrict__ cu, int H,
                          float scale, __bf16* __restrict__ dk, long dks, __bf16* __restrict__ dv, long dvs,
                          int B, int nkb) {
  constexpr int RS = DH + 8, KK = DH / 16, DB = DH / 32, THREADS = 64 * NW;
  __shared__ __attribute__((aligned(16))) __bf16 Qs[2][BT * RS];
  __shared__ __attribute__((aligned(16))) __bf16 Gs[2][BT * RS];     // dO rows
  __shared__ __attribute__((aligned(16))) float lse2s[2][BT];
  __shared__ __attribute__((aligned(16))) float Ds[2][BT];
  __shared__ int s_cu[LPT ? 2 * kLptMaxB + 1 : 1];
  __shared__ int s_pick;
  static_assert(2 * BT >= 32 * NW, "the Q / dO buffers double as the output staging tiles");

  const TileId tile_id = xcd_tile(nkb, H, B);
  if (!tile_id.valid) return;
  const int h = tile_id.h;
  const Segment seg = LPT ? lpt_segment<THREADS>(tile_id.rank, B, cu, nullptr, 0, s_cu, &s_pick)
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
  gst.load(gh, seg.row0, seg.nq, C);
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
    const int buf = t & 1, qt = t * BT;
    if (t + 1 < nt) {
      qst.load(qh, seg.row0 + qt + BT, seg.nq - qt - BT, qs);
      gst.load(gh, seg.row0 + qt + BT, seg.nq - qt - BT, C);
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
      qst.store(Qs[buf ^ 1]);
      gst.store(Gs[buf ^ 1]);
      store_stats(buf ^ 1);
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
    flush_tile<DH, RS>(ktile, dk + (seg.row0 + k0 + wv * 32) * dks + h * DH, dks, nrows, lane);
    flush_tile<DH, RS>(vtile, dv + (seg.row0 + k0 + wv * 32) * dvs + h * DH, dvs, nrows, lane);
  }
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
                    float* __restrict__ g1, long g1s) {
  constexpr int BM = 128, BN = 32;
  __shared__ __attribute__((aligned(16))) float As[BN * DH];   // K (query side) or Q (key side)
  __shared__ __attribute__((aligned(16))) float Bs[BN * DH];   // V (query side) or dO (key side)
  __shared__ float lses[BN], Dss[BN];

  const int h = blockIdx.y;
  const Seg seg = seg_of(blockIdx.z, cu);
  const int r0 = blockIdx.x * BM;
  if (r0 >= seg.n) return;
  const int tid = threadIdx.x;
  const int ri = r0 + tid;
  const bool ok = ri < seg.n;
  const long C = (long)H * DH;
  const long grow = seg.row0 + ri;

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
        b[d] = dout[grow * C + h * DH + d];
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
        x = *reinterpret_cast<const floatx4*>(sa + (seg.row0 + t + r) * sa_stride + h * DH + c * 4);
        y = *reinterpret_cast<const floatx4*>(sb + (seg.row0 + t + r) * sb_stride + h * DH + c * 4);
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
    g0[grow * g0s + h * DH + d] = acc0[d];
    if (kKeySide) g1[grow * g1s + h * DH + d] = acc1[d];
  }
}

}  // namespace spa

using namespace spa;

extern "C" size_t spa_attention_bwd_workspace_bytes(int B, int max_seqlen, int H, int Dh, int dtype) {
  (void)Dh; (void)dtype;
  if (B < 1 || max_seqlen < 1 || H < 1) return 0;
  return (size_t)H * (size_t)B * (size_t)max_seqlen * sizeof(float);   // D_i for every (head, row)
}

extern "C" int spa_packed_attention_bwd(const void* q, const void* k, const void* v, int64_t q_row_stride,
                                        int64_t k_row_stride, int64_t v_row_stride, const void* out,
                                        const void* dout, const float* lse, const int32_t* cu_seqlens, int B,
                                        int max_seqlen, int H, int Dh, int dtype, float softmax_scale,
                                        void* dq, void* dk, void* dv, int64_t dq_row_stride,
                                        int64_t dk_row_stride, int64_t dv_row_stride, void* workspace,
                                        size_t workspace_bytes, void* stream) {
  const char* fn = "spa_packed_attention_bwd";
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
  const size_t need = spa_attention_bwd_workspace_bytes(B, max_seqlen, H, Dh, dtype);
  SPA_REQUIRE(workspace != nullptr && workspace_bytes >= need, SPA_ERR_WORKSPACE,
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
                     (long)dq_row_stride, (float*)nullptr, 0L);                                               \
  hipLaunchKernelGGL((attn_bwd_f32_kernel<D, true>), grid, block, 0, st, (const float*)q, (const float*)k,    \
                     (const float*)v, (long)q_row_stride, (long)k_row_stride, (long)v_row_stride,             \
                     (const float*)out, (const float*)dout, lse, dvec, ls, cu_seqlens, H, scale, (float*)dk,  \
                     (long)dk_row_stride, (float*)dv, (long)dv_row_stride)
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
    const char* env = std::getenv("SPA_ATTN_BWD_SHORT");                 // "tiled" forces the 4-wave kernels
    const bool short_seg = max_seqlen <= 256 && !(env != nullptr && env[0] == 't');
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
    if (Dh == 32) SPA_BWD_BF16(32); else SPA_BWD_BF16(64);
#undef SPA_BWD_BF16
#undef SPA_BWD_ARGS_DQ
#undef SPA_BWD_ARGS_DKDV
  }
  return check_launch(fn);
}
