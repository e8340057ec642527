// Masked multi-head self-attention on packed tokens (Section 3.2, last paragraph): a token
// attends only to tokens of its own image.  The mask is never built: a workgroup works on
// one (image, head, query block) and walks the keys of that image's segment only.
//
// bf16 path (MFMA, fp32 softmax).  One wave owns 32 queries.  It computes the TRANSPOSED
// score tile S^T = K Q^T with v_mfma_f32_32x32x16_bf16, so that in the accumulator layout
// (column = lane % 32, 16 rows per lane) a lane holds 16 keys of ONE query: row max and
// row sum are in-lane reductions plus one exchange with lane ^ 32, the running max / sum /
// rescale factor are one scalar per lane, and the bf16-rounded probabilities are already
// in the B-operand layout of the second product O^T = V^T P^T — no trip through LDS.
// K tiles sit in LDS row-major (A operand: 16-byte reads), V tiles are stored transposed.
//
// fp32 path (reference-grade, used by the small fp32 workload): one thread per query,
// K/V tiles broadcast from LDS, plain fp32 FMA.
#include <cmath>

#include "spa_common.h"

namespace spa {

struct Segment {
  long row0;   // first packed row of the segment
  int nq;      // query rows to compute
  int nk;      // keys to attend to
};

// packed mode: cu_seqlens bounds.  padded mode (key_lens != nullptr): every image owns
// n_pad rows, all are queries, only the first key_lens[b] are keys.
__device__ __forceinline__ Segment segment_of(int b, const int32_t* cu, const int32_t* key_lens, int n_pad) {
  Segment s;
  if (key_lens != nullptr) {
    s.row0 = (long)b * n_pad;
    s.nq = n_pad;
    s.nk = min(max(key_lens[b], 0), n_pad);
  } else {
    const int a = cu[b];
    s.row0 = a;
    s.nq = s.nk = cu[b + 1] - a;
  }
  return s;
}

// ------------------------------------------------------------------------- bf16 / MFMA
constexpr int kBN = 64;   // keys per LDS tile

template <int DH, int NW>
__global__ void __launch_bounds__(64 * NW)
attn_fwd_bf16_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k,
                     const __bf16* __restrict__ v, long qs, long ks, long vs, const int32_t* __restrict__ cu,
                     const int32_t* __restrict__ key_lens, int n_pad, int H, float scale_log2,
                     __bf16* __restrict__ out, float* __restrict__ lse, long lse_stride) {
  constexpr int KS = DH + 8;    // LDS row stride of the K tile (elements): conflict-free b128 reads
  constexpr int VS = kBN + 4;   // LDS row stride of the transposed V tile: conflict-free b64 reads
  constexpr int KK = DH / 16;   // MFMA k-steps over the head dim
  constexpr int DB = DH / 32;   // 32-row blocks of O^T
  __shared__ __attribute__((aligned(16))) __bf16 Ks[kBN * KS];
  __shared__ __attribute__((aligned(16))) __bf16 Vt[DH * VS];

  const int h = blockIdx.y;
  const Segment seg = segment_of(blockIdx.z, cu, key_lens, n_pad);
  const int q0 = blockIdx.x * (32 * NW);
  if (q0 >= seg.nq) return;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wv = tid >> 6;
  const int l32 = lane & 31, hh = lane >> 5;
  const int qi = q0 + wv * 32 + l32;
  const bool wave_live = q0 + wv * 32 < seg.nq;
  const bool q_ok = qi < seg.nq;
  const long C = (long)H * DH;

  bf16x8 qf[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) {
    bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
    qf[kk] = z;
    if (q_ok) qf[kk] = *reinterpret_cast<const bf16x8*>(q + (seg.row0 + qi) * qs + h * DH + kk * 16 + hh * 8);
  }

  floatx16 o[DB];
#pragma unroll
  for (int d = 0; d < DB; ++d)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[d][r] = 0.f;
  float m = -INFINITY, l = 0.f;

  for (int kt = 0; kt < seg.nk; kt += kBN) {
    __syncthreads();
    constexpr int CPR = DH / 8;
    for (int i = tid; i < kBN * CPR; i += 64 * NW) {
      const int r = i / CPR, c = i % CPR;
      bf16x8 kv = {0, 0, 0, 0, 0, 0, 0, 0};
      bf16x8 vv = kv;
      if (kt + r < seg.nk) {
        kv = *reinterpret_cast<const bf16x8*>(k + (seg.row0 + kt + r) * ks + h * DH + c * 8);
        vv = *reinterpret_cast<const bf16x8*>(v + (seg.row0 + kt + r) * vs + h * DH + c * 8);
      }
      *reinterpret_cast<bf16x8*>(&Ks[r * KS + c * 8]) = kv;
#pragma unroll
      for (int e = 0; e < 8; ++e) Vt[(c * 8 + e) * VS + r] = vv[e];
    }
    __syncthreads();
    if (!wave_live) continue;

#pragma unroll
    for (int sb = 0; sb < kBN / 32; ++sb) {
      const int key0 = kt + sb * 32;
      if (key0 >= seg.nk) break;
      // S^T tile: rows = 32 keys, cols = this wave's 32 queries
      floatx16 s;
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(&Ks[(sb * 32 + l32) * KS + kk * 16 + hh * 8]);
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[kk], s, 0, 0, 0);
      }
      // accumulator register r of this lane is key key0 + 8*(r/4) + 4*hh + r%4
      if (key0 + 32 > seg.nk) {
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (key0 + 8 * (r / 4) + 4 * hh + (r % 4) >= seg.nk) s[r] = -INFINITY;
      }
      float mx = s[0];
#pragma unroll
      for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
      const float m_new = fmaxf(m, mx * scale_log2);
      const float alpha = __builtin_amdgcn_exp2f(m - m_new);
      float p[16];
      float psum = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        p[r] = __builtin_amdgcn_exp2f(fmaf(s[r], scale_log2, -m_new));
        psum += p[r];
      }
      l = fmaf(l, alpha, psum);
      m = m_new;
#pragma unroll
      for (int d = 0; d < DB; ++d)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[d][r] *= alpha;
      // O^T += V^T P^T, 16 keys per MFMA: registers 8*mf .. 8*mf+7 are the B operand
#pragma unroll
      for (int mf = 0; mf < 2; ++mf) {
        floatx8 pf;
#pragma unroll
        for (int j = 0; j < 8; ++j) pf[j] = p[8 * mf + j];
        const bf16x8 pb = float_to_bf16x8(pf);
#pragma unroll
        for (int d = 0; d < DB; ++d) {
          const __bf16* vr = &Vt[(d * 32 + l32) * VS + sb * 32 + 16 * mf + 4 * hh];
          const bf16x4 lo = *reinterpret_cast<const bf16x4*>(vr);
          const bf16x4 hi = *reinterpret_cast<const bf16x4*>(vr + 8);
          const bf16x8 a = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb, o[d], 0, 0, 0);
        }
      }
    }
  }

  if (!wave_live) return;
  const float l_tot = l + __shfl_xor(l, 32, kWave);
  if (!q_ok) return;
  const float inv = seg.nk > 0 ? 1.0f / l_tot : 0.f;
  __bf16* orow = out + (seg.row0 + qi) * C + h * DH;
#pragma unroll
  for (int d = 0; d < DB; ++d)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      floatx4 f = {o[d][4 * g] * inv, o[d][4 * g + 1] * inv, o[d][4 * g + 2] * inv, o[d][4 * g + 3] * inv};
      *reinterpret_cast<bf16x4*>(orow + d * 32 + 8 * g + 4 * hh) = __builtin_convertvector(f, bf16x4);
    }
  if (lse != nullptr && hh == 0)
    lse[h * lse_stride + seg.row0 + qi] = seg.nk > 0 ? (m + __log2f(l_tot)) * 0.69314718055994531f : -INFINITY;
}

// ------------------------------------------------------------------------------- fp32
template <int DH>
__global__ void __launch_bounds__(128)
attn_fwd_f32_kernel(const float* __restrict__ q, const float* __restrict__ k,
                    const float* __restrict__ v, long qs, long ks, long vs, const int32_t* __restrict__ cu,
                    const int32_t* __restrict__ key_lens, int n_pad, int H, float scale,
                    float* __restrict__ out, float* __restrict__ lse, long lse_stride) {
  constexpr int BM = 128, BN = 32;
  __shared__ __attribute__((aligned(16))) float Ks[BN * DH];
  __shared__ __attribute__((aligned(16))) float Vs[BN * DH];

  const int h = blockIdx.y;
  const Segment seg = segment_of(blockIdx.z, cu, key_lens, n_pad);
  const int q0 = blockIdx.x * BM;
  if (q0 >= seg.nq) return;
  const int tid = threadIdx.x;
  const int qi = q0 + tid;
  const bool q_ok = qi < seg.nq;
  const long C = (long)H * DH;

  float qr[DH], o[DH];
#pragma unroll
  for (int d = 0; d < DH; ++d) { qr[d] = 0.f; o[d] = 0.f; }
  if (q_ok) {
    const float* qp = q + (seg.row0 + qi) * qs + h * DH;
#pragma unroll
    for (int d = 0; d < DH; d += 4) {
      const floatx4 t = *reinterpret_cast<const floatx4*>(qp + d);
      qr[d] = t[0] * scale; qr[d + 1] = t[1] * scale; qr[d + 2] = t[2] * scale; qr[d + 3] = t[3] * scale;
    }
  }
  float m = -INFINITY, l = 0.f;

  for (int kt = 0; kt < seg.nk; kt += BN) {
    __syncthreads();
    for (int i = tid; i < BN * DH / 4; i += BM) {
      const int r = i / (DH / 4), c = i % (DH / 4);
      floatx4 kv = {0.f, 0.f, 0.f, 0.f}, vv = kv;
      if (kt + r < seg.nk) {
        kv = *reinterpret_cast<const floatx4*>(k + (seg.row0 + kt + r) * ks + h * DH + c * 4);
        vv = *reinterpret_cast<const floatx4*>(v + (seg.row0 + kt + r) * vs + h * DH + c * 4);
      }
      *reinterpret_cast<floatx4*>(&Ks[r * DH + c * 4]) = kv;
      *reinterpret_cast<floatx4*>(&Vs[r * DH + c * 4]) = vv;
    }
    __syncthreads();
    const int kn = min(BN, seg.nk - kt);
    float s[BN];
    float mx = -INFINITY;
#pragma unroll
    for (int j = 0; j < BN; ++j) {
      float acc = 0.f;
#pragma unroll
      for (int d = 0; d < DH; ++d) acc = fmaf(qr[d], Ks[j * DH + d], acc);
      s[j] = j < kn ? acc : -INFINITY;
      mx = fmaxf(mx, s[j]);
    }
    const float m_new = fmaxf(m, mx);
    const float alpha = expf(m - m_new);
    l *= alpha;
#pragma unroll
    for (int d = 0; d < DH; ++d) o[d] *= alpha;
#pragma unroll
    for (int j = 0; j < BN; ++j) {
      const float p = expf(s[j] - m_new);
      l += p;
#pragma unroll
      for (int d = 0; d < DH; ++d) o[d] = fmaf(p, Vs[j * DH + d], o[d]);
    }
    m = m_new;
  }
  if (!q_ok) return;
  const float inv = seg.nk > 0 ? 1.0f / l : 0.f;
  float* op = out + (seg.row0 + qi) * C + h * DH;
#pragma unroll
  for (int d = 0; d < DH; d += 4) {
    floatx4 t = {o[d] * inv, o[d + 1] * inv, o[d + 2] * inv, o[d + 3] * inv};
    *reinterpret_cast<floatx4*>(op + d) = t;
  }
  if (lse != nullptr) lse[h * lse_stride + seg.row0 + qi] = seg.nk > 0 ? m + logf(l) : -INFINITY;
}

// ------------------------------------------------------------------------------- host
static int attention_common(const char* fn, const void* q, const void* k, const void* v,
                            int64_t q_stride, int64_t k_stride, int64_t v_stride, const int32_t* cu, const int32_t* key_lens, int B,
                            int n_max, int H, int Dh, int dtype, float softmax_scale, void* out,
                            float* lse, void* stream) {
  SPA_REQUIRE(q && k && v && out && (cu || key_lens), SPA_ERR_INVALID_ARG, "%s: null pointer", fn);
  SPA_REQUIRE(B >= 1 && n_max >= 1 && H >= 1, SPA_ERR_INVALID_ARG, "%s: B, max_seqlen, H must be >= 1", fn);
  SPA_REQUIRE((long)B * n_max < 2147483647L, SPA_ERR_INVALID_ARG, "%s: B*max_seqlen must be < 2^31", fn);
  SPA_REQUIRE(B <= 65535 && H <= 65535, SPA_ERR_INVALID_ARG, "%s: B and H must be <= 65535", fn);
  SPA_REQUIRE(dtype == SPA_F32 || dtype == SPA_BF16, SPA_ERR_UNSUPPORTED, "%s: unknown dtype %d", fn, dtype);
  SPA_REQUIRE(Dh == 32 || Dh == 64, SPA_ERR_UNSUPPORTED, "%s: head dim %d not supported (32 or 64)", fn, Dh);
  const int64_t strides[3] = {q_stride, k_stride, v_stride};
  for (int64_t rs : strides) {
    SPA_REQUIRE(rs >= (int64_t)H * Dh, SPA_ERR_INVALID_ARG, "%s: row stride %ld < H*Dh", fn, (long)rs);
    SPA_REQUIRE((rs * elem_size(dtype)) % 16 == 0, SPA_ERR_INVALID_ARG, "%s: row stride is not a multiple of 16 bytes", fn);
  }
  SPA_REQUIRE(aligned16(q) && aligned16(k) && aligned16(v) && aligned16(out), SPA_ERR_INVALID_ARG,
              "%s: q/k/v/out not 16-byte aligned", fn);
  SPA_REQUIRE(softmax_scale >= 0.f && std::isfinite(softmax_scale), SPA_ERR_INVALID_ARG,
              "%s: softmax_scale must be finite and >= 0 (0 = 1/sqrt(Dh))", fn);
  const float scale = softmax_scale > 0.f ? softmax_scale : 1.0f / std::sqrt((float)Dh);
  const long lse_stride = (long)B * n_max;
  hipStream_t st = as_stream(stream);
  if (dtype == SPA_F32) {
    const dim3 grid((n_max + 127) / 128, H, B), block(128);
#define SPA_F32_LAUNCH(D)                                                                                \
  hipLaunchKernelGGL((attn_fwd_f32_kernel<D>), grid, block, 0, st, (const float*)q, (const float*)k,    \
                     (const float*)v, (long)q_stride, (long)k_stride, (long)v_stride, cu, key_lens, n_max, H, scale, (float*)out, lse, \
                     lse_stride)
    if (Dh == 32) SPA_F32_LAUNCH(32); else SPA_F32_LAUNCH(64);
#undef SPA_F32_LAUNCH
  } else {
    const float scale_log2 = scale * 1.4426950408889634f;
    const int NW = n_max <= 256 ? 2 : 4;
    const dim3 grid((n_max + 32 * NW - 1) / (32 * NW), H, B), block(64 * NW);
#define SPA_BF16_LAUNCH(D, W)                                                                              \
  hipLaunchKernelGGL((attn_fwd_bf16_kernel<D, W>), grid, block, 0, st, (const __bf16*)q, (const __bf16*)k, \
                     (const __bf16*)v, (long)q_stride, (long)k_stride, (long)v_stride, cu, key_lens, n_max, H, scale_log2, (__bf16*)out, \
                     lse, lse_stride)
    if (Dh == 32) { if (NW == 2) SPA_BF16_LAUNCH(32, 2); else SPA_BF16_LAUNCH(32, 4); }
    else          { if (NW == 2) SPA_BF16_LAUNCH(64, 2); else SPA_BF16_LAUNCH(64, 4); }
#undef SPA_BF16_LAUNCH
  }
  return check_launch(fn);
}

}  // namespace spa

using namespace spa;

extern "C" int spa_packed_attention(const void* q, const void* k, const void* v, int64_t q_row_stride,
                                    int64_t k_row_stride, int64_t v_row_stride, const int32_t* cu_seqlens, int B, int max_seqlen, int H, int Dh,
                                    int dtype, float softmax_scale, void* out, float* lse, void* stream) {
  SPA_REQUIRE(cu_seqlens, SPA_ERR_INVALID_ARG, "spa_packed_attention: cu_seqlens is null");
  return attention_common("spa_packed_attention", q, k, v, q_row_stride, k_row_stride, v_row_stride, cu_seqlens, nullptr, B, max_seqlen,
                          H, Dh, dtype, softmax_scale, out, lse, stream);
}

extern "C" int spa_padded_attention(const void* q, const void* k, const void* v, int64_t row_stride,
                                    const int32_t* seqlens, int B, int n_pad, int H, int Dh, int dtype,
                                    float softmax_scale, void* out, void* stream) {
  SPA_REQUIRE(seqlens, SPA_ERR_INVALID_ARG, "spa_padded_attention: seqlens is null");
  return attention_common("spa_padded_attention", q, k, v, row_stride, row_stride, row_stride, nullptr, seqlens, B, n_pad, H, Dh,
                          dtype, softmax_scale, out, nullptr, stream);
}
