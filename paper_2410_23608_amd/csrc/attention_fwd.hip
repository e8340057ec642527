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
// fp32 path (reference-grade, used by the small fp32 workload): eight lanes per query,
// K/V tiles read from LDS, plain fp32 FMA.
#include <cmath>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <type_traits>

#include "attn_tiles.h"
#include "spa_common.h"

namespace spa {

// Optional fused scatter-back (the unpack step folded into the attention kernel): packed
// output row j goes to y[gather_idx[j]] (plus base), and every workgroup first fills its
// share of the rows that bypass attention (inv_pos < 0) with base or zero.  All-null = off.
// y is the path's final output: nothing here reads it again, so its stores are non-temporal
// (they do not push the packed rows the next launches read out of the caches).
struct Scatter {
  const int32_t* gather_idx;   // [B*N] packed row -> flat token
  const int32_t* inv_pos;      // [B*N] flat token -> packed row or -1
  const void* base;            // [B*N, C] residual or nullptr
  void* y;                     // [B*N, C]
  int N;                       // tokens per image; in flat mode all rows of y (B*N)
  int flat;                    // 0: segment s fills the bypassing rows of image s (segments are images)
                               // 1: segments are not images (containers): the rows of y are dealt
                               //    evenly to all (segment, part) work units
  int gathered;                // 1: q, k, v are NOT packed: the row of packed position j is row
                               //    gather_idx[j] of q, k, v (token positions); packing then only
                               //    builds the index and no row is copied before the attention
  const uint8_t* mask;         // [B*N] or nullptr: when given, a token bypasses attention iff its mask byte is 0
                               //    (used in place of inv_pos by the form that is given no packing index)
};
__device__ __forceinline__ bool bypasses(const Scatter& sc, long row) {
  return sc.mask != nullptr ? sc.mask[row] == 0 : sc.inv_pos[row] < 0;
}

// Row of q / k / v that holds packed position j of a segment starting at packed row row0:
// gi = gather_idx + row0 when the rows are gathered through the index, else null.
// GATHER is a compile-time property of every bf16 kernel: with packed rows the index is known to be
// absent and the row addresses stay affine in the loop counters (pointer increments), with gathered
// rows every row address is a multiply on a loaded index.
template <bool GATHER>
__device__ __forceinline__ const int32_t* gather_base(const Scatter& sc, long row0) {
  return GATHER ? sc.gather_idx + row0 : nullptr;
}
__device__ __forceinline__ long source_row(const int32_t* gi, long row0, int j) {
  return gi != nullptr ? (long)gi[j] : row0 + j;
}
// Element offset of a gathered row: one 32 x 32 -> 64 bit multiply (the host checks that rows and
// strides are below 2^31).
__device__ __forceinline__ long row_offset(int row, long stride) {
  return (long)((unsigned long)(uint32_t)row * (uint32_t)stride);
}

// The rows whose bypass fill falls to work unit (segment `seg` of `nseg`, part `part` of `nparts`):
// tokens [t0, t1) of image b (flat mode: b = 0 and the range is over all rows of y).
struct FillRange {
  int b, t0, t1;
};
__device__ __forceinline__ FillRange fill_range(const Scatter& sc, int seg, int nseg, int part, int nparts) {
  FillRange f = {0, 0, 0};
  if (sc.y == nullptr) return f;
  if (!sc.flat) {
    const int per = (sc.N + nparts - 1) / nparts;
    f.b = seg;
    f.t0 = min(sc.N, part * per);
    f.t1 = min(sc.N, (part + 1) * per);
  } else {
    const long units = (long)nseg * nparts, u = (long)seg * nparts + part;
    const long per = (sc.N + units - 1) / units;
    f.t0 = (int)min((long)sc.N, u * per);
    f.t1 = (int)min((long)sc.N, (u + 1) * per);
  }
  return f;
}

// Fill the head slice [h*DH, (h+1)*DH) of the bypassing rows among tokens [t0, t1) of image b.
// Shared by `nthreads` threads, this one being number `tid` of them.
template <typename T, int DH>
__device__ __forceinline__ void scatter_fill(const Scatter& sc, int b, int t0, int t1, int h, long C, int tid,
                                             int nthreads) {
  constexpr int VE = 16 / sizeof(T), CPR = DH / VE;
  const long tok0 = (long)b * sc.N;
  const int work = (t1 - t0) * CPR;
  for (int i = tid; i < work; i += nthreads) {
    const int t = t0 + i / CPR, c = i % CPR;
    if (bypasses(sc, tok0 + t)) {
      const long off = (tok0 + t) * C + h * DH + c * VE;
      uintx4 val = {0u, 0u, 0u, 0u};
      if (sc.base != nullptr) val = *reinterpret_cast<const uintx4*>(static_cast<const T*>(sc.base) + off);
      __builtin_nontemporal_store(val, reinterpret_cast<uintx4*>(static_cast<T*>(sc.y) + off));
    }
  }
}

// Fill every column of the bypassing rows among the flat token rows [r0, r1).
template <typename T>
__device__ __forceinline__ void scatter_fill_rows(const Scatter& sc, long r0, long r1, long C, int tid, int nthreads) {
  constexpr int VE = 16 / sizeof(T);
  const int cpr = (int)(C / VE);
  const long work = (r1 - r0) * cpr;
  for (long i = tid; i < work; i += nthreads) {
    const long row = r0 + i / cpr;
    const int c = (int)(i % cpr);
    if (bypasses(sc, row)) {
      const long off = row * C + c * VE;
      uintx4 val = {0u, 0u, 0u, 0u};
      if (sc.base != nullptr) val = *reinterpret_cast<const uintx4*>(static_cast<const T*>(sc.base) + off);
      __builtin_nontemporal_store(val, reinterpret_cast<uintx4*>(static_cast<T*>(sc.y) + off));
    }
  }
}

// ------------------------------------------------------------------------- bf16 / MFMA
// Per-wave state of the online softmax: O^T accumulators (rows = head dim, cols = this
// wave's 32 queries), running max m (log2 domain, scale folded in) and running sum l (the
// two halves of the wave keep partial sums that are added at the end).
template <int DH>
struct FwdAcc {
  floatx16 o[DH / 32];
  float m, l;
  __device__ __forceinline__ void init() {
#pragma unroll
    for (int d = 0; d < DH / 32; ++d)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[d][r] = 0.f;
    m = -INFINITY;
    l = 0.f;
  }
};

// Score sub-tiles of one group of GSB*32 keys: S^T = K Q^T (rows = keys, cols = queries).
// key0 = first key of the group inside the LDS tile, rem = valid keys of the tile.
template <int DH, int RS, int GSB, bool FULL>
__device__ __forceinline__ void fwd_scores(const __bf16* kbuf, int key0, int rem, const bf16x8 (&qf)[DH / 16],
                                           floatx16 (&s)[GSB], int l32, int hh) {
#pragma unroll
  for (int sb = 0; sb < GSB; ++sb) {
    const int k0 = key0 + sb * 32;
    if (FULL || k0 < rem) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s[sb][r] = 0.f;
#pragma unroll
      for (int kk = 0; kk < DH / 16; ++kk) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(&kbuf[(k0 + l32) * RS + kk * 16 + hh * 8]);
        s[sb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[kk], s[sb], 0, 0, 0);
      }
      if (!FULL && rem - k0 < 32) {
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (k0 + acc_row(r, hh) >= rem) s[sb][r] = -INFINITY;
      }
    } else {
#pragma unroll
      for (int r = 0; r < 16; ++r) s[sb][r] = -INFINITY;
    }
  }
}

// One online-softmax update (max, rescale, exp, sum) over a group of GSB*32 keys, then
// O^T += V^T P^T for the group.  V^T at vbuf (row stride TS), the group's keys at column vcol; TS == 0:
// V rows as they lie in memory (row stride DH + 8, the group's keys from row vcol), the V^T fragments
// then come from the transposing LDS read.
template <int DH, int TS, int GSB, bool FULL>
__device__ __forceinline__ void fwd_softmax_pv(const floatx16 (&s)[GSB], const __bf16* vbuf, int vcol, int key0,
                                               int rem, FwdAcc<DH>& acc, float scale_log2, int l32, int hh) {
  constexpr int DB = DH / 32;
  float mx = s[0][0];
#pragma unroll
  for (int sb = 0; sb < GSB; ++sb)
#pragma unroll
    for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[sb][r]);
  mx = max_across_halves(mx);
  const float m_new = fmaxf(acc.m, mx * scale_log2);
  if (__ballot(m_new != acc.m) != 0) {       // some query's running max moved: rescale
    const float alpha = __builtin_amdgcn_exp2f(acc.m - m_new);
    acc.l *= alpha;
#pragma unroll
    for (int d = 0; d < DB; ++d)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc.o[d][r] *= alpha;
    acc.m = m_new;
  }
  float psum = 0.f;
#pragma unroll
  for (int sb = 0; sb < GSB; ++sb) {
    if (FULL || key0 + sb * 32 < rem) {
      float p[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        p[r] = __builtin_amdgcn_exp2f(fmaf(s[sb][r], scale_log2, -m_new));
        psum += p[r];
      }
#pragma unroll
      for (int mf = 0; mf < 2; ++mf) {
        floatx8 pf;
#pragma unroll
        for (int j = 0; j < 8; ++j) pf[j] = p[8 * mf + j];
        const bf16x8 pb = float_to_bf16x8(pf);
#pragma unroll
        for (int d = 0; d < DB; ++d) {
          const bf16x8 a = TS == 0 ? transposed_frag_rowmajor<DH + 8>(vbuf, d, vcol + sb * 32, mf, l32 + 32 * hh)
                                   : transposed_frag<TS == 0 ? 1 : TS>(vbuf, d * 32 + l32, vcol + sb * 32, mf, hh);
          acc.o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb, acc.o[d], 0, 0, 0);
        }
      }
    }
  }
  acc.l += psum;
}

// One tile of NSB*32 keys held in LDS (K rows at kbuf, row stride RS; V^T at vbuf, row
// stride TS, the tile's keys starting at column vcol0), processed in groups of 64 keys with
// a two-stage software pipeline: the score MFMAs of group g+1 are issued before the softmax
// VALU work of group g, and that group's P V MFMAs run under the next group's softmax, so
// the matrix pipe and the vector ALU overlap inside one wave.  rem = valid keys in the tile;
// FULL = every key valid (no masking code).
template <int DH, int RS, int TS, int NSB, bool FULL>
__device__ __forceinline__ void fwd_process_tile(const __bf16* kbuf, const __bf16* vbuf, int vcol0, int rem,
                                                 const bf16x8 (&qf)[DH / 16], FwdAcc<DH>& acc,
                                                 float scale_log2, int l32, int hh) {
  constexpr int GSB = NSB >= 4 ? 2 : 1;     // sub-tiles per softmax group
  constexpr int NG = NSB / GSB;
  floatx16 s[2][GSB];
  fwd_scores<DH, RS, GSB, FULL>(kbuf, 0, rem, qf, s[0], l32, hh);
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    const int key0 = g * GSB * 32;
    if (!FULL && key0 >= rem) break;
    if (g + 1 < NG && (FULL || key0 + GSB * 32 < rem))
      fwd_scores<DH, RS, GSB, FULL>(kbuf, key0 + GSB * 32, rem, qf, s[(g + 1) & 1], l32, hh);
    fwd_softmax_pv<DH, TS, GSB, FULL>(s[g & 1], vbuf, vcol0 + key0, key0, rem, acc, scale_log2, l32, hh);
  }
}

// Output stage, phase 1: normalise this wave's O^T accumulators and park the 32 x DH bf16
// tile in LDS (row = query, row stride RS), so that phase 2 can write whole rows.
// Also writes lse.  Called by every lane of a live wave.
template <int DH, int RS>
__device__ __forceinline__ void fwd_park(FwdAcc<DH>& acc, bool q_ok, bool have_keys, __bf16* tile,
                                         float* lse_ptr, int l32, int hh) {
  const float l_tot = sum_across_halves(acc.l);
  const float inv = have_keys ? 1.0f / l_tot : 0.f;
#pragma unroll
  for (int d = 0; d < DH / 32; ++d)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      floatx4 f = {acc.o[d][4 * g] * inv, acc.o[d][4 * g + 1] * inv, acc.o[d][4 * g + 2] * inv,
                   acc.o[d][4 * g + 3] * inv};
      *reinterpret_cast<bf16x4*>(&tile[l32 * RS + d * 32 + 8 * g + 4 * hh]) = __builtin_convertvector(f, bf16x4);
    }
  if (q_ok && lse_ptr != nullptr && hh == 0)
    *lse_ptr = have_keys ? (acc.m + __log2f(l_tot)) * 0.69314718055994531f : -INFINITY;
}

// Output stage, phase 2 (after a barrier): the wave copies its parked tile to global memory,
// consecutive lanes writing consecutive 16-byte chunks of a row.  nrows = valid rows (<= 32);
// prow0 = packed row of the tile's first row.  out may be null when only y is wanted.
template <int DH, int RS>
__device__ __forceinline__ void fwd_flush(const __bf16* tile, __bf16* out, const Scatter& sc, long prow0, int h,
                                          long C, int nrows, int lane) {
  constexpr int CPR = DH / 8;
#pragma unroll
  for (int i = lane; i < 32 * CPR; i += 64) {
    const int r = i / CPR, c = i % CPR;
    if (r < nrows) {
      bf16x8 val = *reinterpret_cast<const bf16x8*>(&tile[r * RS + c * 8]);
      if (out != nullptr) *reinterpret_cast<bf16x8*>(out + (prow0 + r) * C + h * DH + c * 8) = val;
      if (sc.y != nullptr) {
        const long off = (long)sc.gather_idx[prow0 + r] * C + h * DH + c * 8;
        if (sc.base != nullptr) {
          const floatx8 bv = bf16x8_to_float(*reinterpret_cast<const bf16x8*>(static_cast<const __bf16*>(sc.base) + off));
          val = float_to_bf16x8(bf16x8_to_float(val) + bv);
        }
        __builtin_nontemporal_store(val, reinterpret_cast<bf16x8*>(static_cast<__bf16*>(sc.y) + off));
      }
    }
  }
}

// Register staging of key/value rows on their way to LDS: task i = 16-byte chunk column
// c = i % CPR of the row pair (2*(i / CPR), +1); K goes row-major, V transposed.
template <int DH, int THREADS, int TASKS, bool GATHER>
struct KvStage {
  static constexpr int CPR = DH / 8;
  static constexpr int TPT = (TASKS + THREADS - 1) / THREADS;
  static constexpr int RPP = 2 * THREADS / CPR;   // rows one pass of the workgroup covers
  static_assert(THREADS % CPR == 0, "a thread keeps its chunk column over the passes");
  bf16x8 kreg[TPT][2], vreg[TPT][2];

  // The rows the next load() fetches: keys [kt_, kt_ + tile) of a segment of nk_ keys whose packed rows
  // start at row0_.  Packed rows need no per-lane address arithmetic: the address is a uniform base
  // (segment, tile, pass) plus a 32-bit per-lane offset that never changes.  Gathered rows have their
  // token rows loaded here, one tile ahead of load(), so the row loads never wait for an index.
  int tok_rows[TPT][2];
  long row0_;
  int kt_, nk_;

  __device__ __forceinline__ bool valid(int t, int u) const {
    const int i = threadIdx.x + t * THREADS;
    return i < TASKS && kt_ + 2 * (i / CPR) + u < nk_;
  }
  __device__ __forceinline__ void index(const int32_t* gi, long row0, int kt, int nk) {
    row0_ = row0;
    kt_ = kt;
    nk_ = nk;
    if (GATHER) {
      if (TASKS % THREADS == 0 && kt + 2 * TASKS / CPR <= nk) {      // a whole tile: no predicates
#pragma unroll
        for (int t = 0; t < TPT; ++t)
#pragma unroll
          for (int u = 0; u < 2; ++u) tok_rows[t][u] = gi[kt + 2 * ((threadIdx.x + t * THREADS) / CPR) + u];
      } else {
#pragma unroll
        for (int t = 0; t < TPT; ++t)
#pragma unroll
          for (int u = 0; u < 2; ++u)
            if (valid(t, u)) tok_rows[t][u] = gi[kt + 2 * ((threadIdx.x + t * THREADS) / CPR) + u];
      }
    }
  }
  // The row loads; rows past the segment read as zero
  __device__ __forceinline__ void load(const __bf16* kh, const __bf16* vh, long ks, long vs) {
    const int c = threadIdx.x % CPR, lrow = 2 * (threadIdx.x / CPR);
    const uint32_t koff = (uint32_t)lrow * (uint32_t)ks + c * 8, voff = (uint32_t)lrow * (uint32_t)vs + c * 8;
    // a tile that lies wholly inside the segment (all but the last one): no predicates, no zero fill
    if (TASKS % THREADS == 0 && kt_ + 2 * TASKS / CPR <= nk_) {
#pragma unroll
      for (int t = 0; t < TPT; ++t) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const __bf16 *kp, *vp;
          if (GATHER) {
            kp = kh + row_offset(tok_rows[t][u], ks) + c * 8;
            vp = vh + row_offset(tok_rows[t][u], vs) + c * 8;
          } else {
            const long r = row0_ + kt_ + t * RPP + u;     // uniform
            kp = kh + r * ks + koff;
            vp = vh + r * vs + voff;
          }
          kreg[t][u] = *reinterpret_cast<const bf16x8*>(kp);
          vreg[t][u] = *reinterpret_cast<const bf16x8*>(vp);
        }
      }
      return;
    }
#pragma unroll
    for (int t = 0; t < TPT; ++t) {
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        kreg[t][u] = zero_bf16x8();
        vreg[t][u] = zero_bf16x8();
        if (valid(t, u)) {
          const __bf16 *kp, *vp;
          if (GATHER) {
            kp = kh + row_offset(tok_rows[t][u], ks) + c * 8;
            vp = vh + row_offset(tok_rows[t][u], vs) + c * 8;
          } else {
            const long r = row0_ + kt_ + t * RPP + u;     // uniform
            kp = kh + r * ks + koff;
            vp = vh + r * vs + voff;
          }
          kreg[t][u] = *reinterpret_cast<const bf16x8*>(kp);
          vreg[t][u] = *reinterpret_cast<const bf16x8*>(vp);
        }
      }
    }
  }
  // K rows -> kbuf[row * RS], V -> vbuf[d * TS + col0 + row]
  template <int RS, int TS>
  __device__ __forceinline__ void store(__bf16* kbuf, __bf16* vbuf, int col0) const {
#pragma unroll
    for (int t = 0; t < TPT; ++t) {
      const int i = threadIdx.x + t * THREADS;
      if (i < TASKS) {
        const int c = i % CPR, r0 = 2 * (i / CPR);
        *reinterpret_cast<bf16x8*>(&kbuf[r0 * RS + c * 8]) = kreg[t][0];
        *reinterpret_cast<bf16x8*>(&kbuf[(r0 + 1) * RS + c * 8]) = kreg[t][1];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          bf16x2 pr = {vreg[t][0][e], vreg[t][1][e]};
          *reinterpret_cast<bf16x2*>(&vbuf[(c * 8 + e) * TS + col0 + r0]) = pr;
        }
      }
    }
  }
};

template <int DH>
__device__ __forceinline__ void load_q_frags(const __bf16* qrow, bool q_ok, int hh, bf16x8 (&qf)[DH / 16]) {
#pragma unroll
  for (int kk = 0; kk < DH / 16; ++kk) {
    qf[kk] = zero_bf16x8();
    if (q_ok) qf[kk] = *reinterpret_cast<const bf16x8*>(qrow + kk * 16 + hh * 8);
  }
}

// Register staging of BN key and value rows on their way to LDS (both row-major): chunk i =
// 16-byte piece i % CPR of row i / CPR; index() runs one tile ahead of load() (see KvStage).
template <int DH, int THREADS, int BN, bool GATHER>
struct KvRowStage {
  static constexpr int CPR = DH / 8, CHUNKS = BN * CPR, CPT = (CHUNKS + THREADS - 1) / THREADS;
  static constexpr int RPP = THREADS / CPR;
  static_assert(THREADS % CPR == 0, "a thread keeps its chunk column over the passes");
  bf16x8 kreg[CPT], vreg[CPT];
  int tok_rows[CPT];                   // gathered rows only: see KvStage
  long row0_;
  int kt_, nk_;
  __device__ __forceinline__ bool valid(int t) const {
    const int i = threadIdx.x + t * THREADS;
    return i < CHUNKS && kt_ + i / CPR < nk_;
  }
  __device__ __forceinline__ void index(const int32_t* gi, long row0, int kt, int nk) {
    row0_ = row0;
    kt_ = kt;
    nk_ = nk;
    if (GATHER) {
      if (CHUNKS % THREADS == 0 && kt + BN <= nk) {                  // a whole tile: no predicates
#pragma unroll
        for (int t = 0; t < CPT; ++t) tok_rows[t] = gi[kt + (threadIdx.x + t * THREADS) / CPR];
      } else {
#pragma unroll
        for (int t = 0; t < CPT; ++t)
          if (valid(t)) tok_rows[t] = gi[kt + (threadIdx.x + t * THREADS) / CPR];
      }
    }
  }
  __device__ __forceinline__ void load(const __bf16* kh, const __bf16* vh, long ks, long vs) {
    const int c = threadIdx.x % CPR, lrow = threadIdx.x / CPR;
    const uint32_t koff = (uint32_t)lrow * (uint32_t)ks + c * 8, voff = (uint32_t)lrow * (uint32_t)vs + c * 8;
    // a tile that lies wholly inside the segment (all but the last one): no predicates, no zero fill
    if (CHUNKS % THREADS == 0 && kt_ + BN <= nk_) {
#pragma unroll
      for (int t = 0; t < CPT; ++t) {
        const __bf16 *kp, *vp;
        if (GATHER) {
          kp = kh + row_offset(tok_rows[t], ks) + c * 8;
          vp = vh + row_offset(tok_rows[t], vs) + c * 8;
        } else {
          const long r = row0_ + kt_ + t * RPP;           // uniform
          kp = kh + r * ks + koff;
          vp = vh + r * vs + voff;
        }
        kreg[t] = *reinterpret_cast<const bf16x8*>(kp);
        vreg[t] = *reinterpret_cast<const bf16x8*>(vp);
      }
      return;
    }
#pragma unroll
    for (int t = 0; t < CPT; ++t) {
      kreg[t] = zero_bf16x8();
      vreg[t] = zero_bf16x8();
      if (valid(t)) {
        const __bf16 *kp, *vp;
        if (GATHER) {
          kp = kh + row_offset(tok_rows[t], ks) + c * 8;
          vp = vh + row_offset(tok_rows[t], vs) + c * 8;
        } else {
          const long r = row0_ + kt_ + t * RPP;           // uniform
          kp = kh + r * ks + koff;
          vp = vh + r * vs + voff;
        }
        kreg[t] = *reinterpret_cast<const bf16x8*>(kp);
        vreg[t] = *reinterpret_cast<const bf16x8*>(vp);
      }
    }
  }
  __device__ __forceinline__ void store(__bf16* kbuf, __bf16* vbuf) const {
#pragma unroll
    for (int t = 0; t < CPT; ++t) {
      const int i = threadIdx.x + t * THREADS, r = i / CPR, c = i % CPR;
      if (i < CHUNKS) {
        *reinterpret_cast<bf16x8*>(&kbuf[r * (DH + 8) + c * 8]) = kreg[t];
        *reinterpret_cast<bf16x8*>(&vbuf[r * (DH + 8) + c * 8]) = vreg[t];
      }
    }
  }
};

// Long segments.  Workgroup = NW waves x 32 queries; the keys of the segment stream through
// LDS in tiles of BN keys, double-buffered: while a tile is consumed the next one is already
// in flight from global memory into registers, and is written to the other LDS buffer
// before the single barrier that ends the iteration.
// Head dim 32 is compiled for three waves per SIMD (168 registers, no spills): with several
// batches in flight the third wave fills the softmax stalls of the other two.
// V in LDS: at head dim 64 as the rows lie in memory (staging is plain 16-byte copies, the V^T fragments
// come from the transposing LDS read: uniform long segments 521 against 481 TFLOP/s), at head dim 32
// transposed while staging (the detection batch 42.2 against 43.1 us for the launch; the same rate on
// uniform segments).
template <int DH>
constexpr bool kTiledVRows = DH == 64;
template <int DH, int BN>
struct TiledLds {
  static constexpr int RS = DH + 8, TS = transposed_stride(BN);
  static constexpr int VSIZE = kTiledVRows<DH> ? BN * RS : DH * TS;
  __attribute__((aligned(16))) __bf16 Ks[2][BN * RS];
  __attribute__((aligned(16))) __bf16 Vs[2][VSIZE];
};

// The workgroup's work on queries [q0, q0 + 32 NW) of head h of segment seg (q0 < seg.nq).
template <int DH, int NW, int BN, bool GATHER>
__device__ __forceinline__ void
tiled_attention(TiledLds<DH, BN>& lds, const Segment seg, int h, int q0, const __bf16* __restrict__ q,
                const __bf16* __restrict__ k, const __bf16* __restrict__ v, long qs, long ks, long vs, int H,
                float scale_log2, __bf16* __restrict__ out, float* __restrict__ lse, long lse_stride,
                const Scatter& sc) {
  constexpr int RS = DH + 8, NSB = BN / 32;
  constexpr bool VROWS = kTiledVRows<DH>;
  constexpr int TS = VROWS ? 0 : transposed_stride(BN);    // 0: V rows in LDS (see fwd_softmax_pv)
  auto& Ks = lds.Ks;
  auto& Vs = lds.Vs;
  static_assert(2 * BN >= 32 * NW, "the K buffers double as the output staging tile");
  const long C = (long)H * DH;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6, l32 = lane & 31, hh = lane >> 5;
  const int qi = q0 + wv * 32 + l32;
  const bool wave_live = q0 + wv * 32 < seg.nq;
  const bool q_ok = qi < seg.nq;
  const __bf16* kh = k + h * DH;
  const __bf16* vh = v + h * DH;

  const int32_t* gi = gather_base<GATHER>(sc, seg.row0);
  const long q_src = q_ok ? source_row(gi, seg.row0, qi) : 0;   // (gathered: an index load, issued first)
  typename std::conditional<VROWS, KvRowStage<DH, 64 * NW, BN, GATHER>,
                            KvStage<DH, 64 * NW, (BN / 2) * (DH / 8), GATHER>>::type stage;
  auto store = [&](int buf) {
    if constexpr (VROWS) stage.store(Ks[buf], Vs[buf]);
    else stage.template store<RS, transposed_stride(BN)>(Ks[buf], Vs[buf], 0);
  };
  stage.index(gi, seg.row0, 0, seg.nk);
  stage.load(kh, vh, ks, vs);
  stage.index(gi, seg.row0, BN, seg.nk);
  bf16x8 qf[DH / 16];
  load_q_frags<DH>(q + q_src * qs + h * DH, q_ok, hh, qf);
  FwdAcc<DH> acc;
  acc.init();
  store(0);
  __syncthreads();

  const int nt = (seg.nk + BN - 1) / BN;
  for (int t = 0; t < nt; ++t) {
    const int buf = t & 1, kt = t * BN;
    if (t + 1 < nt) {
      stage.load(kh, vh, ks, vs);                           // tile t + 1, whose rows were indexed a tile ago
      stage.index(gi, seg.row0, kt + 2 * BN, seg.nk);
    }
    if (wave_live) {
      const int rem = seg.nk - kt;               // valid keys from this tile on (may exceed BN)
      if (rem >= BN) fwd_process_tile<DH, RS, TS, NSB, true>(Ks[buf], Vs[buf], 0, BN, qf, acc, scale_log2, l32, hh);
      else fwd_process_tile<DH, RS, TS, NSB, false>(Ks[buf], Vs[buf], 0, rem, qf, acc, scale_log2, l32, hh);
    }
    if (t + 1 < nt) store(buf ^ 1);
    __syncthreads();
  }
  // every wave is past its last read of the K buffers (the loop ends with a barrier)
  __bf16* tile = &Ks[0][0] + wv * 32 * RS;
  if (wave_live)
    fwd_park<DH, RS>(acc, q_ok, seg.nk > 0, tile, lse != nullptr ? lse + h * lse_stride + seg.row0 + qi : nullptr,
                     l32, hh);
  __syncthreads();
  if (wave_live)
    fwd_flush<DH, RS>(tile, out, sc, seg.row0 + q0 + wv * 32, h, C, min(32, seg.nq - q0 - wv * 32), lane);
}

template <int DH, int NW, int BN, bool GATHER>
__global__ void __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(DH == 32 ? 3 : 2)))
attn_fwd_bf16_tiled_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k,
                           const __bf16* __restrict__ v, long qs, long ks, long vs,
                           const int32_t* __restrict__ cu, const int32_t* __restrict__ key_lens, int n_pad,
                           int H, float scale_log2, __bf16* __restrict__ out, float* __restrict__ lse,
                           long lse_stride, Scatter sc, int B, int nqb) {
  __shared__ TiledLds<DH, BN> lds;
  __shared__ int s_cu[2 * kLptMaxB + 1];
  __shared__ int s_pick;
  __shared__ LiveTile s_live;

  const long C = (long)H * DH;
  // live blocks first in launch order where the batch allows it (see live_tile_wave); the bypass fill
  // is then whole rows, an even share of all tokens per workgroup.  Otherwise block qb of every
  // (segment, head) pair in turn, the pair's share of its image's bypassing tokens per block.  The
  // fill is done right away by a workgroup without queries, after the main loop by one that has some.
  const bool live = key_lens == nullptr && live_tiles_apply(H, B);
  Segment seg = {0, 0, 0};
  int h = 0, q0 = 0;
  FillRange fr = {0, 0, 0};
  if (live) {
    const LiveTile lt = live_tile_block(blockIdx.x & 7, blockIdx.x >> 3, H, B, cu, 32 * NW, nqb, &s_live);
    if (lt.valid) {
      seg = {lt.row0, lt.len, lt.len};
      h = lt.h;
      q0 = lt.qb * (32 * NW);
    }
  } else {
    const TileId tile_id = xcd_tile(nqb, H, B);
    if (!tile_id.valid) return;
    h = tile_id.h;
    seg = lpt_segment<64 * NW>(tile_id.rank, B, cu, key_lens, n_pad, s_cu, &s_pick);
    const int fill_img = key_lens == nullptr && B > 1 && B <= kLptMaxB ? s_pick : tile_id.rank;
    fr = fill_range(sc, fill_img, B, tile_id.qb, nqb);
    q0 = tile_id.qb * (32 * NW);
  }
  if (q0 < seg.nq)
    tiled_attention<DH, NW, BN, GATHER>(lds, seg, h, q0, q, k, v, qs, ks, vs, H, scale_log2, out, lse, lse_stride, sc);
  if (sc.y == nullptr) return;
  if (live) {
    const long rows = sc.flat ? (long)sc.N : (long)B * sc.N;
    const long per = (rows + gridDim.x - 1) / gridDim.x;
    const long r0 = min(rows, blockIdx.x * per);
    scatter_fill_rows<__bf16>(sc, r0, min(rows, r0 + per), C, threadIdx.x, 64 * NW);
  } else {
    scatter_fill<__bf16, DH>(sc, fr.b, fr.t0, fr.t1, h, C, threadIdx.x, 64 * NW);
  }
}

// Long segments, two query sub-tiles per wave.  A wave owns 64 queries as two independent
// 32-query chains that share every K and V fragment it reads from LDS: half the LDS operand
// reads per MFMA of the one-chain kernel above, and two independent dependency chains in one
// instruction stream, so the score and P V MFMAs of one chain run under the softmax vector
// work of the other even when the wave has its SIMD to itself (the long-segment launches of
// this path keep one to two waves per SIMD resident, too few to hide a single chain's stalls).
// K and V tiles sit row-major in LDS; V^T fragments come from the transposing LDS read, so
// staging is plain 16-byte copies.  One softmax update per 32 keys and chain.
template <int DH, int BN>
struct Tiled2Lds {
  static constexpr int RS = DH + 8;
  __attribute__((aligned(16))) __bf16 Ks[2][BN * RS];
  __attribute__((aligned(16))) __bf16 Vs[2][BN * RS];
};


// Online-softmax update of one chain over one 32-key sub-tile whose first key is k0 of the tile
// (rem = valid keys of the tile): masks keys past the segment, moves the running max, rescales
// the chain's accumulators when some query's max moved, and leaves the bf16 probabilities in
// the B-operand layout of the P V product.
template <int DH, bool FULL>
__device__ __forceinline__ void chain_softmax(floatx16& s, int k0, int rem, FwdAcc<DH>& acc, float scale_log2,
                                              bf16x8 (&pb)[2], int hh) {
  if (!FULL && rem - k0 < 32) {
#pragma unroll
    for (int r = 0; r < 16; ++r)
      if (k0 + acc_row(r, hh) >= rem) s[r] = -INFINITY;
  }
  float mx = s[0];
#pragma unroll
  for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
  mx = max_across_halves(mx);
  // The rescale is unconditional (alpha = 1 when no max moved): skipping it takes a branch per
  // chain and sub-tile, and every branch ends a scheduling region, which is what keeps the two
  // chains, the fragment reads and the MFMAs from overlapping.  The first sub-tile of a tile always
  // holds a valid key, so m_new is finite and alpha well defined.
  const float m_new = fmaxf(acc.m, mx * scale_log2);
  const float alpha = __builtin_amdgcn_exp2f(acc.m - m_new);
  acc.m = m_new;
#pragma unroll
  for (int d = 0; d < DH / 32; ++d)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc.o[d][r] *= alpha;
  float p[16], psum = 0.f;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    p[r] = __builtin_amdgcn_exp2f(fmaf(s[r], scale_log2, -m_new));
    psum += p[r];
  }
  acc.l = fmaf(acc.l, alpha, psum);
#pragma unroll
  for (int mf = 0; mf < 2; ++mf) {
    floatx8 pf;
#pragma unroll
    for (int j = 0; j < 8; ++j) pf[j] = p[8 * mf + j];
    pb[mf] = float_to_bf16x8(pf);
  }
}

// One tile of NSB*32 keys in LDS (K rows at kbuf, V rows at vbuf, both row stride RS) against
// the wave's NC query chains.  The score MFMAs of sub-tile sb + 1 are issued before the softmax of
// sub-tile sb.  FULL = every key of the tile is valid; otherwise keys >= rem are masked (their K and
// V rows in LDS are zero): all sub-tiles are computed, there is no control flow in the tile.
template <int DH, int RS, int NSB, bool FULL, int NC>
__device__ __forceinline__ void fwd_tile_chains(const __bf16* kbuf, const __bf16* vbuf, int rem,
                                                const bf16x8 (&qf)[NC][DH / 16], FwdAcc<DH> (&acc)[NC],
                                                float scale_log2, int lane) {
  constexpr int KK = DH / 16, DB = DH / 32;
  const int l32 = lane & 31, hh = lane >> 5;
  floatx16 s[2][NC];
  auto scores = [&](int sb, floatx16 (&dst)[NC]) {
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
      for (int r = 0; r < 16; ++r) dst[c][r] = 0.f;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      const bf16x8 a = *reinterpret_cast<const bf16x8*>(&kbuf[(sb * 32 + l32) * RS + kk * 16 + hh * 8]);
#pragma unroll
      for (int c = 0; c < NC; ++c) dst[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[c][kk], dst[c], 0, 0, 0);
    }
  };
  scores(0, s[0]);
#pragma unroll
  for (int sb = 0; sb < NSB; ++sb) {
    const int k0 = sb * 32;
    if (sb + 1 < NSB) scores(sb + 1, s[(sb + 1) & 1]);
    bf16x8 vf[2][DB];                                  // V^T fragments of the sub-tile: read before the softmax needs them
#pragma unroll
    for (int mf = 0; mf < 2; ++mf)
#pragma unroll
      for (int d = 0; d < DB; ++d) vf[mf][d] = transposed_frag_rowmajor<RS>(vbuf, d, k0, mf, lane);
    bf16x8 pb[NC][2];
#pragma unroll
    for (int c = 0; c < NC; ++c) chain_softmax<DH, FULL>(s[sb & 1][c], k0, rem, acc[c], scale_log2, pb[c], hh);
#pragma unroll
    for (int mf = 0; mf < 2; ++mf)
#pragma unroll
      for (int d = 0; d < DB; ++d)
#pragma unroll
        for (int c = 0; c < NC; ++c)
          acc[c].o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[mf][d], pb[c][mf], acc[c].o[d], 0, 0, 0);
  }
}

// The key loop of one wave with NC live query chains (NC = 0: a wave without queries, which only
// helps to stage the tiles).  Every instantiation runs the same sequence of barriers.
template <int DH, int NW, int BN, int NC, bool GATHER>
__device__ __forceinline__ void
tiled2_wave(Tiled2Lds<DH, BN>& lds, KvRowStage<DH, 64 * NW, BN, GATHER>& stage, const Segment& seg, const int32_t* gi,
            const __bf16* kh, const __bf16* vh, long ks, long vs, const bf16x8 (&qf)[2][DH / 16], FwdAcc<DH> (&acc2)[2],
            float scale_log2, int lane) {
  constexpr int RS = DH + 8, NSB = BN / 32, KK = DH / 16, NCA = NC > 0 ? NC : 1;
  bf16x8 q[NCA][KK];
  FwdAcc<DH> acc[NCA];
#pragma unroll
  for (int c = 0; c < NCA; ++c) {
    acc[c].init();
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) q[c][kk] = qf[c][kk];
  }
  const int nt = (seg.nk + BN - 1) / BN;
  for (int t = 0; t + 1 < nt; ++t) {                  // all tiles but the last are full
    const int buf = t & 1;
    stage.load(kh, vh, ks, vs);                        // tile t + 1, whose rows were indexed a tile ago
    stage.index(gi, seg.row0, (t + 2) * BN, seg.nk);
    if (NC > 0) fwd_tile_chains<DH, RS, NSB, true, NCA>(lds.Ks[buf], lds.Vs[buf], BN, q, acc, scale_log2, lane);
    stage.store(lds.Ks[buf ^ 1], lds.Vs[buf ^ 1]);
    __syncthreads();
  }
  if (nt > 0) {
    const int buf = (nt - 1) & 1;
    if (NC > 0)
      fwd_tile_chains<DH, RS, NSB, false, NCA>(lds.Ks[buf], lds.Vs[buf], seg.nk - (nt - 1) * BN, q, acc, scale_log2, lane);
  }
  __syncthreads();                                     // every wave is past its last read of the K buffers
#pragma unroll
  for (int c = 0; c < NCA; ++c)
    if (NC > 0) acc2[c] = acc[c];
}

// The workgroup's work on queries [q0, q0 + 64 NW) of head h of segment seg (q0 < seg.nq).
template <int DH, int NW, int BN, bool GATHER>
__device__ __forceinline__ void
tiled2_attention(Tiled2Lds<DH, BN>& lds, const Segment seg, int h, int q0, const __bf16* __restrict__ q,
                 const __bf16* __restrict__ k, const __bf16* __restrict__ v, long qs, long ks, long vs, int H,
                 float scale_log2, __bf16* __restrict__ out, float* __restrict__ lse, long lse_stride,
                 const Scatter& sc) {
  constexpr int RS = DH + 8, KK = DH / 16;
  static_assert(2 * BN >= 64 * NW, "the K buffers double as the output staging tile");
  const long C = (long)H * DH;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6, l32 = lane & 31, hh = lane >> 5;
  const int qw = q0 + wv * 64;                         // the wave's first query
  const int nc = qw >= seg.nq ? 0 : (qw + 32 < seg.nq ? 2 : 1);      // live chains of this wave
  const __bf16* kh = k + h * DH;
  const __bf16* vh = v + h * DH;
  const int32_t* gi = gather_base<GATHER>(sc, seg.row0);

  bool q_ok[2];
  long q_src[2];
#pragma unroll
  for (int c = 0; c < 2; ++c) {
    const int qi = qw + 32 * c + l32;
    q_ok[c] = qi < seg.nq;
    q_src[c] = q_ok[c] ? source_row(gi, seg.row0, qi) : 0;     // (gathered: an index load, issued first)
  }
  KvRowStage<DH, 64 * NW, BN, GATHER> stage;
  stage.index(gi, seg.row0, 0, seg.nk);
  stage.load(kh, vh, ks, vs);
  stage.index(gi, seg.row0, BN, seg.nk);
  bf16x8 qf[2][KK];
#pragma unroll
  for (int c = 0; c < 2; ++c) load_q_frags<DH>(q + q_src[c] * qs + h * DH, q_ok[c], hh, qf[c]);
  FwdAcc<DH> acc[2];
  acc[0].init();
  acc[1].init();
  stage.store(lds.Ks[0], lds.Vs[0]);
  __syncthreads();
  if (nc == 2) tiled2_wave<DH, NW, BN, 2, GATHER>(lds, stage, seg, gi, kh, vh, ks, vs, qf, acc, scale_log2, lane);
  else if (nc == 1) tiled2_wave<DH, NW, BN, 1, GATHER>(lds, stage, seg, gi, kh, vh, ks, vs, qf, acc, scale_log2, lane);
  else tiled2_wave<DH, NW, BN, 0, GATHER>(lds, stage, seg, gi, kh, vh, ks, vs, qf, acc, scale_log2, lane);

  __bf16* tile = &lds.Ks[0][0] + wv * 64 * RS;
#pragma unroll
  for (int c = 0; c < 2; ++c)
    if (c < nc)
      fwd_park<DH, RS>(acc[c], q_ok[c], seg.nk > 0, tile + c * 32 * RS,
                       lse != nullptr ? lse + h * lse_stride + seg.row0 + qw + 32 * c + l32 : nullptr, l32, hh);
  __syncthreads();
#pragma unroll
  for (int c = 0; c < 2; ++c)
    if (c < nc)
      fwd_flush<DH, RS>(tile + c * 32 * RS, out, sc, seg.row0 + qw + 32 * c, h, C, min(32, seg.nq - qw - 32 * c), lane);
}

template <int DH, int NW, int BN, bool GATHER>
__global__ void __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(2)))
attn_fwd_bf16_tiled2_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k,
                            const __bf16* __restrict__ v, long qs, long ks, long vs,
                            const int32_t* __restrict__ cu, const int32_t* __restrict__ key_lens, int n_pad,
                            int H, float scale_log2, __bf16* __restrict__ out, float* __restrict__ lse,
                            long lse_stride, Scatter sc, int B, int nqb) {
  __shared__ Tiled2Lds<DH, BN> lds;
  __shared__ int s_cu[2 * kLptMaxB + 1];
  __shared__ int s_pick;

  const TileId tile_id = xcd_tile(nqb, H, B);
  if (!tile_id.valid) return;
  const int h = tile_id.h;
  const Segment seg = lpt_segment<64 * NW>(tile_id.rank, B, cu, key_lens, n_pad, s_cu, &s_pick);
  const long C = (long)H * DH;
  const int fill_img = key_lens == nullptr && B > 1 && B <= kLptMaxB ? s_pick : tile_id.rank;
  const FillRange fr = fill_range(sc, fill_img, B, tile_id.qb, nqb);
  const int q0 = tile_id.qb * (64 * NW);
  if (q0 < seg.nq)
    tiled2_attention<DH, NW, BN, GATHER>(lds, seg, h, q0, q, k, v, qs, ks, vs, H, scale_log2, out, lse, lse_stride, sc);
  if (sc.y != nullptr) scatter_fill<__bf16, DH>(sc, fr.b, fr.t0, fr.t1, h, C, threadIdx.x, 64 * NW);
}

// Short segments, wave-autonomous.  ONE wave per (image, head, 32-query block), no
// workgroup barriers, no shared state between waves: the wave streams its segment's K and V
// rows in steps of STEP keys through a private LDS tile (coalesced 16-byte row loads, the next
// step's rows already in flight in registers), reads K fragments back as MFMA A operands
// and V fragments through the transposing LDS read, and keeps the online softmax state in
// registers.  Work units are small (<= n/32 steps each), so the load spreads over all SIMDs
// instead of concentrating a heavy (image, head) on one compute unit.
// The wave's work on queries [q0, q0 + 32) of head h of segment seg (q0 < seg.nq): Ks, Vs are
// its private LDS tiles of STEP rows.
template <int DH, int STEP, bool GATHER>
__device__ __forceinline__ void
wave_attention(__bf16* Ks, __bf16* Vs, const Segment seg, int h, int q0, const __bf16* __restrict__ q,
               const __bf16* __restrict__ k, const __bf16* __restrict__ v, long qs, long ks, long vs, int H,
               float scale_log2, __bf16* __restrict__ out, float* __restrict__ lse, long lse_stride,
               const Scatter& sc) {
  constexpr int RS = DH + 8, KK = DH / 16, DB = DH / 32, CPR = DH / 8;
  constexpr int NSB = STEP / 32;                 // 32-key sub-tiles per step (one softmax update)
  constexpr int LPL = STEP * CPR / 64;           // 16-byte loads per lane per tensor per step
  const long C = (long)H * DH;
  const int lane = threadIdx.x, l32 = lane & 31, hh = lane >> 5;
  const int qi = q0 + l32;
  const bool q_ok = qi < seg.nq;
  const __bf16* kh = k + h * DH;
  const __bf16* vh = v + h * DH;

  // lane -> (row, chunk) of the step's tile: 8 (Dh 64) or 4 (Dh 32) lanes cover one row
  bf16x8 kreg[LPL], vreg[LPL];
  const int32_t* gi = gather_base<GATHER>(sc, seg.row0);
  int tok_rows[LPL];                              // gathered rows only: token rows of the next gload
  int kt_next = 0;                                // first key of the step the next gload fetches
  const int c = lane % CPR, lrow = lane / CPR;
  const uint32_t koff = (uint32_t)lrow * (uint32_t)ks + c * 8, voff = (uint32_t)lrow * (uint32_t)vs + c * 8;
  auto iload = [&](int kt) {                      // issued one step ahead of the row loads that use it
    kt_next = kt;
    if (GATHER) {
#pragma unroll
      for (int t = 0; t < LPL; ++t) {
        const int r = kt + lrow + t * (64 / CPR);
        if (r < seg.nk) tok_rows[t] = gi[r];
      }
    }
  };
  auto gload = [&]() {                            // rows past the segment read as zero
#pragma unroll
    for (int t = 0; t < LPL; ++t) {
      kreg[t] = zero_bf16x8();
      vreg[t] = zero_bf16x8();
      if (kt_next + lrow + t * (64 / CPR) < seg.nk) {
        const __bf16 *kp, *vp;
        if (GATHER) {
          kp = kh + row_offset(tok_rows[t], ks) + c * 8;
          vp = vh + row_offset(tok_rows[t], vs) + c * 8;
        } else {
          const long r = seg.row0 + kt_next + t * (64 / CPR);    // uniform: the lane's part is koff / voff
          kp = kh + r * ks + koff;
          vp = vh + r * vs + voff;
        }
        kreg[t] = *reinterpret_cast<const bf16x8*>(kp);
        vreg[t] = *reinterpret_cast<const bf16x8*>(vp);
      }
    }
  };
  auto lstore = [&]() {
#pragma unroll
    for (int t = 0; t < LPL; ++t) {
      const int i = lane + 64 * t, r = i / CPR, c = i % CPR;
      *reinterpret_cast<bf16x8*>(&Ks[r * RS + c * 8]) = kreg[t];
      *reinterpret_cast<bf16x8*>(&Vs[r * RS + c * 8]) = vreg[t];
    }
  };

  const long q_src = q_ok ? source_row(gi, seg.row0, qi) : 0;   // (gathered: an index load, issued first, so that
  iload(0);                                                      // its wait is the one the first row loads need anyway)
  gload();
  iload(STEP);
  bf16x8 qf[KK];
  load_q_frags<DH>(q + q_src * qs + h * DH, q_ok, hh, qf);
  FwdAcc<DH> acc;
  acc.init();

  for (int kt = 0; kt < seg.nk; kt += STEP) {
    lstore();                                     // this step's rows: registers -> LDS
    if (kt + STEP < seg.nk) {
      gload();                                    // next step's rows: in flight during the math
      iload(kt + 2 * STEP);
    }
    const int rem = seg.nk - kt;
    // scores of the step: S^T = K Q^T, NSB 32-key sub-tiles, one softmax update for all
    floatx16 s[NSB];
    fwd_scores<DH, RS, NSB, false>(Ks, 0, rem, qf, s, l32, hh);
    float mx = s[0][0];
#pragma unroll
    for (int sb = 0; sb < NSB; ++sb)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[sb][r]);
    mx = max_across_halves(mx);
    const float m_new = fmaxf(acc.m, mx * scale_log2);
    if (__ballot(m_new != acc.m) != 0) {
      const float alpha = __builtin_amdgcn_exp2f(acc.m - m_new);
      acc.l *= alpha;
#pragma unroll
      for (int d = 0; d < DB; ++d)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc.o[d][r] *= alpha;
      acc.m = m_new;
    }
    float psum = 0.f;
#pragma unroll
    for (int sb = 0; sb < NSB; ++sb) {
      if (sb * 32 < rem) {
        float p[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          p[r] = __builtin_amdgcn_exp2f(fmaf(s[sb][r], scale_log2, -m_new));
          psum += p[r];
        }
#pragma unroll
        for (int mf = 0; mf < 2; ++mf) {
          floatx8 pf;
#pragma unroll
          for (int j = 0; j < 8; ++j) pf[j] = p[8 * mf + j];
          const bf16x8 pb = float_to_bf16x8(pf);
#pragma unroll
          for (int d = 0; d < DB; ++d) {
            const bf16x8 a = transposed_frag_rowmajor<RS>(Vs, d, sb * 32, mf, lane);
            acc.o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb, acc.o[d], 0, 0, 0);
          }
        }
      }
    }
    acc.l += psum;
  }

  // output: park the 32 x DH tile in the (now free) K tile, then write whole rows
  fwd_park<DH, RS>(acc, q_ok, seg.nk > 0, Ks, lse != nullptr ? lse + h * lse_stride + seg.row0 + qi : nullptr, l32,
                   hh);
  fwd_flush<DH, RS>(Ks, out, sc, seg.row0 + q0, h, C, min(32, seg.nq - q0), lane);
}

template <int DH, int STEP, bool GATHER>
__global__ void __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(STEP == 32 ? 3 : 1)))
attn_fwd_bf16_wave_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k,
                          const __bf16* __restrict__ v, long qs, long ks, long vs,
                          const int32_t* __restrict__ cu, const int32_t* __restrict__ key_lens, int n_pad,
                          int H, float scale_log2, __bf16* __restrict__ out, float* __restrict__ lse,
                          long lse_stride, Scatter sc, int B, int nqb) {
  constexpr int RS = DH + 8;
  __shared__ __attribute__((aligned(16))) __bf16 Ks[STEP * RS];
  __shared__ __attribute__((aligned(16))) __bf16 Vs[STEP * RS];

  const TileId tile_id = xcd_tile(nqb, H, B);
  if (!tile_id.valid) return;
  const int h = tile_id.h, img = tile_id.rank;
  const Segment seg = segment_of(img, cu, key_lens, n_pad);
  const long C = (long)H * DH;
  // this wave's share of the image's bypassing tokens: at once if it has no queries, else last
  const FillRange fr = fill_range(sc, img, B, tile_id.qb, nqb);
  const int q0 = tile_id.qb * 32;
  if (q0 < seg.nq)
    wave_attention<DH, STEP, GATHER>(Ks, Vs, seg, h, q0, q, k, v, qs, ks, vs, H, scale_log2, out, lse, lse_stride, sc);
  if (sc.y != nullptr) scatter_fill<__bf16, DH>(sc, fr.b, fr.t0, fr.t1, h, C, threadIdx.x, 64);
}

// The one-wave work units driven by the selection mask itself: no packing launch precedes this
// kernel.  The wave reads its image's N <= 256 mask bytes, ranks the survivors with ballots and
// writes their token rows, in order, to a list in LDS: exactly the image's part of gather_idx, so
// wave_attention runs on it as on gathered rows (packed position j of the image = row list[j] of
// q, k, v and of y), and the bypass fill tests the mask byte instead of inv_pos.  Costs four byte
// loads and four ballots per wave where the other forms cost a kernel launch.
template <int DH, int STEP>
__global__ void __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(3)))
attn_fwd_bf16_wave_mask_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k,
                               const __bf16* __restrict__ v, long qs, long ks, long vs,
                               const uint8_t* __restrict__ mask, int N, int H, float scale_log2, Scatter sc, int B,
                               int nqb) {
  constexpr int RS = DH + 8;
  __shared__ __attribute__((aligned(16))) __bf16 Ks[STEP * RS];
  __shared__ __attribute__((aligned(16))) __bf16 Vs[STEP * RS];
  __shared__ int32_t list[256];

  const TileId tile_id = xcd_tile(nqb, H, B);
  if (!tile_id.valid) return;
  const int h = tile_id.h, img = tile_id.rank, lane = threadIdx.x;
  const long tok0 = (long)img * N;
  int n = 0;                                       // survivors of the image so far
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int t = lane + 64 * i;
    const bool sel = t < N && mask[tok0 + t] != 0;
    const uint64_t bal = __ballot(sel);
    if (sel) list[n + __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0u))] = (int32_t)(tok0 + t);
    n += __popcll(bal);
  }
  __syncthreads();
  const Segment seg = {0, n, n};                   // packed rows numbered inside the image: row j <-> list[j]
  Scatter scl = sc;
  scl.gather_idx = list;
  const long C = (long)H * DH;
  const FillRange fr = fill_range(sc, img, B, tile_id.qb, nqb);
  const int q0 = tile_id.qb * 32;
  if (q0 < n)
    wave_attention<DH, STEP, true>(Ks, Vs, seg, h, q0, q, k, v, qs, ks, vs, H, scale_log2, nullptr, nullptr, 0, scl);
  scatter_fill<__bf16, DH>(sc, fr.b, fr.t0, fr.t1, h, C, lane, 64);
}

// The same work units, dealt to the compute units by weight (batches of up to 64 images, one
// per lane).  All one-wave workgroups of the launch are resident at once and workgroup j of
// an XCD runs on compute unit j % 32 (the hardware id register says so), so which units get
// the long segments is decided by the numbering alone; numbered blindly, the unluckiest SIMDs
// end a third later than the median.  Here every wave ranks the images by their number of
// 32-key steps (9 classes, one ballot each; images of a class in index order), the (image,
// head) pairs of that ranking are dealt to the XCDs in snake order (an XCD's L2 still holds
// all blocks of its pairs), the XCD's live query blocks are listed heaviest first, and the
// m-th workgroup of a unit takes block r = 32 m + (unit, or 31 - unit for odd m).  Workgroups
// past the live blocks only fill; the bypassing rows of y are shared evenly by all.
// One wave fills the bypassing rows among rows [r0, r1) of y: the lanes test 64 rows at a time
// (one load each), then the wave writes the rows that need it, a lane per 16-byte chunk.
template <typename T>
__device__ __forceinline__ void scatter_fill_rows(const Scatter& sc, long r0, long r1, long C, int lane) {
  constexpr int VE = 16 / sizeof(T);
  const int cpr = (int)(C / VE);
  for (long rb = r0; rb < r1; rb += kWave) {
    const long row = rb + lane;
    uint64_t todo = __ballot(row < r1 && bypasses(sc, row));
    while (todo != 0) {
      const long off0 = (rb + __ffsll((unsigned long long)todo) - 1) * C;
      todo &= todo - 1;
      for (int c = lane; c < cpr; c += kWave) {
        uintx4 val = {0u, 0u, 0u, 0u};
        if (sc.base != nullptr) val = *reinterpret_cast<const uintx4*>(static_cast<const T*>(sc.base) + off0 + c * VE);
        __builtin_nontemporal_store(val, reinterpret_cast<uintx4*>(static_cast<T*>(sc.y) + off0 + c * VE));
      }
    }
  }
}

// No tables are needed: with the pairs sorted by
// class, class c holds the ranked images [A_c, A_c + n_c) (n_c from one ballot), hence the
// pairs [A_c H, (A_c + n_c) H), of which this XCD owns a count with a closed form; every pair
// of class c has exactly c live blocks.  Walking the 9 classes with scalar arithmetic finds
// the class, the pair and the block of number r; the image is the k-th set bit of the class
// ballot and its bounds come by readlane.
__device__ __forceinline__ int pairs_below(int X, int x) {        // XCD x's pairs with index < X
  const int g = X >> 3, s = (g & 1) ? 7 - x : x;
  return g + (s < (X & 7) ? 1 : 0);
}
// Block number r of XCD x -> its segment, head and first query (live = false: past the live
// blocks).  QB = queries per block; a segment's class is its number of blocks.  Every wave of
// the workgroup computes the same answer from its own ballots.
struct LptBlock {
  Segment seg;
  int h, q0;
  bool live;
};
template <int QB>
__device__ __forceinline__ LptBlock lpt64_block(const int32_t* __restrict__ cu, const int32_t* __restrict__ key_lens,
                                                int n_pad, int B, int H, int nqb, int x, int r) {
  const int lane = threadIdx.x & 63;
  const bool padded = key_lens != nullptr;
  int start = 0, len = 0, cls = -1;
  if (lane < B) {
    if (padded) {
      start = lane * n_pad;
      len = min(max(key_lens[lane], 0), n_pad);
    } else {
      start = cu[lane];
      len = cu[lane + 1] - start;
    }
    cls = min((max(len, 0) + QB - 1) / QB, nqb);
  }
  LptBlock blk = {{0, 0, 0}, 0, 0, false};
  int ranked = 0, tiles = 0, g0 = 0;             // images, live blocks, this XCD's pairs of the heavier classes
  for (int c = nqb; c >= 0; --c) {
    const uint64_t bal = __ballot(cls == c);
    const int n_c = __popcll(bal);
    const int per_pair = padded ? nqb : c;
    const int pairs_c = pairs_below((ranked + n_c) * H, x) - pairs_below(ranked * H, x);
    const int tiles_c = pairs_c * per_pair;
    if (r < tiles + tiles_c) {
      const int idx = r - tiles, g = g0 + idx / per_pair;
      const int p = 8 * g + ((g & 1) ? 7 - x : x);
      const int img = kth_set_bit(bal, p / H - ranked);
      blk.h = p % H;
      blk.q0 = (idx % per_pair) * QB;
      blk.seg.row0 = __builtin_amdgcn_readlane(start, img);
      blk.seg.nk = __builtin_amdgcn_readlane(len, img);
      blk.seg.nq = padded ? n_pad : blk.seg.nk;
      blk.live = blk.q0 < blk.seg.nq;
      break;
    }
    tiles += tiles_c;
    g0 += pairs_c;
    ranked += n_c;
  }
  return blk;
}
// the grid of such a launch: 8 XCDs x 32 units x enough rounds for all blocks of the XCD with most pairs
static unsigned lpt64_grid(int B, int H, int nqb) {
  const long g8 = ((long)B * H + 7) / 8;
  return (unsigned)(8 * 32 * ((g8 * nqb + 31) / 32));
}

// Compiled for three waves per SIMD (168 registers at head dim 64, no spills): a ViT-B-shaped
// batch has ~2800 live waves for 1024 SIMDs and then runs in one round instead of two.
template <int DH, int STEP, bool GATHER>
__global__ void __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(3)))
attn_fwd_bf16_wave_lpt64_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k,
                                const __bf16* __restrict__ v, long qs, long ks, long vs,
                                const int32_t* __restrict__ cu, const int32_t* __restrict__ key_lens, int n_pad,
                                int H, float scale_log2, __bf16* __restrict__ out, float* __restrict__ lse,
                                long lse_stride, Scatter sc, int B, int nqb) {
  constexpr int RS = DH + 8;
  __shared__ __attribute__((aligned(16))) __bf16 Ks[STEP * RS];
  __shared__ __attribute__((aligned(16))) __bf16 Vs[STEP * RS];
  const int x = blockIdx.x & 7, j = blockIdx.x >> 3, unit = j & 31, m = j >> 5;
  const LptBlock blk = lpt64_block<32>(cu, key_lens, n_pad, B, H, nqb, x, m * 32 + ((m & 1) ? 31 - unit : unit));
  if (blk.live)
    wave_attention<DH, STEP, GATHER>(Ks, Vs, blk.seg, blk.h, blk.q0, q, k, v, qs, ks, vs, H, scale_log2, out, lse, lse_stride,
                             sc);
  if (sc.y != nullptr) {
    const long rows = sc.flat ? (long)sc.N : (long)B * sc.N, per = (rows + gridDim.x - 1) / gridDim.x;
    const long r0 = min(rows, blockIdx.x * per), r1 = min(rows, r0 + per);
    scatter_fill_rows<__bf16>(sc, r0, r1, (long)H * DH, threadIdx.x);
  }
}

// Short segments (every segment <= NKMAX keys).  ONE workgroup per (image, head): all K / V
// rows of the segment are staged once (each element is read from memory exactly once per
// head), one barrier, then wave w owns queries [32w, 32w+32) and walks the keys in LDS with
// no further synchronisation.  No workgroup is launched for nothing.
template <int DH, int NKMAX, bool GATHER>
__global__ void __launch_bounds__(2 * NKMAX)
attn_fwd_bf16_whole_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k,
                           const __bf16* __restrict__ v, long qs, long ks, long vs,
                           const int32_t* __restrict__ cu, const int32_t* __restrict__ key_lens, int n_pad,
                           int H, float scale_log2, __bf16* __restrict__ out, float* __restrict__ lse,
                           long lse_stride, Scatter sc) {
  constexpr int THREADS = 2 * NKMAX;                       // one wave per 32 queries
  constexpr int RS = DH + 8, TS = transposed_stride(NKMAX);
  constexpr int TILE = NKMAX < 128 ? NKMAX : 128;           // keys per softmax update
  constexpr int NSB = TILE / 32;
  __shared__ __attribute__((aligned(16))) __bf16 Ks[NKMAX * RS];
  __shared__ __attribute__((aligned(16))) __bf16 Vt[DH * TS];

  const int h = blockIdx.x;
  Segment seg = segment_of(blockIdx.y, cu, key_lens, n_pad);
  seg.nq = min(seg.nq, NKMAX);   // never index past the LDS tile, whatever cu_seqlens holds
  seg.nk = min(seg.nk, NKMAX);
  const long C = (long)H * DH;
  const FillRange fr = fill_range(sc, blockIdx.y, gridDim.y, 0, 1);
  if (seg.nq <= 0) {
    if (sc.y != nullptr) scatter_fill<__bf16, DH>(sc, fr.b, fr.t0, fr.t1, h, C, threadIdx.x, THREADS);
    return;
  }
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6, l32 = lane & 31, hh = lane >> 5;
  const int qi = wv * 32 + l32;
  const bool wave_live = wv * 32 < seg.nq;
  const bool q_ok = qi < seg.nq;

  const int32_t* gi = gather_base<GATHER>(sc, seg.row0);
  KvStage<DH, THREADS, (NKMAX / 2) * (DH / 8), GATHER> stage;
  stage.index(gi, seg.row0, 0, seg.nk);
  stage.load(k + h * DH, v + h * DH, ks, vs);
  bf16x8 qf[DH / 16];
  load_q_frags<DH>(q + (q_ok ? source_row(gi, seg.row0, qi) : 0) * qs + h * DH, q_ok, hh, qf);
  FwdAcc<DH> acc;
  acc.init();
  stage.template store<RS, TS>(Ks, Vt, 0);
  __syncthreads();
  // the rows that bypass attention are filled by the waves that own no queries while the
  // others compute; if every wave has queries (few rows bypass then) all do it at the end
  const int live_threads = ((seg.nq + 31) / 32) * 64;
  if (!wave_live && sc.y != nullptr)
    scatter_fill<__bf16, DH>(sc, fr.b, fr.t0, fr.t1, h, C, threadIdx.x - live_threads, THREADS - live_threads);
  if (wave_live) {
    for (int kt = 0; kt < seg.nk; kt += TILE) {
      const int rem = seg.nk - kt;
      if (rem >= TILE) fwd_process_tile<DH, RS, TS, NSB, true>(Ks + kt * RS, Vt, kt, TILE, qf, acc, scale_log2, l32, hh);
      else fwd_process_tile<DH, RS, TS, NSB, false>(Ks + kt * RS, Vt, kt, rem, qf, acc, scale_log2, l32, hh);
    }
  }
  __syncthreads();                       // all waves are done reading K: its rows become the output tile
  __bf16* tile = Ks + wv * 32 * RS;
  if (wave_live)
    fwd_park<DH, RS>(acc, q_ok, seg.nk > 0, tile, lse != nullptr ? lse + h * lse_stride + seg.row0 + qi : nullptr,
                     l32, hh);
  __syncthreads();
  if (wave_live) fwd_flush<DH, RS>(tile, out, sc, seg.row0 + wv * 32, h, C, min(32, seg.nq - wv * 32), lane);
  if (sc.y != nullptr && live_threads >= THREADS)
    scatter_fill<__bf16, DH>(sc, fr.b, fr.t0, fr.t1, h, C, threadIdx.x, THREADS);
}

// ------------------------------------------------------------------------------- fp32
// G lanes share one query: lane g takes the keys j = g (mod G) of every tile with its own
// online-softmax state, the G partial states are merged with a butterfly of shuffles at the
// end, and every lane writes DH / G of the query's output elements.
template <int DH>
__global__ void __launch_bounds__(128)
attn_fwd_f32_kernel(const float* __restrict__ q, const float* __restrict__ k,
                    const float* __restrict__ v, long qs, long ks, long vs, const int32_t* __restrict__ cu,
                    const int32_t* __restrict__ key_lens, int n_pad, int H, float scale,
                    float* __restrict__ out, float* __restrict__ lse, long lse_stride, Scatter sc) {
  constexpr int THREADS = 128, G = 8, BM = THREADS / G, BN = 32, JPL = BN / G, EPL = DH / G;
  static_assert(EPL % 4 == 0, "every lane writes whole 16-byte pieces");
  __shared__ __attribute__((aligned(16))) float Ks[BN * DH];
  __shared__ __attribute__((aligned(16))) float Vs[BN * DH];

  const int h = blockIdx.y;
  const long C = (long)H * DH;
  // cu == key_lens == nullptr: no packing index exists; the first wave derives the image's packing
  // order from its n_pad <= 256 mask bytes (see attn_fwd_bf16_wave_mask_kernel) and the workgroup
  // works on that list as on gathered rows
  __shared__ int32_t list[256];
  __shared__ int s_n;
  const bool from_mask = cu == nullptr && key_lens == nullptr;
  Segment seg;
  if (from_mask) {
    if (threadIdx.x < kWave) {
      const long tok0 = (long)blockIdx.z * n_pad;
      int n = 0;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int t = (int)threadIdx.x + 64 * i;
        const bool sel = t < n_pad && sc.mask[tok0 + t] != 0;
        const uint64_t bal = __ballot(sel);
        if (sel) list[n + __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0u))] = (int32_t)(tok0 + t);
        n += __popcll(bal);
      }
      if (threadIdx.x == 0) s_n = n;
    }
    __syncthreads();
    seg = {0, s_n, s_n};
    sc.gather_idx = list;
  } else {
    seg = segment_of(blockIdx.z, cu, key_lens, n_pad);
  }
  if (sc.y != nullptr) {
    const FillRange fr = fill_range(sc, blockIdx.z, gridDim.z, blockIdx.x, gridDim.x);
    scatter_fill<float, DH>(sc, fr.b, fr.t0, fr.t1, h, C, threadIdx.x, THREADS);
  }
  const int q0 = blockIdx.x * BM;
  if (q0 >= seg.nq) return;
  const int tid = threadIdx.x, g = tid % G;
  const int qi = q0 + tid / G;
  const bool q_ok = qi < seg.nq;

  float qr[DH], o[DH];
#pragma unroll
  for (int d = 0; d < DH; ++d) { qr[d] = 0.f; o[d] = 0.f; }
  const int32_t* gi = sc.gathered ? sc.gather_idx + seg.row0 : nullptr;
  if (q_ok) {
    const float* qp = q + source_row(gi, seg.row0, qi) * qs + h * DH;
#pragma unroll
    for (int d = 0; d < DH; d += 4) {
      const floatx4 t = *reinterpret_cast<const floatx4*>(qp + d);
      qr[d] = t[0] * scale; qr[d + 1] = t[1] * scale; qr[d + 2] = t[2] * scale; qr[d + 3] = t[3] * scale;
    }
  }
  float m = -INFINITY, l = 0.f;

  for (int kt = 0; kt < seg.nk; kt += BN) {
    __syncthreads();
    for (int i = tid; i < BN * DH / 4; i += THREADS) {
      const int r = i / (DH / 4), c = i % (DH / 4);
      floatx4 kv = {0.f, 0.f, 0.f, 0.f}, vv = kv;
      if (kt + r < seg.nk) {
        const long src = source_row(gi, seg.row0, kt + r);
        kv = *reinterpret_cast<const floatx4*>(k + src * ks + h * DH + c * 4);
        vv = *reinterpret_cast<const floatx4*>(v + src * vs + h * DH + c * 4);
      }
      *reinterpret_cast<floatx4*>(&Ks[r * DH + c * 4]) = kv;
      *reinterpret_cast<floatx4*>(&Vs[r * DH + c * 4]) = vv;
    }
    __syncthreads();
    const int kn = min(BN, seg.nk - kt);
    float s[JPL];
    float mx = -INFINITY;
#pragma unroll
    for (int jj = 0; jj < JPL; ++jj) {
      const int j = jj * G + g;
      float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
#pragma unroll
      for (int d = 0; d < DH; d += 4) {
        const floatx4 kv = *reinterpret_cast<const floatx4*>(&Ks[j * DH + d]);
        a0 = fmaf(qr[d], kv[0], a0);
        a1 = fmaf(qr[d + 1], kv[1], a1);
        a2 = fmaf(qr[d + 2], kv[2], a2);
        a3 = fmaf(qr[d + 3], kv[3], a3);
      }
      s[jj] = j < kn ? (a0 + a1) + (a2 + a3) : -INFINITY;
      mx = fmaxf(mx, s[jj]);
    }
    const float m_new = fmaxf(m, mx);
    if (m_new > -INFINITY) {          // this lane has seen at least one key
      const float alpha = expf(m - m_new);
      l *= alpha;
#pragma unroll
      for (int d = 0; d < DH; ++d) o[d] *= alpha;
#pragma unroll
      for (int jj = 0; jj < JPL; ++jj) {
        const int j = jj * G + g;
        const float p = expf(s[jj] - m_new);
        l += p;
#pragma unroll
        for (int d = 0; d < DH; d += 4) {
          const floatx4 vv = *reinterpret_cast<const floatx4*>(&Vs[j * DH + d]);
          o[d] = fmaf(p, vv[0], o[d]);
          o[d + 1] = fmaf(p, vv[1], o[d + 1]);
          o[d + 2] = fmaf(p, vv[2], o[d + 2]);
          o[d + 3] = fmaf(p, vv[3], o[d + 3]);
        }
      }
      m = m_new;
    }
  }
  // merge the G partial states of the query (all G lanes end with the merged state)
#pragma unroll
  for (int off = G / 2; off > 0; off >>= 1) {
    const float m_o = __shfl_xor(m, off, kWave), l_o = __shfl_xor(l, off, kWave);
    const float m_new = fmaxf(m, m_o);
    const float a = m > -INFINITY ? expf(m - m_new) : 0.f;
    const float b = m_o > -INFINITY ? expf(m_o - m_new) : 0.f;
    l = l * a + l_o * b;
#pragma unroll
    for (int d = 0; d < DH; ++d) o[d] = o[d] * a + __shfl_xor(o[d], off, kWave) * b;
    m = m_new;
  }
  if (!q_ok) return;
  const float inv = seg.nk > 0 ? 1.0f / l : 0.f;
  float* op = out != nullptr ? out + (seg.row0 + qi) * C + h * DH : nullptr;
  const long yoff = sc.y != nullptr ? (long)sc.gather_idx[seg.row0 + qi] * C + h * DH : 0;
#pragma unroll
  for (int d0 = 0; d0 < DH; d0 += 4) {
    if (d0 / EPL != g) continue;      // this lane's share of the row
    floatx4 t = {o[d0] * inv, o[d0 + 1] * inv, o[d0 + 2] * inv, o[d0 + 3] * inv};
    if (op != nullptr) *reinterpret_cast<floatx4*>(op + d0) = t;
    if (sc.y != nullptr) {
      if (sc.base != nullptr) t += *reinterpret_cast<const floatx4*>(static_cast<const float*>(sc.base) + yoff + d0);
      __builtin_nontemporal_store(t, reinterpret_cast<floatx4*>(static_cast<float*>(sc.y) + yoff + d0));
    }
  }
  if (lse != nullptr && g == 0) lse[h * lse_stride + seg.row0 + qi] = seg.nk > 0 ? m + logf(l) : -INFINITY;
}

// ------------------------------------------------------------------------------- host
static int attention_common(const char* fn, const void* q, const void* k, const void* v,
                            int64_t q_stride, int64_t k_stride, int64_t v_stride, const int32_t* cu, const int32_t* key_lens, int B,
                            int n_max, int H, int Dh, int dtype, float softmax_scale, void* out,
                            float* lse, const Scatter& sc, void* stream) {
  SPA_REQUIRE(q && k && v && (out || sc.y) && (cu || key_lens), SPA_ERR_INVALID_ARG, "%s: null pointer", fn);
  SPA_REQUIRE(B >= 1 && n_max >= 1 && H >= 1, SPA_ERR_INVALID_ARG, "%s: B, max_seqlen, H must be >= 1", fn);
  SPA_REQUIRE((long)B * n_max < 2147483647L, SPA_ERR_INVALID_ARG, "%s: B*max_seqlen must be < 2^31", fn);
  SPA_REQUIRE(B <= 65535 && H <= 65535, SPA_ERR_INVALID_ARG, "%s: B and H must be <= 65535", fn);
  SPA_REQUIRE(((long)H * B + 8) * ((n_max + 31) / 32) < 2147483647L, SPA_ERR_INVALID_ARG,
              "%s: B*H*ceil(max_seqlen/32) must be < 2^31", fn);
  SPA_REQUIRE(dtype == SPA_F32 || dtype == SPA_BF16, SPA_ERR_UNSUPPORTED, "%s: unknown dtype %d", fn, dtype);
  SPA_REQUIRE(Dh == 32 || Dh == 64, SPA_ERR_UNSUPPORTED, "%s: head dim %d not supported (32 or 64)", fn, Dh);
  const int64_t strides[3] = {q_stride, k_stride, v_stride};
  for (int64_t rs : strides) {
    SPA_REQUIRE(rs >= (int64_t)H * Dh, SPA_ERR_INVALID_ARG, "%s: row stride %ld < H*Dh", fn, (long)rs);
    // the kernels keep a lane's offset inside a tile (up to 128 rows) in 32 bits
    SPA_REQUIRE(rs < (1 << 24), SPA_ERR_INVALID_ARG, "%s: row stride %ld must be < 2^24 elements", fn, (long)rs);
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
    const dim3 grid((n_max + 15) / 16, H, B), block(128);   // 16 queries per workgroup, 8 lanes each
#define SPA_F32_LAUNCH(D)                                                                                \
  hipLaunchKernelGGL((attn_fwd_f32_kernel<D>), grid, block, 0, st, (const float*)q, (const float*)k,    \
                     (const float*)v, (long)q_stride, (long)k_stride, (long)v_stride, cu, key_lens, n_max, H, scale, (float*)out, lse, \
                     lse_stride, sc)
    if (Dh == 32) SPA_F32_LAUNCH(32); else SPA_F32_LAUNCH(64);
#undef SPA_F32_LAUNCH
  } else {
    const float scale_log2 = scale * 1.4426950408889634f;
#define SPA_ARGS_PLAIN SPA_ARGS
#define SPA_ARGS_BN SPA_ARGS, B, nqb
#define SPA_LAUNCH(KERNEL, GRID, BLOCK, ARGS, ...)                                                            \
  do {                                                                                                        \
    if (sc.gathered) hipLaunchKernelGGL((KERNEL<__VA_ARGS__, true>), GRID, BLOCK, 0, st, ARGS);               \
    else hipLaunchKernelGGL((KERNEL<__VA_ARGS__, false>), GRID, BLOCK, 0, st, ARGS);                          \
  } while (0)
#define SPA_ARGS                                                                                              \
  (const __bf16*)q, (const __bf16*)k, (const __bf16*)v, (long)q_stride, (long)k_stride, (long)v_stride, cu,   \
      key_lens, n_max, H, scale_log2, (__bf16*)out, lse, lse_stride, sc
    // options attn_fwd_cfg (forces the tiled kernel with that launch shape), attn_fwd_short and
    // attn_fwd_wave_max select among the kernels below; unset, the measured best is taken
    const Options& opt = options();
    int NW = opt.fwd_nw, BN = opt.fwd_bn;
    const bool use_whole = opt.fwd_whole;
    const int wave_max = opt.fwd_wave_max;
    if (NW == 0 && n_max <= wave_max && !use_whole) {
      // short segments: one wave per (image, head, 32 queries)
      const int nqb = (n_max + 31) / 32;
      const dim3 grid(xcd_grid(nqb, H, B));
      // default: blocks dealt to the compute units by weight ("plain": numbered blindly)
      const bool step64 = opt.fwd_step64, plain = opt.fwd_plain;
      if (!step64 && !plain && B <= kWave) {
        const dim3 lgrid(lpt64_grid(B, H, nqb));
        if (Dh == 32) SPA_LAUNCH(attn_fwd_bf16_wave_lpt64_kernel, lgrid, dim3(64), SPA_ARGS_BN, 32, 32);
        else SPA_LAUNCH(attn_fwd_bf16_wave_lpt64_kernel, lgrid, dim3(64), SPA_ARGS_BN, 64, 32);
      } else if (Dh == 32) {
        if (step64) SPA_LAUNCH(attn_fwd_bf16_wave_kernel, grid, dim3(64), SPA_ARGS_BN, 32, 64);
        else SPA_LAUNCH(attn_fwd_bf16_wave_kernel, grid, dim3(64), SPA_ARGS_BN, 32, 32);
      } else {
        if (step64) SPA_LAUNCH(attn_fwd_bf16_wave_kernel, grid, dim3(64), SPA_ARGS_BN, 64, 64);
        else SPA_LAUNCH(attn_fwd_bf16_wave_kernel, grid, dim3(64), SPA_ARGS_BN, 64, 32);
      }
    } else if (NW == 0 && n_max <= 256) {
      // short segments: one workgroup per (image, head), whole segment in LDS
      const dim3 grid(H, B);
#define SPA_WHOLE(D)                                                                                          \
  do {                                                                                                        \
    if (n_max <= 64) SPA_LAUNCH(attn_fwd_bf16_whole_kernel, grid, dim3(128), SPA_ARGS_PLAIN, D, 64);       \
    else if (n_max <= 128) SPA_LAUNCH(attn_fwd_bf16_whole_kernel, grid, dim3(256), SPA_ARGS_PLAIN, D, 128); \
    else SPA_LAUNCH(attn_fwd_bf16_whole_kernel, grid, dim3(512), SPA_ARGS_PLAIN, D, 256);          \
  } while (0)
      if (Dh == 32) SPA_WHOLE(32); else SPA_WHOLE(64);
#undef SPA_WHOLE
    } else if (NW == 0 && opt.fwd_long_two) {
      // long segments: two query chains per wave, 2 waves x 64 queries per workgroup, 64-key tiles
      const int nqb = (n_max + 127) / 128;
      const dim3 grid(xcd_grid(nqb, H, B)), block(128);
      if (Dh == 32) SPA_LAUNCH(attn_fwd_bf16_tiled2_kernel, grid, block, SPA_ARGS_BN, 32, 2, 64);
      else SPA_LAUNCH(attn_fwd_bf16_tiled2_kernel, grid, block, SPA_ARGS_BN, 64, 2, 64);
    } else {
      if (NW == 0) { NW = 4; BN = 128; }
      const int nqb = (n_max + 32 * NW - 1) / (32 * NW);
      const dim3 grid(xcd_grid(nqb, H, B)), block(64 * NW);
#define SPA_TILED(D)                                                                                          \
  do {                                                                                                        \
    if (NW == 2 && BN == 64) SPA_LAUNCH(attn_fwd_bf16_tiled_kernel, grid, block, SPA_ARGS_BN, D, 2, 64);        \
    else if (NW == 2) SPA_LAUNCH(attn_fwd_bf16_tiled_kernel, grid, block, SPA_ARGS_BN, D, 2, 128);              \
    else if (BN == 64) SPA_LAUNCH(attn_fwd_bf16_tiled_kernel, grid, block, SPA_ARGS_BN, D, 4, 64);              \
    else SPA_LAUNCH(attn_fwd_bf16_tiled_kernel, grid, block, SPA_ARGS_BN, D, 4, 128);           \
  } while (0)
      if (Dh == 32) SPA_TILED(32); else SPA_TILED(64);
#undef SPA_TILED
    }
#undef SPA_ARGS
#undef SPA_ARGS_PLAIN
#undef SPA_ARGS_BN
#undef SPA_LAUNCH
  }
  return check_launch(fn);
}

}  // namespace spa

using namespace spa;

extern "C" int spa_packed_attention(const void* q, const void* k, const void* v, int64_t q_row_stride,
                                    int64_t k_row_stride, int64_t v_row_stride, const int32_t* cu_seqlens, int B, int max_seqlen, int H, int Dh,
                                    int dtype, float softmax_scale, void* out, float* lse, void* stream) {
  SPA_REQUIRE(cu_seqlens, SPA_ERR_INVALID_ARG, "spa_packed_attention: cu_seqlens is null");
  SPA_REQUIRE(out, SPA_ERR_INVALID_ARG, "spa_packed_attention: out is null");
  const Scatter none = {nullptr, nullptr, nullptr, nullptr, 0, 0, 0, nullptr};
  return attention_common("spa_packed_attention", q, k, v, q_row_stride, k_row_stride, v_row_stride, cu_seqlens, nullptr, B, max_seqlen,
                          H, Dh, dtype, softmax_scale, out, lse, none, stream);
}

extern "C" int spa_padded_attention(const void* q, const void* k, const void* v, int64_t row_stride,
                                    const int32_t* seqlens, int B, int n_pad, int H, int Dh, int dtype,
                                    float softmax_scale, void* out, void* stream) {
  SPA_REQUIRE(seqlens, SPA_ERR_INVALID_ARG, "spa_padded_attention: seqlens is null");
  SPA_REQUIRE(out, SPA_ERR_INVALID_ARG, "spa_padded_attention: out is null");
  const Scatter none = {nullptr, nullptr, nullptr, nullptr, 0, 0, 0, nullptr};
  return attention_common("spa_padded_attention", q, k, v, row_stride, row_stride, row_stride, nullptr, seqlens, B, n_pad, H, Dh,
                          dtype, softmax_scale, out, nullptr, none, stream);
}

extern "C" int spa_packed_attention_unpack(const void* q, const void* k, const void* v, int64_t q_row_stride,
                                           int64_t k_row_stride, int64_t v_row_stride,
                                           const int32_t* cu_seqlens, const int32_t* gather_idx,
                                           const int32_t* inv_pos, const void* base, int B, int N, int H, int Dh,
                                           int dtype, float softmax_scale, void* out, float* lse, void* y,
                                           void* stream) {
  SPA_REQUIRE(cu_seqlens && gather_idx && inv_pos && y, SPA_ERR_INVALID_ARG,
              "spa_packed_attention_unpack: null pointer");
  SPA_REQUIRE(aligned16(y) && aligned16(base), SPA_ERR_INVALID_ARG,
              "spa_packed_attention_unpack: y / base not 16-byte aligned");
  const Scatter sc = {gather_idx, inv_pos, base, y, N, 0, 0, nullptr};
  return attention_common("spa_packed_attention_unpack", q, k, v, q_row_stride, k_row_stride, v_row_stride,
                          cu_seqlens, nullptr, B, N, H, Dh, dtype, softmax_scale, out, lse, sc, stream);
}

extern "C" int spa_gathered_attention_unpack(const void* q, const void* k, const void* v, int64_t q_row_stride,
                                             int64_t k_row_stride, int64_t v_row_stride,
                                             const int32_t* cu_seqlens, const int32_t* gather_idx,
                                             const int32_t* inv_pos, const void* base, int B, int N, int H, int Dh,
                                             int dtype, float softmax_scale, void* out, float* lse, void* y,
                                             void* stream) {
  const char* fn = "spa_gathered_attention_unpack";
  SPA_REQUIRE(cu_seqlens && gather_idx && inv_pos && y, SPA_ERR_INVALID_ARG, "%s: null pointer", fn);
  SPA_REQUIRE(aligned16(y) && aligned16(base), SPA_ERR_INVALID_ARG, "%s: y / base not 16-byte aligned", fn);
  const Scatter sc = {gather_idx, inv_pos, base, y, N, 0, 1, nullptr};
  return attention_common(fn, q, k, v, q_row_stride, k_row_stride, v_row_stride, cu_seqlens, nullptr, B, N, H, Dh,
                          dtype, softmax_scale, out, lse, sc, stream);
}

extern "C" int spa_selected_attention_unpack(const void* q, const void* k, const void* v, int64_t q_row_stride,
                                             int64_t k_row_stride, int64_t v_row_stride, const uint8_t* mask,
                                             const void* base, int B, int N, int H, int Dh, int dtype,
                                             float softmax_scale, void* y, void* stream) {
  const char* fn = "spa_selected_attention_unpack";
  SPA_REQUIRE(q && k && v && mask && y, SPA_ERR_INVALID_ARG, "%s: null pointer", fn);
  SPA_REQUIRE(B >= 1 && N >= 1 && H >= 1, SPA_ERR_INVALID_ARG, "%s: B, N, H must be >= 1", fn);
  SPA_REQUIRE(dtype == SPA_F32 || dtype == SPA_BF16, SPA_ERR_UNSUPPORTED, "%s: unknown dtype %d", fn, dtype);
  SPA_REQUIRE(N <= 256, SPA_ERR_UNSUPPORTED, "%s: N = %d > 256 tokens per image (use index-only spa_pack + spa_gathered_attention_unpack)", fn, N);
  SPA_REQUIRE(Dh == 32 || Dh == 64, SPA_ERR_UNSUPPORTED, "%s: head dim %d not supported (32 or 64)", fn, Dh);
  SPA_REQUIRE(B <= 65535 && H <= 65535 && (long)B * N < 2147483647L, SPA_ERR_INVALID_ARG, "%s: B, H <= 65535 and B*N < 2^31", fn);
  SPA_REQUIRE(((long)H * B + 8) * ((N + 31) / 32) < 2147483647L, SPA_ERR_INVALID_ARG, "%s: B*H*ceil(N/32) must be < 2^31", fn);
  const int64_t strides[3] = {q_row_stride, k_row_stride, v_row_stride};
  for (int64_t rs : strides) {
    SPA_REQUIRE(rs >= (int64_t)H * Dh && rs < (1 << 24), SPA_ERR_INVALID_ARG, "%s: row stride %ld outside [H*Dh, 2^24)", fn, (long)rs);
    SPA_REQUIRE((rs * elem_size(dtype)) % 16 == 0, SPA_ERR_INVALID_ARG, "%s: row stride is not a multiple of 16 bytes", fn);
  }
  SPA_REQUIRE(aligned16(q) && aligned16(k) && aligned16(v) && aligned16(y) && aligned16(base), SPA_ERR_INVALID_ARG,
              "%s: q / k / v / y / base not 16-byte aligned", fn);
  SPA_REQUIRE(softmax_scale >= 0.f && std::isfinite(softmax_scale), SPA_ERR_INVALID_ARG,
              "%s: softmax_scale must be finite and >= 0 (0 = 1/sqrt(Dh))", fn);
  const float scale = softmax_scale > 0.f ? softmax_scale : 1.0f / std::sqrt((float)Dh);
  const float scale_log2 = scale * 1.4426950408889634f;
  const Scatter sc = {nullptr, nullptr, base, y, N, 0, 1, mask};
  if (dtype == SPA_F32) {
    const dim3 grid((N + 15) / 16, H, B), block(128);   // 16 queries per workgroup, 8 lanes each
    if (Dh == 32)
      hipLaunchKernelGGL((attn_fwd_f32_kernel<32>), grid, block, 0, as_stream(stream), (const float*)q, (const float*)k,
                         (const float*)v, (long)q_row_stride, (long)k_row_stride, (long)v_row_stride, nullptr, nullptr, N,
                         H, scale, (float*)nullptr, (float*)nullptr, 0L, sc);
    else
      hipLaunchKernelGGL((attn_fwd_f32_kernel<64>), grid, block, 0, as_stream(stream), (const float*)q, (const float*)k,
                         (const float*)v, (long)q_row_stride, (long)k_row_stride, (long)v_row_stride, nullptr, nullptr, N,
                         H, scale, (float*)nullptr, (float*)nullptr, 0L, sc);
    return check_launch(fn);
  }
  const int nqb = (N + 31) / 32;
  const dim3 grid(xcd_grid(nqb, H, B));
#define SPA_SEL(D)                                                                                              \
  hipLaunchKernelGGL((attn_fwd_bf16_wave_mask_kernel<D, 32>), grid, dim3(64), 0, as_stream(stream), (const __bf16*)q, \
                     (const __bf16*)k, (const __bf16*)v, (long)q_row_stride, (long)k_row_stride, (long)v_row_stride,    \
                     mask, N, H, scale_log2, sc, B, nqb)
  if (Dh == 32) SPA_SEL(32); else SPA_SEL(64);
#undef SPA_SEL
  return check_launch(fn);
}

extern "C" int spa_segment_attention_unpack(const void* q, const void* k, const void* v, int64_t q_row_stride,
                                            int64_t k_row_stride, int64_t v_row_stride,
                                            const int32_t* seg_cu_seqlens, int n_segments, int max_seqlen,
                                            const int32_t* gather_idx, const int32_t* inv_pos, const void* base,
                                            int64_t rows, int H, int Dh, int dtype, float softmax_scale,
                                            void* out, float* lse, void* y, void* stream) {
  const char* fn = "spa_segment_attention_unpack";
  SPA_REQUIRE(seg_cu_seqlens && gather_idx && inv_pos && y, SPA_ERR_INVALID_ARG, "%s: null pointer", fn);
  SPA_REQUIRE(rows >= 1 && rows < 2147483647L, SPA_ERR_INVALID_ARG, "%s: rows must be in [1, 2^31)", fn);
  SPA_REQUIRE(aligned16(y) && aligned16(base), SPA_ERR_INVALID_ARG, "%s: y / base not 16-byte aligned", fn);
  const Scatter sc = {gather_idx, inv_pos, base, y, (int)rows, 1, 0, nullptr};
  return attention_common(fn, q, k, v, q_row_stride, k_row_stride, v_row_stride, seg_cu_seqlens, nullptr, n_segments,
                          max_seqlen, H, Dh, dtype, softmax_scale, out, lse, sc, stream);
}
