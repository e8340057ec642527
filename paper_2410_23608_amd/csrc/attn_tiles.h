// LDS tile staging for the packed-attention kernels (bf16, gfx950).
//
// Two layouts are used.  Row-major [rows][DH + 8]: feeds MFMA operands whose k-dimension is
// the head dim (a lane reads 16 contiguous bytes of one row; the 16-byte row pad makes those
// reads bank-conflict free).  Transposed [DH][rows + 4]: feeds operands whose k-dimension is
// the token index (a lane reads 4 consecutive tokens of one head-dim column as 8 bytes).
#pragma once

#include "spa_common.h"

namespace spa {

template <int DH> struct TileShape {
  static constexpr int kRowStride = DH + 8;        // elements, row-major tile
  static constexpr int kChunksPerRow = DH / 8;     // 16-byte chunks per row
};

constexpr int transposed_stride(int rows) { return rows + 4; }

__device__ __forceinline__ bf16x8 zero_bf16x8() {
  bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
  return z;
}

// Stage `ROWS` rows (row r = global row row0 + r, zero beyond n_valid) of a [*, stride]
// tensor's head slice into LDS: row-major into `rm` (if kRowMajor) and/or transposed into
// `tr` (if kTransposed).  Called by all THREADS threads of the workgroup.
template <int DH, int ROWS, int THREADS, bool kRowMajor, bool kTransposed>
__device__ __forceinline__ void stage_tile(const __bf16* __restrict__ src, long row0, int n_valid,
                                           long stride, __bf16* rm, __bf16* tr) {
  constexpr int CPR = DH / 8;
  constexpr int RS = DH + 8;
  constexpr int TS = transposed_stride(ROWS);
  // one task = one 16-byte chunk column of a PAIR of rows, so that transposed stores are
  // 4 bytes (two tokens of one head-dim column)
  constexpr int TASKS = (ROWS / 2) * CPR;
  for (int i = threadIdx.x; i < TASKS; i += THREADS) {
    const int c = i % CPR, g = i / CPR;
    const int r0 = 2 * g;
    bf16x8 a = zero_bf16x8(), b = zero_bf16x8();
    if (r0 < n_valid) a = *reinterpret_cast<const bf16x8*>(src + (row0 + r0) * stride + c * 8);
    if (r0 + 1 < n_valid) b = *reinterpret_cast<const bf16x8*>(src + (row0 + r0 + 1) * stride + c * 8);
    if (kRowMajor) {
      *reinterpret_cast<bf16x8*>(&rm[r0 * RS + c * 8]) = a;
      *reinterpret_cast<bf16x8*>(&rm[(r0 + 1) * RS + c * 8]) = b;
    }
    if (kTransposed) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        bf16x2 pr = {a[e], b[e]};
        *reinterpret_cast<bf16x2*>(&tr[(c * 8 + e) * TS + r0]) = pr;
      }
    }
  }
}

// A-operand fragment from a transposed tile: head-dim row `d`, the 8 token slots that pair
// with accumulator registers 8*mf .. 8*mf+7 of a 32x32 tile whose rows are tokens
// (token = 16*mf + 8*(j/4) + 4*hh + j%4 for slot j of half hh).
template <int TS>
__device__ __forceinline__ bf16x8 transposed_frag(const __bf16* tr, int d, int tok0, int mf, int hh) {
  const __bf16* p = &tr[d * TS + tok0 + 16 * mf + 4 * hh];
  const bf16x4 lo = *reinterpret_cast<const bf16x4*>(p);
  const bf16x4 hi = *reinterpret_cast<const bf16x4*>(p + 8);
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// The same A-operand fragment taken from a ROW-MAJOR tile (rows = tokens, row stride RS
// elements) with the transposing LDS read ds_read_b64_tr_b16.  Within each block of 16 lanes
// that instruction hands lane i, element e, the value that lane (4e + i/4) of the block
// addressed at its own element i%4.  So lane s of a block points at token row k0 + s/4,
// head-dim columns d0 + 4*(s%4) .. +3, and lane i receives tokens k0..k0+3 at column d0+i.
// The four 16-lane blocks of the wave cover (d0 = 0 | 16 of the 32-row block) x (hh = 0 | 1).
typedef short shortx4_lds __attribute__((ext_vector_type(4)));
template <int RS>
__device__ __forceinline__ bf16x8 transposed_frag_rowmajor(const __bf16* rows, int dblock, int tok0, int mf,
                                                           int lane) {
  const int blk = lane >> 4, s = lane & 15;
  const int hh = blk >> 1;
  const int d = dblock * 32 + 16 * (blk & 1) + 4 * (s & 3);
  const __bf16* p = rows + (tok0 + 16 * mf + 4 * hh + (s >> 2)) * RS + d;
  typedef shortx4_lds __attribute__((address_space(3))) * lds_ptr;
  const shortx4_lds lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p));
  const shortx4_lds hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p + 8 * RS));
  const bf16x4 l4 = __builtin_bit_cast(bf16x4, lo), h4 = __builtin_bit_cast(bf16x4, hi);
  return __builtin_shufflevector(l4, h4, 0, 1, 2, 3, 4, 5, 6, 7);
}

// Row of a 32x32 fp32 accumulator tile held in register r of a lane in half hh.
__device__ __forceinline__ constexpr int acc_row(int r, int hh) { return 8 * (r / 4) + 4 * hh + (r % 4); }

}  // namespace spa
