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

// One wave zeroes columns [0, C) of the unselected rows among rows [r0, r1): the lanes test 64
// rows at a time, then the wave writes the rows that need it, a lane per 16-byte chunk.
__device__ __forceinline__ void zero_unselected_rows(__bf16* dst, long row_stride, int C, const int32_t* inv_pos, long r0,
                                                     long r1, int lane) {
  const bf16x8 z = zero_bf16x8();
  for (long rb = r0; rb < r1; rb += kWave) {
    const long row = rb + lane;
    uint64_t todo = __ballot(row < r1 && inv_pos[row] < 0);
    while (todo != 0) {
      __bf16* p = dst + (rb + __ffsll((unsigned long long)todo) - 1) * row_stride;
      todo &= todo - 1;
      for (int c = lane; c < C / 8; c += kWave) *reinterpret_cast<bf16x8*>(p + c * 8) = z;
    }
  }
}

// Row of a 32x32 fp32 accumulator tile held in register r of a lane in half hh.
__device__ __forceinline__ constexpr int acc_row(int r, int hh) { return 8 * (r / 4) + 4 * hh + (r % 4); }

// ------------------------------------------------------------------ segments and launch order
// Exchange between lane l and lane l ^ 32 without the LDS crossbar: v_permlane32_swap of a
// value with itself leaves (x[l % 32], x[l % 32 + 32]) in every lane (lane layout checked on
// the GPU), so a reduction over the two halves is one swap and one ALU op, identical in both.
// (The two results are copied to scalars before the bit cast: casting the vector elements in
// place made the compiler read element 0 twice.)
__device__ __forceinline__ void swap_halves(float v, float& lo, float& hi) {
  const unsigned a = __builtin_bit_cast(unsigned, v);
  const auto r = __builtin_amdgcn_permlane32_swap(a, a, false, false);
  const unsigned r0 = r[0], r1 = r[1];
  lo = __builtin_bit_cast(float, r0);
  hi = __builtin_bit_cast(float, r1);
}
__device__ __forceinline__ float max_across_halves(float v) {
  float lo, hi;
  swap_halves(v, lo, hi);
  return fmaxf(lo, hi);
}
__device__ __forceinline__ float sum_across_halves(float v) {
  float lo, hi;
  swap_halves(v, lo, hi);
  return lo + hi;
}

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

// XCD-aware launch order.  Workgroups are handed to the 8 XCDs round-robin by linear id and
// each XCD has its own L2, so the query blocks that share one (image, head)'s K and V must
// sit on the same XCD or every XCD fetches those rows from memory again.  The grid is 1-D:
// id -> (xcd = id % 8, j = id / 8); inside an XCD j walks (pair, query block) with the query
// block fastest, and pair = 8 * (j / nqb) + xcd spreads consecutive pairs over the XCDs.
// pair -> (launch rank of the image = pair / H, head = pair % H).  Ids past the last pair
// (the grid is padded to a multiple of 8 pairs) are invalid.
struct TileId {
  int qb, h, rank;
  bool valid;
};
// (xcd, j): the workgroup's XCD and its number inside the XCD
__device__ __forceinline__ TileId xcd_tile_at(int xcd, int j, int nqb, int H, int B) {
  const int pl = j / nqb;
  TileId t;
  t.qb = j - pl * nqb;
  const int pair = pl * 8 + xcd;
  t.valid = pair < H * B;
  t.h = pair % H;
  t.rank = pair / H;
  return t;
}
__device__ __forceinline__ TileId xcd_tile(int nqb, int H, int B) {
  return xcd_tile_at(blockIdx.x & 7, blockIdx.x >> 3, nqb, H, B);
}
static unsigned xcd_grid(int nqb, int H, int B) {
  const long pairs8 = ((long)H * B + 7) / 8;
  return (unsigned)(pairs8 * 8 * nqb);
}

// Position of the kth set bit of mask (kth < popcount(mask)): binary search on popcounts.
__device__ __forceinline__ int kth_set_bit(uint64_t mask, int kth) {
  int pos = 0;
#pragma unroll
  for (int sh = 32; sh >= 1; sh >>= 1) {
    const int cnt = __popcll((mask >> pos) & ((1ull << sh) - 1ull));
    if (kth >= cnt) {
      kth -= cnt;
      pos += sh;
    }
  }
  return pos;
}

// Heaviest-class-first launch order for up to 64 segments, computed by every wave on its own (no
// LDS, no barrier): lane b holds segment b's bounds, a segment's class is its number of 32-row
// tiles (<= ncls), launch rank r is the (r - #heavier)th segment of its class in index order.
// Returns the segment of launch rank `rank` (< B) with its length.
struct RankedSegment {
  int img, row0, len;
};
__device__ __forceinline__ RankedSegment ranked_segment_wave(int rank, int B, const int32_t* __restrict__ cu, int ncls) {
  const int lane = threadIdx.x & 63;
  int start = 0, len = 0, cls = -1;
  if (lane < B) {
    start = cu[lane];
    len = cu[lane + 1] - start;
    cls = min((max(len, 0) + 31) >> 5, ncls);
  }
  int img = 0, ranked = 0;
  for (int c = ncls; c >= 0; --c) {
    const uint64_t bal = __ballot(cls == c);
    const int n_c = __popcll(bal);
    if (rank < ranked + n_c) {
      img = kth_set_bit(bal, rank - ranked);
      break;
    }
    ranked += n_c;
  }
  return {img, __builtin_amdgcn_readlane(start, img), __builtin_amdgcn_readlane(len, img)};
}

// Compact longest-first numbering of the LIVE (segment, head, block) work units of an XCD, for up
// to 64 segments and 64 (segment, head) pairs per XCD, computed by every wave on its own (no LDS
// memory, no barrier).  Pairs are numbered as in xcd_tile_at: pair = rank * H + h with rank 0 the
// longest segment (ties by index), pair p on XCD p % 8.  Workgroup j of an XCD takes the j-th live
// block of that XCD's pairs in pair order, the ceil(len / rows) blocks of a pair next to each
// other.  The host sizes the grid for the longest possible segment, so most workgroups of a
// sparse batch have no block: numbered this way they all come after the live ones in launch
// order instead of between them (they cost a dispatch slot each: on a batch of eight images with
// 5-40 % of 4200 tokens the launch takes 32 instead of 38 us).  valid = false: no block.
struct LiveTile {
  int qb, h, img, row0, len;
  bool valid;
};
constexpr int kLiveMaxB = 64, kLiveMaxPairs = 512;
__device__ __forceinline__ bool live_tiles_apply(int H, int B) { return B <= kLiveMaxB && H * B <= kLiveMaxPairs; }
__device__ __forceinline__ int lanes_below(uint64_t m) {      // set bits of m below this lane
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}
// nblk: blocks the grid provides per pair (no segment has more).
__device__ __forceinline__ LiveTile live_tile_wave(int xcd, int j, int H, int B, const int32_t* __restrict__ cu,
                                                   int rows, int nblk) {
  const int lane = threadIdx.x & 63;
  int start = 0, len = 0;
  if (lane < B) {
    start = cu[lane];
    len = max(cu[lane + 1] - start, 0);
  }
  // launch rank of segment `lane`.  Few segments: how many are longer, or as long with a lower index
  // (B steps).  Many segments: by number of blocks, most first, equal counts in index order (one
  // ballot per possible count, nblk + 1 steps); the cheaper of the two.
  int r = 0;
  if (B <= nblk) {
    for (int o = 0; o < B; ++o) {
      const int lo = __builtin_amdgcn_readlane(len, o);
      r += (lo > len) | ((lo == len) & (o < lane));
    }
  } else {
    const int mine = lane < B ? min((len + rows - 1) / rows, nblk) : -1;
    int ranked = 0;
    for (int c = nblk; c >= 0; --c) {
      const uint64_t same = __ballot(mine == c);
      if (mine == c) r = ranked + lanes_below(same);
      ranked += __popcll(same);
    }
  }
  if (lane >= B) r = lane;            // (keeps the exchange below a permutation of the 64 lanes)
  // lane r of these = the segment of launch rank r
  const int len_r = __builtin_amdgcn_ds_permute(r << 2, len);
  const int start_r = __builtin_amdgcn_ds_permute(r << 2, start);
  const int img_r = __builtin_amdgcn_ds_permute(r << 2, lane);
  // lane l as pair number l of this XCD: its blocks, and the blocks up to and including it
  const int pair = lane * 8 + xcd;
  const bool ok = pair < H * B;
  const int rank_l = ok ? pair / H : 0;
  const int len_l = __builtin_amdgcn_ds_bpermute(rank_l << 2, len_r);
  const int nb = ok ? (len_l + rows - 1) / rows : 0;
  int incl = nb;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int up = __shfl_up(incl, o, 64);
    if (lane >= o) incl += up;
  }
  LiveTile t = {0, 0, 0, 0, 0, false};
  const uint64_t past = __ballot(incl > j);
  if (past == 0) return t;
  const int pl = __builtin_ctzll(past);
  const int p = pl * 8 + xcd, rank = p / H;
  t.qb = j - (__builtin_amdgcn_readlane(incl, pl) - __builtin_amdgcn_readlane(nb, pl));
  t.h = p - rank * H;
  t.img = __builtin_amdgcn_readlane(img_r, rank);
  t.row0 = __builtin_amdgcn_readlane(start_r, rank);
  t.len = __builtin_amdgcn_readlane(len_r, rank);
  t.valid = true;
  return t;
}

// The same for a workgroup of several waves.  With few segments every wave numbers for itself (no
// barrier: measured 1 % faster on an 8-image batch with other batches in flight); with many, the
// first wave numbers and the others read the answer from LDS (one barrier: a uniform batch of 64
// segments ran 5 % slower with every wave of every workgroup doing the ranking).  All threads call it.
__device__ __forceinline__ LiveTile live_tile_block(int xcd, int j, int H, int B, const int32_t* __restrict__ cu,
                                                    int rows, int nblk, LiveTile* slot) {
  if (B <= 16) return live_tile_wave(xcd, j, H, B, cu, rows, nblk);
  if (threadIdx.x < 64) {
    const LiveTile t = live_tile_wave(xcd, j, H, B, cu, rows, nblk);
    if (threadIdx.x == 0) *slot = t;
  }
  __syncthreads();
  return *slot;
}

// Longest-segment-first launch order.  Work per segment grows like n^2 and workgroups are
// handed to compute units in launch order, so the heaviest images should start first.  Maps
// launch rank -> image by ranking the segment lengths (ties by index) and returns that
// image's segment; all threads of the workgroup call it.  The bounds are staged in LDS once,
// so no second dependent global load is needed.  For B > kLptMaxB the order is the identity.
// Used by the long-segment kernel only: short-segment workgroups are all resident at once
// and the ranking would cost more than it gains.
// s_cu: 2*kLptMaxB + 1 ints of LDS.
constexpr int kLptMaxB = 256;
template <int THREADS>
__device__ __forceinline__ Segment lpt_segment(int rank, int B, const int32_t* cu, const int32_t* key_lens,
                                               int n_pad, int* s_cu, int* s_pick) {
  if (B > kLptMaxB || B == 1) return segment_of(rank, cu, key_lens, n_pad);
  // s_cu[b] = segment start (packed mode only), s_len[b] = segment / key length
  int* s_len = s_cu + kLptMaxB + 1;
  const bool padded = key_lens != nullptr;
  for (int b = threadIdx.x; b < B; b += THREADS) {
    if (padded) {
      s_len[b] = key_lens[b];
    } else {
      const int a = cu[b], e = cu[b + 1];
      s_cu[b] = a;
      s_len[b] = e - a;
    }
  }
  __syncthreads();
  for (int b = threadIdx.x; b < B; b += THREADS) {
    const int nb = s_len[b];
    int r = 0;
#pragma unroll 8
    for (int j = 0; j < B; ++j) {
      const int nj = s_len[j];
      r += (nj > nb) | ((nj == nb) & (j < b));
    }
    if (r == rank) *s_pick = b;
  }
  __syncthreads();
  const int img = *s_pick;
  Segment s;
  if (padded) {
    s.row0 = (long)img * n_pad;
    s.nq = n_pad;
    s.nk = min(max(s_len[img], 0), n_pad);
  } else {
    s.row0 = s_cu[img];
    s.nq = s.nk = s_len[img];
  }
  return s;
}

// Row-major staging of `ROWS` rows of one head slice on their way to LDS: global -> registers
// (16-byte chunks, consecutive lanes on consecutive chunks of a row) -> LDS rows of stride
// DH + 8.  load() and store() are separate so that the next tile's rows can be in flight
// while the current tile is consumed.  Rows >= nrows read as zero.
template <int DH, int THREADS, int ROWS>
struct RowStage {
  static constexpr int CPR = DH / 8;
  static constexpr int CHUNKS = ROWS * CPR;
  static constexpr int CPT = (CHUNKS + THREADS - 1) / THREADS;
  bf16x8 reg[CPT];
  __device__ __forceinline__ void load(const __bf16* src, long base, int nrows, long stride) {
#pragma unroll
    for (int t = 0; t < CPT; ++t) {
      const int i = threadIdx.x + t * THREADS, r = i / CPR, c = i % CPR;
      reg[t] = zero_bf16x8();
      if (i < CHUNKS && r < nrows) reg[t] = *reinterpret_cast<const bf16x8*>(src + (base + r) * stride + c * 8);
    }
  }
  // the same with row r taken at src + row_index[r] * stride (rows gathered through an index)
  __device__ __forceinline__ void load_rows(const __bf16* src, const int32_t* row_index, int nrows, long stride) {
#pragma unroll
    for (int t = 0; t < CPT; ++t) {
      const int i = threadIdx.x + t * THREADS, r = i / CPR, c = i % CPR;
      reg[t] = zero_bf16x8();
      if (i < CHUNKS && r < nrows)
        reg[t] = *reinterpret_cast<const bf16x8*>(src + (long)row_index[r] * stride + c * 8);
    }
  }
  __device__ __forceinline__ void store(__bf16* rows) const {
#pragma unroll
    for (int t = 0; t < CPT; ++t) {
      const int i = threadIdx.x + t * THREADS, r = i / CPR, c = i % CPR;
      if (i < CHUNKS) *reinterpret_cast<bf16x8*>(&rows[r * (DH + 8) + c * 8]) = reg[t];
    }
  }
};

// Park a wave's transposed accumulator tile (rows = head dim, cols = its 32 tokens) in LDS
// as 32 token rows of DH bf16 (row stride RS), scaled; then flush_tile writes whole rows.
template <int DH, int RS>
__device__ __forceinline__ void park_tile(const floatx16 (&acc)[DH / 32], float scale, __bf16* tile, int l32, int hh) {
#pragma unroll
  for (int d = 0; d < DH / 32; ++d)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      floatx4 f = {acc[d][4 * g] * scale, acc[d][4 * g + 1] * scale, acc[d][4 * g + 2] * scale,
                   acc[d][4 * g + 3] * scale};
      *reinterpret_cast<bf16x4*>(&tile[l32 * RS + d * 32 + 8 * g + 4 * hh]) = __builtin_convertvector(f, bf16x4);
    }
}
template <int DH, int RS>
__device__ __forceinline__ void flush_tile(const __bf16* tile, __bf16* dst, long row_stride, int nrows, int lane) {
  constexpr int CPR = DH / 8;
#pragma unroll
  for (int i = lane; i < 32 * CPR; i += 64) {
    const int r = i / CPR, c = i % CPR;
    if (r < nrows)
      *reinterpret_cast<bf16x8*>(dst + r * row_stride + c * 8) = *reinterpret_cast<const bf16x8*>(&tile[r * RS + c * 8]);
  }
}

}  // namespace spa
