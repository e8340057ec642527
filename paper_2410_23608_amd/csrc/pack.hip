// Token packing (Section 3.2 "Token Packing"), the scatter back, and their transposes.
// All kernels move feature rows with 16-byte accesses and are bandwidth-bound.
//
// spa_pack is ONE launch with no scratch memory and no inter-workgroup dependency: a
// workgroup owns one tile of <= 256 consecutive tokens of one image, counts the selected
// tokens that precede its tile (from the per-image counts when the caller has them, else
// from the mask bytes themselves — B*N bytes that sit in L2), ranks its own tokens with
// wave ballots, and copies its survivors' rows to their final place.
#include <cstdlib>

#include "spa_common.h"

namespace spa {

constexpr int kPackThreads = 256;
constexpr int kPackWaves = kPackThreads / kWave;

// number of non-zero bytes in a 32-bit word
__device__ __forceinline__ int nonzero_bytes(uint32_t w) {
  uint32_t t = (((w & 0x7F7F7F7Fu) + 0x7F7F7F7Fu) | w) & 0x80808080u;
  return __popc(t);
}

// Sum over the workgroup; every thread gets the result.  red: kPackWaves ints of LDS.
__device__ __forceinline__ int block_sum(int v, int* red) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  __syncthreads();
  if (lane_id() == 0) red[threadIdx.x / kWave] = v;
  __syncthreads();
  int s = 0;
#pragma unroll
  for (int i = 0; i < kPackWaves; ++i) s += red[i];
  return s;
}

// Non-zero bytes of m[0 .. n), counted cooperatively by the workgroup (partial per thread).
__device__ __forceinline__ int count_bytes_partial(const uint8_t* m, long n) {
  int cnt = 0;
  const uintptr_t a = reinterpret_cast<uintptr_t>(m);
  long head = (16 - (a & 15)) & 15;
  if (head > n) head = n;
  for (long i = threadIdx.x; i < head; i += kPackThreads) cnt += m[i] != 0;
  const long nvec = (n - head) / 16;
  const uintx4* mv = reinterpret_cast<const uintx4*>(m + head);
  for (long i = threadIdx.x; i < nvec; i += kPackThreads) {
    uintx4 v = mv[i];
    cnt += nonzero_bytes(v[0]) + nonzero_bytes(v[1]) + nonzero_bytes(v[2]) + nonzero_bytes(v[3]);
  }
  for (long i = head + nvec * 16 + threadIdx.x; i < n; i += kPackThreads) cnt += m[i] != 0;
  return cnt;
}

// Position in the original map of the p-th token (raster order) of the cyclically shifted map:
// the shifted map holds at (r, c) the token at ((r + sh) mod gh, (c + sw) mod gw).
struct Shift {
  int gh, gw, sh, sw;   // 0 <= sh < gh, 0 <= sw < gw
  __device__ __forceinline__ int orig(int p) const {
    int r = p / gw, c = p - r * gw;
    r += sh;
    if (r >= gh) r -= gh;
    c += sw;
    if (c >= gw) c -= gw;
    return r * gw + c;
  }
};

// Copy of a tile's selected rows (sel_src[r] = position in the image of the r-th survivor) to
// consecutive packed rows: consecutive threads take consecutive 16-byte chunks, up to twelve
// independent loads in flight per thread before the first store (a 16-token tile of q|k|v rows
// of a 384-wide model is nine per thread: one pass, one memory latency).
template <typename T, bool kScale>
__device__ __forceinline__ void copy_selected_rows(const T* __restrict__ xt, T* __restrict__ pt, int C, int nsel,
                                                   const int* sel_src, const float* sel_scale, int tid) {
  constexpr int VE = 16 / sizeof(T);
  constexpr int U = 12;
  const int chunks = C / VE;
  const unsigned work = (unsigned)nsel * (unsigned)chunks;
  for (unsigned i0 = tid; i0 < work; i0 += kPackThreads * U) {
    uintx4 v[U];
    unsigned dst_off[U];
    float sc[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const unsigned i = i0 + u * kPackThreads;
      if (i < work) {
        const unsigned r = i / (unsigned)chunks;
        const unsigned ch = i - r * (unsigned)chunks;
        v[u] = *reinterpret_cast<const uintx4*>(xt + (long)sel_src[r] * C + ch * VE);
        dst_off[u] = r * (unsigned)C + ch * VE;
        if (kScale) sc[u] = sel_scale[r];
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const unsigned i = i0 + u * kPackThreads;
      if (i < work) {
        uintx4 o = v[u];
        if (kScale) {
          if constexpr (sizeof(T) == 2) {
            floatx8 f = bf16x8_to_float(__builtin_bit_cast(bf16x8, o));
#pragma unroll
            for (int e = 0; e < 8; ++e) f[e] *= sc[u];
            o = __builtin_bit_cast(uintx4, float_to_bf16x8(f));
          } else {
            o = __builtin_bit_cast(uintx4, __builtin_bit_cast(floatx4, o) * sc[u]);
          }
        }
        *reinterpret_cast<uintx4*>(pt + dst_off[u]) = o;
      }
    }
  }
}

// kShift: tokens are ranked in the raster order of the shifted map (Section 1: the feature
// map is shifted so that the token pairs sharing a container vary); gather_idx / inv_pos keep
// naming ORIGINAL positions, so the scatter back undoes the shift by itself.
template <typename T, bool kScale, bool kShift, bool kPair>
__global__ void __launch_bounds__(kPackThreads)
pack_kernel(const T* __restrict__ x, const uint8_t* __restrict__ mask,
            const int32_t* __restrict__ counts, const float* __restrict__ gate_scores,
            int B, int N, int C, int tile, int tiles_per_image, int container_len, Shift shift,
            T* __restrict__ packed, int32_t* __restrict__ cu_seqlens,
            int32_t* __restrict__ gather_idx, int32_t* __restrict__ inv_pos,
            int32_t* __restrict__ total, const T* __restrict__ x2, int C2, T* __restrict__ packed2) {
  constexpr int VE = 16 / sizeof(T);
  __shared__ int red[kPackWaves];
  __shared__ int wave_cnt[kPackWaves];
  __shared__ int sel_src[kPackThreads];
  __shared__ float sel_scale[kPackThreads];

  const int b = blockIdx.x / tiles_per_image;
  const int t = blockIdx.x % tiles_per_image;
  const int tile_start = t * tile;
  const int tile_n = min(tile, N - tile_start);
  const long img0 = (long)b * N;

  // 1. selected tokens before this tile
  int part = 0;
  if (counts != nullptr) {
    for (int i = threadIdx.x; i < b; i += kPackThreads) part += counts[i];
    if (!kShift) part += count_bytes_partial(mask + img0, tile_start);
  } else {
    part = count_bytes_partial(mask, kShift ? img0 : img0 + tile_start);
  }
  if (kShift)   // the tile's predecessors inside the image are not contiguous in memory
    for (int p = threadIdx.x; p < tile_start; p += kPackThreads) part += mask[img0 + shift.orig(p)] != 0;
  const int base = block_sum(part, red);

  // 2. rank of each token of the tile among the tile's survivors
  const int tid = threadIdx.x;
  const bool in_tile = tid < tile_n;
  const int src = in_tile ? (kShift ? shift.orig(tile_start + tid) : tile_start + tid) : 0;   // position in the image
  const bool flag = in_tile && mask[img0 + src] != 0;
  const uint64_t bal = __ballot(flag);
  const int wv = tid / kWave;
  if (lane_id() == 0) wave_cnt[wv] = __popcll(bal);
  __syncthreads();
  int wave_off = 0, nsel = 0;
#pragma unroll
  for (int i = 0; i < kPackWaves; ++i) {
    const int c = wave_cnt[i];
    if (i < wv) wave_off += c;
    nsel += c;
  }
  const int local_rank = wave_off + rank_in_ballot(bal);
  if (in_tile && inv_pos != nullptr) inv_pos[img0 + src] = flag ? base + local_rank : -1;
  if (flag) {
    if (gather_idx != nullptr) gather_idx[base + local_rank] = (int32_t)(img0 + src);
    sel_src[local_rank] = src;
    if (kScale) sel_scale[local_rank] = sigmoidf_dev(gate_scores[img0 + src]);
  }
  if (t == 0 && tid == 0 && cu_seqlens != nullptr) cu_seqlens[b] = base;
  __syncthreads();

  const int chunks = C / VE;
  // 3. the last tile knows T: publish it and zero the tail of the last container
  if (b == B - 1 && t == tiles_per_image - 1) {
    const int T_sel = base + nsel;
    if (tid == 0) {
      if (cu_seqlens != nullptr) cu_seqlens[B] = T_sel;
      if (total != nullptr) total[0] = T_sel;
    }
    if (container_len > 0 && packed != nullptr) {
      const long t_pad = ((long)T_sel + container_len - 1) / container_len * container_len;
      const long nz = (t_pad - T_sel) * chunks;
      uintx4* dst = reinterpret_cast<uintx4*>(packed + (long)T_sel * C);
      const uintx4 z = {0u, 0u, 0u, 0u};
      for (long i = tid; i < nz; i += kPackThreads) dst[i] = z;
    }
  }

  // 4. copy the survivors' rows.  kPair: the rows of x go to packed as they are, and the rows
  //    of a second tensor x2 (width C2) of the same tokens, multiplied by Sigmoid(s) when scores
  //    are given, go to packed2, in the same launch (one copy after the other: one list of chunks
  //    over both tensors, with all loads in flight together, measured slower, 13.6 against 12.3 us).
  if (packed != nullptr)
    copy_selected_rows<T, kScale && !kPair>(x + img0 * (long)C, packed + (long)base * C, C, nsel, sel_src, sel_scale, tid);
  if (kPair)
    copy_selected_rows<T, kScale>(x2 + img0 * (long)C2, packed2 + (long)base * C2, C2, nsel, sel_src, sel_scale, tid);
}

// y[i] = base[i] (+ src[inv[i]]) or src[inv[i]] or 0.  A block owns `rpb` consecutive output
// rows; consecutive threads take consecutive 16-byte chunks.
// kStream: y is a final output nothing in the path reads again (spa_unpack): non-temporal
// stores, so it does not displace what the next launches read; the transpose of the pack gather
// (spa_pack_bwd) feeds the gate backward and keeps ordinary stores.
template <typename T, bool kBase, bool kStream>
__global__ void __launch_bounds__(256)
unpack_kernel(const T* __restrict__ src, const int32_t* __restrict__ inv_pos,
              const T* base, long rows, int C, int rpb, T* y) {
  constexpr int VE = 16 / sizeof(T);
  constexpr int U = 4;
  const unsigned chunks = C / VE;
  const long row0 = (long)blockIdx.x * rpb;
  const unsigned nrows = (unsigned)min((long)rpb, rows - row0);
  const unsigned work = nrows * chunks;
  const int32_t* inv = inv_pos + row0;
  const T* bt = kBase ? base + row0 * C : nullptr;
  T* yt = y + row0 * C;
  for (unsigned i0 = threadIdx.x; i0 < work; i0 += 256 * U) {
    uintx4 v[U], bv[U];
    int j[U];
    unsigned off[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const unsigned i = i0 + u * 256;
      if (i < work) {
        const unsigned r = i / chunks, ch = i - r * chunks;
        off[u] = r * (unsigned)C + ch * VE;
        j[u] = inv[r];
        const uintx4 z = {0u, 0u, 0u, 0u};
        v[u] = z;
        if (j[u] >= 0) v[u] = *reinterpret_cast<const uintx4*>(src + (long)j[u] * C + ch * VE);
        if (kBase) bv[u] = *reinterpret_cast<const uintx4*>(bt + off[u]);
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const unsigned i = i0 + u * 256;
      if (i < work) {
        uintx4 o = v[u];
        if (kBase) {
          if (j[u] >= 0) {
            if constexpr (sizeof(T) == 2) {
              floatx8 a = bf16x8_to_float(__builtin_bit_cast(bf16x8, v[u]));
              floatx8 c = bf16x8_to_float(__builtin_bit_cast(bf16x8, bv[u]));
              o = __builtin_bit_cast(uintx4, float_to_bf16x8(a + c));
            } else {
              o = __builtin_bit_cast(uintx4, __builtin_bit_cast(floatx4, v[u]) + __builtin_bit_cast(floatx4, bv[u]));
            }
          } else {
            o = bv[u];
          }
        }
        if (kStream) __builtin_nontemporal_store(o, reinterpret_cast<uintx4*>(yt + off[u]));
        else *reinterpret_cast<uintx4*>(yt + off[u]) = o;
      }
    }
  }
}

// dst[j] = src[idx[j]] for j < *total (rows of `chunks` 16-byte chunks); a block owns rpb rows
__global__ void __launch_bounds__(256)
gather_rows_kernel(const uintx4* __restrict__ src, const int32_t* __restrict__ idx,
                   const int32_t* __restrict__ total, long cap_rows, unsigned chunks, int rpb,
                   uintx4* __restrict__ dst) {
  constexpr int U = 4;
  const long rows = min((long)total[0], cap_rows);
  const long row0 = (long)blockIdx.x * rpb;
  if (row0 >= rows) return;
  const unsigned nrows = (unsigned)min((long)rpb, rows - row0);
  const unsigned work = nrows * chunks;
  const int32_t* id = idx + row0;
  uintx4* dt = dst + row0 * chunks;
  for (unsigned i0 = threadIdx.x; i0 < work; i0 += 256 * U) {
    uintx4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const unsigned i = i0 + u * 256;
      if (i < work) {
        const unsigned r = i / chunks, ch = i - r * chunks;
        v[u] = src[(long)id[r] * chunks + ch];
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const unsigned i = i0 + u * 256;
      if (i < work) dt[i] = v[u];
    }
  }
}

// rows per block for the row-copy kernels: about 4 chunks per thread
static int rows_per_block(long chunks) {
  long r = (1024 + chunks - 1) / chunks;
  return (int)(r < 1 ? 1 : r);
}

static int pick_tile(int B, int N, bool have_counts) {
  // Small tiles give more workgroups (bandwidth), but without per-image counts every
  // workgroup re-reads the mask prefix, so keep tiles larger when B*N is large.
  const long want = (!have_counts && (long)B * N > 16384) ? 512 : 1024;
  int tile = 256;
  while (tile > 16 && (long)B * ((N + tile - 1) / tile) < want) tile >>= 1;
  if (options().pack_tile != 0) tile = options().pack_tile;       // option pack_tile
  return tile;
}

static int check_rows(const char* fn, int B, int N, int C, int dtype) {
  SPA_REQUIRE(B >= 1 && N >= 1 && C >= 1, SPA_ERR_INVALID_ARG, "%s: B, N, C must be >= 1", fn);
  SPA_REQUIRE((long)B * N < 2147483647L, SPA_ERR_INVALID_ARG, "%s: B*N must be < 2^31", fn);
  SPA_REQUIRE(dtype == SPA_F32 || dtype == SPA_BF16, SPA_ERR_UNSUPPORTED, "%s: unknown dtype %d", fn, dtype);
  SPA_REQUIRE(((long)C * elem_size(dtype)) % 16 == 0, SPA_ERR_INVALID_ARG,
              "%s: row length C*elem = %ld bytes is not a multiple of 16", fn, (long)C * elem_size(dtype));
  SPA_REQUIRE(C <= (1 << 20), SPA_ERR_UNSUPPORTED, "%s: C = %d exceeds 2^20", fn, C);
  return SPA_OK;
}

template <typename T, bool kStream>
static void launch_unpack(const void* src, const int32_t* inv, const void* base, long rows, int C,
                          void* y, hipStream_t st) {
  constexpr int VE = 16 / sizeof(T);
  const int rpb = rows_per_block(C / VE);
  const unsigned g = (unsigned)((rows + rpb - 1) / rpb);
  if (base != nullptr)
    hipLaunchKernelGGL((unpack_kernel<T, true, kStream>), dim3(g), dim3(256), 0, st, static_cast<const T*>(src), inv,
                       static_cast<const T*>(base), rows, C, rpb, static_cast<T*>(y));
  else
    hipLaunchKernelGGL((unpack_kernel<T, false, kStream>), dim3(g), dim3(256), 0, st, static_cast<const T*>(src), inv,
                       static_cast<const T*>(nullptr), rows, C, rpb, static_cast<T*>(y));
}

}  // namespace spa

using namespace spa;

static int pack_common(const char* fn, const void* x, const uint8_t* mask, const int32_t* counts,
                       const float* gate_scores, int B, int N, int C, int dtype, int container_len,
                       const Shift& shift, bool shifted, void* packed, int32_t* cu_seqlens,
                       int32_t* gather_idx, int32_t* inv_pos, int32_t* total, void* stream) {
  SPA_REQUIRE(mask && ((x != nullptr) == (packed != nullptr)), SPA_ERR_INVALID_ARG,
              "%s: mask is null, or only one of x / packed is given", fn);
  if (int rc = check_rows(fn, B, N, C, dtype)) return rc;
  SPA_REQUIRE(container_len >= 0, SPA_ERR_INVALID_ARG, "%s: container_len must be >= 0", fn);
  SPA_REQUIRE(aligned16(x) && aligned16(packed), SPA_ERR_INVALID_ARG, "%s: x / packed not 16-byte aligned", fn);
  const int tile = pick_tile(B, N, counts != nullptr);
  const int tpi = (N + tile - 1) / tile;
  SPA_REQUIRE((long)B * tpi < 2147483647L, SPA_ERR_INVALID_ARG, "%s: too many tiles", fn);
  const dim3 grid((unsigned)((long)B * tpi)), block(kPackThreads);
  hipStream_t st = as_stream(stream);
#define SPA_PACK_LAUNCH(T, S, SH)                                                                        \
  hipLaunchKernelGGL((pack_kernel<T, S, SH, false>), grid, block, 0, st, static_cast<const T*>(x), mask, counts, \
                     gate_scores, B, N, C, tile, tpi, container_len, shift, static_cast<T*>(packed),     \
                     cu_seqlens, gather_idx, inv_pos, total, static_cast<const T*>(nullptr), 0,          \
                     static_cast<T*>(nullptr))
#define SPA_PACK_SCALE(T, SH)                                                                            \
  do {                                                                                                   \
    if (gate_scores) SPA_PACK_LAUNCH(T, true, SH); else SPA_PACK_LAUNCH(T, false, SH);                   \
  } while (0)
  if (dtype == SPA_F32) {
    if (shifted) SPA_PACK_SCALE(float, true); else SPA_PACK_SCALE(float, false);
  } else {
    if (shifted) SPA_PACK_SCALE(__bf16, true); else SPA_PACK_SCALE(__bf16, false);
  }
#undef SPA_PACK_SCALE
#undef SPA_PACK_LAUNCH
  return check_launch(fn);
}

extern "C" int spa_pack(const void* x, const uint8_t* mask, const int32_t* counts,
                        const float* gate_scores, int B, int N, int C, int dtype, int container_len,
                        void* packed, int32_t* cu_seqlens, int32_t* gather_idx, int32_t* inv_pos,
                        int32_t* total, void* stream) {
  return pack_common("spa_pack", x, mask, counts, gate_scores, B, N, C, dtype, container_len, Shift{1, 1, 0, 0},
                     false, packed, cu_seqlens, gather_idx, inv_pos, total, stream);
}

extern "C" int spa_pack_pair(const void* x, int C, const void* x2, int C2, const uint8_t* mask, const int32_t* counts,
                             const float* gate_scores, int B, int N, int dtype, void* packed, void* packed2,
                             int32_t* cu_seqlens, int32_t* gather_idx, int32_t* inv_pos, int32_t* total,
                             void* stream) {
  const char* fn = "spa_pack_pair";
  SPA_REQUIRE(mask && x && x2 && packed && packed2, SPA_ERR_INVALID_ARG, "%s: null pointer", fn);
  if (int rc = check_rows(fn, B, N, C, dtype)) return rc;
  if (int rc = check_rows(fn, B, N, C2, dtype)) return rc;
  SPA_REQUIRE(aligned16(x) && aligned16(packed) && aligned16(x2) && aligned16(packed2), SPA_ERR_INVALID_ARG,
              "%s: buffers not 16-byte aligned", fn);
  const int tile = pick_tile(B, N, counts != nullptr);
  const int tpi = (N + tile - 1) / tile;
  SPA_REQUIRE((long)B * tpi < 2147483647L, SPA_ERR_INVALID_ARG, "%s: too many tiles", fn);
  const dim3 grid((unsigned)((long)B * tpi)), block(kPackThreads);
  hipStream_t st = as_stream(stream);
  const Shift shift{1, 1, 0, 0};
#define SPA_PACK_PAIR(T, S)                                                                                    \
  hipLaunchKernelGGL((pack_kernel<T, S, false, true>), grid, block, 0, st, static_cast<const T*>(x), mask, counts, \
                     gate_scores, B, N, C, tile, tpi, 0, shift, static_cast<T*>(packed), cu_seqlens, gather_idx, \
                     inv_pos, total, static_cast<const T*>(x2), C2, static_cast<T*>(packed2))
  if (dtype == SPA_F32) {
    if (gate_scores) SPA_PACK_PAIR(float, true); else SPA_PACK_PAIR(float, false);
  } else {
    if (gate_scores) SPA_PACK_PAIR(__bf16, true); else SPA_PACK_PAIR(__bf16, false);
  }
#undef SPA_PACK_PAIR
  return check_launch(fn);
}

extern "C" int spa_pack_shifted(const void* x, const uint8_t* mask, const int32_t* counts,
                                const float* gate_scores, int B, int grid_h, int grid_w, int shift_h,
                                int shift_w, int C, int dtype, int container_len, void* packed,
                                int32_t* cu_seqlens, int32_t* gather_idx, int32_t* inv_pos, int32_t* total,
                                void* stream) {
  const char* fn = "spa_pack_shifted";
  SPA_REQUIRE(grid_h >= 1 && grid_w >= 1 && (long)grid_h * grid_w < 2147483647L, SPA_ERR_INVALID_ARG,
              "%s: grid_h, grid_w must be >= 1 and grid_h*grid_w < 2^31", fn);
  // any integer shift; reduced to [0, extent)
  const int sh = ((shift_h % grid_h) + grid_h) % grid_h, sw = ((shift_w % grid_w) + grid_w) % grid_w;
  return pack_common(fn, x, mask, counts, gate_scores, B, grid_h * grid_w, C, dtype, container_len,
                     Shift{grid_h, grid_w, sh, sw}, sh != 0 || sw != 0, packed, cu_seqlens, gather_idx, inv_pos,
                     total, stream);
}

// Boundaries of the container-local attention segments: a segment ends where an image ends or a
// container of length L ends.  One workgroup; images are scanned 256 at a time.
__global__ void __launch_bounds__(256)
container_segments_kernel(const int32_t* __restrict__ cu_seqlens, int B, int L, int seg_cap,
                          int32_t* __restrict__ seg_cu, int32_t* __restrict__ n_segments) {
  __shared__ int wave_sum[4];
  __shared__ int carry_s;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  if (tid == 0) carry_s = 0;
  __syncthreads();
  const int T = cu_seqlens[B];
  for (int b0 = 0; b0 < B; b0 += 256) {
    const int b = b0 + tid;
    int start = 0, end = 0, cnt = 0;
    if (b < B) {
      start = cu_seqlens[b];
      end = cu_seqlens[b + 1];
      if (end > start) cnt = (end + L - 1) / L - start / L;   // the image's start, then every multiple of L inside it
    }
    // exclusive scan of cnt over the 256 images of this round
    int inc = cnt;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int up = __shfl_up(inc, o, 64);
      if (lane >= o) inc += up;
    }
    if (lane == 63) wave_sum[wv] = inc;
    __syncthreads();
    int off = carry_s;
    for (int i = 0; i < wv; ++i) off += wave_sum[i];
    const int first = off + inc - cnt;
    for (int i = 0; i < cnt; ++i) {
      const int pos = i == 0 ? start : (start / L + i) * L;
      if (first + i <= seg_cap) seg_cu[first + i] = pos;
    }
    __syncthreads();
    if (tid == 255) carry_s = off + inc;
    __syncthreads();
  }
  const int n = carry_s;
  // closing boundary, then empty segments up to the capacity
  for (int i = n + tid; i <= seg_cap; i += 256) seg_cu[i] = T;
  if (tid == 0) n_segments[0] = n;
}

extern "C" int64_t spa_container_segments_capacity(int B, int64_t max_total, int container_len) {
  if (B < 1 || max_total < 0 || container_len < 1) return -1;
  return (int64_t)B + max_total / container_len;
}

extern "C" int spa_container_segments(const int32_t* cu_seqlens, int B, int container_len, int64_t max_total,
                                      int seg_cap, int32_t* seg_cu_seqlens, int32_t* n_segments, void* stream) {
  const char* fn = "spa_container_segments";
  SPA_REQUIRE(cu_seqlens && seg_cu_seqlens && n_segments, SPA_ERR_INVALID_ARG, "%s: null pointer", fn);
  SPA_REQUIRE(B >= 1 && container_len >= 1 && max_total >= 0, SPA_ERR_INVALID_ARG,
              "%s: B, container_len must be >= 1 and max_total >= 0", fn);
  const int64_t need = spa_container_segments_capacity(B, max_total, container_len);
  SPA_REQUIRE(seg_cap >= need, SPA_ERR_WORKSPACE, "%s: seg_cap = %d, need %lld for B = %d, max_total = %lld, L = %d", fn,
              seg_cap, (long long)need, B, (long long)max_total, container_len);
  hipLaunchKernelGGL(container_segments_kernel, dim3(1), dim3(256), 0, as_stream(stream), cu_seqlens, B,
                     container_len, seg_cap, seg_cu_seqlens, n_segments);
  return check_launch(fn);
}

extern "C" int spa_unpack(const void* packed_out, const int32_t* inv_pos, const void* base,
                          int B, int N, int C, int dtype, void* y, void* stream) {
  SPA_REQUIRE(packed_out && inv_pos && y, SPA_ERR_INVALID_ARG, "spa_unpack: null pointer");
  if (int rc = check_rows("spa_unpack", B, N, C, dtype)) return rc;
  SPA_REQUIRE(aligned16(packed_out) && aligned16(y) && aligned16(base), SPA_ERR_INVALID_ARG,
              "spa_unpack: buffers not 16-byte aligned");
  if (dtype == SPA_F32) launch_unpack<float, true>(packed_out, inv_pos, base, (long)B * N, C, y, as_stream(stream));
  else launch_unpack<__bf16, true>(packed_out, inv_pos, base, (long)B * N, C, y, as_stream(stream));
  return check_launch("spa_unpack");
}

extern "C" int spa_pack_bwd(const void* dpacked, const int32_t* inv_pos, int B, int N, int C,
                            int dtype, void* d_rg, void* stream) {
  SPA_REQUIRE(dpacked && inv_pos && d_rg, SPA_ERR_INVALID_ARG, "spa_pack_bwd: null pointer");
  if (int rc = check_rows("spa_pack_bwd", B, N, C, dtype)) return rc;
  SPA_REQUIRE(aligned16(dpacked) && aligned16(d_rg), SPA_ERR_INVALID_ARG, "spa_pack_bwd: buffers not 16-byte aligned");
  if (dtype == SPA_F32) launch_unpack<float, false>(dpacked, inv_pos, nullptr, (long)B * N, C, d_rg, as_stream(stream));
  else launch_unpack<__bf16, false>(dpacked, inv_pos, nullptr, (long)B * N, C, d_rg, as_stream(stream));
  return check_launch("spa_pack_bwd");
}

extern "C" int spa_unpack_bwd(const void* dy, const int32_t* gather_idx, const int32_t* total,
                              int B, int N, int C, int dtype, void* dout, void* stream) {
  SPA_REQUIRE(dy && gather_idx && total && dout, SPA_ERR_INVALID_ARG, "spa_unpack_bwd: null pointer");
  if (int rc = check_rows("spa_unpack_bwd", B, N, C, dtype)) return rc;
  SPA_REQUIRE(aligned16(dy) && aligned16(dout), SPA_ERR_INVALID_ARG, "spa_unpack_bwd: buffers not 16-byte aligned");
  const int chunks = (int)((long)C * elem_size(dtype) / 16);
  const long cap = (long)B * N;
  const int rpb = rows_per_block(chunks);
  hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)((cap + rpb - 1) / rpb)), dim3(256), 0, as_stream(stream),
                     static_cast<const uintx4*>(dy), gather_idx, total, cap, (unsigned)chunks, rpb,
                     static_cast<uintx4*>(dout));
  return check_launch("spa_unpack_bwd");
}
