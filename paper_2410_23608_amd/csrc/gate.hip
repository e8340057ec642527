// Gate scoring + hard selection (Section 3.2, equations for s and r_p), the 2x2 max-pool
// that resizes up-scale scores, and the gate backward with the selection loss
// (Section 3.3).  All kernels are bandwidth-bound: every feature row is read once with
// 16-byte loads, a group of G lanes per token, fp32 accumulation.
#include <cmath>
#include <mutex>

#include "spa_common.h"

namespace spa {

constexpr int kGateThreads = 256;
constexpr int kMaxGateC = 8192;   // (the gate backward stages w in LDS as fp32)

template <typename T> struct Vec16;
template <> struct Vec16<float> {
  static constexpr int kElems = 4;
  __device__ static __forceinline__ void load(const float* p, float (&f)[4]) {
    floatx4 v = *reinterpret_cast<const floatx4*>(p);
    f[0] = v[0]; f[1] = v[1]; f[2] = v[2]; f[3] = v[3];
  }
  // dx is the last thing the backward pass writes and nothing here reads it again: non-temporal
  __device__ static __forceinline__ void store(float* p, const float (&f)[4]) {
    floatx4 v = {f[0], f[1], f[2], f[3]};
    __builtin_nontemporal_store(v, reinterpret_cast<floatx4*>(p));
  }
};
template <> struct Vec16<__bf16> {
  static constexpr int kElems = 8;
  __device__ static __forceinline__ void load(const __bf16* p, float (&f)[8]) {
    floatx8 v = bf16x8_to_float(*reinterpret_cast<const bf16x8*>(p));
#pragma unroll
    for (int i = 0; i < 8; ++i) f[i] = v[i];
  }
  __device__ static __forceinline__ void store(__bf16* p, const float (&f)[8]) {
    floatx8 v;
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = f[i];
    __builtin_nontemporal_store(float_to_bf16x8(v), reinterpret_cast<bf16x8*>(p));
  }
};

template <int G>
__device__ __forceinline__ float group_sum(float v) {
#pragma unroll
  for (int o = G / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

// One group of G lanes per token; the group strides over the row's 16-byte chunks.
// kPool: s_up is the score map of the finer stage, [B, 2 gh, 2 gw], and is 2x2 max-pooled on
// the fly (Section 3.2: up-scale scores adjusted via max-pooling); the pooled value is also
// written to s_up_pooled when that is given (the backward pass needs it).
struct PoolGrid {
  int gh, gw;            // this stage's grid, N = gh * gw
  float* s_up_pooled;    // [B, N] or null
};

// Packing index built by the gate launch itself (Section 3.2 "Token Packing" needs nothing but the
// selection): the workgroup that finishes LAST (one arrival counter, no waiting anywhere) walks
// the mask once and writes cu_seqlens, gather_idx, inv_pos, total (and counts), exactly what
// spa_pack writes.  arrive == nullptr: off.
struct IndexOut {
  int32_t* cu_seqlens;   // [B+1]
  int32_t* gather_idx;   // [B*N]
  int32_t* inv_pos;      // [B*N]
  int32_t* total;        // [1] or null
  int32_t* counts;       // [B] or null
  unsigned* arrive;      // kArriveWords words, zero before the launch, zero again after it
};
// Arrival is counted in two levels, 16 group counters and a root: atomics on ONE address are served
// one after the other (about 25 ns each here, 50 us for the 2100 workgroups of a 33600-token
// batch), and so are atomics on neighbouring lines (they meet in one memory channel), so the
// counters lie 4352 bytes apart.
constexpr int kArriveGroups = 16, kArriveStride = 1088;             // words between counters (4352 bytes)
constexpr int kArriveWords = (kArriveGroups + 1) * kArriveStride;

// number of non-zero bytes in a 32-bit word
__device__ __forceinline__ int nonzero_bytes_u32(uint32_t w) {
  const uint32_t t = (((w & 0x7F7F7F7Fu) + 0x7F7F7F7Fu) | w) & 0x80808080u;
  return __popc(t);
}

// One workgroup of kGateThreads threads: stable compaction index of mask[0 .. ntok) (tokens of image b
// are [b*N, (b+1)*N)).  In a round, thread t owns the 16 consecutive tokens [4096 r + 16 t, + 16)
// (consecutive threads, consecutive groups: the index stores of a wave are contiguous); the
// mask words of up to kRounds rounds are fetched first, as independent 32-bit agent-scope loads (the
// mask is 16-byte aligned; other XCDs wrote these bytes in this same launch), so 32768 tokens cost
// one trip to memory, then every round is one scan over the workgroup and a walk of 16 tokens.
__device__ __forceinline__ void build_pack_index(const uint8_t* mask, int ntok, int N, int B, const IndexOut& idx) {
  constexpr int kWaves = kGateThreads / kWave;
  constexpr int kRounds = 8, kPerRound = kGateThreads * 16;
  __shared__ int s_wave[2][kWaves];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
  int carry = 0;                                       // selected tokens before the round (the same in every thread)
  const int tail = ntok & ~3;                          // start of the one partial word at the end of the mask
  for (int t_super = 0; t_super < ntok; t_super += kRounds * kPerRound) {
    uint32_t m[kRounds][4];
#pragma unroll
    for (int r = 0; r < kRounds; ++r)
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        m[r][k] = 0u;
        const int tk = t_super + r * kPerRound + tid * 16 + 4 * k;
        if (tk + 4 <= ntok)
          m[r][k] = __hip_atomic_load(reinterpret_cast<const uint32_t*>(mask + tk), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    if (tail < ntok) {                                 // the partial word, by the thread that owns it
#pragma unroll
      for (int r = 0; r < kRounds; ++r)
#pragma unroll
        for (int k = 0; k < 4; ++k)
          if (t_super + r * kPerRound + tid * 16 + 4 * k == tail) {
            uint32_t word = 0u;
            for (int j = 0; j < ntok - tail; ++j)
              word |= (uint32_t)__hip_atomic_load(mask + tail + j, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) << (8 * j);
            m[r][k] = word;
          }
    }
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
      const int t0 = t_super + r * kPerRound + tid * 16;
      if (t_super + r * kPerRound >= ntok) break;      // uniform
      const int cnt = nonzero_bytes_u32(m[r][0]) + nonzero_bytes_u32(m[r][1]) + nonzero_bytes_u32(m[r][2]) +
                      nonzero_bytes_u32(m[r][3]);
      int inc = cnt;                                   // inclusive scan over the wave
#pragma unroll
      for (int o = 1; o < kWave; o <<= 1) {
        const int up = __shfl_up(inc, o, kWave);
        if (lane >= o) inc += up;
      }
      if (lane == kWave - 1) s_wave[r & 1][wv] = inc;
      __syncthreads();                                 // one barrier per round: the wave totals alternate between two rows
      int run = carry + inc - cnt, total = 0;          // selected tokens before this thread's first token
#pragma unroll
      for (int i = 0; i < kWaves; ++i) {
        const int c = s_wave[r & 1][i];
        if (i < wv) run += c;
        total += c;
      }
      carry += total;
      if (t0 < ntok) {
        int b = t0 / N, rr = t0 - b * N;
        int inv[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) {
          const int tok = t0 + k;
          const bool sel = ((m[r][k >> 2] >> (8 * (k & 3))) & 0xFFu) != 0u;   // bytes past ntok are zero: never selected
          if (tok < ntok && rr == 0) idx.cu_seqlens[b] = run;
          inv[k] = -1;
          if (sel) {
            idx.gather_idx[run] = tok;
            inv[k] = run;
            ++run;
          }
          if (++rr == N) { rr = 0; ++b; }
        }
        if (t0 + 16 <= ntok) {
#pragma unroll
          for (int k = 0; k < 16; k += 4) {
            const uintx4 v = {(uint32_t)inv[k], (uint32_t)inv[k + 1], (uint32_t)inv[k + 2], (uint32_t)inv[k + 3]};
            *reinterpret_cast<uintx4*>(idx.inv_pos + t0 + k) = v;
          }
        } else {
          for (int k = 0; k < ntok - t0; ++k) idx.inv_pos[t0 + k] = inv[k];
        }
      }
    }
  }
  if (tid == 0) {
    idx.cu_seqlens[B] = carry;
    if (idx.total != nullptr) idx.total[0] = carry;
  }
  if (idx.counts != nullptr) {                       // counts[b] = cu[b+1] - cu[b], from this workgroup's own writes
    __syncthreads();
    for (int b = tid; b < B; b += kGateThreads) idx.counts[b] = idx.cu_seqlens[b + 1] - idx.cu_seqlens[b];
  }
}

template <typename T, int G, bool kPool, bool kIndex>
__global__ void __launch_bounds__(kGateThreads)
gate_select_kernel(const T* __restrict__ x, const T* __restrict__ w, float bias,
                   const float* __restrict__ s_up, const float* __restrict__ noise, float theta, int ntok, int N, int C,
                   PoolGrid pool, float* __restrict__ scores, uint8_t* __restrict__ mask, IndexOut idx) {
  constexpr int VE = Vec16<T>::kElems;
  constexpr int kGroups = kGateThreads / G;
  const int grp = threadIdx.x / G;
  const int gl = threadIdx.x % G;
  const int chunks = C / VE;
  static_assert(kGroups % 4 == 0, "a pass of the workgroup covers whole 4-token words of the mask");
  __shared__ uint8_t s_sel[kGroups];
  for (long base = (long)blockIdx.x * kGroups; base < ntok; base += (long)gridDim.x * kGroups) {
    const long tok = base + grp;
    float acc = 0.f;
    if (tok < ntok) {
      // the lane's chunks of w come from memory like its chunks of the row (w is a few KB that every
      // workgroup reads: cache hits), issued together with them: no staging of w in LDS, no barrier
      // between the launch and the first row load
      const T* row = x + tok * (long)C;
#pragma unroll 4
      for (int ch = gl; ch < chunks; ch += G) {
        float f[VE], wv[VE];
        Vec16<T>::load(row + ch * VE, f);
        Vec16<T>::load(w + ch * VE, wv);
#pragma unroll
        for (int i = 0; i < VE; ++i) acc = fmaf(f[i], wv[i], acc);
      }
    }
    acc = group_sum<G>(acc);
    if (gl == 0 && tok < ntok) {
      float s = acc + bias;
      if (kPool) {
        const int b = (int)(tok / N), n = (int)(tok - (long)b * N);
        const int oy = n / pool.gw, ox = n - oy * pool.gw;
        const float* p = s_up + (long)b * N * 4 + (long)(2 * oy) * (2 * pool.gw) + 2 * ox;
        const float2 top = *reinterpret_cast<const float2*>(p);
        const float2 bot = *reinterpret_cast<const float2*>(p + 2 * pool.gw);
        const float up = fmaxf(fmaxf(top.x, top.y), fmaxf(bot.x, bot.y));
        if (pool.s_up_pooled != nullptr) pool.s_up_pooled[tok] = up;
        s = fmaxf(s, up);
      } else if (s_up != nullptr) {
        s = fmaxf(s, s_up[tok]);
      }
      // noise: logistic variate of the two-class Gumbel-Softmax; theta already carries the temperature
      const bool sel = (noise != nullptr ? s + noise[tok] : s) > theta;
      scores[tok] = s;
      if (kIndex) s_sel[grp] = sel ? 1 : 0;
      else mask[tok] = sel ? 1 : 0;
    }
    if (kIndex) {
      // With the index built in this launch the mask is written with agent-scope stores, whole
      // 4-token words (byte stores past the caches cost a partial write to memory each): such a
      // store goes through the XCD's write-back L2, so that the last workgroup, on whatever XCD it
      // runs, reads the bytes without any workgroup having to flush its L2.  The pass covers tokens
      // [base, base + kGroups), base a multiple of 4; the mask is 16-byte aligned.
      __syncthreads();
      if (threadIdx.x < kGroups / 4) {
        const long t4 = base + 4 * threadIdx.x;
        if (t4 + 4 <= ntok) {
          const uint32_t word = (uint32_t)s_sel[4 * threadIdx.x] | ((uint32_t)s_sel[4 * threadIdx.x + 1] << 8) |
                                ((uint32_t)s_sel[4 * threadIdx.x + 2] << 16) | ((uint32_t)s_sel[4 * threadIdx.x + 3] << 24);
          __hip_atomic_store(reinterpret_cast<uint32_t*>(mask + t4), word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        } else {
          for (long t = t4; t < ntok; ++t)
            __hip_atomic_store(mask + t, s_sel[t - base], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __builtin_amdgcn_s_waitcnt(0);               // the stores have completed before this thread goes on
      }
      __syncthreads();
    }
  }
  if (kIndex) {
    // sign off: this workgroup's mask stores have completed (see above; the barrier that ends the
    // last pass orders them before what follows) before its arrival is counted; the workgroup whose
    // arrival completes the count reads the mask with agent-scope loads and builds the index.  No
    // workgroup waits for another.
    __shared__ int s_last;
    if (threadIdx.x == 0) {
      const unsigned g = blockIdx.x % kArriveGroups, groups = min((unsigned)kArriveGroups, gridDim.x);
      const unsigned members = (gridDim.x - g + kArriveGroups - 1) / kArriveGroups;      // workgroups of group g
      unsigned* mine = idx.arrive + (1 + g) * kArriveStride;
      int last = 0;
      if (atomicAdd(mine, 1u) == members - 1) {      // last of its group: nobody touches this counter again
        __hip_atomic_store(mine, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (atomicAdd(idx.arrive, 1u) == groups - 1) {
          __hip_atomic_store(idx.arrive, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // counters left as found
          last = 1;
        }
      }
      s_last = last;
    }
    __syncthreads();
    if (s_last) build_pack_index(mask, ntok, N, ntok / N, idx);
  }
}

// counts[b] = selected tokens of image b: one workgroup per image, no atomics.
__global__ void __launch_bounds__(256)
count_selected_kernel(const uint8_t* __restrict__ mask, int N, int32_t* __restrict__ counts) {
  __shared__ int red[4];
  const uint8_t* m = mask + (long)blockIdx.x * N;
  int c = 0;
  for (int i = threadIdx.x; i < N; i += 256) c += m[i] != 0;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) c += __shfl_xor(c, o, kWave);
  if (lane_id() == 0) red[threadIdx.x / kWave] = c;
  __syncthreads();
  if (threadIdx.x == 0) counts[blockIdx.x] = red[0] + red[1] + red[2] + red[3];
}

__global__ void maxpool2x2_kernel(const float* __restrict__ s, int B, int h, int w,
                                  float* __restrict__ out) {
  const int ho = h / 2, wo = w / 2;
  const long n = (long)B * ho * wo;
  for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (long)gridDim.x * blockDim.x) {
    const int b = i / (ho * wo);
    const int r = i % (ho * wo);
    const int oy = r / wo, ox = r % wo;
    const float* p = s + (long)b * h * w + (long)(2 * oy) * w + 2 * ox;
    out[i] = fmaxf(fmaxf(p[0], p[1]), fmaxf(p[w], p[w + 1]));
  }
}


// ---------------------------------------------------------------------- gate backward
// Selection loss (binary cross-entropy on sigmoid(s)) + gradient of r_g = sigmoid(s) . r.
// A group of G lanes owns a token; the row's chunks live in registers (IT per lane), so x
// and d_rg are read once.  dw / db / loss are reduced without atomics: lanes accumulate
// over their tokens, groups are folded in a fixed order into LDS, every workgroup writes one
// partial row, and a second kernel adds the partial rows in order.
// Straight-through estimator of the hard selection: selected tokens differentiate the relaxed
// weight sigmoid((s + noise) / T) in place of the 0/1 mask.  mask == nullptr: off.
struct StraightThrough {
  const uint8_t* mask;
  const float* noise;   // may be null (noise-free selection)
  float inv_temperature;
};

template <typename T, int G, int IT>
__global__ void __launch_bounds__(kGateThreads)
gate_bwd_kernel(const T* __restrict__ x, const T* __restrict__ w, float bias,
                const float* __restrict__ scores, const float* __restrict__ s_up,
                const uint8_t* __restrict__ labels, const T* __restrict__ d_rg, int gate_scaled,
                float loss_scale, StraightThrough st, int ntok, int C, T* __restrict__ dx,
                float* __restrict__ partial, int fold_parallel) {
  constexpr int VE = Vec16<T>::kElems;
  constexpr int kGroups = kGateThreads / G;
  extern __shared__ float lds[];
  float* w_lds = lds;            // [C]
  float* sdw = lds + C;          // [C]
  __shared__ float s_loss[kGroups], s_db[kGroups];
  for (int c = threadIdx.x; c < C; c += kGateThreads) { w_lds[c] = static_cast<float>(w[c]); sdw[c] = 0.f; }
  __syncthreads();

  const int grp = threadIdx.x / G, gl = threadIdx.x % G;
  const int chunks = C / VE;
  const bool scaled = gate_scaled != 0 && d_rg != nullptr;
  float dwa[IT][VE];
#pragma unroll
  for (int it = 0; it < IT; ++it)
#pragma unroll
    for (int e = 0; e < VE; ++e) dwa[it][e] = 0.f;
  float loss_acc = 0.f, db_acc = 0.f;

  for (long tok = (long)blockIdx.x * kGroups + grp; tok < ntok; tok += (long)gridDim.x * kGroups) {
    float xr[IT][VE], dr[IT][VE];
    float dot = 0.f, g = 0.f;
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      const int ch = gl + it * G;
#pragma unroll
      for (int e = 0; e < VE; ++e) { xr[it][e] = 0.f; dr[it][e] = 0.f; }
      if (ch < chunks) {
        Vec16<T>::load(x + tok * (long)C + ch * VE, xr[it]);
        if (scaled) Vec16<T>::load(d_rg + tok * (long)C + ch * VE, dr[it]);
#pragma unroll
        for (int e = 0; e < VE; ++e) {
          dot = fmaf(dr[it][e], xr[it][e], dot);
          g = fmaf(xr[it][e], w_lds[ch * VE + e], g);
        }
      }
    }
    dot = group_sum<G>(dot);
    const float s = scores[tok];
    bool own = true;
    if (s_up != nullptr) {
      g = group_sum<G>(g) + bias;
      own = g >= s_up[tok];                 // the up-scale score won the max: no gradient to (w, b)
    }
    const float p = sigmoidf_dev(s);
    const float y = labels[tok] != 0 ? 1.f : 0.f;
    float ds = loss_scale * (p - y);
    if (scaled) {
      float coef = p * (1.f - p);                      // through r_g = sigmoid(s) . r
      if (st.mask != nullptr && st.mask[tok] != 0) {   // through the relaxed selection weight: <d_rg, r_g> = p dot
        const float pt = sigmoidf_dev((s + (st.noise != nullptr ? st.noise[tok] : 0.f)) * st.inv_temperature);
        coef = fmaf(pt * (1.f - pt) * st.inv_temperature, p, coef);
      }
      ds = fmaf(coef, dot, ds);
    }
    const float dsg = own ? ds : 0.f;
    const float pg = scaled ? p : 0.f;
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      const int ch = gl + it * G;
      if (ch < chunks) {
        float o[VE];
#pragma unroll
        for (int e = 0; e < VE; ++e) {
          o[e] = fmaf(dsg, w_lds[ch * VE + e], pg * dr[it][e]);
          dwa[it][e] = fmaf(dsg, xr[it][e], dwa[it][e]);
        }
        Vec16<T>::store(dx + tok * (long)C + ch * VE, o);
      }
    }
    if (gl == 0) {
      loss_acc += fmaxf(s, 0.f) - y * s + log1pf(__expf(-fabsf(s)));
      db_acc += dsg;
    }
  }

  // fold the groups in a fixed order (group 0, 1, ...).  When the per-group partials fit in
  // LDS every group parks its partial row and each thread adds a column top to bottom; else
  // the groups take turns adding into one LDS row.
  if (fold_parallel) {
    float* grows = sdw + C;                       // [kGroups][C]
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      const int ch = gl + it * G;
      if (ch < chunks) {
#pragma unroll
        for (int e = 0; e < VE; ++e) grows[grp * C + ch * VE + e] = dwa[it][e];
      }
    }
    __syncthreads();
    for (int c = threadIdx.x; c < C; c += kGateThreads) {
      float a = 0.f;
#pragma unroll
      for (int g2 = 0; g2 < kGroups; ++g2) a += grows[g2 * C + c];
      sdw[c] = a;
    }
    __syncthreads();
  } else {
    for (int gsel = 0; gsel < kGroups; ++gsel) {
      if (grp == gsel) {
#pragma unroll
        for (int it = 0; it < IT; ++it) {
          const int ch = gl + it * G;
          if (ch < chunks) {
#pragma unroll
            for (int e = 0; e < VE; ++e) sdw[ch * VE + e] += dwa[it][e];
          }
        }
      }
      __syncthreads();
    }
  }
  if (gl == 0) { s_loss[grp] = loss_acc; s_db[grp] = db_acc; }
  __syncthreads();
  float* prow = partial + (long)blockIdx.x * (C + 2);
  for (int c = threadIdx.x; c < C; c += kGateThreads) prow[c] = sdw[c];
  if (threadIdx.x == 0) {
    float a = 0.f, b = 0.f;
    for (int i = 0; i < kGroups; ++i) { a += s_loss[i]; b += s_db[i]; }
    prow[C] = a;
    prow[C + 1] = b;
  }
}

// Adds the partial rows in a fixed order: a block owns 16 columns; 16 row slices run in
// parallel (slice s adds rows s, s+16, ...), then the slices are added 0..15.
__global__ void __launch_bounds__(256)
gate_bwd_reduce_kernel(const float* __restrict__ partial, int nparts, int C, float loss_scale,
                       float* __restrict__ loss, float* __restrict__ dw, float* __restrict__ db) {
  __shared__ float red[16][17];
  const int cl = threadIdx.x & 15, sl = threadIdx.x >> 4;
  const int c = blockIdx.x * 16 + cl;
  float a = 0.f;
  if (c < C + 2) {
#pragma unroll 8
    for (int i = sl; i < nparts; i += 16) a += partial[(long)i * (C + 2) + c];
  }
  red[sl][cl] = a;
  __syncthreads();
  if (sl == 0 && c < C + 2) {
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) t += red[i][cl];
    if (c < C) dw[c] = t;
    else if (c == C) loss[0] = t * loss_scale;
    else db[0] = t;
  }
}

constexpr int kGateBwdMaxParts = 512;

static int gate_bwd_parts(long ntok) {
  long p = (ntok + 15) / 16;
  if (p > kGateBwdMaxParts) p = kGateBwdMaxParts;
  if (p < 1) p = 1;
  return (int)p;
}

template <typename T>
static int launch_gate(const char* fn, const void* x, const void* w, float bias, const float* s_up,
                       const float* noise, float theta, int B, int N, int C, PoolGrid pool, bool pooled,
                       float* scores, uint8_t* mask, int32_t* counts, hipStream_t st,
                       IndexOut idx = IndexOut{nullptr, nullptr, nullptr, nullptr, nullptr, nullptr}) {
  constexpr int VE = Vec16<T>::kElems;
  const int chunks = C / VE;
  const long ntok = (long)B * N;
  const size_t lds = 0;      // (the gate weight is read from memory, nothing is staged)
  auto go = [&](auto gtag) {
    constexpr int G = decltype(gtag)::value;
    const long per_wg = kGateThreads / G;
    long wgs = (ntok + per_wg - 1) / per_wg;
    if (wgs > 4096) wgs = 4096;
    if (pooled)
      hipLaunchKernelGGL((gate_select_kernel<T, G, true, false>), dim3((unsigned)wgs), dim3(kGateThreads), lds, st,
                         static_cast<const T*>(x), static_cast<const T*>(w), bias, s_up, noise, theta,
                         (int)ntok, N, C, pool, scores, mask, idx);
    else if (idx.arrive != nullptr)
      hipLaunchKernelGGL((gate_select_kernel<T, G, false, true>), dim3((unsigned)wgs), dim3(kGateThreads), lds, st,
                         static_cast<const T*>(x), static_cast<const T*>(w), bias, s_up, noise, theta,
                         (int)ntok, N, C, pool, scores, mask, idx);
    else
      hipLaunchKernelGGL((gate_select_kernel<T, G, false, false>), dim3((unsigned)wgs), dim3(kGateThreads), lds, st,
                         static_cast<const T*>(x), static_cast<const T*>(w), bias, s_up, noise, theta,
                         (int)ntok, N, C, pool, scores, mask, idx);
  };
  if (chunks <= 8) go(std::integral_constant<int, 8>{});
  else if (chunks <= 64) go(std::integral_constant<int, 16>{});
  else if (chunks <= 256) go(std::integral_constant<int, 32>{});
  else go(std::integral_constant<int, 64>{});
  if (counts != nullptr && idx.arrive == nullptr)
    hipLaunchKernelGGL(count_selected_kernel, dim3(B), dim3(256), 0, st, mask, N, counts);
  return check_launch(fn);
}

}  // namespace spa

using namespace spa;

static int gate_select_common(const char* fn, const void* x, const void* w, float bias, const float* s_up,
                              const float* noise, float temperature, float tau, int B, int N, int C, int dtype,
                              float* scores, uint8_t* mask, int32_t* counts, void* stream,
                              PoolGrid pool = PoolGrid{0, 0, nullptr}, bool pooled = false,
                              IndexOut idx = IndexOut{nullptr, nullptr, nullptr, nullptr, nullptr, nullptr}) {
  SPA_REQUIRE(x && w && scores && mask, SPA_ERR_INVALID_ARG, "%s: null pointer", fn);
  SPA_REQUIRE(B >= 1 && N >= 1 && C >= 1, SPA_ERR_INVALID_ARG, "%s: B, N, C must be >= 1", fn);
  SPA_REQUIRE((long)B * N < 2147483647L, SPA_ERR_INVALID_ARG, "%s: B*N must be < 2^31", fn);
  SPA_REQUIRE(tau > 0.f && tau < 1.f, SPA_ERR_INVALID_ARG, "%s: tau must lie in (0,1), got %g", fn, (double)tau);
  SPA_REQUIRE(temperature > 0.f && std::isfinite(temperature), SPA_ERR_INVALID_ARG,
              "%s: temperature must be positive and finite, got %g", fn, (double)temperature);
  SPA_REQUIRE(dtype == SPA_F32 || dtype == SPA_BF16, SPA_ERR_UNSUPPORTED, "%s: unknown dtype %d", fn, dtype);
  SPA_REQUIRE(((long)C * elem_size(dtype)) % 16 == 0, SPA_ERR_INVALID_ARG,
              "%s: row length C*elem = %ld bytes is not a multiple of 16", fn, (long)C * elem_size(dtype));
  SPA_REQUIRE(aligned16(x), SPA_ERR_INVALID_ARG, "%s: x is not 16-byte aligned", fn);
  SPA_REQUIRE(C <= kMaxGateC, SPA_ERR_UNSUPPORTED, "%s: C = %d exceeds %d", fn, C, kMaxGateC);
  // sigmoid((s + e) / T) > tau  <=>  s + e > T * logit(tau)
  const float theta = (float)((double)temperature * std::log((double)tau / (1.0 - (double)tau)));
  hipStream_t st = as_stream(stream);
  if (dtype == SPA_F32)
    return launch_gate<float>(fn, x, w, bias, s_up, noise, theta, B, N, C, pool, pooled, scores, mask, counts, st, idx);
  return launch_gate<__bf16>(fn, x, w, bias, s_up, noise, theta, B, N, C, pool, pooled, scores, mask, counts, st, idx);
}

extern "C" int spa_gate_select(const void* x, const void* w, float bias, const float* s_up,
                               float tau, int B, int N, int C, int dtype, float* scores,
                               uint8_t* mask, int32_t* counts, void* stream) {
  return gate_select_common("spa_gate_select", x, w, bias, s_up, nullptr, 1.f, tau, B, N, C, dtype, scores, mask,
                            counts, stream);
}

extern "C" int spa_gate_select_index(const void* x, const void* w, float bias, const float* s_up, float tau, int B,
                                     int N, int C, int dtype, float* scores, uint8_t* mask, int32_t* counts,
                                     int32_t* cu_seqlens, int32_t* gather_idx, int32_t* inv_pos, int32_t* total,
                                     void* workspace, size_t workspace_bytes, void* stream) {
  const char* fn = "spa_gate_select_index";
  SPA_REQUIRE(cu_seqlens && gather_idx && inv_pos, SPA_ERR_INVALID_ARG, "%s: null index pointer", fn);
  SPA_REQUIRE(workspace != nullptr && workspace_bytes >= kArriveWords * sizeof(unsigned), SPA_ERR_WORKSPACE,
              "%s: workspace of %zu bytes needed (zero-filled once, left zero by every call), %zu given", fn,
              kArriveWords * sizeof(unsigned), workspace_bytes);
  SPA_REQUIRE((reinterpret_cast<uintptr_t>(workspace) & 3u) == 0 && aligned16(mask) && aligned16(inv_pos),
              SPA_ERR_INVALID_ARG, "%s: mask / inv_pos not 16-byte aligned or workspace not 4-byte aligned", fn);
  const IndexOut idx = {cu_seqlens, gather_idx, inv_pos, total, counts, static_cast<unsigned*>(workspace)};
  return gate_select_common(fn, x, w, bias, s_up, nullptr, 1.f, tau, B, N, C, dtype, scores, mask, counts, stream,
                            PoolGrid{0, 0, nullptr}, false, idx);
}

extern "C" int spa_gate_select_gumbel(const void* x, const void* w, float bias, const float* s_up,
                                      const float* noise, float temperature, float tau, int B, int N, int C,
                                      int dtype, float* scores, uint8_t* mask, int32_t* counts, void* stream) {
  SPA_REQUIRE(noise != nullptr, SPA_ERR_INVALID_ARG, "spa_gate_select_gumbel: noise is null");
  return gate_select_common("spa_gate_select_gumbel", x, w, bias, s_up, noise, temperature, tau, B, N, C, dtype,
                            scores, mask, counts, stream);
}

extern "C" int spa_gate_select_pooled(const void* x, const void* w, float bias, const float* s_fine,
                                      float tau, int B, int grid_h, int grid_w, int C, int dtype, float* scores,
                                      uint8_t* mask, int32_t* counts, float* s_up_pooled, void* stream) {
  const char* fn = "spa_gate_select_pooled";
  SPA_REQUIRE(s_fine != nullptr, SPA_ERR_INVALID_ARG, "%s: s_fine is null", fn);
  SPA_REQUIRE(grid_h >= 1 && grid_w >= 1 && (long)grid_h * grid_w < 2147483647L / 4, SPA_ERR_INVALID_ARG,
              "%s: grid_h, grid_w must be >= 1", fn);
  SPA_REQUIRE((reinterpret_cast<uintptr_t>(s_fine) & 7) == 0, SPA_ERR_INVALID_ARG, "%s: s_fine not 8-byte aligned", fn);
  return gate_select_common(fn, x, w, bias, s_fine, nullptr, 1.f, tau, B, grid_h * grid_w, C, dtype, scores, mask,
                            counts, stream, PoolGrid{grid_h, grid_w, s_up_pooled}, true);
}

extern "C" int spa_maxpool2x2(const float* s, int B, int h, int w, float* pooled, void* stream) {
  SPA_REQUIRE(s && pooled, SPA_ERR_INVALID_ARG, "spa_maxpool2x2: null pointer");
  SPA_REQUIRE(B >= 1 && h >= 2 && w >= 2 && h % 2 == 0 && w % 2 == 0, SPA_ERR_INVALID_ARG,
              "spa_maxpool2x2: need B >= 1 and even h, w >= 2 (got %d, %d, %d)", B, h, w);
  const long n = (long)B * (h / 2) * (w / 2);
  long wgs = (n + 255) / 256;
  if (wgs > 2048) wgs = 2048;
  hipLaunchKernelGGL(maxpool2x2_kernel, dim3((unsigned)wgs), dim3(256), 0, as_stream(stream), s, B, h, w, pooled);
  return check_launch("spa_maxpool2x2");
}

extern "C" size_t spa_gate_bwd_workspace_bytes(int B, int N, int C, int dtype) {
  (void)dtype;
  if (B < 1 || N < 1 || C < 1) return 0;
  return (size_t)gate_bwd_parts((long)B * N) * (size_t)(C + 2) * sizeof(float);
}

template <typename T>
static int launch_gate_bwd(const void* x, const void* w, float bias, const float* scores, const float* s_up,
                           const uint8_t* labels, const void* d_rg, int gate_scaled, float loss_scale,
                           StraightThrough stt, long ntok, int C, float* loss, void* dx, float* dw, float* db,
                           float* partial, hipStream_t st) {
  constexpr int VE = Vec16<T>::kElems;
  const int chunks = C / VE;
  const int parts = gate_bwd_parts(ntok);
  // LDS: w [C] + dw row [C] (+ one partial row per group when that fits in 64 KB)
  const int groups = chunks <= 128 ? 16 : 4;
  const int fold_parallel = (size_t)(2 + groups) * C * sizeof(float) <= 65536 ? 1 : 0;
  const size_t lds = (size_t)(fold_parallel ? 2 + groups : 2) * C * sizeof(float);
#define SPA_GB(G, IT)                                                                                         \
  hipLaunchKernelGGL((gate_bwd_kernel<T, G, IT>), dim3(parts), dim3(kGateThreads), lds, st,                  \
                     static_cast<const T*>(x), static_cast<const T*>(w), bias, scores, s_up, labels,         \
                     static_cast<const T*>(d_rg), gate_scaled, loss_scale, stt, (int)ntok, C,                \
                     static_cast<T*>(dx), partial, fold_parallel)
  if (chunks <= 16) SPA_GB(16, 1);
  else if (chunks <= 32) SPA_GB(16, 2);
  else if (chunks <= 64) SPA_GB(16, 4);
  else if (chunks <= 128) SPA_GB(16, 8);
  else if (chunks <= 256) SPA_GB(64, 4);
  else if (chunks <= 512) SPA_GB(64, 8);
  else return fail(SPA_ERR_UNSUPPORTED, "spa_gate_bwd: C = %d too large (at most %d)", C, 512 * VE);
#undef SPA_GB
  hipLaunchKernelGGL(gate_bwd_reduce_kernel, dim3((C + 2 + 15) / 16), dim3(256), 0, st, partial, parts, C,
                     loss_scale, loss, dw, db);
  return check_launch("spa_gate_bwd");
}

static int gate_bwd_common(const char* fn, const void* x, const void* w, float bias, const float* scores,
                           const float* s_up, const uint8_t* labels, const void* d_rg, int gate_scaled,
                           float loss_scale, StraightThrough stt, int B, int N, int C, int dtype, float* loss,
                           void* dx, float* dw, float* db, void* workspace, size_t workspace_bytes, void* stream) {
  SPA_REQUIRE(x && w && scores && labels && loss && dx && dw && db, SPA_ERR_INVALID_ARG, "%s: null pointer", fn);
  SPA_REQUIRE(B >= 1 && N >= 1 && C >= 1, SPA_ERR_INVALID_ARG, "%s: B, N, C must be >= 1", fn);
  SPA_REQUIRE((long)B * N < 2147483647L, SPA_ERR_INVALID_ARG, "%s: B*N must be < 2^31", fn);
  SPA_REQUIRE(dtype == SPA_F32 || dtype == SPA_BF16, SPA_ERR_UNSUPPORTED, "%s: unknown dtype %d", fn, dtype);
  SPA_REQUIRE(((long)C * elem_size(dtype)) % 16 == 0, SPA_ERR_INVALID_ARG,
              "%s: row length C*elem = %ld bytes is not a multiple of 16", fn, (long)C * elem_size(dtype));
  SPA_REQUIRE(aligned16(x) && aligned16(dx) && aligned16(d_rg), SPA_ERR_INVALID_ARG,
              "%s: x / dx / d_rg not 16-byte aligned", fn);
  SPA_REQUIRE(!(gate_scaled && !d_rg), SPA_ERR_INVALID_ARG, "%s: gate_scaled needs d_rg", fn);
  SPA_REQUIRE(C <= kMaxGateC, SPA_ERR_UNSUPPORTED, "%s: C = %d exceeds %d", fn, C, kMaxGateC);
  const size_t need = spa_gate_bwd_workspace_bytes(B, N, C, dtype);
  SPA_REQUIRE(workspace != nullptr && workspace_bytes >= need, SPA_ERR_WORKSPACE,
              "%s: workspace of %zu bytes needed, %zu given", fn, need, workspace_bytes);
  hipStream_t st = as_stream(stream);
  float* partial = static_cast<float*>(workspace);
  if (dtype == SPA_F32)
    return launch_gate_bwd<float>(x, w, bias, scores, s_up, labels, d_rg, gate_scaled, loss_scale, stt, (long)B * N,
                                  C, loss, dx, dw, db, partial, st);
  return launch_gate_bwd<__bf16>(x, w, bias, scores, s_up, labels, d_rg, gate_scaled, loss_scale, stt, (long)B * N,
                                 C, loss, dx, dw, db, partial, st);
}

extern "C" int spa_gate_bwd(const void* x, const void* w, float bias, const float* scores,
                            const float* s_up, const uint8_t* labels, const void* d_rg, int gate_scaled,
                            float loss_scale, int B, int N, int C, int dtype, float* loss, void* dx,
                            float* dw, float* db, void* workspace, size_t workspace_bytes, void* stream) {
  return gate_bwd_common("spa_gate_bwd", x, w, bias, scores, s_up, labels, d_rg, gate_scaled, loss_scale,
                         StraightThrough{nullptr, nullptr, 1.f}, B, N, C, dtype, loss, dx, dw, db, workspace,
                         workspace_bytes, stream);
}

// ---- the gate backward for callers that cannot allocate --------------------------------
// The partial rows of the two-stage reduction live in a file-scope device array instead of a
// caller workspace.  The array's name is a host-side stand-in, not a device address: its
// address on the current device is looked up once per device with hipGetSymbolAddress and that
// pointer is what the kernels get.
namespace spa {
constexpr int kNoAllocMaxC = 1024;
constexpr int kNoAllocMaxDevices = 64;
static __device__ __align__(256) float scratch[(size_t)kGateBwdMaxParts * (kNoAllocMaxC + 2)];
static float* g_scratch_ptr[kNoAllocMaxDevices] = {};
static std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device (looked up on the first call on that device).
static int scratch_on_current_device(const char* fn, float** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(SPA_ERR_HIP, "%s: hipGetDevice: %s", fn, hipGetErrorString(e));
  SPA_REQUIRE(dev >= 0 && dev < kNoAllocMaxDevices, SPA_ERR_UNSUPPORTED, "%s: device %d beyond %d", fn, dev,
              kNoAllocMaxDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || p == nullptr)
      return fail(SPA_ERR_HIP, "%s: hipGetSymbolAddress(scratch): %s", fn, hipGetErrorString(e));
    g_scratch_ptr[dev] = static_cast<float*>(p);
  }
  *out = g_scratch_ptr[dev];
  return SPA_OK;
}
}  // namespace spa

extern "C" int spa_gate_bwd_static(const void* x, const void* w, float bias, const float* scores,
                                   const float* s_up, const uint8_t* labels, const void* d_rg, int gate_scaled,
                                   float loss_scale, int B, int N, int C, int dtype, float* loss, void* dx,
                                   float* dw, float* db, void* stream) {
  const char* fn = "spa_gate_bwd_static";
  SPA_REQUIRE(C >= 1 && C <= kNoAllocMaxC, SPA_ERR_WORKSPACE,
              "%s: C = %d exceeds the built-in scratch (C <= %d); use spa_gate_bwd with a workspace", fn, C,
              kNoAllocMaxC);
  SPA_REQUIRE(B >= 1 && N >= 1, SPA_ERR_INVALID_ARG, "%s: B, N must be >= 1", fn);
  const size_t need = spa_gate_bwd_workspace_bytes(B, N, C, dtype);
  SPA_REQUIRE(need <= sizeof(float) * (size_t)kGateBwdMaxParts * (kNoAllocMaxC + 2), SPA_ERR_WORKSPACE,
              "%s: %zu bytes of scratch needed, more than the built-in array holds", fn, need);
  float* ptr = nullptr;
  if (int rc = scratch_on_current_device(fn, &ptr)) return rc;
  // every partial row the reduction reads is written by this call's first kernel: nothing to clear
  return gate_bwd_common(fn, x, w, bias, scores, s_up, labels, d_rg, gate_scaled, loss_scale,
                         StraightThrough{nullptr, nullptr, 1.f}, B, N, C, dtype, loss, dx, dw, db, ptr, need, stream);
}

extern "C" int spa_gate_bwd_straight_through(const void* x, const void* w, float bias, const float* scores,
                                             const float* s_up, const uint8_t* labels, const void* d_rg,
                                             float loss_scale, const uint8_t* mask, const float* noise,
                                             float temperature, int B, int N, int C, int dtype, float* loss,
                                             void* dx, float* dw, float* db, void* workspace,
                                             size_t workspace_bytes, void* stream) {
  const char* fn = "spa_gate_bwd_straight_through";
  SPA_REQUIRE(mask && d_rg, SPA_ERR_INVALID_ARG, "%s: mask and d_rg are required", fn);
  SPA_REQUIRE(temperature > 0.f && std::isfinite(temperature), SPA_ERR_INVALID_ARG,
              "%s: temperature must be positive and finite, got %g", fn, (double)temperature);
  return gate_bwd_common(fn, x, w, bias, scores, s_up, labels, d_rg, 1, loss_scale,
                         StraightThrough{mask, noise, 1.f / temperature}, B, N, C, dtype, loss, dx, dw, db, workspace,
                         workspace_bytes, stream);
}
