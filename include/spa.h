/*
 * libspa — Select-and-Pack Attention (SPA) hot path for AMD MI355X (gfx950).
 *
 * The calls follow the paper's statement of the SPA / SnP block (Section 3.2):
 *   scores  s   = Max(f_g(r), s_up)                      spa_gate_select
 *   select  r_p = hard(Gumbel-Softmax(s)) . r_g          spa_gate_select (mask) + spa_pack
 *   pack    survivors of every image, in order, no padding to the batch maximum
 *                                                        spa_pack
 *   masked multi-head self-attention on the packed tokens, a token attends only to
 *   tokens of its own image                              spa_packed_attention
 *   selected tokens return to their positions, the others bypass attention
 *                                                        spa_unpack
 * and, for training, the transposes of those steps plus the selection loss of
 * Section 3.3.
 *
 * Conventions (all entry points)
 *   - Every pointer is a DEVICE pointer unless it is said to be a host value; scalars are
 *     passed by value.  The caller owns every buffer; the library allocates, frees and
 *     retains nothing.  Buffers must not overlap unless stated.
 *   - Row-major, innermost dimension contiguous.  Token t of image b is flat token b*N + t.
 *   - dtype is SPA_F32 or SPA_BF16 and names the storage type of the feature tensors
 *     (x, packed, q/k/v, out, y, their gradients).  Scores, lse, loss, dw, db are fp32.
 *     Arithmetic accumulates in fp32; bf16 attention uses bf16 MFMA with fp32 softmax.
 *   - `stream` is a hipStream_t (NULL = the null stream).  Calls enqueue work and return
 *     without synchronising.  No call reads device memory on the host: output buffers are
 *     sized by the capacity B*N, and the number of selected tokens stays on the device.
 *   - Return value: SPA_OK, or a negative SPA_ERR_* code.  Arguments are validated before
 *     anything is launched; on error nothing has been enqueued and spa_last_error() (a
 *     thread-local, host string) says what was wrong.
 *   - Feature rows must be 16-byte aligned: base pointers 16-byte aligned and row length
 *     in bytes (C * element size, row_stride * element size) a multiple of 16.
 *   - B >= 1, N >= 1, B*N < 2^31.
 */
#ifndef SPA_H
#define SPA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SPA_OK 0
#define SPA_ERR_INVALID_ARG (-1)  /* null pointer, bad size, misalignment, tau outside (0,1) */
#define SPA_ERR_UNSUPPORTED (-2)  /* dtype / head dim the kernels do not cover */
#define SPA_ERR_WORKSPACE (-3)    /* workspace missing or too small */
#define SPA_ERR_HIP (-4)          /* the HIP runtime reported an error at launch */

#define SPA_F32 0
#define SPA_BF16 1

/* Library version (major*10000 + minor*100 + patch). Host. */
int spa_version(void);

/* Message of the last failing call on this thread ("" if none). Host string owned by the
 * library; valid until the next failing call on the same thread. */
const char* spa_last_error(void);

/*
 * Launch options (host, process-wide; not part of the method).  Every option has a default
 * that is the measured best; the alternatives select other kernels of the library for the same
 * call (used by the parity tests to cover them, and for tuning).  Each option is also read ONCE,
 * when the library is loaded, from the environment variable SPA_<NAME IN CAPITALS>; nothing on a
 * launch path reads the environment.  value NULL or "" restores the default.  Not synchronised
 * with calls running on other host threads.  Returns SPA_ERR_INVALID_ARG for an unknown name or a
 * malformed value (nothing changes then).
 *   attn_fwd_short     words of: "whole" (one workgroup per (image, head)), "64" (64-key steps),
 *                      "plain" (one-wave blocks numbered blindly instead of by weight)
 *   attn_fwd_long      "two": the long-segment forward kernel with two chains of 32 queries per wave
 *                      sharing every K / V fragment (default: one chain per wave)
 *   attn_fwd_cfg       "NW,BN": the one-chain tiled forward kernel with NW in {2,4} waves, BN in {64,128} keys
 *   attn_fwd_wave_max  longest segment (<= 256) the one-wave forward kernels take
 *   attn_bwd_short     "split" | "tiled": two-kernel / long-segment backward for segments <= 256
 *   attn_bwd_long      "two": the dq and dkdv roles of the long-segment backward as two launches
 *   gemm_tm            2 | 4 | 8: 128x128, 256x128, 256x256 projection tiles
 *   gemm_splits        1..16 token chunks of the weight-side GEMM
 *   pack_tile          16 | 32 | 64 | 128 | 256 tokens per packing workgroup
 */
int spa_set_option(const char* name, const char* value);

/*
 * Bytes of workspace that call `op` needs for a batch of B images x N tokens, width C, H heads
 * (the one query over the per-call ones below; Section 3.2 / 3.3 name the calls).  0 for the
 * calls that need none (all forward calls and the row-moving transposes), and for bad arguments.
 * The projection ops take M_cap = B*N rows, K = C and N_out = 3C (QKV) or C (output).  Host.
 */
#define SPA_OP_GATE_SELECT 0
#define SPA_OP_PACK 1
#define SPA_OP_PACKED_ATTENTION 2
#define SPA_OP_UNPACK 3
#define SPA_OP_PACKED_ATTENTION_BWD 4
#define SPA_OP_GATE_BWD 5
#define SPA_OP_QKV_PROJECTION_BWD_WEIGHT 6
#define SPA_OP_OUT_PROJECTION_BWD_WEIGHT 7
size_t spa_workspace_bytes(int op, int B, int N, int C, int H, int dtype);

/*
 * Gate scoring and selection (Section 3.2, equations for s and r_p).
 *   g_i      = bias + sum_c w[c] * x[i,c]            (linear gating layer f_g)
 *   scores_i = max(g_i, s_up[i]) if s_up else g_i    (s = Max(f_g(r), s_up))
 *   mask_i   = scores_i > ln(tau/(1-tau))            (hard, noise-free Gumbel-Softmax
 *                                                     decision sigmoid(s) > tau; a tie is
 *                                                     not selected)
 *   counts_b = number of selected tokens of image b
 * in:  x [B,N,C] dtype; w [C] dtype; bias (host float); s_up [B,N] fp32 or NULL (scores of
 *      the finer stage already max-pooled to this stage's grid, see spa_maxpool2x2);
 *      tau in (0,1) (host float).
 * out: scores [B,N] fp32 logits; mask [B,N] uint8 (0/1); counts [B] int32 or NULL.
 */
int spa_gate_select(const void* x, const void* w, float bias, const float* s_up, float tau,
                    int B, int N, int C, int dtype,
                    float* scores, uint8_t* mask, int32_t* counts, void* stream);

/*
 * spa_gate_select and the index-only spa_pack in ONE launch (Section 3.2: scores s, hard selection,
 * and the order in which "Token Packing" lines the survivors up): the workgroup of the gate kernel
 * that finishes last walks the finished mask once and writes the packing index.  There is no
 * waiting between workgroups; one arrival counter in `workspace` tells which workgroup is last.
 * in:  as spa_gate_select (mask and inv_pos 16-byte aligned); workspace: at least 73984 bytes of
 *      device memory, 4-byte aligned, ZERO before the first call; every call leaves it zero, so
 *      consecutive calls on one stream may share it (calls that overlap in time must not).
 * out: scores, mask, counts (or NULL) as spa_gate_select; cu_seqlens [B+1], gather_idx [B*N],
 *      inv_pos [B*N], total [1] (or NULL) exactly as spa_pack writes them (bit for bit).
 */
int spa_gate_select_index(const void* x, const void* w, float bias, const float* s_up, float tau,
                          int B, int N, int C, int dtype, float* scores, uint8_t* mask, int32_t* counts,
                          int32_t* cu_seqlens, int32_t* gather_idx, int32_t* inv_pos, int32_t* total,
                          void* workspace, size_t workspace_bytes, void* stream);

/*
 * Stochastic selection (Section 3.2, r_p = Gumbel-Softmax(s) . r_g): Gumbel-Softmax of the
 * two-class logits [s, 0].  With e_i = g1 - g2 the difference of two Gumbel(0,1) draws (a
 * Logistic(0,1) variate) the relaxed weight of the 'select' class is
 *   p~_i = sigmoid((scores_i + e_i) / temperature)
 * and the token is selected when p~_i > tau, decided as scores_i + e_i > temperature*logit(tau)
 * in fp32 (strict).  The library draws no random numbers: the caller supplies e.
 * in:  as spa_gate_select, plus noise [B,N] fp32 (e_i) and temperature > 0 (host float).
 * out: scores [B,N] fp32 (the logits s, WITHOUT the noise); mask; counts as spa_gate_select.
 * spa_gate_select is the noise-free case e = 0, temperature = 1.
 */
int spa_gate_select_gumbel(const void* x, const void* w, float bias, const float* s_up,
                           const float* noise, float temperature, float tau, int B, int N, int C,
                           int dtype, float* scores, uint8_t* mask, int32_t* counts, void* stream);

/*
 * 2x2 stride-2 max-pooling of a score map, used to hand the scores of a finer stage to
 * the next one (Section 3.2: up-scale scores "adjusted via max-pooling").
 * in:  s [B, h*w] fp32 (h, w even).   out: pooled [B, (h/2)*(w/2)] fp32.
 */
int spa_maxpool2x2(const float* s, int B, int h, int w, float* pooled, void* stream);

/*
 * spa_gate_select with the 2x2 max-pooling of the finer stage's score map folded in
 * (Section 3.2: s = Max(f_g(r), s_up) with s_up "adjusted via max-pooling"): one launch per
 * stage of a hierarchy instead of two.  This stage's tokens form a grid_h x grid_w map
 * (N = grid_h*grid_w); s_fine is the score map of the previous, 2x finer stage.
 * in:  x [B,N,C], w [C] dtype; bias; s_fine [B, 2*grid_h, 2*grid_w] fp32 (8-byte aligned); tau.
 * out: scores, mask, counts as spa_gate_select; s_up_pooled [B,N] fp32 or NULL: the pooled
 *      scores, which spa_gate_bwd takes as s_up.
 * Results equal spa_maxpool2x2 followed by spa_gate_select bit for bit.
 */
int spa_gate_select_pooled(const void* x, const void* w, float bias, const float* s_fine, float tau,
                           int B, int grid_h, int grid_w, int C, int dtype, float* scores,
                           uint8_t* mask, int32_t* counts, float* s_up_pooled, void* stream);

/*
 * Token packing (Section 3.2 "Token Packing").  Stable compaction of the selected tokens:
 * images in batch order, tokens in ascending position.
 *   cu_seqlens[b]  = number of selected tokens in images < b    (cu_seqlens[B] = T)
 *   gather_idx[j]  = flat token id of packed row j              (j < T)
 *   inv_pos[i]     = packed row of flat token i, or -1
 *   packed[j,:]    = x[gather_idx[j],:]  (times sigmoid(gate_scores[gather_idx[j]]) when
 *                    gate_scores is given: r_g = Sigmoid(s) . r), rounded to dtype
 *   rows T .. ceil(T/container_len)*container_len - 1 of packed are zero (only the last
 *   container is padded); container_len = 0 means no padding.  Rows beyond that are left
 *   untouched.
 * in:  x [B,N,C] dtype (C may be a fused row such as 3*C of q|k|v), or NULL together with
 *      packed = NULL to compute the indices only; mask [B,N] uint8
 *      (non-zero = selected); counts [B] int32 or NULL: the per-image selected counts that
 *      spa_gate_select wrote for this mask (when given, a workgroup scans only its own
 *      image's mask instead of the whole prefix; results are identical);
 *      gate_scores [B,N] fp32 or NULL.
 * out: packed [B*N (+ container_len - 1 if padding), C] dtype; cu_seqlens [B+1] int32;
 *      gather_idx [B*N] int32 (first T valid); inv_pos [B*N] int32; total [1] int32.
 *      gather_idx, inv_pos, cu_seqlens, total may each be NULL if not wanted.
 */
int spa_pack(const void* x, const uint8_t* mask, const int32_t* counts, const float* gate_scores,
             int B, int N, int C, int dtype, int container_len,
             void* packed, int32_t* cu_seqlens, int32_t* gather_idx, int32_t* inv_pos,
             int32_t* total, void* stream);

/*
 * spa_pack of TWO tensors of the same tokens in one launch (Section 3.2 "Token Packing": the
 * same selection, the same packed order): the rows of x go to packed as they are, the rows of
 * x2, multiplied by sigmoid(gate_scores) when gate_scores is given (Eq. r_g = Sigmoid(s) . r),
 * go to packed2.  Equal, bit for bit, to spa_pack(x, gate_scores = NULL) followed by
 * spa_pack(x2, gate_scores); the survivors are counted and ranked once.
 * in:  x [B,N,C], x2 [B,N,C2] dtype (C*elem, C2*elem multiples of 16 bytes); mask, counts,
 *      gate_scores as in spa_pack.  No container padding.
 * out: packed [B*N, C], packed2 [B*N, C2] dtype; cu_seqlens, gather_idx, inv_pos, total as in
 *      spa_pack (each may be NULL).
 */
int spa_pack_pair(const void* x, int C, const void* x2, int C2, const uint8_t* mask,
                  const int32_t* counts, const float* gate_scores, int B, int N, int dtype,
                  void* packed, void* packed2, int32_t* cu_seqlens, int32_t* gather_idx,
                  int32_t* inv_pos, int32_t* total, void* stream);

/*
 * Token packing of a cyclically shifted feature map (Section 1: the feature maps are shifted
 * every two blocks so that the token pairs that share a container vary).  Every image is a
 * grid_h x grid_w map, N = grid_h*grid_w; the shifted map holds at (r, c) the token that sits
 * at ((r + shift_h) mod grid_h, (c + shift_w) mod grid_w) of the original (the window-shift
 * convention of the Swin design the paper builds on).  Tokens are packed in the raster order
 * of the SHIFTED map; gather_idx and inv_pos keep naming positions of the ORIGINAL layout, so
 * x is read in place and spa_unpack puts results back unshifted.  Everything else, and every
 * argument not named here, is as in spa_pack; shift (0, 0) is spa_pack.  shift_h, shift_w:
 * any integers (reduced modulo the grid).
 */
int spa_pack_shifted(const void* x, const uint8_t* mask, const int32_t* counts, const float* gate_scores,
                     int B, int grid_h, int grid_w, int shift_h, int shift_w, int C, int dtype,
                     int container_len, void* packed, int32_t* cu_seqlens, int32_t* gather_idx,
                     int32_t* inv_pos, int32_t* total, void* stream);

/*
 * Container-local attention segments (Section 3.2 "Token Packing" and the B'(2 L^2 C) term of
 * the complexity formula): the packed stream is cut into containers of length L and a token
 * attends to the tokens of its own image inside its own container.  The segment boundaries are
 * the distinct values among the image boundaries cu_seqlens[0..B] and the multiples of L below
 * T = cu_seqlens[B]; feeding them to spa_packed_attention / spa_packed_attention_bwd as
 * cu_seqlens (with B = seg_cap and max_seqlen = min(L, longest image)) evaluates that mask.
 *   seg_cu_seqlens[0 .. n]       = the boundaries, ascending, seg[0] = 0, seg[n] = T
 *   seg_cu_seqlens[n+1 .. seg_cap] = T   (empty segments, so that seg_cap can be used as the
 *                                    segment count without reading n back to the host)
 * in:  cu_seqlens [B+1] int32 (device); container_len L >= 1; max_total: an upper bound of T
 *      known to the host (B*N); seg_cap >= spa_container_segments_capacity(B, max_total, L)
 *      = B + max_total / L, else SPA_ERR_WORKSPACE.
 * out: seg_cu_seqlens [seg_cap+1] int32 (device); n_segments [1] int32 (device).
 */
int64_t spa_container_segments_capacity(int B, int64_t max_total, int container_len);
int spa_container_segments(const int32_t* cu_seqlens, int B, int container_len, int64_t max_total, int seg_cap,
                           int32_t* seg_cu_seqlens, int32_t* n_segments, void* stream);

/*
 * Multi-head self-attention on packed tokens in which a token attends only to tokens of
 * its own image (Section 3.2, last paragraph).  For every image b and head h, over packed
 * rows [cu_seqlens[b], cu_seqlens[b+1]):
 *   O = softmax(Q K^T * softmax_scale) V,   lse = log sum_j exp(S_ij)
 * The attention mask is never materialised; segments are addressed by cu_seqlens.
 * in:  q, k, v: packed rows, element (j, h, d) of q at q[j*q_row_stride + h*Dh + d] (likewise
 *      k, v); the three may point into one fused [*, 3*H*Dh] buffer or into separate ones.
 *      Row strides in elements.
 *      cu_seqlens [B+1] int32; max_seqlen >= every segment length (N); Dh in {32, 64};
 *      softmax_scale (host float; 0 means 1/sqrt(Dh)).
 * out: out [>= T, H*Dh] dtype, contiguous rows; lse [H, B*max_seqlen] fp32 or NULL
 *      (entry (h, j) for packed row j).  Rows >= T are not written.
 */
int spa_packed_attention(const void* q, const void* k, const void* v, int64_t q_row_stride,
                         int64_t k_row_stride, int64_t v_row_stride, const int32_t* cu_seqlens, int B, int max_seqlen, int H, int Dh,
                         int dtype, float softmax_scale, void* out, float* lse, void* stream);

/*
 * Scatter back (Section 3.2: positive tokens undergo attention, negative tokens go on
 * directly).  y[i,:] = packed_out[inv_pos[i],:] if inv_pos[i] >= 0 else 0; with base given,
 * y[i,:] = base[i,:] (+ packed_out[inv_pos[i],:] on selected rows).
 * in:  packed_out [>= T, C] dtype; inv_pos [B*N] int32; base [B,N,C] dtype or NULL.
 * out: y [B,N,C] dtype (may alias base).
 */
int spa_unpack(const void* packed_out, const int32_t* inv_pos, const void* base,
               int B, int N, int C, int dtype, void* y, void* stream);

/*
 * spa_packed_attention followed by spa_unpack, in one launch: packed output row j is written
 * to y[gather_idx[j], :] (plus base) by the attention kernel itself, and the rows that
 * bypass attention (inv_pos < 0) are filled with base or zero by the same kernel.  Results
 * equal the two separate calls (same arithmetic, same roundings).
 * in:  q, k, v, strides, cu_seqlens, softmax_scale as in spa_packed_attention; gather_idx,
 *      inv_pos [B*N] int32 from spa_pack; base [B,N,C] dtype or NULL; N tokens per image
 *      (also the bound on every segment length); C = H*Dh.
 * out: y [B,N,C] dtype; out [>= T, H*Dh] dtype or NULL (the packed output, kept when a
 *      backward pass needs it); lse [H, B*N] fp32 or NULL.  y may alias base.
 */
int spa_packed_attention_unpack(const void* q, const void* k, const void* v, int64_t q_row_stride,
                                int64_t k_row_stride, int64_t v_row_stride,
                                const int32_t* cu_seqlens, const int32_t* gather_idx,
                                const int32_t* inv_pos, const void* base, int B, int N, int H, int Dh,
                                int dtype, float softmax_scale, void* out, float* lse, void* y,
                                void* stream);

/*
 * spa_packed_attention_unpack on rows that were never copied (Section 3.2 "Token Packing": packing
 * re-arranges tokens, it computes nothing): q, k, v stay where the projections wrote them, at the
 * token positions, and the kernel fetches the row of packed position j from row gather_idx[j].
 * Together with the index-only spa_pack (x = packed = NULL) the forward pass moves no row twice.
 * Results equal spa_pack of q|k|v followed by spa_packed_attention_unpack, bit for bit.
 * in:  q, k, v: element (i, h, d) of q at q[i*q_row_stride + h*Dh + d] for TOKEN i = b*N + n
 *      (likewise k, v; e.g. three column slices of one [B*N, 3*H*Dh] tensor); every other
 *      argument, and every output, as in spa_packed_attention_unpack (out and lse are in packed
 *      order).
 */
int spa_gathered_attention_unpack(const void* q, const void* k, const void* v, int64_t q_row_stride,
                                  int64_t k_row_stride, int64_t v_row_stride,
                                  const int32_t* cu_seqlens, const int32_t* gather_idx,
                                  const int32_t* inv_pos, const void* base, int B, int N, int H, int Dh,
                                  int dtype, float softmax_scale, void* out, float* lse, void* y,
                                  void* stream);

/*
 * Packing order, attention and scatter in ONE call, for images of at most 256 tokens (Section 3.2:
 * the positive tokens, in token order, attend to each other inside their image; the negative tokens
 * go on directly): spa_gathered_attention_unpack without a packing index.  Every wave derives its
 * image's part of gather_idx from the mask bytes themselves (survivors in token order, exactly what
 * spa_pack writes), so no packing launch precedes the call: gate + this call = a forward step in two
 * launches.  y is bit for bit what spa_pack (index only) + spa_gathered_attention_unpack give.
 * in:  q, k, v at TOKEN positions (row i = flat token i; strides in elements, as spa_packed_attention);
 *      mask [B,N] uint8 as spa_gate_select writes it; base [B,N,C] or NULL; N <= 256 (larger images:
 *      SPA_ERR_UNSUPPORTED, use the index-only spa_pack + spa_gathered_attention_unpack).
 * out: y [B,N,C] as spa_packed_attention_unpack.  No packed output, no lse (forward only).
 */
int spa_selected_attention_unpack(const void* q, const void* k, const void* v, int64_t q_row_stride,
                                  int64_t k_row_stride, int64_t v_row_stride, const uint8_t* mask,
                                  const void* base, int B, int N, int H, int Dh, int dtype,
                                  float softmax_scale, void* y, void* stream);

/*
 * spa_packed_attention_unpack for segments that are not whole images (the container-local
 * segments of spa_container_segments): attention inside every segment of seg_cu_seqlens and,
 * in the same launch, the scatter back to y with the fill of the bypassing rows.  Results equal
 * spa_packed_attention on the segments followed by spa_unpack, bit for bit.
 * in:  q, k, v, strides, softmax_scale as in spa_packed_attention; seg_cu_seqlens
 *      [n_segments + 1] int32 (empty segments allowed); max_seqlen >= every segment length;
 *      gather_idx, inv_pos [rows] int32 from spa_pack / spa_pack_shifted; base [rows, H*Dh]
 *      dtype or NULL; rows = B*N, the rows of y.
 * out: y [rows, H*Dh] dtype; out [>= T, H*Dh] dtype or NULL; lse [H, n_segments*max_seqlen]
 *      fp32 or NULL.  y may alias base.
 */
int spa_segment_attention_unpack(const void* q, const void* k, const void* v, int64_t q_row_stride,
                                 int64_t k_row_stride, int64_t v_row_stride,
                                 const int32_t* seg_cu_seqlens, int n_segments, int max_seqlen,
                                 const int32_t* gather_idx, const int32_t* inv_pos, const void* base,
                                 int64_t rows, int H, int Dh, int dtype, float softmax_scale, void* out,
                                 float* lse, void* y, void* stream);

/*
 * Linear projection of packed tokens (the 3 L C^2 / N C^2 terms of the SPA complexity
 * formula, Section 3.2), with the packing gather and the gate scaling optionally folded into
 * the operand load:
 *   a_j     = x[gather_idx[j], :] (or x[j, :] when gather_idx is NULL)
 *   s_j      = sigmoid(gate_scores[gather_idx[j]]) when gate_scores is given, else 1
 *              (r_g = Sigmoid(s) . r; the bf16 kernel applies s_j to the fp32 accumulator,
 *              one rounding fewer than multiplying a materialised packed r_g)
 *   out[j,:] = s_j (a_j W^T) + bias                for j < min(*total, M_cap)
 * in:  x [*, K] dtype; gather_idx [>= rows] int32 or NULL; gate_scores fp32 indexed by token
 *      or NULL (needs gather_idx); total [1] int32 (device) or NULL (= M_cap rows);
 *      W [N_out, K] dtype (row n = weights of output n); bias [N_out] dtype or NULL.
 *      bf16: K, N_out and out_row_stride multiples of 8.
 * out: out[j*out_row_stride + n] dtype; rows >= min(*total, M_cap) are not written.
 */
int spa_linear_packed(const void* x, const int32_t* gather_idx, const float* gate_scores,
                      const int32_t* total, const void* W, const void* bias, int M_cap, int K,
                      int N_out, int dtype, void* out, int64_t out_row_stride, void* stream);

/*
 * Output projection of the packed rows with the scatter back and the residual add folded into
 * the store (Section 3.2: unselected tokens bypass the block; selected tokens receive the
 * block's output at their original position):
 *   y[scatter_idx[j], :] = residual[scatter_idx[j], :] + (x[j, :] W^T + bias)   for j < min(*total, M_cap)
 * Rows of y that no j names are not touched, so with y == residual (the residual stream updated
 * in place) the bypassing tokens keep their values without any copy.  The bf16 kernel rounds the
 * projection to bf16 before the residual is added (two roundings, as a separate unpack would).
 * in:  x [M_cap, K] dtype (packed rows); total [1] int32 (device) or NULL; W [N_out, K], bias
 *      [N_out] or NULL; scatter_idx [>= rows] int32 (gather_idx of spa_pack: distinct rows);
 *      residual: same layout as y, or NULL (then y[scatter_idx[j]] = projection only).
 * out: y[row*y_row_stride + n] dtype; y may alias residual.
 */
int spa_linear_packed_scatter(const void* x, const int32_t* total, const void* W, const void* bias,
                              int M_cap, int K, int N_out, int dtype, const int32_t* scatter_idx,
                              const void* residual, void* y, int64_t y_row_stride, void* stream);

/* ----------------------------------------------------------------- training ---- */

/*
 * Backward of the projections with respect to the rows that were multiplied (the 3 L C^2 /
 * N C^2 terms of Section 3.2; chain rule of out_j = r_j W^T + bias):
 *   g_j             = dout[dout_idx[j], :]  (dout[j, :] when dout_idx is NULL)
 *   dx[o(j), :]     = g_j W                 for j < min(*total, M_cap), o(j) = dx_idx[j] or j
 * For spa_linear_packed with gate_scores, r_j is the gated row Sigmoid(s) . r, so the result is
 * the gradient of r_g (the d_rg of spa_gate_bwd, which applies the sigmoid factor), written at
 * the token positions when dx_idx = gather_idx.  For spa_linear_packed_scatter, dout is the
 * gradient at token positions and dout_idx = scatter_idx gathers it.
 * in:  dout [*, N_out] dtype, row stride dout_row_stride; dout_idx [>= rows used] int32 or NULL;
 *      total [1] int32 (device) or NULL (= M_cap rows); W [N_out, K] dtype; dx_idx int32
 *      (distinct rows) or NULL; inv_pos [rows] int32 or NULL: when given (needs dx_idx), every
 *      row i < rows of dx with inv_pos[i] < 0 is set to zero (the rows of unselected tokens).
 *      bf16: K, N_out and both row strides multiples of 8.
 * out: dx[o(j)*dx_row_stride + k] dtype; other rows untouched unless inv_pos is given.
 */
int spa_linear_packed_bwd_input(const void* dout, const int32_t* dout_idx, int64_t dout_row_stride,
                                const int32_t* total, const void* W, int M_cap, int K, int N_out,
                                int dtype, const int32_t* dx_idx, const int32_t* inv_pos, int64_t rows,
                                void* dx, int64_t dx_row_stride, void* stream);

/* Bytes of workspace spa_linear_packed_bwd_weight needs (0 for fp32). Host. */
size_t spa_linear_bwd_weight_workspace_bytes(int M_cap, int K, int N_out, int dtype);

/*
 * Backward of the projections with respect to the weights and the bias (same chain rule):
 *   r_j   = s_j x[x_idx[j], :]  (x[j, :] when x_idx is NULL), s_j = sigmoid(gate_scores[x_idx[j]])
 *           when gate_scores is given, else 1 (bf16: r_j is rounded to bf16, as a packed r_g is)
 *   dW    = sum_j g_j^T r_j,  dbias = sum_j g_j      over j < min(*total, M_cap), g_j as above
 * in:  dout, dout_idx, dout_row_stride, total as in spa_linear_packed_bwd_input; x [*, K] dtype
 *      contiguous rows; x_idx int32 or NULL; gate_scores fp32 indexed by token or NULL (needs
 *      x_idx); workspace (device, 256-byte aligned) of at least
 *      spa_linear_bwd_weight_workspace_bytes bytes (bf16).
 * out: dW [N_out, K] fp32; dbias [N_out] fp32 or NULL.  Sums run in a fixed order: run-to-run
 *      bit-stable.  With no rows (*total = 0) both are zero.
 */
int spa_linear_packed_bwd_weight(const void* dout, const int32_t* dout_idx, int64_t dout_row_stride,
                                 const void* x, const int32_t* x_idx, const float* gate_scores,
                                 const int32_t* total, int M_cap, int K, int N_out, int dtype,
                                 float* dW, float* dbias, void* workspace, size_t workspace_bytes,
                                 void* stream);

/*
 * Transpose of spa_unpack: dout[j,:] = dy[gather_idx[j],:] for j < total.
 * in:  dy [B,N,C] dtype; gather_idx [B*N] int32; total [1] int32 (device).
 * out: dout [B*N, C] dtype (rows >= T untouched).
 */
int spa_unpack_bwd(const void* dy, const int32_t* gather_idx, const int32_t* total,
                   int B, int N, int C, int dtype, void* dout, void* stream);

/*
 * Transpose of spa_pack's row gather: d_rg[i,:] = dpacked[inv_pos[i],:] or 0.  The
 * sigmoid factor of a gate-scaled pack is applied by spa_gate_bwd, not here.
 * in:  dpacked [>= T, C] dtype; inv_pos [B*N] int32.   out: d_rg [B,N,C] dtype.
 */
int spa_pack_bwd(const void* dpacked, const int32_t* inv_pos, int B, int N, int C, int dtype,
                 void* d_rg, void* stream);

/* Bytes of workspace spa_packed_attention_bwd needs. Host. */
size_t spa_attention_bwd_workspace_bytes(int B, int max_seqlen, int H, int Dh, int dtype);

/*
 * Backward of spa_packed_attention (softmax-attention calculus per image and head):
 *   P = exp(S - lse), dV = P^T dO, dP = dO V^T, D_i = sum_d dO_id O_id,
 *   dS = P * (dP - D), dQ = dS K * scale, dK = dS^T Q * scale.
 * in:  q, k, v as in the forward (with their row strides); out, dout [>= T, H*Dh] dtype
 *      contiguous;
 *      lse [H, B*max_seqlen] fp32 from the forward; workspace (device, 256-byte aligned)
 *      of at least spa_attention_bwd_workspace_bytes bytes.
 * out: dq, dk, dv: element (j,h,d) of dq at dq[j*dq_row_stride + h*Dh + d] (likewise dk,
 *      dv; they may point into one fused buffer).  Rows >= T are not written.  Results are
 *      run-to-run bit-stable.
 */
int spa_packed_attention_bwd(const void* q, const void* k, const void* v, int64_t q_row_stride,
                             int64_t k_row_stride, int64_t v_row_stride,
                             const void* out, const void* dout, const float* lse,
                             const int32_t* cu_seqlens, int B, int max_seqlen, int H, int Dh,
                             int dtype, float softmax_scale,
                             void* dq, void* dk, void* dv, int64_t dq_row_stride,
                             int64_t dk_row_stride, int64_t dv_row_stride,
                             void* workspace, size_t workspace_bytes, void* stream);

/*
 * spa_unpack_bwd, spa_packed_attention_bwd and spa_pack_bwd (of dq, dk and dv) in one launch:
 * the upstream gradient is read at the token positions and the gradients are written at the
 * token positions (the transposes of the scatter and gather of Section 3.2 folded into the
 * attention backward).  workspace as for spa_packed_attention_bwd; bf16 with max_seqlen <= 256
 * needs none and NULL may be passed.
 * in:  q, k, v, out, lse, cu_seqlens as in spa_packed_attention_bwd; dy [rows, H*Dh] dtype
 *      contiguous, the gradient of the spa_unpack output; gather_idx, inv_pos [rows] int32
 *      from spa_pack; rows = B*N.
 * out: dq, dk, dv at token positions: element (i,h,d) of dq at dq[i*dq_row_stride + h*Dh + d]
 *      for token i = b*N + n (likewise dk, dv; they may point into one fused buffer, but not
 *      into dy).  Rows of unselected tokens are zero.  Run-to-run bit-stable.
 */
int spa_packed_attention_bwd_tokens(const void* q, const void* k, const void* v, int64_t q_row_stride,
                                    int64_t k_row_stride, int64_t v_row_stride,
                                    const void* out, const void* dy, const float* lse,
                                    const int32_t* cu_seqlens, int B, int max_seqlen, int H, int Dh,
                                    int dtype, float softmax_scale, const int32_t* gather_idx,
                                    const int32_t* inv_pos, int64_t rows,
                                    void* dq, void* dk, void* dv, int64_t dq_row_stride,
                                    int64_t dk_row_stride, int64_t dv_row_stride,
                                    void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of workspace spa_gate_bwd needs. Host. */
size_t spa_gate_bwd_workspace_bytes(int B, int N, int C, int dtype);

/*
 * Backward of the gate with the selection loss (Section 3.3: binary cross-entropy between
 * sigmoid(s) and the selection label, summed over tokens, weighted by loss_scale):
 *   p_i  = sigmoid(scores_i)
 *   loss = loss_scale * sum_i [ max(s_i,0) - y_i s_i + log(1 + exp(-|s_i|)) ]
 *   ds_i = loss_scale (p_i - y_i) + [gate_scaled] p_i (1-p_i) <d_rg[i,:], x[i,:]>
 *   dx_i = [gate_scaled] p_i d_rg[i,:] + own_i ds_i w
 *   dw   = sum_i own_i ds_i x[i,:],  db = sum_i own_i ds_i
 * own_i = 0 where the up-scale score won the max (scores_i came from s_up, i.e.
 * g_i < s_up_i), else 1; the hard mask is a constant.
 * in:  x [B,N,C], w [C] dtype; bias; scores [B,N] fp32 (output of spa_gate_select);
 *      s_up [B,N] fp32 or NULL; labels [B,N] uint8; d_rg [B,N,C] dtype or NULL (gradient of
 *      r_g = Sigmoid(s) . r, zero rows for unselected tokens); gate_scaled 0/1;
 *      workspace of at least spa_gate_bwd_workspace_bytes bytes.
 * out: loss [1] fp32; dx [B,N,C] dtype; dw [C] fp32; db [1] fp32.  Deterministic.
 */
int spa_gate_bwd(const void* x, const void* w, float bias, const float* scores,
                 const float* s_up, const uint8_t* labels, const void* d_rg, int gate_scaled,
                 float loss_scale, int B, int N, int C, int dtype,
                 float* loss, void* dx, float* dw, float* db,
                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * spa_gate_bwd for callers that cannot allocate device memory or hand in a workspace: code under
 * HIP graph capture, tight serving / training loops, harnesses that forbid hipMalloc.  Same
 * arguments, kernels and results (bit for bit) as spa_gate_bwd, but the partial rows of the
 * dw / db / loss reduction live in a device array built into the library (2.1 MB per GPU, held
 * until the process ends; its address on the current device is looked up on the first call on
 * that device).  The call allocates and frees nothing.
 * Limits: C <= 1024 (any B, N); beyond that SPA_ERR_WORKSPACE and nothing is launched.
 * Every call on a GPU uses that GPU's one array: calls that overlap in time on the same GPU
 * (different streams, different threads) race; calls on one stream, or ordered by events, do not.
 * Nothing in the array needs clearing between calls (every row read is written first).
 */
int spa_gate_bwd_static(const void* x, const void* w, float bias, const float* scores,
                        const float* s_up, const uint8_t* labels, const void* d_rg, int gate_scaled,
                        float loss_scale, int B, int N, int C, int dtype,
                        float* loss, void* dx, float* dw, float* db, void* stream);

/*
 * spa_gate_bwd with the straight-through estimator of the hard selection (Section 3.2, the
 * Gumbel-Softmax with hard samples): the forward pass multiplied r_g by the 0/1 mask, the
 * backward pass differentiates the relaxed weight p~_i = sigmoid((s_i + e_i)/temperature) in
 * its place, which adds on selected tokens
 *   ds_i += <d_rg[i,:], r_g[i,:]> p~_i (1 - p~_i) / temperature,   r_g[i,:] = p_i x[i,:]
 * to the ds_i of spa_gate_bwd with gate_scaled = 1 (d_rg[i,:] is the gradient of the packed
 * row there).  Everything else as spa_gate_bwd.
 * in:  as spa_gate_bwd (d_rg required), plus mask [B,N] uint8 (the selection of the forward
 *      pass), noise [B,N] fp32 or NULL (the e_i of spa_gate_select_gumbel; NULL = 0),
 *      temperature > 0.
 */
int spa_gate_bwd_straight_through(const void* x, const void* w, float bias, const float* scores,
                                  const float* s_up, const uint8_t* labels, const void* d_rg,
                                  float loss_scale, const uint8_t* mask, const float* noise,
                                  float temperature, int B, int N, int C, int dtype, float* loss,
                                  void* dx, float* dw, float* db, void* workspace,
                                  size_t workspace_bytes, void* stream);

/* -------------------------------------------------- comparison baseline -------- */

/*
 * Padded-to-max masked attention, the scheme the paper contrasts SPA with (Section 1:
 * padding every image's selected tokens to the batch maximum).  q, k, v, out are
 * [B, n_pad, H*Dh] with n_pad >= every seqlens[b]; all n_pad query rows of every image are
 * computed, keys >= seqlens[b] are masked.  Same kernels as spa_packed_attention.
 * in:  seqlens [B] int32.  out rows of padded queries hold finite, meaningless values.
 */
int spa_padded_attention(const void* q, const void* k, const void* v, int64_t row_stride,
                         const int32_t* seqlens, int B, int n_pad, int H, int Dh, int dtype,
                         float softmax_scale, void* out, void* stream);

/*
 * Measurement aids (not part of the method): the yardstick kernels bench.py times on the box to
 * report achievable ceilings beside the published peaks.
 * spa_ceiling_copy: dst[0..bytes) = src[0..bytes) with 16-byte accesses (device pointers,
 * 16-byte aligned, bytes a multiple of 16).
 * spa_ceiling_mfma: an MFMA-only loop (four independent v_mfma_f32_32x32x16_bf16 chains per
 * wave, `iters` rounds, `waves_per_simd` waves on every SIMD of 256 CUs); sink [1] fp32 device
 * (never written).  Returns the flops the launch issues, or -1 on a bad argument.
 */
int spa_ceiling_copy(const void* src, void* dst, size_t bytes, void* stream);
double spa_ceiling_mfma(float* sink, int waves_per_simd, int iters, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SPA_H */
