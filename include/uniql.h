/*
 * uniql.h — C ABI of the MI355X (gfx950) library for the inference hot path of
 * UniQL (arxiv 2512.03383): linear layers of 4-bit group-quantised, structurally
 * pruned models, and the fused rotary embedding on pruned Q/K heads.
 *
 * Because the model's channels are sorted by importance once (Sec. 3.2), an
 * on-device pruning rate only truncates each weight matrix to leading rows /
 * columns (Sec. 3.4, "On-device adaptive pruning").  Here that truncation is a
 * run-time argument: nothing is repacked when the rate changes.
 *
 * General rules for every entry point
 *   - All data pointers are DEVICE pointers on the current HIP device; the
 *     descriptor structs themselves are HOST memory, read during the call only.
 *   - The caller owns every buffer.  The library allocates nothing, keeps no
 *     reference after return and never synchronises: work is enqueued on
 *     `hip_stream` (a hipStream_t passed as void*, NULL = default stream).
 *   - Arguments are validated on the host before anything is launched.  Return
 *     value 0 = enqueued; negative = error, nothing was launched.
 *   - Values inside device tables (kept_idx entries, zeros > 15) are not
 *     checked; out-of-range table entries are undefined behaviour.
 *   - Results are deterministic: no atomics, fixed reduction order, so repeated
 *     calls with the same arguments return the same bits.
 */
#ifndef UNIQL_H
#define UNIQL_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  UNIQL_OK = 0,
  UNIQL_E_NULL = -1,  /* a required pointer is NULL                                   */
  UNIQL_E_SHAPE = -2, /* impossible size: group != 128, K_total % 128, M < 1, ld < dim */
  UNIQL_E_KEEP = -3,  /* kept dims inconsistent with totals / segment rule / heads     */
  UNIQL_E_ALIGN = -4, /* qweight not 16-byte, scales / x / y / q / k not 2-byte,
                         positions / kept_idx / ids not 4-byte aligned, embedding
                         output not 16-byte aligned or its ld not a multiple of 8     */
  UNIQL_E_ARCH = -5,  /* current device is not gfx950                                  */
  UNIQL_E_HIP = -6    /* HIP runtime / launch error; see uniql_last_hip_error()        */
};

/*
 * One quantised linear with N_total outputs and K_total inputs (the paper's
 * W in R^{D_in x D_out}, Sec. 3.1, stored output-major).  Group-wise uniform
 * 4-bit weights, group = 128 along the input dimension (Sec. 3.4, Eq. 3); the
 * 4-bit codes are packed eight to a 32-bit word (Sec. 3.4).
 *
 *   qweight [N_total][K_total/8] : nibble j (bits 4j..4j+3) of word w of a row is
 *                                  the code q of input column 8w+j, 0..15
 *   scales  [N_total][K_total/128]: scale s of the group, 16-bit float bits in the format `dtype`
 *   zeros   [N_total][K_total/128]: zero point z, 0..15; or NULL: every zero point is 8,
 *                                  which is Eq. 3's symmetric scheme with stored code =
 *                                  signed code + 8 (no zero point is read at all)
 * The dequantised weight is the fp16 number nearest (ties to even) to (q - z) * s.
 * Groups are those of the unpruned matrix (quantisation precedes pruning).
 *
 * dtype selects the 16-bit floating-point format of everything that goes with the matrix: its
 * scales, the activations multiplied with it and the outputs (all the `_f16` arguments of the calls
 * below).  UNIQL_F16 (0, so a zero-initialised field keeps its meaning) is IEEE binary16;
 * UNIQL_BF16 is bfloat16, the compute type the paper names (Sec. 4.1): the dequantised weight is then
 * the bfloat16 nearest (ties to even) to (q - z) * s, sums are still fp32 and rounded once.
 * Matrices that share a call (multi, qkv_rope, gate_up_silu) must share the format, except in
 * uniql_w4_linear_multi, which then runs them one by one.
 *
 * col_interleave = H > 0 is a second storage order of the SAME matrix, for the linear that reads the attention heads
 * (o_proj, Eq. 2; Sec. 3.4 prunes the head dimension D_hd of its inputs and leaves D_h): the K_total inputs are H heads
 * of D = K_total / H dims, and the 32-bit words of a row are stored dim-block-major, word (d / 8) * H + h holding the
 * dims 8 (d / 8) .. 8 (d / 8) + 7 of head h (nibble j = dim 8 (d / 8) + j), instead of head-major (word h * D / 8 + d / 8).
 * Nothing else changes: input column numbers, the keep rule, groups, scales and zero points all refer to the
 * head-major matrix (column h * D + d, group (h * D + d) / 128), x and y are what they are for that matrix.  What it buys:
 * keeping the leading D' dims of every head (column segments of stride D) keeps the leading ceil(D' / 8) * H words of
 * every row, so the pruned codes are not fetched at all, where the head-major order fetches them with the 32-byte
 * sectors they share with kept ones.  uniql_w4_interleave converts (a permutation of words, exact) and
 * uniql_w4_deinterleave converts back.  Served: uniql_w4_linear for H a multiple of 4 that divides 256, D = 128,
 * unpruned rows, and either no column pruning or column segments of stride 128, with the one-token kernel (1..64 tokens
 * run it with one token per grid row of one launch; more tokens: E_SHAPE, convert back for a prompt); uniql_w4_dequant for any H; every other call
 * returns E_SHAPE for such a matrix.
 *
 * bits = 8 (Eq. 3 with N = 8; Sec. 3.4 and App. C name 8, 6, 4 and 3 bits as widths the method covers): qweight is
 * [N_total][K_total/4], byte j of word w of a row is input column 4 w + j; zeros are 0..255, or NULL: every zero
 * point is 128.  Groups, the keep rule and the weight RN16((q - z) * s) are as for 4-bit codes.  Served by
 * uniql_w4_linear (any M; at most 32768 stored columns up to the last kept one, else E_SHAPE) and uniql_w4_dequant;
 * every other call, and col_interleave > 0, return E_SHAPE for such a matrix.
 *
 * bits = 3 or 6 (Eq. 3 with N = 3, 6; the same passages): the paper fixes no packing for these widths; here a row's
 * codes are one little-endian bit stream over its words, qweight [N_total][K_total * bits / 32]: code k occupies bits
 * [bits * k, bits * k + bits) of the stream, bit b of the stream = bit b % 32 of word b / 32 (a code may run over a
 * word boundary; a group of 128 columns is 12 or 24 whole words).  Zeros are 0..2^bits - 1, or NULL: every zero point
 * is 2^(bits - 1).  Served like 8-bit codes: uniql_w4_linear (any M; at most 32768 stored columns up to the last kept
 * one) and uniql_w4_dequant; every other call, and col_interleave > 0, return E_SHAPE.
 * Any other value of bits: E_SHAPE.
 */
enum { UNIQL_F16 = 0, UNIQL_BF16 = 1 };

typedef struct uniql_w4 {
  const uint32_t* qweight; /* device, 16-byte aligned */
  const uint16_t* scales;  /* device */
  const uint8_t* zeros;    /* device, or NULL (symmetric) */
  int32_t N_total, K_total, group;
  int32_t dtype;           /* UNIQL_F16 or UNIQL_BF16; anything else: E_SHAPE */
  int32_t col_interleave;  /* 0: words in column order; H > 0: head-interleaved over H heads (see above) */
  int32_t bits;            /* width of a code: 0 or 4 = the 4-bit format above; 8, 6 or 3: see above */
} uniql_w4_t;

/*
 * Which stored rows (outputs) and columns (inputs) survive pruning.  An
 * all-zero struct (or a NULL pointer) means unpruned.
 *
 * rows: row_seg_stride == 0 : the first n_keep rows (n_keep == 0 -> all)
 *       row_seg_stride  > 0 : row r < row_seg_limit is kept iff
 *                             (r % row_seg_stride) < row_seg_keep; row_seg_limit must
 *                             be a multiple of the stride.  With row_seg2_stride > 0 a
 *                             second family follows: row_seg_limit <= r < row_seg2_limit
 *                             is kept iff ((r - row_seg_limit) % row_seg2_stride) <
 *                             row_seg2_keep (row_seg2_limit - row_seg_limit a multiple
 *                             of that stride).  Every row behind the last family is
 *                             kept.  n_keep must be 0 or the resulting count.
 *       (MLP gate/up: prefix of D_int.  Q/K heads: stride D_hd/2, keep D'_hd/2 —
 *        the leading channels of each half, Alg. 2.  V heads: stride D_hd, keep
 *        D'_hd.  Mamba in_proj [z | x | B | C | dt]: first family over the z and x
 *        parts (per head, Alg. 5: stride D_hd, keep D'_hd), second family over the B and
 *        C parts when the state dimension is pruned too (per SSM group, Alg. 4: stride
 *        D_s, keep D'_s), the step-size rows behind them kept whole.)
 * cols: col_seg_stride == 0 : the first k_keep columns (k_keep == 0 -> all)
 *       col_seg_stride  > 0 : column k is kept iff (k % col_seg_stride) <
 *                             col_seg_keep; the stride is at least 8 and divides
 *                             K_total; k_keep must be 0 or the resulting count.
 *       (MLP down / Mamba out_proj: prefix.  Attention o_proj: per-head segments.)
 * Kept rows / columns appear in the compact y / x in increasing stored order.
 */
typedef struct uniql_keep {
  int32_t n_keep, k_keep;
  int32_t row_seg_stride, row_seg_keep, row_seg_limit;
  int32_t col_seg_stride, col_seg_keep;
  int32_t row_seg2_stride, row_seg2_keep, row_seg2_limit;
} uniql_keep_t;

/*
 * y[m][r'] = sum over kept columns k' of x[m][k'] * w[row(r')][col(k')]   (Y = X W
 * of Sec. 3.1 on the truncated matrix; the linears of Eq. 1, Eq. 2 and the Mamba
 * block).  w is the fp16 dequantised weight defined above, products are summed
 * in fp32 and y is rounded once to fp16.
 *   x_f16 : device, fp16 [M][ldx], first k_keep entries of a row are the kept inputs
 *   y_f16 : device, fp16 [M][ldy], first n_keep entries of a row are written
 *   ldx >= k_keep, ldy >= n_keep (elements); x and y must not overlap (this is not checked:
 *   with overlapping buffers the result is undefined).
 * M = 1 runs the streaming GEMV; M >= 2 the MFMA dequant-GEMM: 2..32 tokens the decode-batch
 * kernels (a wave owns 16 rows and part of K; tall matrices above 8 tokens a slab kernel), up to
 * 64 tokens tiles whose K range is split over the waves of a block, large tiles for prefill.
 * Errors: E_NULL, E_SHAPE, E_KEEP, E_ALIGN, E_ARCH, E_HIP.  E_SHAPE also at M = 1 when the last
 * kept column lies past stored column 81920 (the block's image of the activations in LDS holds
 * 40 tiles of 2048 columns), and for codes of 8, 6 or 3 bits past column 32768 at any M.
 */
int uniql_w4_linear(const uniql_w4_t* W, const uniql_keep_t* keep, const void* x_f16, int64_t ldx,
                    void* y_f16, int64_t ldy, int32_t M, void* hip_stream);

/*
 * n (1..4) independent linears with the same token count in one call, e.g. the q, k and v
 * projections of a layer (Eq. 2) or gate and up (Eq. 1), which read the same x.  W, keep (or NULL
 * = all unpruned), x_f16, ldx, y_f16, ldy are host arrays of n entries; each entry follows the
 * rules of uniql_w4_linear.  At M = 1 linears that stream rows of the same length are served by
 * ONE kernel launch (a decode step is launch-latency bound), and so are the linears of a decode
 * batch (M = 2..32) when each keeps a column prefix of at least 8 columns and is one the
 * decode-batch kernel takes; otherwise they are launched one after the other on the stream.
 * Results are identical to n separate uniql_w4_linear calls.
 * Errors: E_SHAPE also for n outside 1..4; otherwise as uniql_w4_linear (nothing is launched if
 * any entry is invalid).
 */
int uniql_w4_linear_multi(int32_t n, const uniql_w4_t* W, const uniql_keep_t* keep,
                          const void* const* x_f16, const int64_t* ldx, void* const* y_f16,
                          const int64_t* ldy, int32_t M, void* hip_stream);

/*
 * Bit-exact dequantised weights of the kept sub-matrix:
 *   w_f16[r'][k'] = RN_fp16((q - z) * s), fp16 [n_keep][k_keep] compact, device.
 * (Sec. 3.4: the unpack step of "unpack, prune channels, repack".)
 * Errors: as uniql_w4_linear.
 */
int uniql_w4_dequant(const uniql_w4_t* W, const uniql_keep_t* keep, void* w_f16, void* hip_stream);

/*
 * On-device repack (Sec. 3.4: INT4 weights are unpacked, the pruned channels dropped and the rest packed
 * again into INT32).  Nothing in this library needs it -- every call takes the pruning as an argument --
 * but a deployment that settles on a rate can reclaim the memory of the pruned channels.  The compact
 * matrix has the format of uniql_w4_t (group 128), which fixes the granularity:
 *   rows    : exactly the kept rows, in order (N_out = n_keep)
 *   columns : a quantisation group is carried whole (its scale and zero point serve all of its
 *             columns).  Column prefix: the ceil(k_keep / 128) leading groups.  Column segments whose
 *             stride is a multiple of 128: the leading ceil(col_seg_keep / 128) groups of every segment.
 *             Any other column segments (e.g. o_proj, where a head is one group): all columns stay.
 * keep_out is the descriptor to pass with the compact matrix: all rows kept, the same kept columns at
 * their new positions; every entry point then returns exactly what it returns for (W, keep).
 *
 * uniql_w4_repack_plan: host arithmetic only, no GPU needed; only the sizes of W are read (its data
 *   pointers may be NULL).  Errors: E_NULL, E_SHAPE, E_KEEP.
 * uniql_w4_repack: out_qweight [N_out][K_out/8] (16-byte aligned), out_scales / out_zeros
 *   [N_out][K_out/128] (out_zeros is not written, and may be NULL, when W has no zero points),
 *   device, caller-allocated with the sizes of the plan (E_SHAPE if N_out / K_out
 *   differ from it); must not overlap the source.  Bit-exact.  Errors: as uniql_w4_dequant.
 */
int uniql_w4_repack_plan(const uniql_w4_t* W, const uniql_keep_t* keep, int32_t* N_out, int32_t* K_out,
                         uniql_keep_t* keep_out);
int uniql_w4_repack(const uniql_w4_t* W, const uniql_keep_t* keep, uint32_t* out_qweight, uint16_t* out_scales,
                    uint8_t* out_zeros, int32_t N_out, int32_t K_out, void* hip_stream);

/*
 * Rows of a quantised table gathered by token id (Sec. 3.4: the embedding layer is quantised like
 * the linears; the hidden dimension is never pruned, so rows are K_total wide):
 *   out[i][k] = RN_fp16((q - z) * s) of row ids[i], k < K_total
 *   ids     : device int32 [n], entries in [0, N_total) (not checked: see the general rules)
 *   out_f16 : device fp16 [n][ld], ld >= K_total; 16-byte aligned, ld a multiple of 8
 * Bit-exact like uniql_w4_dequant.  Errors: E_NULL, E_SHAPE (n < 1, ld < K_total), E_ALIGN, E_ARCH, E_HIP.
 */
int uniql_w4_embedding(const uniql_w4_t* W, const int32_t* ids, int32_t n, void* out_f16, int64_t ld,
                       void* hip_stream);

/*
 * Fused rotary embedding on pruned heads, in place (Sec. 3.2 MHSA paragraph,
 * Alg. 2 / Alg. A1, Fig. 4a).  A head keeps D_keep of D_full channels: the
 * leading D_keep/2 of each half in sorted order, so kept pair i of a head is
 * (v[i], v[i + D_keep/2]).  Its original pair index j = kept_idx[h_tab][i] picks
 * the frequency: phi = positions[t] * theta^(-2j / D_full), and
 *   v[i]            <- v[i] cos(phi) - v[i + D_keep/2] sin(phi)
 *   v[i + D_keep/2] <- v[i + D_keep/2] cos(phi) + v[i] sin(phi)
 * (RoPE(X) = cos * X + sin * R(X), R([x1, x2]) = [-x2, x1]).  Only half of the
 * symmetric index vector is stored.  Q and K are rotated by the same launch.
 *   q_f16     : device fp16 [T][Hq][D_keep], rotated in place
 *   k_f16     : device fp16 [T][Hkv][D_keep] or NULL (then Hkv must be 0)
 *   positions : device int32 [T]
 *   kept_idx  : device int32 [H_tab][D_keep/2], entries in [0, D_full/2)
 *   H_tab     : table rows; head h of a tensor with H heads uses row
 *               h / (H / H_tab) (one row per KV head under GQA, per head for MHSA),
 *               so Hq and Hkv must be multiples of H_tab
 * The angle is formed in fp64, in revolutions; its fraction is rounded to fp32 for the sin/cos.
 * Errors: E_NULL, E_SHAPE (T < 1, Hq < 1), E_KEEP (D_keep odd, < 2 or > D_full,
 * D_full odd, head counts not multiples of H_tab, theta <= 0), E_ALIGN, E_ARCH, E_HIP.
 */
int uniql_pruned_rope(void* q_f16, void* k_f16, const int32_t* positions, const int32_t* kept_idx,
                      int32_t T, int32_t Hq, int32_t Hkv, int32_t H_tab, int32_t D_full,
                      int32_t D_keep, double theta, void* hip_stream);

/*
 * Debug aid, host only (no GPU work, no launch): checks a kept-index table that lies in HOST memory for
 * what the rotary kernels assume and never check on the device (Alg. 2 / Alg. A1: a row holds the
 * original pair indices of the kept pairs of one (KV-)head, in importance order): every entry in
 * [0, D_full / 2) and the entries of a row distinct.  kept_idx_host: int32 [H_tab][D_keep / 2].
 * Errors: E_NULL, E_KEEP (the shape rules of uniql_pruned_rope, or a bad entry).
 */
int uniql_rope_table_check(const int32_t* kept_idx_host, int32_t H_tab, int32_t D_full, int32_t D_keep);

/* The same rotation (Sec. 3.2, Alg. 2 / Alg. A1) of bfloat16 tensors (Sec. 4.1's compute type): every
 * argument, layout and error as in uniql_pruned_rope; q and k hold bfloat16 and are rounded to
 * bfloat16 (nearest even) once, after the fp32 rotation. */
int uniql_pruned_rope_bf16(void* q_bf16, void* k_bf16, const int32_t* positions, const int32_t* kept_idx,
                           int32_t T, int32_t Hq, int32_t Hkv, int32_t H_tab, int32_t D_full,
                           int32_t D_keep, double theta, void* hip_stream);

/*
 * Decode step of an attention block's input side in ONE launch (Eq. 2 followed by the rotary
 * embedding of Sec. 3.2 / Alg. 2 / Alg. A1, one token):
 *   q = RoPE(x Wq'),  k = RoPE(x Wk'),  v = x Wv'
 * with the linears of uniql_w4_linear and the rotation of uniql_pruned_rope.  The rotation is applied
 * to the fp32 sums, so q and k are rounded to fp16 once (the separate calls round them before the
 * rotation as well).
 *   W, keep   : host arrays of 3 entries (q, k, v); keep may be NULL (all unpruned).  The kept rows
 *               of q must number Hq * D_keep and those of k Hkv * D_keep: the compact outputs are
 *               [heads][D_keep], kept pair i of a head = (y[i], y[i + D_keep / 2]).  The three
 *               matrices read the same x, so their kept columns must agree in number.
 *   x_f16     : device fp16 [k_keep], one token
 *   q_f16, k_f16, v_f16 : device fp16 [Hq * D_keep], [Hkv * D_keep], [n_keep of v]
 *   position  : device int32 [1];  kept_idx, H_tab, D_full, D_keep, theta as in uniql_pruned_rope
 * One launch needs the three matrices to stream rows of the same length class (the same number of
 * 2048-column pieces, at most 8) with a group count per row that is a multiple of 4; otherwise the
 * call enqueues uniql_w4_linear_multi and uniql_pruned_rope instead: the same definition, but q and k
 * are then rounded to fp16 before the rotation (an extra error of up to 2^-11 of each member of a pair).
 * Errors: as uniql_w4_linear and uniql_pruned_rope; E_KEEP also when the kept rows of q / k do not
 * match the head counts; E_SHAPE when Hkv < 1 or the kept column counts differ.
 */
int uniql_w4_qkv_rope(const uniql_w4_t* W, const uniql_keep_t* keep, const void* x_f16, void* q_f16,
                      void* k_f16, void* v_f16, const int32_t* position, const int32_t* kept_idx,
                      int32_t Hq, int32_t Hkv, int32_t H_tab, int32_t D_full, int32_t D_keep,
                      double theta, void* hip_stream);

/*
 * Hidden vector of the gated MLP for one token in ONE launch (Eq. 1):
 *   h = sigma(x W_gate') * (x W_up'),  sigma = SiLU: g / (1 + exp(-g))
 * with the linears of uniql_w4_linear; gate and up sums stay in fp32 until h is rounded to fp16 once.
 *   W, keep : host arrays of 2 entries (gate, up); keep may be NULL.  Both must keep the same number of
 *             rows and the same columns (they read one x and fill one h).
 *   x_f16   : device fp16 [k_keep], one token;  h_f16 : device fp16 [n_keep]
 * The library has no scratch memory for separate gate and up vectors, so shapes that cannot share one
 * launch are refused (E_SHAPE; run uniql_w4_linear_multi and the activation yourself): rows longer than
 * 16384 kept columns; with fewer than 4096 kept rows (or more than 8192 kept columns, or pruned rows that
 * are not a prefix, or pruned columns that are not a prefix) also a group count per row that is not a
 * multiple of 4, and two members of which only one has zero points.
 * Errors: as uniql_w4_linear; E_KEEP when the two members keep different rows in number or different
 * columns; E_SHAPE as above.
 */
int uniql_w4_gate_up_silu(const uniql_w4_t* W, const uniql_keep_t* keep, const void* x_f16, void* h_f16,
                          void* hip_stream);

/*
 * The same hidden vectors for a decode batch of M tokens in ONE launch (Eq. 1, row by row):
 *   h[m] = sigma(x[m] W_gate') * (x[m] W_up'),  sigma = SiLU
 * gate and up sums stay in fp32 until h is rounded once.
 *   x_f16 : device [M][ldx], the first k_keep entries of a row are the kept inputs;  h_f16 : device [M][ldh], the first
 *   n_keep entries of a row are written;  W, keep as in uniql_w4_gate_up_silu.
 * M = 1 is uniql_w4_gate_up_silu (ldx, ldh unused).  M = 2..16 is served where a block of the decode-batch kernel
 * can hold the activations of all its rows' groups: the kept columns are a prefix of at least 8 and at most 4096
 * stored columns, rows have at least 8 groups, and the K range of a row goes over at most two waves of a block (at
 * least 10225 kept rows, or rows of at most 12 groups up to their last kept column).  Everything else returns E_SHAPE: the library has no scratch memory for separate gate and up
 * results (run uniql_w4_linear_multi and the activation yourself).
 * Errors: as uniql_w4_gate_up_silu.
 */
int uniql_w4_gate_up_silu_batch(const uniql_w4_t* W, const uniql_keep_t* keep, const void* x_f16, int64_t ldx,
                                void* h_f16, int64_t ldh, int32_t M, void* hip_stream);

/*
 * Measurement aid, not part of the method: reads `bytes` of device memory at `src`
 * (16-byte aligned) once with wave-wide 128-bit loads, the access shape of the GEMV's
 * weight stream, and writes one xor word per 8 KB to `out_words` (device, at least
 * ceil(bytes / 8192) uint32).  Its duration is the read-stream ceiling that the
 * benchmark reports beside the GEMV.  Errors: E_NULL, E_SHAPE, E_ALIGN, E_ARCH, E_HIP.
 */
int uniql_stream_read_probe(const void* src, int64_t bytes, void* out_words, void* hip_stream);

/*
 * The words of a matrix in head-interleaved order (uniql_w4_t.col_interleave = heads): out_qweight[r][(d / 8) * heads + h]
 * = W->qweight[r][h * (K_total / heads / 8) + d / 8] for every stored row r.  A permutation of 32-bit words, exact; the
 * scales and zero points are shared with W as they are (they are indexed by the head-major column either way).  The
 * on-device step of Sec. 3.4 (unpack, drop the pruned channels, pack again) for the one linear whose pruned channels
 * cannot be dropped in place: after it, head-dimension pruning of o_proj is a truncation of every row.
 * W must not be interleaved itself; K_total / heads must be a multiple of 8; out_qweight: device, 16-byte aligned,
 * [N_total][K_total / 8], must not overlap W->qweight.  Errors: E_NULL, E_SHAPE, E_ALIGN, E_ARCH, E_HIP.
 */
int uniql_w4_interleave(const uniql_w4_t* W, int32_t heads, uint32_t* out_qweight, void* hip_stream);

/*
 * The inverse of uniql_w4_interleave: the words of a head-interleaved matrix (W->col_interleave = H > 0) back in column
 * order, out_qweight[r][h * (K_total / H / 8) + d / 8] = W->qweight[r][(d / 8) * H + h].  For the calls that do not read
 * interleaved words (more than 64 tokens, the fused launches, repack, embedding): a caller that keeps o_proj
 * interleaved for decoding converts it into a scratch matrix for a prompt, the cost of one pass over the words.
 * out_qweight: device, 16-byte aligned, [N_total][K_total / 8], must not overlap W->qweight; scales and zero points
 * are shared as they are.  Errors: E_NULL, E_SHAPE (W is not interleaved), E_ALIGN, E_ARCH, E_HIP.
 */
int uniql_w4_deinterleave(const uniql_w4_t* W, uint32_t* out_qweight, void* hip_stream);

/*
 * The gated MLP of one token (Eq. 1): y = W_down' (SiLU(W_gate' x) * (W_up' x)), W[0] = gate, W[1] = up, W[2] = down,
 * keep[0..2] their pruning rules (keep = NULL: unpruned).  The kept hidden dimension is the same for the three:
 * n_keep(gate) = n_keep(up) = k_keep(down), which is how the method prunes the MLP (Sec. 3.1: the intermediate channels
 * are sorted once, a rate keeps the leading ones of all three matrices).  x is [k_keep(gate)], y is [n_keep(down)],
 * device pointers, 16-bit elements in the matrices' format.  The hidden vector is rounded to 16 bits once, like every
 * activation of the path, and is bit-identical to what uniql_w4_gate_up_silu writes; y is bit-identical to
 * uniql_w4_linear on that vector.
 *
 * `workspace` is device memory owned by the caller, 256-byte aligned, at least uniql_w4_mlp_workspace_bytes(n_keep(gate))
 * bytes, zero-filled ONCE before its first use (not between calls) and used by one call at a time: calls that share a
 * workspace must not overlap on the device (same stream, or ordered by events).  It holds the hidden vector and, for
 * the single persistent launch that serves tall row-prefix x column-prefix matrices (hidden widths of 2049..4096
 * columns, at least 4096 kept intermediate channels, at least 2048 outputs), a few control words and a word per block
 * through which the launch's blocks tell each other that their part of the hidden vector has reached memory.  That launch occupies every compute unit
 * and its blocks wait for each other, for at most 0.2 s: on a device that other work keeps busy beyond that, a block
 * gives up, y is then incomplete, and uniql_w4_mlp_status reports it.  The launch keeps its serial number in the
 * workspace, so a captured call may be replayed.  Other shapes run uniql_w4_gate_up_silu and uniql_w4_linear one after
 * the other through the same workspace.
 * Errors: as uniql_w4_gate_up_silu and uniql_w4_linear; E_KEEP also when k_keep(down) differs from n_keep(gate);
 * E_SHAPE also when the workspace is too small; E_ALIGN for a workspace that is not 256-byte aligned.
 */
int uniql_w4_mlp(const uniql_w4_t* W, const uniql_keep_t* keep, const void* x_f16, void* y_f16,
                 void* workspace, int64_t workspace_bytes, void* hip_stream);

/* Bytes of workspace uniql_w4_mlp needs for n_hidden_keep kept intermediate channels (0 for a count below 1). */
int64_t uniql_w4_mlp_workspace_bytes(int32_t n_hidden_keep);

/*
 * uniql_w4_mlp for callers that cannot allocate device memory or pass a workspace along: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  The workspace is a static array in device memory that the
 * library's code object carries (68 KB; every device the library runs on holds its own copy until the process ends),
 * large enough for uniql_w4_mlp_static_max_hidden() = 32768 kept intermediate channels: a larger n_keep(gate) returns
 * E_SHAPE and launches nothing.  The call allocates nothing and frees nothing.  Everything else is uniql_w4_mlp: same
 * arguments, same results bit for bit, same errors.  All calls on one device share that device's array, which keeps
 * what the last call left in it (the serial number of the persistent launch among it, so nothing needs clearing):
 * calls that overlap on one device -- two streams, two host threads -- race on it and must be ordered by the caller.
 */
int uniql_w4_mlp_static(const uniql_w4_t* W, const uniql_keep_t* keep, const void* x_f16, void* y_f16,
                        void* hip_stream);

/* Largest n_keep(gate) that uniql_w4_mlp_static accepts. */
int32_t uniql_w4_mlp_static_max_hidden(void);

/*
 * Where the last uniql_w4_mlp call with n_hidden_keep kept intermediate channels left its hidden vector inside
 * `workspace`: *h_f16 receives a device pointer to n_hidden_keep 16-bit elements (valid once that call has finished).
 * Host arithmetic only.  Errors: E_NULL, E_SHAPE.
 */
int uniql_w4_mlp_hidden(const void* workspace, int32_t n_hidden_keep, const void** h_f16);

/*
 * Waits for `hip_stream` and writes to *gave_up_serial (host) the give-up word of `workspace`: 0 when no call on that
 * workspace ever gave up waiting, else the serial number (counted per workspace, from 1) of the last call that did.
 * Errors: E_NULL, E_HIP.
 */
int uniql_w4_mlp_status(const void* workspace, uint32_t* gave_up_serial, void* hip_stream);

/*
 * Measurement aid, not part of the method: the launch of uniql_w4_gate_up_silu on its persistent streaming kernel
 * (fp16 matrices with zero points, row prefix x column prefix, at least 4096 kept rows, rows of at most 8192 kept
 * columns) with every load it issues -- codes, scales, zero points, activations -- and none of its arithmetic: the
 * loads are folded into one meaningless 16-bit word per kept row, written to `h_f16`.  Same grid, same walk over the
 * rows, same loads in flight, so its duration is the read-stream ceiling of exactly that launch.  Arguments as for
 * uniql_w4_gate_up_silu.  Errors: E_NULL, E_SHAPE (also: a shape the streaming kernel does not serve), E_KEEP,
 * E_ALIGN, E_ARCH, E_HIP.
 */
int uniql_w4_gate_up_stream_probe(const uniql_w4_t* W, const uniql_keep_t* keep, const void* x_f16, void* h_f16,
                                  void* hip_stream);

/* Static string for an error code (never NULL). */
const char* uniql_strerror(int code);

/* Raw hipError_t of the last UNIQL_E_HIP on this thread (0 if none). */
int uniql_last_hip_error(void);

/* Library version, e.g. 100 = 0.1.0. */
int uniql_version(void);

#ifdef __cplusplus
}
#endif
#endif /* UNIQL_H */
