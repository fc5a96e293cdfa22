/*
 * uref — the CPU oracle for the pruned W4A16 linear and the pruned RoPE.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * GPU library must compute; only the tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it.  It shares no code, header, table or helper
 * with the HIP library and the product path never calls it.
 *
 * Everything is scalar C.  Floating point is fp64 except where the format
 * fixes it: a dequantised weight is the fp16 value nearest (ties to even) to
 * (q - z) * s, where the product is exact in fp64 (|q - z| <= 15 times an
 * 11-bit significand).  Sums run in index order; the only parallelism is an
 * OpenMP loop over independent output rows / tokens, which reorders no sum.
 *
 * The *_fmt functions take the 16-bit floating-point format of scales, activations and dequantised
 * weights as an argument: fmt 0 = IEEE binary16 (the functions without the suffix), fmt 1 = bfloat16
 * (Sec. 4.1 names BF16 as the compute type of the paper's kernels): 1 sign, 8 exponent and 7 fraction
 * bits, i.e. the upper half of a binary32.  Nothing else changes: a weight is the bfloat16 nearest
 * (ties to even) to (q - z) * s, sums are fp64.
 *
 * What each function follows in the paper (UniQL, arxiv 2512.03383):
 *   uref_w4_dequant / uref_w4_linear   Sec. 3.1 (Y = X W), Eq. 1 / Eq. 2 (where
 *        the linears sit), Sec. 3.4 (group-wise 4-bit weights, group 128, pruned
 *        channels dropped from D_int / D_hd while D_h stays, INT4 packed in INT32)
 *   uref_w4_embedding                  Sec. 3.4 (the embedding layer is quantised as well): rows of a
 *        quantised table gathered by token id and dequantised
 *   uref_w4_repack_plan / uref_w4_repack   Sec. 3.4, on-device pruning of INT4 weights: unpack, drop
 *        the pruned channels, pack again into INT32 -- here at the granularity the format can hold
 *        (kept rows; whole quantisation groups that still hold a kept column)
 *   uref_pruned_rope                   Sec. 3.2 MHSA paragraph: RoPE(X) =
 *        cos * X + sin * R(X), R([x1,x2]) = [-x2,x1]; Alg. 2 / Alg. A1 (symmetric
 *        index vector, one half stored; one table per KV head under GQA); Fig. 4a
 *   uref_pruned_rope_f64               the same rotation on fp64 inputs: the second half of the
 *        fused step y = RoPE(X W) (Eq. 2, then Sec. 3.2), no rounding in between
 *   uref_wq_dequant / uref_wq_linear / uref_quantize_sym_bits   the same with codes of 8, 6 or 3 bits (Eq. 3 with
 *        N = bits; Sec. 3.4 and App. C name 8, 6, 4 and 3 bits as the widths the method covers; the paper states a
 *        packing for none but INT4-in-INT32, the bit-stream order below is this build's reading)
 *   uref_quantize_sym                  Eq. 3 (symmetric, N = 4)
 *   uref_quantize_asym                 the min/max asymmetric variant the
 *        benchmark configuration asks for (not in the paper; Eq. 3 is the case
 *        zero = 8)
 *
 * Storage convention (the paper only says INT4 is repacked into INT32):
 *   qweight uint32 [N_total][K_total/8]; nibble j (bits 4j..4j+3) of word w of a
 *   row is input column 8w+j.  scales fp16 bits [N_total][K_total/group]; zeros
 *   uint8 0..15, same shape, or NULL: every zero point is 8, i.e. the stored code is Eq. 3's signed
 *   code + 8 (the paper's own, symmetric, scheme).  Groups are those of the unpruned matrix.
 *
 * keep[10] = { n_keep, k_keep, row_seg_stride, row_seg_keep, row_seg_limit,
 *              col_seg_stride, col_seg_keep, row_seg2_stride, row_seg2_keep, row_seg2_limit }:
 *   stored row r is kept iff  row_seg_stride == 0 ? r < n_keep
 *                           : r < row_seg_limit ? r % row_seg_stride < row_seg_keep
 *                           : (row_seg2_stride != 0 && r < row_seg2_limit)
 *                                 ? (r - row_seg_limit) % row_seg2_stride < row_seg2_keep
 *                           : 1
 *   (the second family of segments serves the Mamba block's in_proj, Sec. 3.4: besides the head
 *   dimension of the z and x parts, the state dimension D_s is pruned, i.e. the leading D_s' rows of
 *   every SSM group of the B and of the C part survive, in the order Alg. 4 sorted them; the
 *   step-size rows behind them are kept whole)
 *   stored col k is kept iff  col_seg_stride == 0 ? k < k_keep
 *                           : (k % col_seg_stride < col_seg_keep)
 *   n_keep == 0 / k_keep == 0 with stride 0 mean "all".  Kept rows and columns
 *   appear in compact y / x in increasing stored order.
 *
 * Head-interleaved words (the *_il functions, il_heads = H > 0): a second storage order of the same matrix, for the
 *   linear that reads the attention heads (o_proj, Eq. 2; Sec. 3.4 prunes the head dimension of its inputs).  The K_total
 *   input columns are H heads of D = K_total / H dims; column numbers, the keep rule, groups, scales and zero points all
 *   refer to this head-major matrix (column c = h * D + d).  Only where a code is STORED differs: the 32-bit words of a
 *   row are kept dim-block-major, word (d / 8) * H + h holding dims 8 (d / 8) .. + 7 of head h, so the code of column c is
 *   nibble d % 8 of that word.  il_heads = 0 is the plain order above.  uref_w4_interleave converts, uref_w4_deinterleave converts back.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static int g_threads = 1;

void uref_set_threads(int n) { g_threads = n < 1 ? 1 : n; }

int uref_get_max_threads(void) {
#ifdef _OPENMP
  return omp_get_num_procs();
#else
  return 1;
#endif
}

/* ---- fp16 <-> fp64, written from the IEEE 754 binary16 definition ---- */

double uref_half_to_double(uint16_t h) {
  int sign = h >> 15, e = (h >> 10) & 31, m = h & 1023;
  double v;
  if (e == 0)
    v = ldexp((double)m, -24); /* zero and subnormals: m * 2^-24 */
  else if (e == 31)
    v = m ? NAN : INFINITY;
  else
    v = ldexp((double)(1024 + m), e - 25); /* (1 + m/1024) * 2^(e-15) */
  return sign ? -v : v;
}

/* round to nearest, ties to even (the default fenv rounding of rint) */
uint16_t uref_double_to_half(double x) {
  uint16_t sign = signbit(x) ? 0x8000 : 0;
  double a = fabs(x);
  if (isnan(x)) return 0x7e00;
  if (a >= 65520.0) return sign | 0x7c00; /* 65504 + half an ulp rounds up to inf */
  if (a == 0.0) return sign;
  int e;
  (void)frexp(a, &e); /* a = f * 2^e, f in [0.5,1) -> floor(log2 a) = e-1 */
  e -= 1;
  if (e < -14) { /* subnormal range: multiples of 2^-24 */
    double m = rint(ldexp(a, 24));
    return sign | (uint16_t)m; /* m == 1024 is the smallest normal, same bits */
  }
  double m = rint(ldexp(a, 10 - e)); /* in [1024, 2048] */
  if (m == 2048.0) { m = 1024.0; e += 1; }
  return sign | (uint16_t)(((e + 15) << 10) | ((int)m - 1024));
}

/* ---- bfloat16 <-> fp64, from the format's definition: sign, 8 exponent bits (bias 127), 7 fraction
 * bits; exponent 0 = zero and subnormals (multiples of 2^-133), exponent 255 = inf / nan ---- */

double uref_bf16_to_double(uint16_t h) {
  int sign = h >> 15, e = (h >> 7) & 255, m = h & 127;
  double v;
  if (e == 0)
    v = ldexp((double)m, -133);
  else if (e == 255)
    v = m ? NAN : INFINITY;
  else
    v = ldexp((double)(128 + m), e - 134); /* (1 + m/128) * 2^(e-127) */
  return sign ? -v : v;
}

uint16_t uref_double_to_bf16(double x) {
  uint16_t sign = signbit(x) ? 0x8000 : 0;
  double a = fabs(x);
  if (isnan(x)) return 0x7fc0;
  if (a == 0.0) return sign;
  if (isinf(x)) return sign | 0x7f80;
  int e;
  (void)frexp(a, &e);
  e -= 1; /* floor(log2 a) */
  if (e > 127) return sign | 0x7f80;
  if (e < -126) { /* subnormal range: multiples of 2^-133 */
    double m = rint(ldexp(a, 133));
    return sign | (uint16_t)m; /* m == 128 is the smallest normal, same bits */
  }
  double m = rint(ldexp(a, 7 - e)); /* in [128, 256] */
  if (m == 256.0) { m = 128.0; e += 1; }
  if (e > 127) return sign | 0x7f80; /* the largest finite value plus half an ulp rounds up to inf */
  return sign | (uint16_t)(((e + 127) << 7) | ((int)m - 128));
}

static double f16_to_double(uint16_t h, int fmt) { return fmt ? uref_bf16_to_double(h) : uref_half_to_double(h); }
static uint16_t double_to_f16(double x, int fmt) { return fmt ? uref_double_to_bf16(x) : uref_double_to_half(x); }

/* ---- kept rows / columns: the definition, written as a scan ---- */

static int row_kept(const int32_t* keep, int N_total, int r) {
  if (keep[2] == 0) return r < (keep[0] ? keep[0] : N_total);
  if (r < keep[4]) return (r % keep[2]) < keep[3];
  if (keep[7] != 0 && r < keep[9]) return ((r - keep[4]) % keep[7]) < keep[8];
  return 1;
}

static int col_kept(const int32_t* keep, int K_total, int k) {
  if (keep[5] == 0) return k < (keep[1] ? keep[1] : K_total);
  return (k % keep[5]) < keep[6];
}

/* returns the number of kept indices, fills list (size >= total) */
static int kept_rows(const int32_t* keep, int N_total, int32_t* list) {
  int n = 0;
  for (int r = 0; r < N_total; ++r)
    if (row_kept(keep, N_total, r)) list[n++] = r;
  return n;
}

static int kept_cols(const int32_t* keep, int K_total, int32_t* list) {
  int n = 0;
  for (int k = 0; k < K_total; ++k)
    if (col_kept(keep, K_total, k)) list[n++] = k;
  return n;
}

int uref_count_kept(int N_total, int K_total, const int32_t* keep, int32_t* n_out, int32_t* k_out) {
  static const int32_t none[10] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  if (!keep) keep = none;
  int32_t* tmp = (int32_t*)malloc(sizeof(int32_t) * (size_t)(N_total > K_total ? N_total : K_total));
  if (!tmp) return -1;
  *n_out = kept_rows(keep, N_total, tmp);
  *k_out = kept_cols(keep, K_total, tmp);
  free(tmp);
  return 0;
}

/* word of a row that stores column k */
static int word_of_col(int K_total, int il_heads, int k) {
  if (il_heads <= 0) return k / 8;
  int D = K_total / il_heads, h = k / D, d = k % D;
  return (d / 8) * il_heads + h;
}

/* one dequantised weight as 16-bit float bits of format fmt: RN16((q - z) * s).  bits = 3, 4, 6 or 8 is the width
 * of a code (Eq. 3's N).  A row's codes form one little-endian bit stream over its 32-bit words: code k occupies bits
 * [bits * k, bits * k + bits) of the stream, bit b of the stream being bit b % 32 of word b / 32 (for 4 and 8 bits
 * that is the nibble / byte order above; codes of 3 and 6 bits may run over a word boundary, low part in the earlier
 * word).  Without zero points z = 2^(bits - 1), the offset that stores Eq. 3's signed code as an unsigned one.  The
 * product is exact in fp64 for every width (|q - z| <= 255 times an 11-bit significand). */
static int code_width_ok(int bits) { return bits == 3 || bits == 4 || bits == 6 || bits == 8; }

static uint16_t dequant_bits(int bits, const uint32_t* qweight, const uint16_t* scales, const uint8_t* zeros,
                             int K_total, int group, int r, int k, int fmt, int il_heads) {
  size_t words_per_row = (size_t)K_total * (size_t)bits / 32;
  const uint32_t* row = qweight + (size_t)r * words_per_row;
  int q;
  if (bits == 4) {
    q = (int)((row[word_of_col(K_total, il_heads, k)] >> (4 * (k % 8))) & 15u);
  } else {
    q = 0;
    for (int b = 0; b < bits; ++b) {          /* bit by bit from the stream */
      size_t pos = (size_t)bits * (size_t)k + (size_t)b;
      q |= (int)((row[pos / 32] >> (pos % 32)) & 1u) << b;
    }
  }
  size_t g = (size_t)r * (K_total / group) + k / group;
  int z = zeros ? zeros[g] : 1 << (bits - 1);   /* no zero points: the symmetric codes of Eq. 3, stored as signed code + 2^(N-1) */
  double s = f16_to_double(scales[g], fmt);
  return double_to_f16((double)(q - z) * s, fmt);
}

static uint16_t dequant_one(const uint32_t* qweight, const uint16_t* scales, const uint8_t* zeros,
                            int K_total, int group, int r, int k, int fmt, int il_heads) {
  return dequant_bits(4, qweight, scales, zeros, K_total, group, r, k, fmt, il_heads);
}

/* w_f16: [n_keep][k_keep] compact, 16-bit float bits */
int uref_w4_dequant_il(const uint32_t* qweight, const uint16_t* scales, const uint8_t* zeros,
                       int N_total, int K_total, int group, const int32_t* keep, uint16_t* w_f16, int fmt, int il_heads) {
  if (il_heads < 0 || (il_heads > 0 && (K_total % il_heads || (K_total / il_heads) % 8))) return -3;
  static const int32_t none[10] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  if (!keep) keep = none;
  int32_t* rows = (int32_t*)malloc(sizeof(int32_t) * (size_t)N_total);
  int32_t* cols = (int32_t*)malloc(sizeof(int32_t) * (size_t)K_total);
  if (!rows || !cols) { free(rows); free(cols); return -1; }
  int nk = kept_rows(keep, N_total, rows), kk = kept_cols(keep, K_total, cols);
#pragma omp parallel for num_threads(g_threads) schedule(static)
  for (int i = 0; i < nk; ++i)
    for (int j = 0; j < kk; ++j)
      w_f16[(size_t)i * kk + j] = dequant_one(qweight, scales, zeros, K_total, group, rows[i], cols[j], fmt, il_heads);
  free(rows); free(cols);
  return 0;
}

int uref_w4_dequant_fmt(const uint32_t* qweight, const uint16_t* scales, const uint8_t* zeros,
                        int N_total, int K_total, int group, const int32_t* keep, uint16_t* w_f16, int fmt) {
  return uref_w4_dequant_il(qweight, scales, zeros, N_total, K_total, group, keep, w_f16, fmt, 0);
}

int uref_w4_dequant(const uint32_t* qweight, const uint16_t* scales, const uint8_t* zeros,
                    int N_total, int K_total, int group, const int32_t* keep, uint16_t* w_f16) {
  return uref_w4_dequant_fmt(qweight, scales, zeros, N_total, K_total, group, keep, w_f16, 0);
}

/* Rows of a quantised table gathered by token id (Sec. 3.4 also quantises the embedding layer):
 * out[i][k] = RN16((q - z) * s) of row ids[i], every column; fp16 bits [n][K_total]. */
int uref_w4_embedding_fmt(const uint32_t* qweight, const uint16_t* scales, const uint8_t* zeros,
                          int N_total, int K_total, int group, const int32_t* ids, int n, uint16_t* out, int fmt) {
  for (int i = 0; i < n; ++i) {
    if (ids[i] < 0 || ids[i] >= N_total) return -3;
    for (int k = 0; k < K_total; ++k)
      out[(size_t)i * K_total + k] = dequant_one(qweight, scales, zeros, K_total, group, ids[i], k, fmt, 0);
  }
  return 0;
}

int uref_w4_embedding(const uint32_t* qweight, const uint16_t* scales, const uint8_t* zeros,
                      int N_total, int K_total, int group, const int32_t* ids, int n, uint16_t* out) {
  return uref_w4_embedding_fmt(qweight, scales, zeros, N_total, K_total, group, ids, n, out, 0);
}

/* y[m][r'] = sum_{k'} x[m][k'] * w[row(r')][col(k')], fp64, index order.
 * x: fp16 bits [M][ldx] compact columns; y: fp64 [M][ldy] compact rows.
 * If row_list != NULL only the compact rows row_list[0..n_list) are computed,
 * and written to y[m][i] (i = position in the list) -- used to sample large cases. */
int uref_w4_linear_il(const uint32_t* qweight, const uint16_t* scales, const uint8_t* zeros,
                      int N_total, int K_total, int group, const int32_t* keep,
                      const uint16_t* x, int64_t ldx, double* y, int64_t ldy, int M,
                      const int32_t* row_list, int n_list, int fmt, int il_heads) {
  if (il_heads < 0 || (il_heads > 0 && (K_total % il_heads || (K_total / il_heads) % 8))) return -3;
  static const int32_t none[10] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  if (!keep) keep = none;
  int32_t* rows = (int32_t*)malloc(sizeof(int32_t) * (size_t)N_total);
  int32_t* cols = (int32_t*)malloc(sizeof(int32_t) * (size_t)K_total);
  if (!rows || !cols) { free(rows); free(cols); return -1; }
  int nk = kept_rows(keep, N_total, rows), kk = kept_cols(keep, K_total, cols);
  int n_out = row_list ? n_list : nk;
  int bad = 0;
#pragma omp parallel for num_threads(g_threads) schedule(static) reduction(| : bad)
  for (int i = 0; i < n_out; ++i) {
    int rc = row_list ? row_list[i] : i;
    if (rc < 0 || rc >= nk) { bad = 1; continue; }
    int r = rows[rc];
    for (int m = 0; m < M; ++m) {
      double acc = 0.0;
      for (int j = 0; j < kk; ++j) {
        double w = f16_to_double(dequant_one(qweight, scales, zeros, K_total, group, r, cols[j], fmt, il_heads), fmt);
        acc += f16_to_double(x[(size_t)m * ldx + j], fmt) * w;
      }
      y[(size_t)m * ldy + i] = acc;
    }
  }
  free(rows); free(cols);
  return bad ? -2 : 0;
}

int uref_w4_linear_fmt(const uint32_t* qweight, const uint16_t* scales, const uint8_t* zeros,
                       int N_total, int K_total, int group, const int32_t* keep,
                       const uint16_t* x, int64_t ldx, double* y, int64_t ldy, int M,
                       const int32_t* row_list, int n_list, int fmt) {
  return uref_w4_linear_il(qweight, scales, zeros, N_total, K_total, group, keep, x, ldx, y, ldy, M,
                           row_list, n_list, fmt, 0);
}

/* The words of every row in head-interleaved order: out[r][(d / 8) * heads + h] = qweight[r][h * (D / 8) + d / 8],
 * D = K_total / heads.  A permutation of words; scales and zero points are not touched. */
int uref_w4_interleave(const uint32_t* qweight, int N_total, int K_total, int heads, uint32_t* out) {
  if (heads < 1 || K_total % heads || (K_total / heads) % 8) return -3;
  int wpr = K_total / 8, wph = wpr / heads;
  for (int r = 0; r < N_total; ++r)
    for (int h = 0; h < heads; ++h)
      for (int b = 0; b < wph; ++b)
        out[(size_t)r * wpr + (size_t)b * heads + h] = qweight[(size_t)r * wpr + (size_t)h * wph + b];
  return 0;
}

/* The inverse: the words of a head-interleaved matrix back in column order, out[r][h * (D / 8) + d / 8] =
 * qweight_il[r][(d / 8) * heads + h]. */
int uref_w4_deinterleave(const uint32_t* qweight_il, int N_total, int K_total, int heads, uint32_t* out) {
  if (heads < 1 || K_total % heads || (K_total / heads) % 8) return -3;
  int wpr = K_total / 8, wph = wpr / heads;
  for (int r = 0; r < N_total; ++r)
    for (int h = 0; h < heads; ++h)
      for (int b = 0; b < wph; ++b)
        out[(size_t)r * wpr + (size_t)h * wph + b] = qweight_il[(size_t)r * wpr + (size_t)b * heads + h];
  return 0;
}

int uref_w4_linear(const uint32_t* qweight, const uint16_t* scales, const uint8_t* zeros,
                   int N_total, int K_total, int group, const int32_t* keep,
                   const uint16_t* x, int64_t ldx, double* y, int64_t ldy, int M,
                   const int32_t* row_list, int n_list) {
  return uref_w4_linear_fmt(qweight, scales, zeros, N_total, K_total, group, keep, x, ldx, y, ldy, M,
                            row_list, n_list, 0);
}

/* ---- other code widths (Sec. 3.4 / App. C: the method quantises to 8, 6, 4 and 3 bits; Eq. 3 with N = bits).
 * qweight uint32 [N_total][K_total * bits / 32], a row's codes as one bit stream (see dequant_bits; bits = 8: byte j of
 * word w is input column 4w+j); zeros uint8 0..2^bits - 1 or NULL (every zero point 2^(bits-1)).  bits = 4 is the
 * format above.  K_total must be a multiple of 32 so that rows are whole words (it is a multiple of the group).
 * Everything else -- groups, the keep rule, RN16 of
 * (q - z) * s, fp64 sums in index order -- is as in uref_w4_dequant_fmt / uref_w4_linear_fmt. */
int uref_wq_dequant(int bits, const uint32_t* qweight, const uint16_t* scales, const uint8_t* zeros,
                    int N_total, int K_total, int group, const int32_t* keep, uint16_t* w_f16, int fmt) {
  if (!code_width_ok(bits)) return -3;
  static const int32_t none[10] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  if (!keep) keep = none;
  int32_t* rows = (int32_t*)malloc(sizeof(int32_t) * (size_t)N_total);
  int32_t* cols = (int32_t*)malloc(sizeof(int32_t) * (size_t)K_total);
  if (!rows || !cols) { free(rows); free(cols); return -1; }
  int nk = kept_rows(keep, N_total, rows), kk = kept_cols(keep, K_total, cols);
#pragma omp parallel for num_threads(g_threads) schedule(static)
  for (int i = 0; i < nk; ++i)
    for (int j = 0; j < kk; ++j)
      w_f16[(size_t)i * kk + j] = dequant_bits(bits, qweight, scales, zeros, K_total, group, rows[i], cols[j], fmt, 0);
  free(rows); free(cols);
  return 0;
}

int uref_wq_linear(int bits, const uint32_t* qweight, const uint16_t* scales, const uint8_t* zeros,
                   int N_total, int K_total, int group, const int32_t* keep,
                   const uint16_t* x, int64_t ldx, double* y, int64_t ldy, int M,
                   const int32_t* row_list, int n_list, int fmt) {
  if (!code_width_ok(bits)) return -3;
  static const int32_t none[10] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  if (!keep) keep = none;
  int32_t* rows = (int32_t*)malloc(sizeof(int32_t) * (size_t)N_total);
  int32_t* cols = (int32_t*)malloc(sizeof(int32_t) * (size_t)K_total);
  if (!rows || !cols) { free(rows); free(cols); return -1; }
  int nk = kept_rows(keep, N_total, rows), kk = kept_cols(keep, K_total, cols);
  int n_out = row_list ? n_list : nk;
  int bad = 0;
#pragma omp parallel for num_threads(g_threads) schedule(static) reduction(| : bad)
  for (int i = 0; i < n_out; ++i) {
    int rc = row_list ? row_list[i] : i;
    if (rc < 0 || rc >= nk) { bad = 1; continue; }
    int r = rows[rc];
    for (int m = 0; m < M; ++m) {
      double acc = 0.0;
      for (int j = 0; j < kk; ++j) {
        double w = f16_to_double(dequant_bits(bits, qweight, scales, zeros, K_total, group, r, cols[j], fmt, 0), fmt);
        acc += f16_to_double(x[(size_t)m * ldx + j], fmt) * w;
      }
      y[(size_t)m * ldy + i] = acc;
    }
  }
  free(rows); free(cols);
  return bad ? -2 : 0;
}

/* Eq. 3 with N = bits: s = max|W| / (2^(N-1) - 1), code = clamp(rint(W / s), -2^(N-1), 2^(N-1) - 1), stored as
 * code + 2^(N-1) with zero point 2^(N-1).  The scale is stored in fp16 and the codes are taken against the stored
 * scale.  (Only used to build test inputs and for the round-trip pin.) */
int uref_quantize_sym_bits(int bits, const double* w, int N, int K, int group, uint32_t* qweight,
                           uint16_t* scales, uint8_t* zeros) {
  if (!code_width_ok(bits)) return -3;
  int half = 1 << (bits - 1);
  size_t words_per_row = (size_t)K * (size_t)bits / 32;
  memset(qweight, 0, sizeof(uint32_t) * (size_t)N * words_per_row);
  for (int r = 0; r < N; ++r)
    for (int g = 0; g < K / group; ++g) {
      const double* wg = w + (size_t)r * K + (size_t)g * group;
      double mx = 0.0;
      for (int j = 0; j < group; ++j) mx = fmax(mx, fabs(wg[j]));
      uint16_t s16 = uref_double_to_half(mx / (double)(half - 1));
      double s = uref_half_to_double(s16);
      scales[(size_t)r * (K / group) + g] = s16;
      zeros[(size_t)r * (K / group) + g] = (uint8_t)half;
      for (int j = 0; j < group; ++j) {
        double qv = s > 0.0 ? rint(wg[j] / s) : 0.0;
        if (qv < -(double)half) qv = -(double)half;
        if (qv > (double)(half - 1)) qv = (double)(half - 1);
        int k = g * group + j;
        uint32_t code = (uint32_t)((int)qv + half);
        for (int b = 0; b < bits; ++b) {        /* bit by bit into the row's stream */
          size_t pos = (size_t)bits * (size_t)k + (size_t)b;
          qweight[(size_t)r * words_per_row + pos / 32] |= ((code >> b) & 1u) << (pos % 32);
        }
      }
    }
  return 0;
}

/* Pruned RoPE.  q: fp16 bits [T][Hq][D_keep]; k: [T][Hkv][D_keep] or NULL.
 * Kept pair i of a head is (x[i], x[i + D_keep/2]); its original pair index is
 * j = kept_idx[h_tab][i] and its angle pos * theta^(-2j/D_full).  Heads map to
 * table rows in contiguous blocks: h_tab = h / (H / H_tab).  Outputs are fp64. */
static void rope_tensor(const uint16_t* x, double* out, const int32_t* pos, const int32_t* kept_idx,
                        int T, int H, int H_tab, int D_full, int D_keep, double theta, int fmt) {
  int half = D_keep / 2, per = H / H_tab;
#pragma omp parallel for num_threads(g_threads) schedule(static)
  for (int t = 0; t < T; ++t)
    for (int h = 0; h < H; ++h) {
      const uint16_t* xv = x + ((size_t)t * H + h) * D_keep;
      double* ov = out + ((size_t)t * H + h) * D_keep;
      const int32_t* tab = kept_idx + (size_t)(h / per) * half;
      for (int i = 0; i < half; ++i) {
        int j = tab[i];
        double phi = (double)pos[t] * pow(theta, -2.0 * (double)j / (double)D_full);
        double a = f16_to_double(xv[i], fmt), b = f16_to_double(xv[i + half], fmt);
        ov[i] = a * cos(phi) - b * sin(phi);
        ov[i + half] = b * cos(phi) + a * sin(phi);
      }
    }
}

int uref_pruned_rope_fmt(const uint16_t* q, const uint16_t* k, const int32_t* positions,
                         const int32_t* kept_idx, int T, int Hq, int Hkv, int H_tab, int D_full,
                         int D_keep, double theta, double* q_out, double* k_out, int fmt) {
  if (D_keep % 2 || D_keep > D_full || H_tab < 1 || Hq % H_tab) return -3;
  rope_tensor(q, q_out, positions, kept_idx, T, Hq, H_tab, D_full, D_keep, theta, fmt);
  if (k) {
    if (Hkv % H_tab) return -3;
    rope_tensor(k, k_out, positions, kept_idx, T, Hkv, H_tab, D_full, D_keep, theta, fmt);
  }
  return 0;
}

int uref_pruned_rope(const uint16_t* q, const uint16_t* k, const int32_t* positions,
                     const int32_t* kept_idx, int T, int Hq, int Hkv, int H_tab, int D_full,
                     int D_keep, double theta, double* q_out, double* k_out) {
  return uref_pruned_rope_fmt(q, k, positions, kept_idx, T, Hq, Hkv, H_tab, D_full, D_keep, theta, q_out, k_out, 0);
}

/* The same rotation on fp64 inputs, in place: x [T][H][D_keep].  It defines the fused
 * "project, then rotate" step (Eq. 2 followed by the RoPE of Sec. 3.2 / Alg. 2) without an
 * intermediate rounding of the projected values: y = RoPE(X W) evaluated in fp64. */
int uref_pruned_rope_f64(double* x, const int32_t* positions, const int32_t* kept_idx, int T, int H,
                         int H_tab, int D_full, int D_keep, double theta) {
  if (D_keep % 2 || D_keep > D_full || H_tab < 1 || H % H_tab) return -3;
  int half = D_keep / 2, per = H / H_tab;
  for (int t = 0; t < T; ++t)
    for (int h = 0; h < H; ++h) {
      double* v = x + ((size_t)t * H + h) * D_keep;
      const int32_t* tab = kept_idx + (size_t)(h / per) * half;
      for (int i = 0; i < half; ++i) {
        int j = tab[i];
        double phi = (double)positions[t] * pow(theta, -2.0 * (double)j / (double)D_full);
        double a = v[i], b = v[i + half];
        v[i] = a * cos(phi) - b * sin(phi);
        v[i + half] = b * cos(phi) + a * sin(phi);
      }
    }
  return 0;
}

/* ---- quantisers (only used to build test inputs / the round-trip pin) ---- */

static void put_nibble(uint32_t* qweight, int K_total, int r, int k, int v) {
  uint32_t* w = &qweight[(size_t)r * (K_total / 8) + k / 8];
  int sh = 4 * (k % 8);
  *w = (*w & ~(15u << sh)) | ((uint32_t)v << sh);
}

/* Eq. 3 with N = 4: s = max|W| / 7, q = clamp(rint(W / s), -8, 7); stored nibble q + 8, zero 8.
 * The scale is stored in fp16 and the codes are taken against the stored scale. */
int uref_quantize_sym(const double* w, int N, int K, int group, uint32_t* qweight,
                      uint16_t* scales, uint8_t* zeros) {
  for (int r = 0; r < N; ++r)
    for (int g = 0; g < K / group; ++g) {
      const double* wg = w + (size_t)r * K + (size_t)g * group;
      double mx = 0.0;
      for (int j = 0; j < group; ++j) mx = fmax(mx, fabs(wg[j]));
      uint16_t s16 = uref_double_to_half(mx / 7.0);
      double s = uref_half_to_double(s16);
      scales[(size_t)r * (K / group) + g] = s16;
      zeros[(size_t)r * (K / group) + g] = 8;
      for (int j = 0; j < group; ++j) {
        double qv = s > 0.0 ? rint(wg[j] / s) : 0.0;
        if (qv < -8.0) qv = -8.0;
        if (qv > 7.0) qv = 7.0;
        put_nibble(qweight, K, r, g * group + j, (int)qv + 8);
      }
    }
  return 0;
}

/* min/max: s = (max - min) / 15, z = clamp(rint(-min / s), 0, 15), q = clamp(rint(W / s) + z, 0, 15) */
int uref_quantize_asym(const double* w, int N, int K, int group, uint32_t* qweight,
                       uint16_t* scales, uint8_t* zeros) {
  for (int r = 0; r < N; ++r)
    for (int g = 0; g < K / group; ++g) {
      const double* wg = w + (size_t)r * K + (size_t)g * group;
      double mn = wg[0], mx = wg[0];
      for (int j = 1; j < group; ++j) { mn = fmin(mn, wg[j]); mx = fmax(mx, wg[j]); }
      uint16_t s16 = uref_double_to_half((mx - mn) / 15.0);
      double s = uref_half_to_double(s16);
      double z = s > 0.0 ? rint(-mn / s) : 0.0;
      if (z < 0.0) z = 0.0;
      if (z > 15.0) z = 15.0;
      scales[(size_t)r * (K / group) + g] = s16;
      zeros[(size_t)r * (K / group) + g] = (uint8_t)z;
      for (int j = 0; j < group; ++j) {
        double qv = (s > 0.0 ? rint(wg[j] / s) : 0.0) + z;
        if (qv < 0.0) qv = 0.0;
        if (qv > 15.0) qv = 15.0;
        put_nibble(qweight, K, r, g * group + j, (int)qv);
      }
    }
  return 0;
}

/* ---- repack: the compact matrix of the kept channels (Sec. 3.4, "unpack, prune channels, repackage") ----
 * Rows: exactly the kept rows, in order.  Columns: a quantisation group stays whole (its scale and zero
 * point belong to all of its columns), so the compact matrix holds, in order, every source group that
 * still has a kept column -- when the kept columns are a prefix, or segments whose stride is a multiple
 * of the group.  For any other column pattern the compact groups could not be described by one segment
 * rule, and all columns stay in place.  plan[0] = N_out, plan[1] = K_out, plan[2..8] = the keep
 * descriptor to use with the compact matrix (rows: all; columns: the same kept columns at their new
 * positions). */
static int cols_compactable(const int32_t* keep, int group) {
  return keep[5] == 0 || keep[5] % group == 0;
}

static int group_carried(const int32_t* keep, int K_total, int group, int g) {
  if (!cols_compactable(keep, group)) return 1;
  for (int k = g * group; k < (g + 1) * group; ++k)
    if (col_kept(keep, K_total, k)) return 1;
  return 0;
}

int uref_w4_repack_plan(int N_total, int K_total, int group, const int32_t* keep, int32_t* plan) {
  static const int32_t none[10] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  if (!keep) keep = none;
  int n = 0, kept_cols_total = 0, groups = 0;
  for (int r = 0; r < N_total; ++r) n += row_kept(keep, N_total, r);
  for (int k = 0; k < K_total; ++k) kept_cols_total += col_kept(keep, K_total, k);
  for (int g = 0; g < K_total / group; ++g) groups += group_carried(keep, K_total, group, g);
  plan[0] = n;
  plan[1] = groups * group;
  for (int i = 2; i < 9; ++i) plan[i] = 0;
  if (keep[5] == 0) {
    plan[3] = kept_cols_total == plan[1] ? 0 : kept_cols_total;   /* prefix (0 = all) */
  } else {
    int per_seg = (keep[6] + group - 1) / group * group;          /* groups that survive per segment */
    plan[3] = kept_cols_total;
    plan[7] = cols_compactable(keep, group) ? per_seg : keep[5];
    plan[8] = keep[6];
  }
  return 0;
}

/* out_q [N_out][K_out/8], out_s / out_z [N_out][K_out/group], sizes from uref_w4_repack_plan */
int uref_w4_repack(const uint32_t* qweight, const uint16_t* scales, const uint8_t* zeros,
                   int N_total, int K_total, int group, const int32_t* keep,
                   uint32_t* out_q, uint16_t* out_s, uint8_t* out_z) {
  static const int32_t none[10] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  if (!keep) keep = none;
  int32_t plan[9];
  uref_w4_repack_plan(N_total, K_total, group, keep, plan);
  const int K_out = plan[1];
  int ro = 0;
  for (int r = 0; r < N_total; ++r) {
    if (!row_kept(keep, N_total, r)) continue;
    int go = 0;
    for (int g = 0; g < K_total / group; ++g) {
      if (!group_carried(keep, K_total, group, g)) continue;
      out_s[(size_t)ro * (K_out / group) + go] = scales[(size_t)r * (K_total / group) + g];
      if (zeros) out_z[(size_t)ro * (K_out / group) + go] = zeros[(size_t)r * (K_total / group) + g];
      for (int j = 0; j < group; ++j) {
        int k = g * group + j;
        uint32_t word = qweight[(size_t)r * (K_total / 8) + k / 8];
        int q = (int)((word >> (4 * (k % 8))) & 15u);                 /* unpack */
        put_nibble(out_q, K_out, ro, go * group + j, q);              /* pack at the compact position */
      }
      ++go;
    }
    ++ro;
  }
  return 0;
}
