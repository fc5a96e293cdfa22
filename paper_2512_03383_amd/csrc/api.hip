// C ABI of libuniql: host-side validation and dispatch (declared in include/uniql.h).
// All checks that do not need the device run before the first HIP call, so the
// error paths behave the same on a machine without a GPU.
#include "../../include/uniql.h"
#include "common.h"
#include <algorithm>
#include <atomic>
#include <cmath>

#include <string.h>
#include <vector>

using namespace uniql;

static thread_local int g_last_hip_error = 0;

static int hip_fail(hipError_t e) {
  g_last_hip_error = (int)e;
  return UNIQL_E_HIP;
}

// gfx950 check, cached per device ordinal.
static int check_arch() {
  static std::atomic<int> cached[64];   // 0 unknown, 1 ok, -1 wrong arch (host threads may race on the first call)
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e);
  const int known = (dev >= 0 && dev < 64) ? cached[dev].load(std::memory_order_relaxed) : 0;
  if (known != 0) return known > 0 ? UNIQL_OK : UNIQL_E_ARCH;
  hipDeviceProp_t prop;
  e = hipGetDeviceProperties(&prop, dev);
  if (e != hipSuccess) return hip_fail(e);
  int ok = strncmp(prop.gcnArchName, "gfx950", 6) == 0;
  if (dev >= 0 && dev < 64) cached[dev].store(ok ? 1 : -1, std::memory_order_relaxed);
  return ok ? UNIQL_OK : UNIQL_E_ARCH;
}

static bool aligned(const void* p, uintptr_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

// Validate W / keep and normalise the keep rule.  Pure host arithmetic.
// allow8: the caller serves codes of 8, 6 and 3 bits as well (uniql_w4_linear and uniql_w4_dequant do)
static int code_bits(const uniql_w4_t* W) { return W->bits == 0 ? 4 : W->bits; }
static int make_keepmap(const uniql_w4_t* W, const uniql_keep_t* keep, KeepMap* km, bool allow8 = false) {
  if (!W || !W->qweight || !W->scales) return UNIQL_E_NULL;   // zeros may be NULL: every zero point is 8 (128 for 8-bit codes)
  if (W->group != kGroup || W->N_total < 1 || W->K_total < kGroup || W->K_total % kGroup) return UNIQL_E_SHAPE;
  if (code_bits(W) != 4 && !((code_bits(W) == 8 || code_bits(W) == 6 || code_bits(W) == 3) && allow8 && W->col_interleave == 0)) return UNIQL_E_SHAPE;
  if (W->dtype != UNIQL_F16 && W->dtype != UNIQL_BF16) return UNIQL_E_SHAPE;
  if (W->col_interleave < 0 || (W->col_interleave > 0 && (W->K_total % W->col_interleave || (W->K_total / W->col_interleave) % 8)))
    return UNIQL_E_SHAPE;
  if (!aligned(W->qweight, 16) || !aligned(W->scales, 2)) return UNIQL_E_ALIGN;
  uniql_keep_t none;
  memset(&none, 0, sizeof(none));
  if (!keep) keep = &none;
  const int N = W->N_total, K = W->K_total;
  if (keep->n_keep < 0 || keep->k_keep < 0 || keep->row_seg_stride < 0 || keep->col_seg_stride < 0) return UNIQL_E_KEEP;

  km->rs_stride = keep->row_seg_stride;
  km->rs_keep = km->rs_limit = km->rs_segrows = 0;
  km->rs2_stride = km->rs2_keep = km->rs2_limit = km->rs2_segrows = 0;
  if (keep->row_seg2_stride < 0 || (keep->row_seg2_stride > 0 && keep->row_seg_stride == 0)) return UNIQL_E_KEEP;
  if (keep->row_seg_stride == 0) {
    if (keep->n_keep > N) return UNIQL_E_KEEP;
    km->n_keep = keep->n_keep ? keep->n_keep : N;
  } else {
    if (keep->row_seg_keep < 1 || keep->row_seg_keep > keep->row_seg_stride) return UNIQL_E_KEEP;
    if (keep->row_seg_limit < 0 || keep->row_seg_limit > N || keep->row_seg_limit % keep->row_seg_stride) return UNIQL_E_KEEP;
    km->rs_keep = keep->row_seg_keep;
    km->rs_limit = keep->row_seg_limit;
    km->rs_segrows = (keep->row_seg_limit / keep->row_seg_stride) * keep->row_seg_keep;
    km->rs2_limit = keep->row_seg_limit;
    if (keep->row_seg2_stride > 0) {
      const int span = keep->row_seg2_limit - keep->row_seg_limit;
      if (keep->row_seg2_keep < 1 || keep->row_seg2_keep > keep->row_seg2_stride) return UNIQL_E_KEEP;
      if (span < 0 || keep->row_seg2_limit > N || span % keep->row_seg2_stride) return UNIQL_E_KEEP;
      km->rs2_stride = keep->row_seg2_stride;
      km->rs2_keep = keep->row_seg2_keep;
      km->rs2_limit = keep->row_seg2_limit;
      km->rs2_segrows = (span / keep->row_seg2_stride) * keep->row_seg2_keep;
    }
    km->n_keep = km->rs_segrows + km->rs2_segrows + (N - km->rs2_limit);
    if (keep->n_keep && keep->n_keep != km->n_keep) return UNIQL_E_KEEP;
  }

  km->cs_stride = keep->col_seg_stride;
  km->cs_keep = 0;
  if (keep->col_seg_stride == 0) {
    if (keep->k_keep > K) return UNIQL_E_KEEP;
    km->k_keep = keep->k_keep ? keep->k_keep : K;
    km->k_span = km->k_keep;
  } else {
    if (keep->col_seg_keep < 1 || keep->col_seg_keep > keep->col_seg_stride) return UNIQL_E_KEEP;
    if (K % keep->col_seg_stride || keep->col_seg_stride < 8) return UNIQL_E_KEEP;
    km->cs_keep = keep->col_seg_keep;
    km->k_keep = (K / keep->col_seg_stride) * keep->col_seg_keep;
    if (keep->k_keep && keep->k_keep != km->k_keep) return UNIQL_E_KEEP;
    km->k_span = K - (keep->col_seg_stride - keep->col_seg_keep);   // last kept column + 1
  }
  return UNIQL_OK;
}

// Validate one linear call and fill the kernel arguments.  Host arithmetic only.
static int fill_linear(const uniql_w4_t* W, const uniql_keep_t* keep, const void* x_f16, int64_t ldx,
                       void* y_f16, int64_t ldy, int32_t M, LinearArgs* a, bool allow8 = false) {
  int rc = make_keepmap(W, keep, &a->km, allow8);
  if (rc) return rc;
  if (!x_f16 || !y_f16) return UNIQL_E_NULL;
  if (M < 1 || ldx < a->km.k_keep || ldy < a->km.n_keep) return UNIQL_E_SHAPE;
  if (!aligned(x_f16, 2) || !aligned(y_f16, 2)) return UNIQL_E_ALIGN;
  a->qweight = W->qweight;
  a->scales = W->scales;
  a->zeros = W->zeros;
  a->x = (const half_t*)x_f16;
  a->y = (half_t*)y_f16;
  a->ldx = ldx;
  a->ldy = ldy;
  a->N_total = W->N_total;
  a->K_total = W->K_total;
  a->M = M;
  a->bf16 = W->dtype == UNIQL_BF16;
  a->il_heads = W->col_interleave;
  a->bits = code_bits(W);
  return UNIQL_OK;
}

constexpr int kInterleavedMaxTokens = 64;   // a matrix with head-interleaved words: tokens per call

static int run_linear(const LinearArgs& a, hipStream_t s) {
  if (a.bits != 4) {
    hipError_t e8 = a.bits == 8 ? launch_w8_linear(a, s) : launch_wb_linear(a, s);
    if (e8 == hipErrorInvalidValue) return UNIQL_E_SHAPE;   // more kept columns than the kernel's staging holds
    return e8 == hipSuccess ? UNIQL_OK : hip_fail(e8);
  }
  if (a.il_heads > 0 && a.M != 1) {
    // head-interleaved words are read by the one-token kernel only: a decode batch runs it with one token per grid
    // row (the later tokens' words come from the caches); prompts want the words in column order
    if (a.M > kInterleavedMaxTokens) return UNIQL_E_SHAPE;
    hipError_t et = launch_w4_gemv(a, s);
    if (et == hipErrorInvalidValue) return UNIQL_E_SHAPE;
    return et == hipSuccess ? UNIQL_OK : hip_fail(et);
  }
  hipError_t e = (a.M == 1) ? launch_w4_gemv(a, s) : launch_w4_gemm(a, s);
  if (e == hipErrorInvalidValue && a.M == 1) return UNIQL_E_SHAPE;   // K too long for the GEMV's staging
  return e == hipSuccess ? UNIQL_OK : hip_fail(e);
}

extern "C" int uniql_w4_linear(const uniql_w4_t* W, const uniql_keep_t* keep, const void* x_f16, int64_t ldx,
                               void* y_f16, int64_t ldy, int32_t M, void* hip_stream) {
  LinearArgs a;
  int rc = fill_linear(W, keep, x_f16, ldx, y_f16, ldy, M, &a, true);
  if (rc) return rc;
  rc = check_arch();
  if (rc) return rc;
  return run_linear(a, (hipStream_t)hip_stream);
}

extern "C" int uniql_w4_linear_multi(int32_t n, const uniql_w4_t* W, const uniql_keep_t* keep,
                                     const void* const* x_f16, const int64_t* ldx, void* const* y_f16,
                                     const int64_t* ldy, int32_t M, void* hip_stream) {
  if (n < 1 || n > kMaxBatch) return UNIQL_E_SHAPE;
  if (!W || !x_f16 || !ldx || !y_f16 || !ldy) return UNIQL_E_NULL;
  LinearArgs a[kMaxBatch];
  for (int i = 0; i < n; ++i) {
    int rc = fill_linear(&W[i], keep ? &keep[i] : nullptr, x_f16[i], ldx[i], y_f16[i], ldy[i], M, &a[i]);
    if (rc) return rc;
    if (a[i].il_heads > 0 && n > 1) return UNIQL_E_SHAPE;   // a head-interleaved matrix does not share a launch
  }
  int rc = check_arch();
  if (rc) return rc;
  hipStream_t s = (hipStream_t)hip_stream;
  if (M == 1) {
    hipError_t e = launch_w4_gemv_batch(a, n, s);
    if (e == hipErrorInvalidValue) return UNIQL_E_SHAPE;
    return e == hipSuccess ? UNIQL_OK : hip_fail(e);
  }
  if (n > 1 && M <= 32) {
    // a decode batch: one launch when the decode-batch kernel takes every member (the same format: fill_linear's
    // entries of one call may differ in it, then they go one by one)
    bool same = true, done = false;
    for (int i = 1; i < n; ++i) same = same && a[i].bf16 == a[0].bf16;
    if (same) {
      hipError_t e = launch_w4_gemm_batch(a, n, s, &done);
      if (e != hipSuccess) return hip_fail(e);
      if (done) return UNIQL_OK;
    }
  }
  for (int i = 0; i < n; ++i) {
    rc = run_linear(a[i], s);
    if (rc) return rc;
  }
  return UNIQL_OK;
}

extern "C" int uniql_w4_dequant(const uniql_w4_t* W, const uniql_keep_t* keep, void* w_f16, void* hip_stream) {
  LinearArgs a;
  int rc = make_keepmap(W, keep, &a.km, true);
  if (rc) return rc;
  if (!w_f16) return UNIQL_E_NULL;
  if (!aligned(w_f16, 2)) return UNIQL_E_ALIGN;
  rc = check_arch();
  if (rc) return rc;
  a.qweight = W->qweight;
  a.scales = W->scales;
  a.zeros = W->zeros;
  a.x = nullptr;
  a.y = (half_t*)w_f16;
  a.ldx = 0;
  a.ldy = a.km.k_keep;
  a.N_total = W->N_total;
  a.K_total = W->K_total;
  a.M = 0;
  a.bf16 = W->dtype == UNIQL_BF16;
  a.il_heads = W->col_interleave;
  a.bits = code_bits(W);
  hipError_t e = a.bits == 8 ? launch_w8_dequant(a, (hipStream_t)hip_stream)
                 : a.bits == 4 ? launch_w4_dequant(a, (hipStream_t)hip_stream) : launch_wb_dequant(a, (hipStream_t)hip_stream);
  return e == hipSuccess ? UNIQL_OK : hip_fail(e);
}

// Sizes, group mapping and keep descriptor of the compact matrix.  Host arithmetic only.
struct RepackPlan {
  int N_out, K_out, gps_src, gps_out;
  uniql_keep_t keep_out;
};
static int make_repack_plan(const uniql_w4_t* W, const uniql_keep_t* keep, KeepMap* km, RepackPlan* p) {
  int rc = make_keepmap(W, keep, km);
  if (rc) return rc;
  if (W->col_interleave > 0) return UNIQL_E_SHAPE;
  memset(p, 0, sizeof(*p));
  p->N_out = km->n_keep;
  const int K = W->K_total;
  if (km->cs_stride == 0) {
    // column prefix: the groups that reach into it, whole
    p->K_out = (km->k_keep + kGroup - 1) / kGroup * kGroup;
    p->keep_out.k_keep = km->k_keep == p->K_out ? 0 : km->k_keep;
  } else if (km->cs_stride % kGroup == 0) {
    // segments made of whole groups: the leading groups of each segment that hold kept columns
    p->gps_src = km->cs_stride / kGroup;
    p->gps_out = (km->cs_keep + kGroup - 1) / kGroup;
    p->K_out = (K / km->cs_stride) * p->gps_out * kGroup;
    p->keep_out.k_keep = km->k_keep;
    p->keep_out.col_seg_stride = p->gps_out * kGroup;
    p->keep_out.col_seg_keep = km->cs_keep;
  } else {
    // groups straddle segments: every group still holds kept columns or could not be described; columns stay
    p->K_out = K;
    p->keep_out.k_keep = km->k_keep;
    p->keep_out.col_seg_stride = km->cs_stride;
    p->keep_out.col_seg_keep = km->cs_keep;
  }
  return UNIQL_OK;
}

extern "C" int uniql_w4_repack_plan(const uniql_w4_t* W, const uniql_keep_t* keep, int32_t* N_out, int32_t* K_out,
                                    uniql_keep_t* keep_out) {
  if (!N_out || !K_out || !keep_out) return UNIQL_E_NULL;
  KeepMap km;
  RepackPlan p;
  // the plan needs the sizes only: the data pointers of W may be NULL here
  if (!W) return UNIQL_E_NULL;
  uniql_w4_t shape = *W;
  static const uint32_t dummy[4] __attribute__((aligned(16))) = {0, 0, 0, 0};
  shape.qweight = dummy;
  shape.scales = reinterpret_cast<const uint16_t*>(dummy);
  shape.zeros = reinterpret_cast<const uint8_t*>(dummy);
  int rc = make_repack_plan(&shape, keep, &km, &p);
  if (rc) return rc;
  *N_out = p.N_out;
  *K_out = p.K_out;
  *keep_out = p.keep_out;
  return UNIQL_OK;
}

extern "C" int uniql_w4_repack(const uniql_w4_t* W, const uniql_keep_t* keep, uint32_t* out_qweight,
                               uint16_t* out_scales, uint8_t* out_zeros, int32_t N_out, int32_t K_out,
                               void* hip_stream) {
  RepackArgs a;
  RepackPlan p;
  int rc = make_repack_plan(W, keep, &a.km, &p);
  if (rc) return rc;
  if (!out_qweight || !out_scales || (W->zeros && !out_zeros)) return UNIQL_E_NULL;
  if (N_out != p.N_out || K_out != p.K_out) return UNIQL_E_SHAPE;
  if (!aligned(out_qweight, 16) || !aligned(out_scales, 2)) return UNIQL_E_ALIGN;
  rc = check_arch();
  if (rc) return rc;
  a.qweight = W->qweight;
  a.scales = W->scales;
  a.zeros = W->zeros;
  a.out_qweight = out_qweight;
  a.out_scales = out_scales;
  a.out_zeros = out_zeros;
  a.K_total = W->K_total;
  a.K_out = p.K_out;
  a.gps_src = p.gps_src;
  a.gps_out = p.gps_out;
  hipError_t e = launch_w4_repack(a, (hipStream_t)hip_stream);
  return e == hipSuccess ? UNIQL_OK : hip_fail(e);
}

extern "C" int uniql_w4_embedding(const uniql_w4_t* W, const int32_t* ids, int32_t n, void* out_f16, int64_t ld,
                                  void* hip_stream) {
  KeepMap km;
  int rc = make_keepmap(W, nullptr, &km);
  if (rc) return rc;
  if (!ids || !out_f16) return UNIQL_E_NULL;
  if (n < 1 || ld < W->K_total || W->col_interleave > 0) return UNIQL_E_SHAPE;
  // every lane writes 64-byte pieces with 128-bit stores
  if (!aligned(ids, 4) || !aligned(out_f16, 16) || ld % 8) return UNIQL_E_ALIGN;
  rc = check_arch();
  if (rc) return rc;
  hipError_t e = launch_w4_embedding(W->qweight, W->scales, W->zeros, W->K_total, ids, n, (half_t*)out_f16, ld,
                                     W->dtype == UNIQL_BF16, (hipStream_t)hip_stream);
  if (e == hipErrorInvalidValue) return UNIQL_E_SHAPE;
  return e == hipSuccess ? UNIQL_OK : hip_fail(e);
}

static int pruned_rope(void* q_f16, void* k_f16, const int32_t* positions, const int32_t* kept_idx,
                       int32_t T, int32_t Hq, int32_t Hkv, int32_t H_tab, int32_t D_full,
                       int32_t D_keep, double theta, int bf16, void* hip_stream) {
  if (!q_f16 || !positions || !kept_idx) return UNIQL_E_NULL;
  if ((Hkv > 0) != (k_f16 != nullptr)) return Hkv > 0 ? UNIQL_E_NULL : UNIQL_E_SHAPE;
  if (T < 1 || Hq < 1 || Hkv < 0) return UNIQL_E_SHAPE;
  if (D_full < 2 || D_full % 2 || D_keep < 2 || D_keep % 2 || D_keep > D_full) return UNIQL_E_KEEP;
  if (H_tab < 1 || Hq % H_tab || Hkv % H_tab) return UNIQL_E_KEEP;
  if (!(theta > 0.0)) return UNIQL_E_KEEP;
  if (!aligned(q_f16, 2) || !aligned(k_f16, 2) || !aligned(positions, 4) || !aligned(kept_idx, 4)) return UNIQL_E_ALIGN;
  int rc = check_arch();
  if (rc) return rc;
  RopeArgs a;
  a.q = (half_t*)q_f16;
  a.k = (half_t*)k_f16;
  a.positions = positions;
  a.kept_idx = kept_idx;
  a.T = T; a.Hq = Hq; a.Hkv = Hkv; a.H_tab = H_tab; a.D_full = D_full; a.D_keep = D_keep;
  a.theta = theta;
  a.bf16 = bf16;
  hipError_t e = launch_pruned_rope(a, (hipStream_t)hip_stream);
  return e == hipSuccess ? UNIQL_OK : hip_fail(e);
}

extern "C" int uniql_pruned_rope(void* q_f16, void* k_f16, const int32_t* positions, const int32_t* kept_idx,
                                 int32_t T, int32_t Hq, int32_t Hkv, int32_t H_tab, int32_t D_full,
                                 int32_t D_keep, double theta, void* hip_stream) {
  return pruned_rope(q_f16, k_f16, positions, kept_idx, T, Hq, Hkv, H_tab, D_full, D_keep, theta, 0, hip_stream);
}

extern "C" int uniql_rope_table_check(const int32_t* kept_idx_host, int32_t H_tab, int32_t D_full, int32_t D_keep) {
  if (!kept_idx_host) return UNIQL_E_NULL;
  if (D_full < 2 || D_full % 2 || D_keep < 2 || D_keep % 2 || D_keep > D_full || H_tab < 1) return UNIQL_E_KEEP;
  const int hk = D_keep / 2, half = D_full / 2;
  std::vector<unsigned char> seen((size_t)half);
  for (int h = 0; h < H_tab; ++h) {
    std::fill(seen.begin(), seen.end(), 0);
    for (int i = 0; i < hk; ++i) {
      const int32_t j = kept_idx_host[(size_t)h * hk + i];
      if (j < 0 || j >= half || seen[(size_t)j]) return UNIQL_E_KEEP;
      seen[(size_t)j] = 1;
    }
  }
  return UNIQL_OK;
}

extern "C" int uniql_pruned_rope_bf16(void* q_bf16, void* k_bf16, const int32_t* positions, const int32_t* kept_idx,
                                      int32_t T, int32_t Hq, int32_t Hkv, int32_t H_tab, int32_t D_full,
                                      int32_t D_keep, double theta, void* hip_stream) {
  return pruned_rope(q_bf16, k_bf16, positions, kept_idx, T, Hq, Hkv, H_tab, D_full, D_keep, theta, 1, hip_stream);
}

extern "C" int uniql_w4_qkv_rope(const uniql_w4_t* W, const uniql_keep_t* keep, const void* x_f16, void* q_f16,
                                 void* k_f16, void* v_f16, const int32_t* position, const int32_t* kept_idx,
                                 int32_t Hq, int32_t Hkv, int32_t H_tab, int32_t D_full, int32_t D_keep,
                                 double theta, void* hip_stream) {
  if (!W || !position || !kept_idx) return UNIQL_E_NULL;
  if (Hq < 1 || Hkv < 1) return UNIQL_E_SHAPE;
  if (D_full < 2 || D_full % 2 || D_keep < 2 || D_keep % 2 || D_keep > D_full) return UNIQL_E_KEEP;
  if (H_tab < 1 || Hq % H_tab || Hkv % H_tab) return UNIQL_E_KEEP;
  if (!(theta > 0.0)) return UNIQL_E_KEEP;
  if (!aligned(position, 4) || !aligned(kept_idx, 4)) return UNIQL_E_ALIGN;
  void* y[3] = {q_f16, k_f16, v_f16};
  LinearArgs a[3];
  for (int i = 0; i < 3; ++i) {
    // one token: the leading dimensions are the kept dimensions themselves
    KeepMap km;
    int rc = make_keepmap(&W[i], keep ? &keep[i] : nullptr, &km);
    if (rc) return rc;
    rc = fill_linear(&W[i], keep ? &keep[i] : nullptr, x_f16, km.k_keep, y[i], km.n_keep, 1, &a[i]);
    if (rc) return rc;
    if (km.k_keep != a[0].km.k_keep) return UNIQL_E_SHAPE;   // one x for all three
    if (a[i].il_heads > 0) return UNIQL_E_SHAPE;
    if (a[i].bf16 != a[0].bf16) return UNIQL_E_SHAPE;        // ... in one format
  }
  // q and k come out as [heads][D_keep]
  if ((long long)a[0].km.n_keep != (long long)Hq * D_keep || (long long)a[1].km.n_keep != (long long)Hkv * D_keep) return UNIQL_E_KEEP;
  int rc = check_arch();
  if (rc) return rc;
  hipStream_t s = (hipStream_t)hip_stream;
  RopeFuse rf = {};
  rf.positions = position;
  rf.kept_idx = kept_idx;
  rf.H_tab = H_tab;
  rf.D_keep = D_keep;
  rf.base = pow(theta, -2.0 / (double)D_full);
  rf.heads[0] = Hq;
  rf.heads[1] = Hkv;
  bool fused = false;
  // the persistent walk for the sizes it serves, else the block kernel with the rotation as epilogue
  hipError_t e = launch_w4_qkv_rope_stream(a, rf, s, &fused);
  if (e != hipSuccess) return e == hipErrorInvalidValue ? UNIQL_E_SHAPE : hip_fail(e);
  if (fused) return UNIQL_OK;
  e = launch_w4_qkv_rope(a, rf, s, &fused);
  if (e != hipSuccess) return e == hipErrorInvalidValue ? UNIQL_E_SHAPE : hip_fail(e);
  if (fused) return UNIQL_OK;
  // shapes that cannot share one launch: the three projections, then the stand-alone rotation
  e = launch_w4_gemv_batch(a, 3, s);
  if (e != hipSuccess) return e == hipErrorInvalidValue ? UNIQL_E_SHAPE : hip_fail(e);
  RopeArgs r;
  r.q = (half_t*)q_f16;
  r.k = (half_t*)k_f16;
  r.positions = position;
  r.kept_idx = kept_idx;
  r.T = 1; r.Hq = Hq; r.Hkv = Hkv; r.H_tab = H_tab; r.D_full = D_full; r.D_keep = D_keep;
  r.theta = theta;
  r.bf16 = a[0].bf16;
  e = launch_pruned_rope(r, s);
  return e == hipSuccess ? UNIQL_OK : hip_fail(e);
}

extern "C" int uniql_w4_gate_up_silu(const uniql_w4_t* W, const uniql_keep_t* keep, const void* x_f16, void* h_f16,
                                     void* hip_stream) {
  if (!W) return UNIQL_E_NULL;
  LinearArgs a[2];
  for (int i = 0; i < 2; ++i) {
    KeepMap km;
    int rc = make_keepmap(&W[i], keep ? &keep[i] : nullptr, &km);
    if (rc) return rc;
    // both members write their sums to LDS only; h takes the place of y in the descriptor of either
    rc = fill_linear(&W[i], keep ? &keep[i] : nullptr, x_f16, km.k_keep, h_f16, km.n_keep, 1, &a[i]);
    if (rc) return rc;
    if (a[i].il_heads > 0) return UNIQL_E_SHAPE;
  }
  // one x and one h: the same kept rows in number, the same rule for the kept columns
  if (a[0].km.n_keep != a[1].km.n_keep || a[0].K_total != a[1].K_total || a[0].km.k_keep != a[1].km.k_keep ||
      a[0].km.cs_stride != a[1].km.cs_stride || a[0].km.cs_keep != a[1].km.cs_keep) return UNIQL_E_KEEP;
  if (a[0].bf16 != a[1].bf16) return UNIQL_E_SHAPE;
  int rc = check_arch();
  if (rc) return rc;
  bool fused = false;
  hipError_t e = launch_w4_gate_up_silu(a, (hipStream_t)hip_stream, &fused);
  if (e != hipSuccess) return e == hipErrorInvalidValue ? UNIQL_E_SHAPE : hip_fail(e);
  return fused ? UNIQL_OK : UNIQL_E_SHAPE;   // no scratch to fall back on: the caller runs the two linears itself
}

extern "C" int uniql_w4_gate_up_silu_batch(const uniql_w4_t* W, const uniql_keep_t* keep, const void* x_f16, int64_t ldx,
                                           void* h_f16, int64_t ldh, int32_t M, void* hip_stream) {
  if (!W) return UNIQL_E_NULL;
  LinearArgs a[2];
  for (int i = 0; i < 2; ++i) {
    int rc = fill_linear(&W[i], keep ? &keep[i] : nullptr, x_f16, ldx, h_f16, ldh, M, &a[i]);
    if (rc) return rc;
    if (a[i].il_heads > 0) return UNIQL_E_SHAPE;
  }
  if (a[0].km.n_keep != a[1].km.n_keep || a[0].K_total != a[1].K_total || a[0].km.k_keep != a[1].km.k_keep ||
      a[0].km.cs_stride != a[1].km.cs_stride || a[0].km.cs_keep != a[1].km.cs_keep) return UNIQL_E_KEEP;
  if (a[0].bf16 != a[1].bf16) return UNIQL_E_SHAPE;
  if (M == 1) return uniql_w4_gate_up_silu(W, keep, x_f16, h_f16, hip_stream);
  int rc = check_arch();
  if (rc) return rc;
  bool done = false;
  hipError_t e = launch_w4_gate_up_silu_batch(a, (hipStream_t)hip_stream, &done);
  if (e != hipSuccess) return hip_fail(e);
  return done ? UNIQL_OK : UNIQL_E_SHAPE;   // no scratch to fall back on: the caller runs the two linears itself
}

extern "C" int uniql_w4_interleave(const uniql_w4_t* W, int32_t heads, uint32_t* out_qweight, void* hip_stream) {
  KeepMap km;
  int rc = make_keepmap(W, nullptr, &km);
  if (rc) return rc;
  if (!out_qweight) return UNIQL_E_NULL;
  if (W->col_interleave != 0 || heads < 1 || W->K_total % heads || (W->K_total / heads) % 8) return UNIQL_E_SHAPE;
  if (!aligned(out_qweight, 16)) return UNIQL_E_ALIGN;
  rc = check_arch();
  if (rc) return rc;
  hipError_t e = launch_w4_interleave(W->qweight, out_qweight, W->N_total, W->K_total, heads, false, (hipStream_t)hip_stream);
  return e == hipSuccess ? UNIQL_OK : hip_fail(e);
}

extern "C" int uniql_w4_deinterleave(const uniql_w4_t* W, uint32_t* out_qweight, void* hip_stream) {
  KeepMap km;
  int rc = make_keepmap(W, nullptr, &km);
  if (rc) return rc;
  if (!out_qweight) return UNIQL_E_NULL;
  if (W->col_interleave < 1) return UNIQL_E_SHAPE;
  if (!aligned(out_qweight, 16)) return UNIQL_E_ALIGN;
  rc = check_arch();
  if (rc) return rc;
  hipError_t e = launch_w4_interleave(W->qweight, out_qweight, W->N_total, W->K_total, W->col_interleave, true, (hipStream_t)hip_stream);
  return e == hipSuccess ? UNIQL_OK : hip_fail(e);
}

// ---- the gated MLP of one token (Eq. 1): gate + up + activation, then down, in one launch when the shapes allow
// workspace: 256 bytes of control words and 4096 bytes of per-block arrival words (see mlp_stream_kernel.h), then the
// hidden vector, padded to whole units of eight 16-bit elements
static const int64_t kMlpHeader = 4352;
static int64_t mlp_units(int32_t n) { return ((int64_t)n + 7) / 8 * 8; }

extern "C" int64_t uniql_w4_mlp_workspace_bytes(int32_t n_hidden_keep) {
  if (n_hidden_keep < 1) return 0;
  return (kMlpHeader + mlp_units(n_hidden_keep) * 2 + 255) / 256 * 256;
}

static int mlp_run(const uniql_w4_t* W, const uniql_keep_t* keep, const void* x_f16, void* y_f16, void* scratch,
                   int64_t scratch_bytes, hipStream_t stream) {
  if (!W || !scratch) return UNIQL_E_NULL;
  if (!aligned(scratch, 256)) return UNIQL_E_ALIGN;
  LinearArgs a[3];
  KeepMap km0;
  int rc = make_keepmap(&W[0], keep ? &keep[0] : nullptr, &km0);
  if (rc) return rc;
  if (scratch_bytes < uniql_w4_mlp_workspace_bytes(km0.n_keep)) return UNIQL_E_SHAPE;
  uint16_t* h = reinterpret_cast<uint16_t*>(reinterpret_cast<char*>(scratch) + kMlpHeader);
  for (int i = 0; i < 2; ++i) {
    KeepMap km;
    rc = make_keepmap(&W[i], keep ? &keep[i] : nullptr, &km);
    if (rc) return rc;
    rc = fill_linear(&W[i], keep ? &keep[i] : nullptr, x_f16, km.k_keep, h, km.n_keep, 1, &a[i]);
    if (rc) return rc;
  }
  if (a[0].km.n_keep != a[1].km.n_keep || a[0].K_total != a[1].K_total || a[0].km.k_keep != a[1].km.k_keep ||
      a[0].km.cs_stride != a[1].km.cs_stride || a[0].km.cs_keep != a[1].km.cs_keep) return UNIQL_E_KEEP;
  {
    KeepMap km;
    rc = make_keepmap(&W[2], keep ? &keep[2] : nullptr, &km);
    if (rc) return rc;
    if (km.k_keep != a[0].km.n_keep) return UNIQL_E_KEEP;   // down reads exactly the hidden vector gate / up write
    rc = fill_linear(&W[2], keep ? &keep[2] : nullptr, h, km.k_keep, y_f16, km.n_keep, 1, &a[2]);
    if (rc) return rc;
  }
  if (a[0].bf16 != a[1].bf16 || a[0].bf16 != a[2].bf16) return UNIQL_E_SHAPE;
  if (a[0].il_heads > 0 || a[1].il_heads > 0 || a[2].il_heads > 0) return UNIQL_E_SHAPE;
  rc = check_arch();
  if (rc) return rc;
  bool done = false;
  hipError_t e = launch_w4_mlp_fused(a, scratch, stream, &done);
  if (e != hipSuccess) return e == hipErrorInvalidValue ? UNIQL_E_SHAPE : hip_fail(e);
  if (done) return UNIQL_OK;
  // shapes the fused launch does not serve: the two launches one after the other, h through the same scratch memory
  bool fused = false;
  e = launch_w4_gate_up_silu(a, stream, &fused);
  if (e != hipSuccess) return e == hipErrorInvalidValue ? UNIQL_E_SHAPE : hip_fail(e);
  if (!fused) return UNIQL_E_SHAPE;
  return run_linear(a[2], stream);
}

extern "C" int uniql_w4_mlp(const uniql_w4_t* W, const uniql_keep_t* keep, const void* x_f16, void* y_f16,
                            void* workspace, int64_t workspace_bytes, void* hip_stream) {
  return mlp_run(W, keep, x_f16, y_f16, workspace, workspace_bytes, (hipStream_t)hip_stream);
}

// ---- the same call for callers that cannot allocate: the workspace is a static array in device memory
static const int32_t kMlpStaticMaxHidden = 32768;                       // kept intermediate channels the array holds
static const int64_t kMlpStaticBytes = 4352 + 2 * (int64_t)32768;       // = uniql_w4_mlp_workspace_bytes(32768)
static __device__ __align__(256) unsigned char scratch[kMlpStaticBytes];   // zero until the first launch on the device

// Device address of `scratch` on the current device, looked up once per device ordinal (each device holds its own copy
// of the array at its own address).  Host code must use this pointer, never the array's name.
static int scratch_ptr(void** out) {
  static std::atomic<void*> cached[64];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e);
  if (dev < 0 || dev >= 64) return UNIQL_E_SHAPE;
  void* p = cached[dev].load(std::memory_order_acquire);
  if (!p) {
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_fail(e);
    if (!p) return UNIQL_E_NULL;
    cached[dev].store(p, std::memory_order_release);   // (host threads that race on the first call store the same address)
  }
  *out = p;
  return UNIQL_OK;
}

extern "C" int uniql_w4_mlp_static(const uniql_w4_t* W, const uniql_keep_t* keep, const void* x_f16, void* y_f16,
                                   void* hip_stream) {
  if (!W) return UNIQL_E_NULL;
  // the size check comes first and needs no device: a hidden dimension beyond the array is refused, not truncated
  KeepMap km;
  int rc = make_keepmap(&W[0], keep ? &keep[0] : nullptr, &km);
  if (rc) return rc;
  if (km.n_keep > kMlpStaticMaxHidden) return UNIQL_E_SHAPE;
  rc = check_arch();
  if (rc) return rc;
  void* ws = nullptr;
  rc = scratch_ptr(&ws);
  if (rc) return rc;
  return mlp_run(W, keep, x_f16, y_f16, ws, kMlpStaticBytes, (hipStream_t)hip_stream);
}

extern "C" int32_t uniql_w4_mlp_static_max_hidden(void) { return kMlpStaticMaxHidden; }

extern "C" int uniql_w4_mlp_hidden(const void* workspace, int32_t n_hidden_keep, const void** h_f16) {
  if (!workspace || !h_f16) return UNIQL_E_NULL;
  if (n_hidden_keep < 1) return UNIQL_E_SHAPE;
  *h_f16 = reinterpret_cast<const char*>(workspace) + kMlpHeader;
  return UNIQL_OK;
}

extern "C" int uniql_w4_mlp_status(const void* workspace, uint32_t* gave_up_serial, void* hip_stream) {
  if (!workspace || !gave_up_serial) return UNIQL_E_NULL;
  hipStream_t s = (hipStream_t)hip_stream;
  hipError_t e = hipMemcpyAsync(gave_up_serial, reinterpret_cast<const char*>(workspace) + 8, 4, hipMemcpyDeviceToHost, s);
  if (e != hipSuccess) return hip_fail(e);
  e = hipStreamSynchronize(s);
  return e == hipSuccess ? UNIQL_OK : hip_fail(e);
}

extern "C" int uniql_w4_gate_up_stream_probe(const uniql_w4_t* W, const uniql_keep_t* keep, const void* x_f16, void* h_f16,
                                             void* hip_stream) {
  if (!W) return UNIQL_E_NULL;
  LinearArgs a[2];
  for (int i = 0; i < 2; ++i) {
    KeepMap km;
    int rc = make_keepmap(&W[i], keep ? &keep[i] : nullptr, &km);
    if (rc) return rc;
    rc = fill_linear(&W[i], keep ? &keep[i] : nullptr, x_f16, km.k_keep, h_f16, km.n_keep, 1, &a[i]);
    if (rc) return rc;
  }
  int rc = check_arch();
  if (rc) return rc;
  bool done = false;
  hipError_t e = launch_w4_gate_up_stream_probe(a, (hipStream_t)hip_stream, &done);
  if (e != hipSuccess) return hip_fail(e);
  return done ? UNIQL_OK : UNIQL_E_SHAPE;
}

extern "C" int uniql_stream_read_probe(const void* src, int64_t bytes, void* out_words, void* hip_stream) {
  if (!src || !out_words) return UNIQL_E_NULL;
  if (bytes < 0) return UNIQL_E_SHAPE;
  if (!aligned(src, 16) || !aligned(out_words, 4)) return UNIQL_E_ALIGN;
  int rc = check_arch();
  if (rc) return rc;
  hipError_t e = launch_stream_read(src, bytes, (uint32_t*)out_words, (hipStream_t)hip_stream);
  return e == hipSuccess ? UNIQL_OK : hip_fail(e);
}

extern "C" const char* uniql_strerror(int code) {
  switch (code) {
    case UNIQL_OK: return "ok";
    case UNIQL_E_NULL: return "a required pointer is NULL";
    case UNIQL_E_SHAPE: return "impossible shape (group != 128, K_total % 128, unknown dtype, M < 1, leading dimension too small, or K too long)";
    case UNIQL_E_KEEP: return "kept dimensions inconsistent with totals, segment rule or head counts";
    case UNIQL_E_ALIGN: return "pointer alignment (qweight 16 B; 16-bit tensors 2 B; int32 tables 4 B)";
    case UNIQL_E_ARCH: return "current device is not gfx950";
    case UNIQL_E_HIP: return "HIP runtime error (see uniql_last_hip_error)";
    default: return "unknown uniql error code";
  }
}

extern "C" int uniql_last_hip_error(void) { return g_last_hip_error; }

extern "C" int uniql_version(void) { return 220; }
