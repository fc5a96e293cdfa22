// MFMA dequant-GEMM for M > 4 tokens: y[M][n_keep] = x[M][k_keep] * W'^T.
//
// A block owns a BM x BN tile of y and walks the kept input columns one
// quantisation group (128 columns) at a time.  Per step every thread loads 16
// bytes of packed codes (32 weights of one row and group), dequantises them to
// the canonical fp16 weights in registers and writes them to LDS; activations
// are gathered to their stored column positions (zeros where pruned) in LDS;
// the four waves then run 32x32x16 fp16 MFMAs with fp32 accumulators.
#include "common.h"

namespace uniql {

constexpr int BM = 64, BN = 64, BK = 128;
constexpr int LDT = BK + 8;   // padded LDS row (halves): 272 B keeps 128-bit reads conflict-free
constexpr int kGemmThreads = 256;

__global__ __launch_bounds__(kGemmThreads) void w4_gemm_kernel(LinearArgs a) {
  __shared__ __align__(16) half_t As[BM * LDT];
  __shared__ __align__(16) half_t Bs[BN * LDT];

  const KeepMap& km = a.km;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int n_base = blockIdx.x * BN, m_base = blockIdx.y * BM;
  const int words_per_row = a.K_total >> 3;
  const int groups_per_row = a.K_total / kGroup;

  // loader roles: one row (of A or B) per 4 threads, 32 columns per thread
  const int lrow = tid >> 2, lpart = tid & 3;
  int rc = n_base + lrow;
  rc = rc < km.n_keep ? rc : km.n_keep - 1;
  const size_t srow = (size_t)stored_row(km, rc);
  const int tok = m_base + lrow;
  const bool tok_ok = tok < a.M;
  const half_t* xrow = a.x + (size_t)(tok_ok ? tok : 0) * a.ldx;

  float16_t acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;

  const int ksteps = (km.k_span + BK - 1) / BK;
  for (int kt = 0; kt < ksteps; ++kt) {
    const int k0 = kt * BK + lpart * 32;
    // ---- B: packed codes -> canonical fp16 weights -> LDS (natural column order)
    {
      const uint4 wq = *reinterpret_cast<const uint4*>(a.qweight + srow * words_per_row + (k0 >> 3));
      const size_t g = srow * groups_per_row + kt;
      const GroupQ gq = make_groupq(a.scales[g], a.zeros[g]);
      const Magic mg = make_magic();
      const uint32_t wv[4] = {wq.x, wq.y, wq.z, wq.w};
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        half2_t d[4];
        dequant_word(wv[t], gq, mg, d);
        half8_t o = {d[0].x, d[1].x, d[2].x, d[3].x, d[0].y, d[1].y, d[2].y, d[3].y};
        *reinterpret_cast<half8_t*>(&Bs[lrow * LDT + lpart * 32 + t * 8]) = o;
      }
    }
    // ---- A: activations at stored column positions, zeros where pruned
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      half8_t o;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int k = k0 + t * 8 + j;
        const int kc = k < km.k_span ? compact_col(km, k) : -1;
        o[j] = (kc >= 0 && tok_ok) ? xrow[kc] : (half_t)0;
      }
      *reinterpret_cast<half8_t*>(&As[lrow * LDT + lpart * 32 + t * 8]) = o;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      const int col = kk * 16 + 8 * (lane >> 5);
      const half8_t av = *reinterpret_cast<const half8_t*>(&As[(wm * 32 + (lane & 31)) * LDT + col]);
      const half8_t bv = *reinterpret_cast<const half8_t*>(&Bs[(wn * 32 + (lane & 31)) * LDT + col]);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(av, bv, acc, 0, 0, 0);
    }
    __syncthreads();
  }

  // D[i][j]: j = lane % 32 (weight row), i = 8 * (v / 4) + 4 * (lane / 32) + v % 4 (token)
  const int j = n_base + wn * 32 + (lane & 31);
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int i = m_base + wm * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
    if (i < a.M && j < km.n_keep) a.y[(size_t)i * a.ldy + j] = (half_t)acc[v];
  }
}

hipError_t launch_w4_gemm(const LinearArgs& a, hipStream_t stream) {
  dim3 grid((a.km.n_keep + BN - 1) / BN, (a.M + BM - 1) / BM);
  hipLaunchKernelGGL(w4_gemm_kernel, grid, dim3(kGemmThreads), 0, stream, a);
  return hipGetLastError();
}

}  // namespace uniql
