// Streaming W4A16 GEMV for M = 1..4 tokens (decode).
//
// The op is bound by the HBM stream of packed nibbles, so the kernel is built
// around that stream: a wave reads a kept row in contiguous 1 KB pieces (64
// lanes x 128-bit), i.e. every lane owns 32 consecutive input columns that lie
// in one quantisation group.  Pruned rows are never touched (row truncation
// saves their bytes); pruned columns are handled by staging the activations
// once per block into LDS at their *stored* column positions with zeros in the
// pruned slots, so the weight stream needs no per-element masking.
//
// Per 32-bit word (8 weights): 1 shift + 4 and-or build exact fp16 codes, 4
// packed subtracts and 4 packed multiplies give the canonical fp16 weights
// RN16((q - z) s), and 4 two-way dot instructions per token accumulate in fp32.
#include "common.h"

namespace uniql {

constexpr int kGemvThreads = 256;
constexpr int kGemvWaves = kGemvThreads / kWave;
constexpr int kChunk = kWave * 32;   // stored columns one wave covers with one 128-bit load per lane

__device__ __forceinline__ float dpp_xor_reduce(float v) {
  // butterfly within each row of 16 lanes with DPP, then across rows through the LDS crossbar
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true));  // row_half_mirror
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, true));  // row_mirror
  v += __shfl_xor(v, 16);
  v += __shfl_xor(v, 32);
  return v;
}

struct RowRegs {
  uint4 w;          // 32 packed codes
  uint32_t sbits;   // fp16 scale bits of the lane's group
  uint32_t z;       // zero point of the lane's group
};

template <int MT, int R>
__global__ __launch_bounds__(kGemvThreads) void w4_gemv_kernel(LinearArgs a, int m0, int nchunk) {
  extern __shared__ __align__(16) unsigned char smem[];
  uint4* xs = reinterpret_cast<uint4*>(smem);   // [MT][nchunk][4][64] units of 8 halves

  const KeepMap& km = a.km;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int rg = blockIdx.x * kGemvWaves + wave;   // row group of this wave
  const int k_span32 = (km.k_span + 31) & ~31;
  const int words_per_row = a.K_total >> 3;
  const int groups_per_row = a.K_total / kGroup;

  // stored rows of this wave (clamped so that every address is valid)
  int srow[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    int rc = rg * R + r;
    rc = rc < km.n_keep ? rc : km.n_keep - 1;
    srow[r] = stored_row(km, rc);
  }

  auto load_rows = [&](int c, RowRegs (&rr)[R]) {
    const int kb = c * kChunk + lane * 32;
    const bool act = kb < k_span32;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      if (act) {
        const size_t row = (size_t)srow[r];
        rr[r].w = *reinterpret_cast<const uint4*>(a.qweight + row * words_per_row + (kb >> 3));
        rr[r].sbits = a.scales[row * groups_per_row + (kb >> 7)];
        rr[r].z = a.zeros[row * groups_per_row + (kb >> 7)];
      } else {
        rr[r].w = make_uint4(0, 0, 0, 0);
        rr[r].sbits = 0;
        rr[r].z = 0;
      }
    }
  };

  // start the first weight loads before touching x: they do not depend on it
  RowRegs cur[R], nxt[R];
  load_rows(0, cur);

  // ---- stage x (MT tokens) into LDS at stored column positions, zeros where pruned.
  // unit u of a token = 8 stored columns k0..k0+7, k0 = c*2048 + lane*32 + t*8, stored
  // at [c][t][lane] with halves ordered (k0,k0+4,k0+1,k0+5,k0+2,k0+6,k0+3,k0+7) so that
  // dword p pairs with the dequantised pair (w_p, w_{p+4}).
  const int units = nchunk * 256;
  for (int u = tid; u < units * MT; u += kGemvThreads) {
    const int m = u / units, uu = u - m * units;
    const int c = uu >> 8, l = (uu >> 2) & 63, t = uu & 3;
    const int k0 = c * kChunk + l * 32 + t * 8;
    const int mg = m0 + m;
    half_t v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      int kc = (k0 + j < k_span32) ? compact_col(km, k0 + j) : -1;
      v[j] = (kc >= 0 && mg < a.M) ? a.x[(size_t)mg * a.ldx + kc] : (half_t)0;
    }
    half2_t p0 = {v[0], v[4]}, p1 = {v[1], v[5]}, p2 = {v[2], v[6]}, p3 = {v[3], v[7]};
    xs[((m * nchunk + c) * 4 + t) * 64 + l] = make_uint4(as_u32(p0), as_u32(p1), as_u32(p2), as_u32(p3));
  }
  __syncthreads();

  float acc[R][MT];
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int m = 0; m < MT; ++m) acc[r][m] = 0.f;

  for (int c = 0; c < nchunk; ++c) {
    if (c + 1 < nchunk) load_rows(c + 1, nxt);
    uint4 xr[MT][4];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
      for (int t = 0; t < 4; ++t) xr[m][t] = xs[((m * nchunk + c) * 4 + t) * 64 + lane];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const GroupQ g = make_groupq(cur[r].sbits, cur[r].z);
      const uint32_t wv[4] = {cur[r].w.x, cur[r].w.y, cur[r].w.z, cur[r].w.w};
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        half2_t d[4];
        dequant_word(wv[t], g, d);
#pragma unroll
        for (int m = 0; m < MT; ++m) {
          float s = acc[r][m];
          s = __builtin_amdgcn_fdot2(d[0], as_half2(xr[m][t].x), s, false);
          s = __builtin_amdgcn_fdot2(d[1], as_half2(xr[m][t].y), s, false);
          s = __builtin_amdgcn_fdot2(d[2], as_half2(xr[m][t].z), s, false);
          s = __builtin_amdgcn_fdot2(d[3], as_half2(xr[m][t].w), s, false);
          acc[r][m] = s;
        }
      }
    }
    if (c + 1 < nchunk) {
#pragma unroll
      for (int r = 0; r < R; ++r) cur[r] = nxt[r];
    }
  }

#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int m = 0; m < MT; ++m) {
      const float v = dpp_xor_reduce(acc[r][m]);
      const int rc = rg * R + r;
      if (lane == 0 && rc < km.n_keep && m0 + m < a.M) a.y[(size_t)(m0 + m) * a.ldy + rc] = (half_t)v;
    }
}

template <int MT, int R>
static hipError_t launch_one(const LinearArgs& a, int m0, int nchunk, hipStream_t stream) {
  const size_t smem = (size_t)MT * nchunk * 4096;
  auto kern = w4_gemv_kernel<MT, R>;
  if (smem > 160 * 1024) return hipErrorInvalidValue;
  if (smem > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
  }
  const int row_groups = (a.km.n_keep + R - 1) / R;
  const int blocks = (row_groups + kGemvWaves - 1) / kGemvWaves;
  hipLaunchKernelGGL(kern, dim3(blocks), dim3(kGemvThreads), smem, stream, a, m0, nchunk);
  return hipGetLastError();
}

hipError_t launch_w4_gemv(const LinearArgs& a, hipStream_t stream) {
  const int k_span32 = (a.km.k_span + 31) & ~31;
  const int nchunk = (k_span32 + kChunk - 1) / kChunk;
  // tokens per pass: as many as fit the LDS staging (4 KB per token and chunk)
  int mt = a.M >= 4 ? 4 : (a.M >= 2 ? 2 : 1);
  while (mt > 1 && (size_t)mt * nchunk * 4096 > 160 * 1024) mt >>= 1;
  for (int m0 = 0; m0 < a.M; m0 += mt) {
    hipError_t e;
    if (mt == 4) e = launch_one<4, 2>(a, m0, nchunk, stream);
    else if (mt == 2) e = launch_one<2, 4>(a, m0, nchunk, stream);
    else e = launch_one<1, 4>(a, m0, nchunk, stream);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace uniql
