// Bit-exact dequantisation of the kept sub-matrix: w = RN_fp16((q - z) * s), or RN_bf16 when scales and
// output are bfloat16.
// The product of the small integer (q - z) and the 11-bit (8-bit) significand of s is
// exact in fp32, so the single fp32 -> 16-bit conversion is the only rounding.
// (Written with scalar fp32 arithmetic on purpose: it is the independent check
// of the packed-fp16 dequantisation used inside the GEMV / GEMM kernels.)
#include "common.h"

namespace uniql {

template <bool BF16>
__global__ __launch_bounds__(256) void w4_dequant_kernel(LinearArgs a) {
  const KeepMap& km = a.km;
  const int words_span = (km.k_span + 7) >> 3;
  const long long total = (long long)km.n_keep * words_span;
  const int words_per_row = a.K_total >> 3;
  const int groups_per_row = a.K_total / kGroup;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (long long)gridDim.x * blockDim.x) {
    const int rc = (int)(i / words_span);
    const int w = (int)(i - (long long)rc * words_span);
    const size_t row = (size_t)stored_row(km, rc);
    // w counts words in column order; a head-interleaved row stores word (h, d / 8) at (d / 8) * H + h
    int ws = w;
    if (a.il_heads > 0) {
      const int wph = words_per_row / a.il_heads, h = w / wph;
      ws = (w - h * wph) * a.il_heads + h;
    }
    const uint32_t word = a.qweight[row * words_per_row + ws];
    const size_t g = row * groups_per_row + (w >> 4);
    const float s = in16<BF16>(__builtin_bit_cast(half_t, a.scales[g]));
    const int z = a.zeros ? a.zeros[g] : 8;   // no zero points: the symmetric scheme
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int kc = compact_col(km, w * 8 + j);
      if (kc >= 0) {
        const int q = (int)((word >> (4 * j)) & 15u);
        a.y[(size_t)rc * km.k_keep + kc] = out16<BF16>((float)(q - z) * s);
      }
    }
  }
}

hipError_t launch_w4_dequant(const LinearArgs& a, hipStream_t stream) {
  const long long total = (long long)a.km.n_keep * ((a.km.k_span + 7) >> 3);
  long long blocks = (total + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  if (blocks < 1) blocks = 1;
  if (a.bf16) hipLaunchKernelGGL(w4_dequant_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, stream, a);
  else hipLaunchKernelGGL(w4_dequant_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, stream, a);
  return hipGetLastError();
}

// Rows of a quantised table gathered by token id: out[i][:] = dequantised row ids[i].
// A wave handles one (token, 2048-column chunk): a lane reads 16 bytes of codes and the scale and
// zero point of its group, dequantises with the packed path of the GEMV, puts the 32 halves back
// into column order and writes 64 contiguous bytes.  Rows are K_total wide (the hidden dimension
// is never pruned).  BF16: the table's scales and the output are bfloat16 (fp32 arithmetic, subtract then
// multiply, so that a zero weight has the sign of (q - z) * s as in the fp16 path).
template <bool BF16>
__global__ __launch_bounds__(256) void w4_embedding_kernel(const uint32_t* qweight, const uint16_t* scales,
                                                           const uint8_t* zeros, int K_total, const int32_t* ids,
                                                           int n, half_t* out, long long ld) {
  const int lane = threadIdx.x & 63;
  const int chunks = (K_total + 2047) / 2048;
  const long long item = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);   // (token, chunk)
  if (item >= (long long)n * chunks) return;
  const int tok = (int)(item / chunks), c = (int)(item - (long long)tok * chunks);
  const int k0 = c * 2048 + lane * 32;
  if (k0 >= K_total) return;                      // K_total is a multiple of 128: a lane's 32 columns are all in or all out
  const size_t row = (size_t)ids[tok];
  const uint4 w = *reinterpret_cast<const uint4*>(qweight + row * (size_t)(K_total >> 3) + (k0 >> 3));
  const size_t g = row * (size_t)(K_total / kGroup) + (k0 >> 7);
  const uint32_t z = zeros ? zeros[g] : 8u;
  const typename GroupOf<BF16>::type gq = make_group<BF16>(scales[g], z);
  const Magic mg = make_magic();
  const uint32_t words[4] = {w.x, w.y, w.z, w.w};
  uint4* dst = reinterpret_cast<uint4*>(out + (size_t)tok * ld + k0);   // 16-byte aligned: checked by the host
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    uint4 d;                                      // (w0,w4) (w1,w5) (w2,w6) (w3,w7)
    if constexpr (BF16) d = dequant_word_bf16<true>(words[q], gq, (float)z);
    else d = dequant_word4<false>(words[q], gq, mg);
    const uint32_t a = d.x, b = d.y, cc = d.z, e = d.w;
    dst[q] = make_uint4(__builtin_amdgcn_perm(b, a, 0x05040100u), __builtin_amdgcn_perm(e, cc, 0x05040100u),
                        __builtin_amdgcn_perm(b, a, 0x07060302u), __builtin_amdgcn_perm(e, cc, 0x07060302u));
  }
}

hipError_t launch_w4_embedding(const uint32_t* qweight, const uint16_t* scales, const uint8_t* zeros, int K_total,
                               const int32_t* ids, int n, half_t* out, long long ld, int bf16, hipStream_t stream) {
  const long long items = (long long)n * ((K_total + 2047) / 2048);
  const long long blocks = (items + 3) / 4;
  if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  if (bf16)
    hipLaunchKernelGGL(w4_embedding_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, stream, qweight, scales, zeros,
                       K_total, ids, n, out, ld);
  else
    hipLaunchKernelGGL(w4_embedding_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, stream, qweight, scales, zeros,
                       K_total, ids, n, out, ld);
  return hipGetLastError();
}

// Compact copy of the kept channels.  Output row r' is stored row stored_row(r'); output group g' is source
// group (g' / gps_out) * gps_src + g' % gps_out (gps_out = 0: groups stay in place).  A thread moves one
// 16-byte unit (32 codes, a quarter of a group); the thread of a group's first unit also moves the
// group's scale and zero point.  Rows are contiguous on both sides, so the copy streams.
__global__ __launch_bounds__(256) void w4_repack_kernel(RepackArgs a) {
  const int units_out = a.K_out >> 5;
  const long long total = (long long)a.km.n_keep * units_out;
  const int units_src = a.K_total >> 5;
  const int groups_src = a.K_total / kGroup, groups_out = a.K_out / kGroup;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (long long)gridDim.x * blockDim.x) {
    const int rc = (int)(i / units_out);
    const int u = (int)(i - (long long)rc * units_out);
    const int go = u >> 2;
    const int g = a.gps_out ? (go / a.gps_out) * a.gps_src + go % a.gps_out : go;
    const size_t row = (size_t)stored_row(a.km, rc);
    const uint4* src = reinterpret_cast<const uint4*>(a.qweight) + row * units_src + (size_t)g * 4 + (u & 3);
    reinterpret_cast<uint4*>(a.out_qweight)[(size_t)rc * units_out + u] = *src;
    if ((u & 3) == 0) {
      a.out_scales[(size_t)rc * groups_out + go] = a.scales[row * groups_src + g];
      if (a.zeros) a.out_zeros[(size_t)rc * groups_out + go] = a.zeros[row * groups_src + g];
    }
  }
}

// Words of every row from head-major [heads][words per head] to [words per head][heads], or back (INV).  A thread
// moves one word; consecutive threads write consecutive words (the reads stride: the pass runs once per matrix).
template <bool INV>
__global__ __launch_bounds__(256) void w4_interleave_kernel(const uint32_t* __restrict__ qweight, uint32_t* __restrict__ out,
                                                            long long total, int words_per_row, int heads) {
  const int wph = words_per_row / heads;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
    const long long row = i / words_per_row;
    const int wo = (int)(i - row * words_per_row);    // output word
    int src;
    if constexpr (INV) {                              // wo = h * wph + d / 8
      const int h = wo / wph, db = wo - h * wph;
      src = db * heads + h;
    } else {                                          // wo = (d / 8) * heads + h
      const int db = wo / heads, h = wo - db * heads;
      src = h * wph + db;
    }
    out[i] = qweight[row * words_per_row + src];
  }
}

hipError_t launch_w4_interleave(const uint32_t* qweight, uint32_t* out, int N_total, int K_total, int heads, bool inverse,
                                hipStream_t stream) {
  const long long total = (long long)N_total * (K_total >> 3);
  long long blocks = (total + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  if (blocks < 1) blocks = 1;
  if (inverse)
    hipLaunchKernelGGL(w4_interleave_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, stream, qweight, out, total, K_total >> 3, heads);
  else
    hipLaunchKernelGGL(w4_interleave_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, stream, qweight, out, total, K_total >> 3, heads);
  return hipGetLastError();
}

hipError_t launch_w4_repack(const RepackArgs& a, hipStream_t stream) {
  const long long total = (long long)a.km.n_keep * (a.K_out >> 5);
  long long blocks = (total + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(w4_repack_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, a);
  return hipGetLastError();
}

}  // namespace uniql
