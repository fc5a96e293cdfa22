// Bit-exact dequantisation of the kept sub-matrix: w = RN_fp16((q - z) * s).
// The product of the small integer (q - z) and the 11-bit significand of s is
// exact in fp32, so the single fp32 -> fp16 conversion is the only rounding.
// (Written with scalar fp32 arithmetic on purpose: it is the independent check
// of the packed-fp16 dequantisation used inside the GEMV / GEMM kernels.)
#include "common.h"

namespace uniql {

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
    const uint32_t word = a.qweight[row * words_per_row + w];
    const size_t g = row * groups_per_row + (w >> 4);
    const float s = (float)__builtin_bit_cast(half_t, a.scales[g]);
    const int z = a.zeros[g];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int kc = compact_col(km, w * 8 + j);
      if (kc >= 0) {
        const int q = (int)((word >> (4 * j)) & 15u);
        a.y[(size_t)rc * km.k_keep + kc] = (half_t)((float)(q - z) * s);
      }
    }
  }
}

hipError_t launch_w4_dequant(const LinearArgs& a, hipStream_t stream) {
  const long long total = (long long)a.km.n_keep * ((a.km.k_span + 7) >> 3);
  long long blocks = (total + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(w4_dequant_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, a);
  return hipGetLastError();
}

}  // namespace uniql
