// W4A16 GEMM launchers: the fp16 instantiations of mfma_kernel.h and the dispatch to the bfloat16 ones
// (mfma_gemm_bf16.hip).
#include "mfma_kernel.h"

namespace uniql {

hipError_t launch_w4_gemm(const LinearArgs& a, hipStream_t stream) {
  if (a.bf16) return launch_w4_gemm_bf16(a, stream);
  return launch_gemm_fmt<false>(a, stream);
}

// n linears of one decode batch (2..32 tokens, the same format) in one launch when the decode-batch kernel takes them
// all; *done = false: nothing was launched, run them one by one
hipError_t launch_w4_gemm_batch(const LinearArgs* a, int n, hipStream_t stream, bool* done) {
  if (a[0].bf16) return launch_w4_gemm_batch_bf16(a, n, stream, done);
  return smallm_batch<false>(a, n, stream, done);
}

// gate and up of a decode batch with h = SiLU(g) * u (Eq. 1) in one launch; *done = false: nothing was launched
hipError_t launch_w4_gate_up_silu_batch(const LinearArgs* p, hipStream_t stream, bool* done) {
  if (p[0].bf16) return launch_w4_gate_up_silu_batch_bf16(p, stream, done);
  return smallm_glu<false>(p, stream, done);
}

}  // namespace uniql
