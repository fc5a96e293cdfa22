// The bfloat16 instantiations of mfma_kernel.h.
#include "mfma_kernel.h"

namespace uniql {

hipError_t launch_w4_gemm_bf16(const LinearArgs& a, hipStream_t stream) { return launch_gemm_fmt<true>(a, stream); }
hipError_t launch_w4_gemm_batch_bf16(const LinearArgs* a, int n, hipStream_t stream, bool* done) {
  return smallm_batch<true>(a, n, stream, done);
}

hipError_t launch_w4_gate_up_silu_batch_bf16(const LinearArgs* p, hipStream_t stream, bool* done) {
  return smallm_glu<true>(p, stream, done);
}

}  // namespace uniql
