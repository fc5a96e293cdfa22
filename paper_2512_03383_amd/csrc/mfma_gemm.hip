// W4A16 GEMM launchers: the fp16 instantiations of mfma_kernel.h and the dispatch to the bfloat16 ones
// (mfma_gemm_bf16.hip).
#include "mfma_kernel.h"

namespace uniql {

hipError_t launch_w4_gemm(const LinearArgs& a, hipStream_t stream) {
  if (a.bf16) return launch_w4_gemm_bf16(a, stream);
  return launch_gemm_fmt<false>(a, stream);
}

}  // namespace uniql
