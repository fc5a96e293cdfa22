// The bfloat16 instantiations of mfma_kernel.h.  (No hand-scheduled prefill kernel in this format: large
// token counts run the generic kernel with 128 x 256 tiles.)
#include "mfma_kernel.h"

namespace uniql {

hipError_t launch_w4_gemm_bf16(const LinearArgs& a, hipStream_t stream) { return launch_gemm_fmt<true>(a, stream, nullptr); }

}  // namespace uniql
