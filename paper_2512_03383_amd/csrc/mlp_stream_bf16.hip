// The bfloat16 instantiations of the fused gated MLP (mlp_stream_kernel.h).
#include "mlp_stream_kernel.h"

namespace uniql {

hipError_t launch_w4_mlp_fused_bf16(const LinearArgs* probs, void* scratch, hipStream_t stream, bool* done) {
  return gemv::mlp_fused<true>(probs, scratch, stream, done);
}

}  // namespace uniql
