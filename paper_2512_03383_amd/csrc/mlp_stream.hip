// Launchers of the fused gated MLP (mlp_stream_kernel.h): the fp16 instantiations, and the dispatch to the bfloat16
// ones (mlp_stream_bf16.hip).
#include "mlp_stream_kernel.h"

namespace uniql {

hipError_t launch_w4_mlp_fused(const LinearArgs* probs, void* scratch, hipStream_t stream, bool* done) {
  if (probs[0].bf16) return launch_w4_mlp_fused_bf16(probs, scratch, stream, done);
  return gemv::mlp_fused<false>(probs, scratch, stream, done);
}

}  // namespace uniql
