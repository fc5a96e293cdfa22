// The bfloat16 instantiations of the persistent streaming GEMV (gemv_stream_kernel.h).
#include "gemv_stream_kernel.h"

namespace uniql {

hipError_t launch_w4_gemv_stream_bf16(const LinearArgs& a, hipStream_t stream, bool* done) {
  return gemv::stream_one<true>(a, stream, done);
}

hipError_t launch_w4_gate_up_stream_bf16(const LinearArgs* probs, hipStream_t stream, bool* done) {
  return gemv::stream_gate_up<true>(probs, stream, done);
}

hipError_t launch_w4_qkv_rope_stream_bf16(const LinearArgs* probs, const RopeFuse& rf, hipStream_t stream, bool* done) {
  return gemv::stream_qkv_rope<true>(probs, rf, stream, done);
}

}  // namespace uniql
