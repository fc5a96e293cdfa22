// Launchers of the persistent streaming GEMV (gemv_stream_kernel.h): the fp16 instantiations, and the
// dispatch to the bfloat16 ones (gemv_stream_bf16.hip).
#include "gemv_stream_kernel.h"

namespace uniql {

hipError_t launch_w4_gemv_stream(const LinearArgs& a, hipStream_t stream, bool* done) {
  return a.bf16 ? launch_w4_gemv_stream_bf16(a, stream, done) : gemv::stream_one<false>(a, stream, done);
}

hipError_t launch_w4_gate_up_stream(const LinearArgs* probs, hipStream_t stream, bool* done) {
  if (probs[0].bf16 != probs[1].bf16) {
    *done = false;
    return hipSuccess;
  }
  return probs[0].bf16 ? launch_w4_gate_up_stream_bf16(probs, stream, done) : gemv::stream_gate_up<false>(probs, stream, done);
}

// the loads of the gate + up launch without its arithmetic (fp16 matrices with zero points): the read-stream ceiling
hipError_t launch_w4_gate_up_stream_probe(const LinearArgs* probs, hipStream_t stream, bool* done) {
  if (probs[0].bf16 || probs[1].bf16) {
    *done = false;
    return hipSuccess;
  }
  return gemv::stream_gate_up<false, true>(probs, stream, done);
}

// q, k, v of one token with the rotation of q and k on the walk; *done = false (nothing launched) for other shapes
hipError_t launch_w4_qkv_rope_stream(const LinearArgs* probs, const RopeFuse& rf, hipStream_t stream, bool* done) {
  return probs[0].bf16 ? launch_w4_qkv_rope_stream_bf16(probs, rf, stream, done) : gemv::stream_qkv_rope<false>(probs, rf, stream, done);
}

}  // namespace uniql
