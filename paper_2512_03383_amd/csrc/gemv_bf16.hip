// GEMV launchers for bfloat16 matrices with zero points: instantiations of gemv_kernel.h in a
// translation unit of their own, so that the variants build in parallel.
#include "gemv_kernel.h"

namespace uniql {

hipError_t launch_w4_gemv_bf16(const LinearArgs& a, hipStream_t stream) { return gemv::gemv_one<true, true>(a, stream); }
hipError_t launch_w4_gemv_batch_bf16(const LinearArgs* probs, int n, hipStream_t stream) {
  return gemv::gemv_batch<true, true>(probs, n, stream);
}
hipError_t launch_w4_gate_up_silu_bf16(const LinearArgs* probs, hipStream_t stream, bool* fused) {
  return gemv::gate_up_silu<true, true>(probs, stream, fused);
}
hipError_t launch_w4_qkv_rope_bf16(const LinearArgs* probs, const RopeFuse& rf, hipStream_t stream, bool* fused) {
  return gemv::qkv_rope<true, true>(probs, rf, stream, fused);
}

}  // namespace uniql
