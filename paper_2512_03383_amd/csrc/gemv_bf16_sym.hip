// GEMV launchers for bfloat16 matrices without zero points (every z = 8): instantiations of gemv_kernel.h in a
// translation unit of their own, so that the variants build in parallel.
#include "gemv_kernel.h"

namespace uniql {

hipError_t launch_w4_gemv_bf16_sym(const LinearArgs& a, hipStream_t stream) { return gemv::gemv_one<false, true>(a, stream); }
hipError_t launch_w4_gemv_batch_bf16_sym(const LinearArgs* probs, int n, hipStream_t stream) {
  return gemv::gemv_batch<false, true>(probs, n, stream);
}
hipError_t launch_w4_gate_up_silu_bf16_sym(const LinearArgs* probs, hipStream_t stream, bool* fused) {
  return gemv::gate_up_silu<false, true>(probs, stream, fused);
}
hipError_t launch_w4_qkv_rope_bf16_sym(const LinearArgs* probs, const RopeFuse& rf, hipStream_t stream, bool* fused) {
  return gemv::qkv_rope<false, true>(probs, rf, stream, fused);
}

}  // namespace uniql
