// GEMV launchers for matrices without zero points (Eq. 3's symmetric scheme: every z = 8, nothing
// loaded): the second half of the instantiations of gemv_kernel.h.
#include "gemv_kernel.h"

namespace uniql {

hipError_t launch_w4_gemv_sym(const LinearArgs& a, hipStream_t stream) { return gemv::gemv_one<false, false>(a, stream); }
hipError_t launch_w4_gemv_batch_sym(const LinearArgs* probs, int n, hipStream_t stream) {
  return gemv::gemv_batch<false, false>(probs, n, stream);
}
hipError_t launch_w4_gate_up_silu_sym(const LinearArgs* probs, hipStream_t stream, bool* fused) {
  return gemv::gate_up_silu<false, false>(probs, stream, fused);
}
hipError_t launch_w4_qkv_rope_sym(const LinearArgs* probs, const RopeFuse& rf, hipStream_t stream, bool* fused) {
  return gemv::qkv_rope<false, false>(probs, rf, stream, fused);
}

}  // namespace uniql
