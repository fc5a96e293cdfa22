// GEMV launchers for fp16 matrices WITH zero points, and the dispatch on the format and on whether a matrix has them.
// (The kernel template lives in gemv_kernel.h; its instantiations for matrices without zero points
// are compiled in gemv_sym.hip, so that the two halves build in parallel.)
#include "gemv_kernel.h"

namespace uniql {

static bool any_bf16(const LinearArgs* p, int n) {
  for (int i = 0; i < n; ++i)
    if (p[i].bf16) return true;
  return false;
}
static bool all_bf16(const LinearArgs* p, int n) {
  for (int i = 0; i < n; ++i)
    if (!p[i].bf16) return false;
  return true;
}
static bool all_have_zeros(const LinearArgs* p, int n) {
  for (int i = 0; i < n; ++i)
    if (!p[i].zeros) return false;
  return true;
}
static bool none_has_zeros(const LinearArgs* p, int n) {
  for (int i = 0; i < n; ++i)
    if (p[i].zeros) return false;
  return true;
}

hipError_t launch_w4_gemv(const LinearArgs& a, hipStream_t stream) {
  bool done = false;
  hipError_t e = launch_w4_gemv_stream(a, stream, &done);
  if (done || e != hipSuccess) return e;
  if (a.bf16) return a.zeros ? launch_w4_gemv_bf16(a, stream) : launch_w4_gemv_bf16_sym(a, stream);
  return a.zeros ? gemv::gemv_one<true, false>(a, stream) : launch_w4_gemv_sym(a, stream);
}

hipError_t launch_w4_gemv_batch(const LinearArgs* probs, int n, hipStream_t stream) {
  if (n == 1) return launch_w4_gemv(probs[0], stream);
  if (all_bf16(probs, n)) {
    if (all_have_zeros(probs, n)) return launch_w4_gemv_batch_bf16(probs, n, stream);
    if (none_has_zeros(probs, n)) return launch_w4_gemv_batch_bf16_sym(probs, n, stream);
  } else if (!any_bf16(probs, n)) {
    if (all_have_zeros(probs, n)) return gemv::gemv_batch<true, false>(probs, n, stream);
    if (none_has_zeros(probs, n)) return launch_w4_gemv_batch_sym(probs, n, stream);
  }
  for (int i = 0; i < n; ++i) {   // mixed: no common kernel instantiation
    hipError_t e = launch_w4_gemv(probs[i], stream);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_w4_gate_up_silu(const LinearArgs* probs, hipStream_t stream, bool* fused) {
  hipError_t e = launch_w4_gate_up_stream(probs, stream, fused);
  if (*fused || e != hipSuccess) return e;
  if (all_bf16(probs, 2)) {
    if (all_have_zeros(probs, 2)) return launch_w4_gate_up_silu_bf16(probs, stream, fused);
    if (none_has_zeros(probs, 2)) return launch_w4_gate_up_silu_bf16_sym(probs, stream, fused);
  } else if (!any_bf16(probs, 2)) {
    if (all_have_zeros(probs, 2)) return gemv::gate_up_silu<true, false>(probs, stream, fused);
    if (none_has_zeros(probs, 2)) return launch_w4_gate_up_silu_sym(probs, stream, fused);
  }
  *fused = false;
  return hipSuccess;
}

hipError_t launch_w4_qkv_rope(const LinearArgs* probs, const RopeFuse& rf, hipStream_t stream, bool* fused) {
  if (all_bf16(probs, 3)) {
    if (all_have_zeros(probs, 3)) return launch_w4_qkv_rope_bf16(probs, rf, stream, fused);
    if (none_has_zeros(probs, 3)) return launch_w4_qkv_rope_bf16_sym(probs, rf, stream, fused);
  } else if (!any_bf16(probs, 3)) {
    if (all_have_zeros(probs, 3)) return gemv::qkv_rope<true, false>(probs, rf, stream, fused);
    if (none_has_zeros(probs, 3)) return launch_w4_qkv_rope_sym(probs, rf, stream, fused);
  }
  *fused = false;
  return hipSuccess;
}

}  // namespace uniql
