// Fused pruned RoPE: gather the frequency of each kept pair by its original
// index and rotate Q and K in place, one launch.
//
// A block owns one row of the kept-index table (one KV-head group) and a chunk
// of tokens.  Thread i owns kept pair i: it reads its original index once,
// forms theta^(-2j/D) once in fp64, and per token computes the angle in fp64,
// reduces it to [-pi, pi] with a two-term 2*pi, and takes one fp32 sin/cos that
// is reused by every Q head of the group and by the K head.
#include "common.h"

namespace uniql {

constexpr int kRopeTokens = 8;   // tokens per block

__device__ __forceinline__ void rotate_pair(half_t* v, int half_keep, float c, float s) {
  const float a = (float)v[0], b = (float)v[half_keep];
  v[0] = (half_t)(a * c - b * s);
  v[half_keep] = (half_t)(b * c + a * s);
}

__global__ __launch_bounds__(256) void pruned_rope_kernel(RopeArgs a) {
  const int hk = a.D_keep >> 1;
  const int g = blockIdx.y;
  const int t0 = blockIdx.x * kRopeTokens;
  const int qper = a.Hq / a.H_tab, kper = a.Hkv / a.H_tab;
  for (int i = threadIdx.x; i < hk; i += blockDim.x) {
    const int j = a.kept_idx[(size_t)g * hk + i];
    const double inv_freq = exp2(-(2.0 * (double)j / (double)a.D_full) * log2(a.theta));
    for (int t = t0; t < t0 + kRopeTokens && t < a.T; ++t) {
      const double phi = (double)a.positions[t] * inv_freq;
      // phi - 2*pi*n with 2*pi split in two doubles (Cody-Waite)
      const double n = rint(phi * 0.15915494309189534561);
      double r = fma(-n, 6.28318530717958623200, phi);
      r = fma(-n, 2.44929359829470635445e-16, r);
      float sn, cs;
      sincosf((float)r, &sn, &cs);
      for (int h = 0; h < qper; ++h)
        rotate_pair(a.q + ((size_t)t * a.Hq + g * qper + h) * a.D_keep + i, hk, cs, sn);
      for (int h = 0; h < kper; ++h)
        rotate_pair(a.k + ((size_t)t * a.Hkv + g * kper + h) * a.D_keep + i, hk, cs, sn);
    }
  }
}

hipError_t launch_pruned_rope(const RopeArgs& a, hipStream_t stream) {
  const int hk = a.D_keep >> 1;
  int threads = ((hk + 63) / 64) * 64;
  if (threads > 256) threads = 256;
  dim3 grid((a.T + kRopeTokens - 1) / kRopeTokens, a.H_tab);
  hipLaunchKernelGGL(pruned_rope_kernel, grid, dim3(threads), 0, stream, a);
  return hipGetLastError();
}

}  // namespace uniql
