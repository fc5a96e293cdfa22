// Fused pruned RoPE: gather the frequency of each kept pair by its original
// index and rotate Q and K in place, one launch.
//
// A block owns one row of the kept-index table (one KV-head group) and a chunk
// of tokens.  The block first forms theta^(-2j/D) for its kept pairs once, in
// fp64, into LDS.  A work item is (token, pair) -- or (token, two adjacent
// pairs) when D_keep/2 is even, so that every access is a 32-bit half2: per item
// the angle is formed and reduced in fp64 (in revolutions), and one fp32 sin/cos is
// reused by every Q head of the group and by the K head.
#include "common.h"

namespace uniql {

constexpr int kRopeThreads = 256;

// sin / cos of pos * inv_freq.  The angle is formed in fp64 and reduced there, in revolutions:
// rev = phi / (2 pi) - rint(phi / (2 pi)) lies in [-0.5, 0.5] with an error below 1e-11, and the
// hardware sin / cos take their argument in revolutions (absolute error of order 1e-6, far below
// the fp16 rounding of the result).
__device__ __forceinline__ void angle_sincos(double pos, double inv_freq, float* sn, float* cs) {
  const double rev = pos * inv_freq * 0.15915494309189534561;
  const float r = (float)(rev - rint(rev));
  *sn = __builtin_amdgcn_sinf(r);
  *cs = __builtin_amdgcn_cosf(r);
}

// V2: two adjacent pairs per item (needs an even number of kept pairs and 4-byte aligned tensors)
template <bool V2>
__global__ __launch_bounds__(kRopeThreads) void pruned_rope_kernel(RopeArgs a, int tokens_per_block) {
  extern __shared__ __align__(8) unsigned char rope_smem[];
  double* invf = reinterpret_cast<double*>(rope_smem);   // [D_keep / 2]

  const int hk = a.D_keep >> 1;
  const int g = blockIdx.y;
  const int t0 = blockIdx.x * tokens_per_block;
  const int qper = a.Hq / a.H_tab, kper = a.Hkv / a.H_tab;
  const double l2t = log2(a.theta);
  for (int i = threadIdx.x; i < hk; i += kRopeThreads) {
    const int j = a.kept_idx[(size_t)g * hk + i];
    invf[i] = exp2(-(2.0 * (double)j / (double)a.D_full) * l2t);
  }
  __syncthreads();

  const int per_tok = V2 ? hk >> 1 : hk;
  const int tb = min(tokens_per_block, a.T - t0);
  for (int item = threadIdx.x; item < tb * per_tok; item += kRopeThreads) {
    const int tl = item / per_tok, ii = item - tl * per_tok;
    const int t = t0 + tl;
    const double pos = (double)a.positions[t];
    if constexpr (V2) {
      const int i0 = 2 * ii;
      float s0, c0, s1, c1;
      angle_sincos(pos, invf[i0], &s0, &c0);
      angle_sincos(pos, invf[i0 + 1], &s1, &c1);
      // The rotation is in place, so the compiler cannot move a later head's loads above an
      // earlier head's stores: heads are processed four at a time, all loads first.
      auto rot2_heads = [&](half_t* base, int H, int h_first, int count) {
        for (int hb = 0; hb < count; hb += 4) {
          half2_t x1[4], x2[4];
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int h = h_first + (hb + u < count ? hb + u : count - 1);
            const half_t* v = base + ((size_t)t * H + h) * a.D_keep;
            x1[u] = *reinterpret_cast<const half2_t*>(v + i0);
            x2[u] = *reinterpret_cast<const half2_t*>(v + i0 + hk);
          }
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            if (hb + u < count) {
              half_t* v = base + ((size_t)t * H + h_first + hb + u) * a.D_keep;
              const float a0 = (float)x1[u].x, a1 = (float)x1[u].y, b0 = (float)x2[u].x, b1 = (float)x2[u].y;
              *reinterpret_cast<half2_t*>(v + i0) = half2_t{(half_t)(a0 * c0 - b0 * s0), (half_t)(a1 * c1 - b1 * s1)};
              *reinterpret_cast<half2_t*>(v + i0 + hk) = half2_t{(half_t)(b0 * c0 + a0 * s0), (half_t)(b1 * c1 + a1 * s1)};
            }
          }
        }
      };
      rot2_heads(a.q, a.Hq, g * qper, qper);
      if (kper) rot2_heads(a.k, a.Hkv, g * kper, kper);
    } else {
      float sn, cs;
      angle_sincos(pos, invf[ii], &sn, &cs);
      auto rot1_heads = [&](half_t* base, int H, int h_first, int count) {
        for (int hb = 0; hb < count; hb += 4) {
          float x1[4], x2[4];
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int h = h_first + (hb + u < count ? hb + u : count - 1);
            const half_t* v = base + ((size_t)t * H + h) * a.D_keep;
            x1[u] = (float)v[ii];
            x2[u] = (float)v[ii + hk];
          }
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            if (hb + u < count) {
              half_t* v = base + ((size_t)t * H + h_first + hb + u) * a.D_keep;
              v[ii] = (half_t)(x1[u] * cs - x2[u] * sn);
              v[ii + hk] = (half_t)(x2[u] * cs + x1[u] * sn);
            }
          }
        }
      };
      rot1_heads(a.q, a.Hq, g * qper, qper);
      if (kper) rot1_heads(a.k, a.Hkv, g * kper, kper);
    }
  }
}

hipError_t launch_pruned_rope(const RopeArgs& a, hipStream_t stream) {
  const int hk = a.D_keep >> 1;
  // half2 accesses need an even pair count (then every head row and both halves start on a
  // 4-byte boundary, since D_keep is a multiple of 4) and 4-byte aligned tensors
  const bool v2 = (hk % 2 == 0) && (reinterpret_cast<uintptr_t>(a.q) % 4 == 0) &&
                  (a.k == nullptr || reinterpret_cast<uintptr_t>(a.k) % 4 == 0);
  // tokens per block: enough items to fill the block, enough blocks to fill the chip
  const int per_tok = v2 ? hk >> 1 : hk;
  int tpb = (4 * kRopeThreads + per_tok - 1) / per_tok;
  if (tpb > a.T) tpb = a.T;
  if (tpb < 1) tpb = 1;
  dim3 grid((a.T + tpb - 1) / tpb, a.H_tab);
  const size_t smem = (size_t)hk * sizeof(double);
  if (v2) hipLaunchKernelGGL(pruned_rope_kernel<true>, grid, dim3(kRopeThreads), smem, stream, a, tpb);
  else hipLaunchKernelGGL(pruned_rope_kernel<false>, grid, dim3(kRopeThreads), smem, stream, a, tpb);
  return hipGetLastError();
}

}  // namespace uniql
