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
#include <type_traits>

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

// V2: two adjacent pairs per item (needs an even number of kept pairs and 4-byte aligned tensors).
// A thread owns up to kBatch items of its block and handles them TOGETHER: all loads of a chunk of
// heads for all of its items are issued before anything is stored (the rotation is in place, so
// the compiler would not move a load above an earlier store), which keeps tens of loads per wave
// in flight instead of a chain of load - rotate - store round trips.  The first chunk's loads are
// issued before the block builds its frequency table, whose latency they hide.
// (The launcher uses kBatch = 1: on a 4096-token prompt one item per thread and nine tokens per block measured
// 18.8 us against 22.2 us for four items per thread; more, smaller blocks hide the latencies better than
// longer threads do.)
constexpr int kHeadChunk = 4;

// BF16: q and k are bfloat16 (half_t / half2_t then only carry the bits).
template <bool V2, int kBatch, bool BF16>
__global__ __launch_bounds__(kRopeThreads) void pruned_rope_kernel(RopeArgs a, int tokens_per_block) {
  extern __shared__ __align__(8) unsigned char rope_smem[];
  double* invf = reinterpret_cast<double*>(rope_smem);   // [D_keep / 2]
  typedef typename std::conditional<V2, half2_t, half_t>::type elem_t;   // one or two adjacent channels
  constexpr int W = V2 ? 2 : 1;

  const int hk = a.D_keep >> 1;
  const int g = blockIdx.y;
  const int t0 = blockIdx.x * tokens_per_block;
  const int qper = a.Hq / a.H_tab, kper = a.Hkv / a.H_tab;
  const int nheads = qper + kper;                 // heads that share this table row: Q heads, then K heads
  const int per_tok = hk / W;
  const int tb = min(tokens_per_block, a.T - t0);
  const int n_items = tb * per_tok;               // one batch (kBatch * kRopeThreads) unless a single token has more

  // this thread's items of a batch: token and first channel of each, and whether it exists
  int tok[kBatch], ch[kBatch];
  bool live[kBatch];
  auto take_items = [&](int base) {
#pragma unroll
    for (int b = 0; b < kBatch; ++b) {
      const int item = base + threadIdx.x + b * kRopeThreads;
      live[b] = item < n_items;
      const int tl = live[b] ? item / per_tok : 0;
      tok[b] = t0 + tl;
      ch[b] = live[b] ? (item - tl * per_tok) * W : 0;
    }
  };
  take_items(0);
  // head hh of the group (0 .. nheads-1): address of channel ch[b] of token tok[b]
  auto elem_ptr = [&](int b, int hh) -> half_t* {
    return hh < qper ? a.q + ((size_t)tok[b] * a.Hq + g * qper + hh) * a.D_keep + ch[b]
                     : a.k + ((size_t)tok[b] * a.Hkv + g * kper + (hh - qper)) * a.D_keep + ch[b];
  };
  elem_t x1[kBatch][kHeadChunk] = {}, x2[kBatch][kHeadChunk] = {};
  auto load_chunk = [&](int h0) {
#pragma unroll
    for (int u = 0; u < kHeadChunk; ++u) {
      if (h0 + u < nheads) {   // uniform
#pragma unroll
        for (int b = 0; b < kBatch; ++b) {
          if (live[b]) {
            const half_t* v = elem_ptr(b, h0 + u);
            x1[b][u] = *reinterpret_cast<const elem_t*>(v);
            x2[b][u] = *reinterpret_cast<const elem_t*>(v + hk);
          }
        }
      }
    }
  };
  double pos[kBatch];
  auto load_pos = [&]() {
#pragma unroll
    for (int b = 0; b < kBatch; ++b) pos[b] = (double)a.positions[tok[b]];
  };
  load_pos();
  load_chunk(0);

  // theta^(-2j/D) of the block's kept pairs, once, in fp64
  const double l2t = log2(a.theta);
  for (int i = threadIdx.x; i < hk; i += kRopeThreads) {
    const int j = a.kept_idx[(size_t)g * hk + i];
    invf[i] = exp2(-(2.0 * (double)j / (double)a.D_full) * l2t);
  }
  __syncthreads();

  for (int base = 0;;) {
    float sn[kBatch][W], cs[kBatch][W];
#pragma unroll
    for (int b = 0; b < kBatch; ++b)
#pragma unroll
      for (int w = 0; w < W; ++w) angle_sincos(pos[b], invf[ch[b] + w], &sn[b][w], &cs[b][w]);

    for (int h0 = 0; h0 < nheads; h0 += kHeadChunk) {
      // rotate into registers, fetch the next chunk, then store: the next chunk's loads are in
      // flight while this one is written back
      elem_t y1[kBatch][kHeadChunk], y2[kBatch][kHeadChunk];
#pragma unroll
      for (int u = 0; u < kHeadChunk; ++u)
#pragma unroll
        for (int b = 0; b < kBatch; ++b) {
          if constexpr (V2) {
            const float a0 = in16<BF16>(x1[b][u].x), a1 = in16<BF16>(x1[b][u].y), b0 = in16<BF16>(x2[b][u].x), b1 = in16<BF16>(x2[b][u].y);
            y1[b][u] = half2_t{out16<BF16>(a0 * cs[b][0] - b0 * sn[b][0]), out16<BF16>(a1 * cs[b][1] - b1 * sn[b][1])};
            y2[b][u] = half2_t{out16<BF16>(b0 * cs[b][0] + a0 * sn[b][0]), out16<BF16>(b1 * cs[b][1] + a1 * sn[b][1])};
          } else {
            const float a0 = in16<BF16>(x1[b][u]), b0 = in16<BF16>(x2[b][u]);
            y1[b][u] = out16<BF16>(a0 * cs[b][0] - b0 * sn[b][0]);
            y2[b][u] = out16<BF16>(b0 * cs[b][0] + a0 * sn[b][0]);
          }
        }
      if (h0 + kHeadChunk < nheads) load_chunk(h0 + kHeadChunk);
#pragma unroll
      for (int u = 0; u < kHeadChunk; ++u) {
        if (h0 + u < nheads) {
#pragma unroll
          for (int b = 0; b < kBatch; ++b) {
            if (live[b]) {
              half_t* v = elem_ptr(b, h0 + u);
              *reinterpret_cast<elem_t*>(v) = y1[b][u];
              *reinterpret_cast<elem_t*>(v + hk) = y2[b][u];
            }
          }
        }
      }
    }
    base += kBatch * kRopeThreads;
    if (base >= n_items) break;
    take_items(base);
    load_pos();
    load_chunk(0);
  }
}

template <bool BF16>
static hipError_t launch_rope_fmt(const RopeArgs& a, bool v2, dim3 grid, size_t smem, int tpb, hipStream_t stream) {
  if (v2) hipLaunchKernelGGL((pruned_rope_kernel<true, 1, BF16>), grid, dim3(kRopeThreads), smem, stream, a, tpb);
  else hipLaunchKernelGGL((pruned_rope_kernel<false, 1, BF16>), grid, dim3(kRopeThreads), smem, stream, a, tpb);
  return hipGetLastError();
}

hipError_t launch_pruned_rope(const RopeArgs& a, hipStream_t stream) {
  const int hk = a.D_keep >> 1;
  // half2 accesses need an even pair count (then every head row and both halves start on a
  // 4-byte boundary, since D_keep is a multiple of 4) and 4-byte aligned tensors
  const bool v2 = (hk % 2 == 0) && (reinterpret_cast<uintptr_t>(a.q) % 4 == 0) &&
                  (a.k == nullptr || reinterpret_cast<uintptr_t>(a.k) % 4 == 0);
  // tokens per block: one item per thread
  const int per_tok = v2 ? hk >> 1 : hk;
  int tpb = kRopeThreads / per_tok;   // a thread owns one item
  if (tpb > a.T) tpb = a.T;
  if (tpb < 1) tpb = 1;
  dim3 grid((a.T + tpb - 1) / tpb, a.H_tab);
  const size_t smem = (size_t)hk * sizeof(double);
  return a.bf16 ? launch_rope_fmt<true>(a, v2, grid, smem, tpb, stream) : launch_rope_fmt<false>(a, v2, grid, smem, tpb, stream);
}

}  // namespace uniql
