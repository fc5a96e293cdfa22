// Fused pruned RoPE: gather the frequency of each kept pair by its original
// index and rotate Q and K in place, one launch.
//
// Two kernels: the per-pair kernel described here serves single tokens and short
// calls (and shapes the other one does not take); prompt-sized calls go to the
// whole-row kernel further down.
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
constexpr int kRopeRowsMinTokens = 32;     // from here on a wave owns whole head rows
constexpr int kRopeRowsBlocks = 1024;      // blocks of such a launch: four per compute unit

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


// Prompt-sized calls: a wave owns whole head rows.  A head row is D_keep/4 units of 8 bytes (two 32-bit
// words of two adjacent channels each); a lane holds one unit of a row, D_keep/4 lanes hold the row
// and a wave as many rows as fit (two of 108 channels), so one store instruction writes whole rows
// as one contiguous run and the rows of a group's Q heads follow each other in memory -- the
// per-pair kernel above writes runs of half a row, and every run end that falls inside a cache
// line costs a fill of that line.  A word of the first half of a row holds x1 of two pairs and
// takes the partner word x2 from the lane half a row further on (a lane permute); a word of the
// second half the other way round; both compute the same sin / cos, each keeps its own output:
//   first half:  x1 cos - x2 sin        second half:  x2 cos + x1 sin
// With an odd number of words per half row the middle unit has one word of either half and the
// partner of a lane's word 0 is the other lane's word 1; that is uniform over the wave.
//
// A block builds its frequency table once and its waves then walk over token pairs (wave-strided
// over the grid); Q and K are addressed through buffer resources with a per-token lane offset and
// a scalar offset per head step; a lane without a row and a token past the end carry an offset
// beyond the tensor, which the hardware turns into a load of zero and a dropped store, so the
// walk has no divergent branch.  The loads of the next token pair are issued before the stores of
// the current one.  Measured on [4096 tokens, 32 + 8 heads, 108 of 128 channels] (70.8 MB read and
// written in place, eight rotating copies so that no cache holds them): 16.9 us against 18.8 us for
// the per-pair kernel; the memory counters read 1.01 x the algorithmic bytes in either direction
// (1.45 x before), and an in-place elementwise pass of the framework's own vectorised kernel over
// tensors that large streams at 4.4 TB/s where this kernel reaches 4.2 TB/s.  Tokens per wave
// (1, 2, 4) and the number of blocks (512 .. 4096) moved the time by less than 3 %, and so did
// taking the sin / cos out: what is left is the memory system's rate for a read-modify-write pass.
constexpr uint32_t kRopeRsrcWord3 = 0x00020000u;   // raw buffer, 32-bit data format
constexpr int kNoRow = (int)0x80000000u;  // as an unsigned offset: beyond any tensor the kernel accepts, also after a head step is added
typedef uint32_t rope_u32x2_t __attribute__((ext_vector_type(2)));

// kSteps: Q head steps whose loads are in flight together (then one K step)
template <bool BF16, int kSteps>
__global__ __launch_bounds__(kRopeThreads) void pruned_rope_rows_kernel(RopeArgs a) {
  constexpr int kTok = 2;
  extern __shared__ __align__(8) unsigned char rope_smem[];
  double* invf = reinterpret_cast<double*>(rope_smem);   // [D_keep / 2]
  const int hk = a.D_keep >> 1;        // pairs of a head = 32-bit words of a head row
  const int hw = hk >> 1;              // words of half a row = 8-byte units of a row
  const int g = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int hps = 64 / hw;             // head rows a wave covers per step
  const int hsub = lane / hw, unit = lane - hsub * hw;
  const bool active = hsub < hps;
  const bool hw_odd = hw & 1;
  // word e of the unit: which half of the row, which word of that half (pairs 2 pw and 2 pw + 1), the partner's lane
  bool second[2];
  int pw[2], partner_lane4[2];
#pragma unroll
  for (int e = 0; e < 2; ++e) {
    const int d = 2 * unit + e;
    second[e] = d >= hw;
    pw[e] = second[e] ? d - hw : d;
    partner_lane4[e] = 4 * (hsub * hw + ((second[e] ? d - hw : d + hw) >> 1));
  }
  const int qper = a.Hq / a.H_tab, kper = a.Hkv / a.H_tab;
  const int row_bytes = a.D_keep * 2;
  const int step_bytes = hps * row_bytes;

  const __amdgpu_buffer_rsrc_t rq = __builtin_amdgcn_make_buffer_rsrc(a.q, 0, a.T * a.Hq * row_bytes, kRopeRsrcWord3);
  const __amdgpu_buffer_rsrc_t rk = __builtin_amdgcn_make_buffer_rsrc(a.k, 0, a.k ? a.T * a.Hkv * row_bytes : 0, kRopeRsrcWord3);
  // this lane's unit in the group's first head step of token 0
  const int q_lane = (g * qper + hsub) * row_bytes + 8 * unit, k_lane = (g * kper + hsub) * row_bytes + 8 * unit;
  const int q_tok = a.Hq * row_bytes, k_tok = a.Hkv * row_bytes;
  const int q_steps = (qper + hps - 1) / hps, k_steps = (kper + hps - 1) / hps;

  struct Set {   // what a wave holds of one token pair
    rope_u32x2_t own[kTok][kSteps + 1];   // slot kSteps: the first K step
    int q_own[kTok], k_own[kTok];         // lane offsets of head step 0, or kNoRow
    int pos[kTok];                        // converted when used: nothing waits for it at once
  };
  // offset of head step `step` for this lane: heads past the group's (only in a shared last step) have no row
  auto at_step = [&](int base, int step, int per) -> int { return step * hps + hsub < per ? base : kNoRow; };
  auto load_step = [&](Set& s, __amdgpu_buffer_rsrc_t r, const int (&o_own)[kTok], int u, int step, int per) {
#pragma unroll
    for (int b = 0; b < kTok; ++b)
      s.own[b][u] = __builtin_amdgcn_raw_buffer_load_b64(r, at_step(o_own[b], step, per), step * step_bytes, 0);
  };
  auto take = [&](Set& s, int tp) {   // token pair tp: offsets, positions, the first Q chunk and the first K step
#pragma unroll
    for (int b = 0; b < kTok; ++b) {
      const int t = tp * kTok + b;
      const bool there = active && t < a.T;
      s.q_own[b] = there ? t * q_tok + q_lane : kNoRow;
      s.k_own[b] = there ? t * k_tok + k_lane : kNoRow;
      s.pos[b] = a.positions[min(t, a.T - 1)];
    }
#pragma unroll
    for (int u = 0; u < kSteps; ++u) load_step(s, rq, s.q_own, u, u, qper);
    load_step(s, rk, s.k_own, kSteps, 0, kper);
  };
  float sn[kTok][2][2], cs[kTok][2][2];   // [token][word of the unit][pair of the word]
  auto rotate_store_step = [&](Set& s, __amdgpu_buffer_rsrc_t r, const int (&o_own)[kTok], int u, int step, int per) {
#pragma unroll
    for (int b = 0; b < kTok; ++b) {
      const uint32_t w0 = s.own[b][u].x, w1 = s.own[b][u].y;
      rope_u32x2_t y;
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        // the partner word sits half a row further on: the other word of that lane's unit if half a row is an odd number of words
        const uint32_t src = (e == 0) == hw_odd ? w1 : w0;
        const uint32_t oth = (uint32_t)__builtin_amdgcn_ds_bpermute(partner_lane4[e], (int)src);
        const half2_t o = __builtin_bit_cast(half2_t, e == 0 ? w0 : w1), x = __builtin_bit_cast(half2_t, oth);
        const half_t ox = o.x, oy = o.y, xx = x.x, xy = x.y;
        const half2_t v{out16<BF16>(in16<BF16>(ox) * cs[b][e][0] + in16<BF16>(xx) * sn[b][e][0]),
                        out16<BF16>(in16<BF16>(oy) * cs[b][e][1] + in16<BF16>(xy) * sn[b][e][1])};
        if (e == 0) y.x = __builtin_bit_cast(uint32_t, v); else y.y = __builtin_bit_cast(uint32_t, v);
      }
      __builtin_amdgcn_raw_buffer_store_b64(y, r, at_step(o_own[b], step, per), step * step_bytes, 0);
    }
  };
  double f[2][2];
  // finish a token pair: sin / cos, the chunk that travelled with take(), then whatever heads are left
  auto finish = [&](Set& s) {
#pragma unroll
    for (int b = 0; b < kTok; ++b)
#pragma unroll
      for (int e = 0; e < 2; ++e)
#pragma unroll
        for (int w = 0; w < 2; ++w) {
          angle_sincos((double)s.pos[b], f[e][w], &sn[b][e][w], &cs[b][e][w]);
          if (!second[e]) sn[b][e][w] = -sn[b][e][w];
        }
#pragma unroll
    for (int u = 0; u < kSteps; ++u) rotate_store_step(s, rq, s.q_own, u, u, qper);
    rotate_store_step(s, rk, s.k_own, kSteps, 0, kper);
    for (int s0 = kSteps; s0 < q_steps; s0 += kSteps) {
#pragma unroll
      for (int u = 0; u < kSteps; ++u) load_step(s, rq, s.q_own, u, s0 + u, qper);
#pragma unroll
      for (int u = 0; u < kSteps; ++u) rotate_store_step(s, rq, s.q_own, u, s0 + u, qper);
    }
    for (int s0 = 1; s0 < k_steps; s0 += kSteps) {
#pragma unroll
      for (int u = 0; u < kSteps; ++u) load_step(s, rk, s.k_own, u, s0 + u, kper);
#pragma unroll
      for (int u = 0; u < kSteps; ++u) rotate_store_step(s, rk, s.k_own, u, s0 + u, kper);
    }
  };

  const int n_pairs = (a.T + kTok - 1) / kTok;
  const int stride = gridDim.x * (kRopeThreads / 64);
  int tp = blockIdx.x * (kRopeThreads / 64) + wave;
  // the table's index is the first load to return; the first token pair is requested before the table is built
  // (at most 128 pairs: one per thread)
  const int j = (int)threadIdx.x < hk ? a.kept_idx[(size_t)g * hk + threadIdx.x] : 0;
  Set cur, nxt;
  take(cur, tp);
  if ((int)threadIdx.x < hk) invf[threadIdx.x] = exp2(-(2.0 * (double)j / (double)a.D_full) * log2(a.theta));
  __syncthreads();
#pragma unroll
  for (int e = 0; e < 2; ++e) {
    // a lane without a row (its unit index can lie past the row) reads entry 0
    const int i = active ? 2 * pw[e] : 0;
    f[e][0] = invf[i];
    f[e][1] = invf[i + 1];
  }
  // a wave past the end still carries offsets without rows: its loads and stores touch nothing
  while (tp < n_pairs) {
    take(nxt, tp + stride);
    finish(cur);
    tp += stride;
    if (tp >= n_pairs) break;
    take(cur, tp + stride);
    finish(nxt);
    tp += stride;
  }
}

template <bool BF16>
static hipError_t launch_rope_fmt(const RopeArgs& a, bool v2, dim3 grid, size_t smem, int tpb, hipStream_t stream) {
  if (v2) hipLaunchKernelGGL((pruned_rope_kernel<true, 1, BF16>), grid, dim3(kRopeThreads), smem, stream, a, tpb);
  else hipLaunchKernelGGL((pruned_rope_kernel<false, 1, BF16>), grid, dim3(kRopeThreads), smem, stream, a, tpb);
  return hipGetLastError();
}

// the whole-row kernel addresses a tensor with signed 32-bit byte offsets
static bool rows_addressable(const RopeArgs& a) {
  const long long row = (long long)a.D_keep * 2;
  return (long long)a.T * a.Hq * row < (1ll << 31) && (long long)a.T * a.Hkv * row < (1ll << 31);
}

template <bool BF16>
static hipError_t launch_rope_rows(const RopeArgs& a, hipStream_t stream) {
  const size_t smem = (size_t)(a.D_keep >> 1) * sizeof(double);
  const int waves = kRopeThreads / 64;
  const int n_pairs = (a.T + 1) / 2;
  // about kRopeRowsBlocks blocks over all table rows; a wave walks over token pairs
  int bx = (n_pairs + waves - 1) / waves;
  const int cap = (kRopeRowsBlocks + a.H_tab - 1) / a.H_tab;
  if (bx > cap) bx = cap;
  const int hps = 64 / (a.D_keep >> 2);
  const int q_steps = (a.Hq / a.H_tab + hps - 1) / hps;
  if (q_steps <= 2) hipLaunchKernelGGL((pruned_rope_rows_kernel<BF16, 2>), dim3(bx, a.H_tab), dim3(kRopeThreads), smem, stream, a);
  else hipLaunchKernelGGL((pruned_rope_rows_kernel<BF16, 4>), dim3(bx, a.H_tab), dim3(kRopeThreads), smem, stream, a);
  return hipGetLastError();
}

hipError_t launch_pruned_rope(const RopeArgs& a, hipStream_t stream) {
  const int hk = a.D_keep >> 1;
  // half2 accesses need an even pair count (then every head row and both halves start on a
  // 4-byte boundary, since D_keep is a multiple of 4) and 4-byte aligned tensors
  const bool v2 = (hk % 2 == 0) && (reinterpret_cast<uintptr_t>(a.q) % 4 == 0) &&
                  (a.k == nullptr || reinterpret_cast<uintptr_t>(a.k) % 4 == 0);
  // prompt-sized calls whose head rows fit a wave (8-byte units: 8-byte aligned tensors): whole rows per wave
  const bool a8 = (reinterpret_cast<uintptr_t>(a.q) % 8 == 0) && (a.k == nullptr || reinterpret_cast<uintptr_t>(a.k) % 8 == 0);
  if (v2 && a8 && hk <= 128 && a.T >= kRopeRowsMinTokens && rows_addressable(a))
    return a.bf16 ? launch_rope_rows<true>(a, stream) : launch_rope_rows<false>(a, stream);
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
