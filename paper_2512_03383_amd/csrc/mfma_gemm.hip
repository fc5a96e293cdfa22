// W4A16 GEMM launchers: the fp16 instantiations of mfma_kernel.h, the hand-scheduled fp16 prefill kernel,
// and the dispatch to the bfloat16 instantiations (mfma_gemm_bf16.hip).
#include "mfma_kernel.h"

namespace uniql {

// ---- prefill kernel -------------------------------------------------------------------------
// 128 tokens x 256 rows per block; eight waves side by side over rows, each 8 x 2 fragments, two
// waves per SIMD (at most 256 registers), so that one wave's LDS / memory / scalar instructions and
// waits overlap the other's MFMAs.  A wave issues at most one instruction per 4 clocks and the
// matrix pipe takes 16 clocks per MFMA, so the body of a slab (one quantisation group, four MFMA
// steps) is written in the order it should issue and pinned with scheduling barriers: every MFMA
// is followed by the one or two VALU instructions of the NEXT step's dequantisation (in the last
// steps also the staging of the next activation slab and the next slab's first step), and every
// second MFMA by the LDS read that refills the activation fragment it just consumed.
// Column prefix only (XVEC staging); weights and activations are addressed as a uniform base plus
// a 32-bit per-lane offset, which the host checks for.
// ZP = false: the matrix has no zero points (every z = 8, the symmetric scheme) and none is loaded.
template <bool ZP>
__global__ __launch_bounds__(512) void w4_mfma_prefill_kernel(LinearArgs a) {
  constexpr int AF = 8, BF = 2, WN = 8, NT = WN * 64, BM = 16 * AF, BN = WN * BF * 16, SC = 128, NCH = 16;
  constexpr int UPT = BM * NCH / NT;          // 16-byte staging units per thread and slab
  constexpr int SLOTS = AF * BF;              // MFMAs per step
  constexpr int DQ = 13 * BF;                 // dequantisation micro-ops per step
  extern __shared__ __align__(16) unsigned char smem[];
  uint4* xs = reinterpret_cast<uint4*>(smem);   // [2][NCH][BM], swizzled as in w4_mfma_kernel

  const KeepMap& km = a.km;
  const int tid = threadIdx.x, lane = tid & 63, wn = tid >> 6;
  const int n = lane & 15, ks = lane >> 4;
  const int n0 = blockIdx.x * BN, m0 = blockIdx.y * BM;
  const int words_per_row = a.K_total >> 3, groups_per_row = a.K_total / kGroup;
  const int kv = km.k_keep & ~7;
  const int nit = (km.k_span + kGroup - 1) / kGroup;
  auto swz = [](int chunk) { return ((chunk >> 2) & 3) | ((chunk & 3) << 2); };

  // per-lane byte offsets of this lane's weight fragments (rows clamped: every address is valid)
  auto frag_row = [&](int bf) {
    int rc = n0 + (wn * BF + bf) * 16 + n;
    rc = rc < km.n_keep ? rc : km.n_keep - 1;
    return (size_t)stored_row(km, rc);
  };
  uint32_t woff[BF], zoff[BF];
#pragma unroll
  for (int bf = 0; bf < BF; ++bf) {
    const size_t r = frag_row(bf);
    woff[bf] = (uint32_t)(r * words_per_row * 4 + ks * 16);
    zoff[bf] = (uint32_t)(r * groups_per_row);
  }
  const char* qbase = reinterpret_cast<const char*>(a.qweight);
  const char* sbase = reinterpret_cast<const char*>(a.scales);
  const char* zbase = reinterpret_cast<const char*>(a.zeros);
  struct WSet {
    uint32_t w[BF][4];
  };
  auto load_w = [&](int g, WSet& t) {
    g = g < nit ? g : nit - 1;
#pragma unroll
    for (int bf = 0; bf < BF; ++bf) {
      const uint4 v = *reinterpret_cast<const uint4*>(qbase + (size_t)g * 64 + woff[bf]);
      t.w[bf][0] = v.x; t.w[bf][1] = v.y; t.w[bf][2] = v.z; t.w[bf][3] = v.w;
    }
  };
  // Scales and zero points.  A load instruction whose 64 lanes touch 16 different rows costs the
  // memory pipeline about 4 clocks per row whatever its width, so a lane fetches those of EIGHT
  // consecutive groups of its row at once (16 + 8 bytes) and shifts the set down by one group per
  // slab: element 0 is always the next group to be used.  A set that would run past the row's last
  // group starts early and is shifted into place when it is loaded.
  uint4 sc[BF];
  uint2 zz[BF];
  auto shift_set = [&](int bf) {
    sc[bf].x = __builtin_amdgcn_alignbit(sc[bf].y, sc[bf].x, 16);
    sc[bf].y = __builtin_amdgcn_alignbit(sc[bf].z, sc[bf].y, 16);
    sc[bf].z = __builtin_amdgcn_alignbit(sc[bf].w, sc[bf].z, 16);
    sc[bf].w >>= 16;
    zz[bf].x = __builtin_amdgcn_alignbit(zz[bf].y, zz[bf].x, 8);
    zz[bf].y >>= 8;
  };
  auto load_set = [&](int g0) {   // g0: first group the set must hold (a multiple of 8)
    const int start = g0 + 8 <= groups_per_row ? g0 : groups_per_row - 8;
#pragma unroll
    for (int bf = 0; bf < BF; ++bf) {
      sc[bf] = load_u4_unaligned(reinterpret_cast<const half_t*>(sbase + ((size_t)start + zoff[bf]) * 2));
      if constexpr (ZP) {
        const uint32_t* zp = reinterpret_cast<const uint32_t*>(zbase + (size_t)start + zoff[bf]);
        zz[bf] = make_uint2(load_u32_unaligned(zp), load_u32_unaligned(zp + 1));
      } else {
        zz[bf] = make_uint2(0x08080808u, 0x08080808u);
      }
    }
    for (int i = start; i < g0; ++i) {   // only the last set of a row whose group count is not a multiple of 8
#pragma unroll
      for (int bf = 0; bf < BF; ++bf) shift_set(bf);
    }
  };
  auto groupq_from_set = [&](int bf) {
    GroupQ g;
    const uint32_t zp = __builtin_amdgcn_perm(0u, zz[bf].x, 0x0c000c00u);   // (z, z) as 16-bit integers
    g.zlo = as_half2(zp | 0x64006400u);
    g.zhi = as_half2((zp << 4) | 0x54005400u);
    g.s2 = as_half2(__builtin_amdgcn_perm(0u, sc[bf].x, 0x01000100u));      // (s, s)
    return g;
  };

  // activation staging: unit u = token u / 16, chunk u % 16 of the slab; per-unit constants
  const char* xbase = reinterpret_cast<const char*>(a.x + (size_t)m0 * a.ldx);
  uint32_t xoff[UPT];
#pragma unroll
  for (int i = 0; i < UPT; ++i) {
    const int u = tid + i * NT, tk = u / NCH, cb = u % NCH;
    const int tok = m0 + tk < a.M ? tk : a.M - 1 - m0;    // rows past M are never stored: any valid row will do
    xoff[i] = (uint32_t)(((size_t)tok * a.ldx + cb * 8) * 2);
  }
  // unit i of a thread is token tid / 16 + i * NT / 16 of the same chunk: the swizzle only touches the low 4 bits
  const int lds_slot0 = (tid % NCH) * BM + ((tid / NCH) ^ swz(tid % NCH));
  uint4 xr[UPT];
  auto fetch_x = [&](int it, bool masked) {
    it = it < nit ? it : nit - 1;
#pragma unroll
    for (int i = 0; i < UPT; ++i) {
      const int cb = (tid + i * NT) % NCH;
      if (!masked) {
        xr[i] = load_u4_unaligned(reinterpret_cast<const half_t*>(xbase + (size_t)it * (SC * 2) + xoff[i]));
      } else {
        // a chunk that is not entirely below kv reads the first chunk of its row instead (zeroed when stored)
        const bool full = it * SC + cb * 8 + 8 <= kv;
        const uint32_t o = full ? (uint32_t)it * (SC * 2) + xoff[i] : xoff[i] - (uint32_t)cb * 16;
        xr[i] = load_u4_unaligned(reinterpret_cast<const half_t*>(xbase + o));
      }
    }
  };
  // one unit: permute the 8 halves to (0,4,1,5,2,6,3,7), zero it when its columns are not all kept
  auto store_unit = [&](int i, int it, int buf, bool masked) {
    const uint4 r = xr[i];
    uint32_t o0 = __builtin_amdgcn_perm(r.z, r.x, 0x05040100u), o1 = __builtin_amdgcn_perm(r.z, r.x, 0x07060302u);
    uint32_t o2 = __builtin_amdgcn_perm(r.w, r.y, 0x05040100u), o3 = __builtin_amdgcn_perm(r.w, r.y, 0x07060302u);
    if (masked) {
      const int cb = (tid + i * NT) % NCH;
      const uint32_t m = it * SC + cb * 8 + 8 <= kv ? 0xffffffffu : 0u;
      o0 &= m; o1 &= m; o2 &= m; o3 &= m;
    }
    xs[buf * (NCH * BM) + lds_slot0 + i * (NT / NCH)] = make_uint4(o0, o1, o2, o3);
  };

  float4_t acc[AF][BF];
#pragma unroll
  for (int af = 0; af < AF; ++af)
#pragma unroll
    for (int bf = 0; bf < BF; ++bf) acc[af][bf] = float4_t{0.f, 0.f, 0.f, 0.f};

  const Magic mg = make_magic();
  WSet wa, wb;              // the weights of the current and of the next slab, roles alternate
  GroupQ ga[BF], gb[BF];
  uint4 av[AF], bfr[2][BF];
  uint32_t w8[BF];
  half2_t h[BF][4];

  // micro-op o (0 .. DQ-1) of dequantising word t of every row fragment of W into out[]
  auto dq_op = [&](int o, const WSet& W, const GroupQ (&G)[BF], int t, uint4 (&out)[BF]) {
    const int bf = o / 13, k = o % 13;
    const uint32_t w = W.w[bf][t];
    if (k == 0) w8[bf] = w >> 8;
    else if (k == 1) h[bf][0] = as_half2(and_or(w, 0x000F000Fu, mg.m1024));
    else if (k == 2) h[bf][1] = as_half2(and_or(w, 0x00F000F0u, mg.m64));
    else if (k == 3) h[bf][2] = as_half2(and_or(w8[bf], 0x000F000Fu, mg.m1024));
    else if (k == 4) h[bf][3] = as_half2(and_or(w8[bf], 0x00F000F0u, mg.m64));
    else if (k <= 8) h[bf][k - 5] = h[bf][k - 5] - ((k - 5) & 1 ? G[bf].zhi : G[bf].zlo);
    else {
      const uint32_t d = as_u32(h[bf][k - 9] * G[bf].s2);
      if (k == 9) out[bf].x = d; else if (k == 10) out[bf].y = d; else if (k == 11) out[bf].z = d; else out[bf].w = d;
    }
  };
  auto read_a = [&](int buf, int t, int af) {
    return xs[(buf * NCH + ks * 4 + t) * BM + af * 16 + (n ^ (ks | (t << 2)))];
  };

  // prologue: slab 0 staged, its first step dequantised
  load_w(0, wa);
  fetch_x(0, true);
#pragma unroll
  for (int i = 0; i < UPT; ++i) store_unit(i, 0, 0, true);
  load_set(0);
#pragma unroll
  for (int bf = 0; bf < BF; ++bf) {
    ga[bf] = groupq_from_set(bf);
    shift_set(bf);
  }
#pragma unroll
  for (int o = 0; o < DQ; ++o) dq_op(o, wa, ga, 0, bfr[0]);
  __syncthreads();

  // One slab.  cur / gq: this slab's weights and group constants; nxt / gqn: the next slab's, loaded
  // and derived here.  masked = the next slab (staged during this one) has columns at or past kv.
  auto slab = [&](int it, WSet& cur, GroupQ (&gq)[BF], WSet& nxt, GroupQ (&gqn)[BF], auto masked_tag) {
    constexpr bool masked = decltype(masked_tag)::value;
    const int buf = it & 1;
#pragma unroll
    for (int af = 0; af < AF; ++af) av[af] = read_a(buf, 0, af);
    fetch_x(it + 1, masked);
    load_w(it + 1, nxt);
    if (((it + 1) & 7) == 0 && it + 1 < nit) load_set(it + 1);   // the previous set has no element left
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int t = 0; t < 4; ++t) {
#pragma unroll
      for (int af = 0; af < AF; ++af) {
#pragma unroll
        for (int bf = 0; bf < BF; ++bf) {
          const int s = af * BF + bf;   // slot 0 .. SLOTS-1 of the step
          acc[af][bf] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, av[af]),
                                                              __builtin_bit_cast(half8_t, bfr[t & 1][bf]),
                                                              acc[af][bf], 0, 0, 0);
          if (t < 3) {
            for (int o = s * DQ / SLOTS; o < (s + 1) * DQ / SLOTS; ++o) dq_op(o, cur, gq, t + 1, bfr[(t + 1) & 1]);
            if (bf == BF - 1) av[af] = read_a(buf, t + 1, af);   // refill the fragment just consumed
            // the first half of the next slab's staging rides on the third step
            if (t == 2 && s % (2 * SLOTS / UPT) == 1) store_unit(s / (2 * SLOTS / UPT), it + 1, buf ^ 1, masked);
          } else {
            // last step: the next slab's group constants and first step, the rest of the staging
            if (s < BF) {
              gqn[s] = groupq_from_set(s);
              shift_set(s);
            }
            else for (int o = (s - BF) * DQ / (SLOTS - BF); o < (s - BF + 1) * DQ / (SLOTS - BF); ++o) dq_op(o, nxt, gqn, 0, bfr[0]);
            if (s % (2 * SLOTS / UPT) == 1) store_unit(UPT / 2 + s / (2 * SLOTS / UPT), it + 1, buf ^ 1, masked);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    __syncthreads();
  };
  // slabs it < n_plain stage a next slab that lies entirely below kv; roles of (wa, ga) / (wb, gb) alternate
  const int n_plain = kv / SC - 1;
  int it = 0;
  for (; it + 1 < n_plain; it += 2) {
    slab(it, wa, ga, wb, gb, std::false_type{});
    slab(it + 1, wb, gb, wa, ga, std::false_type{});
  }
  for (; it < nit; ++it) {
    if (it & 1) slab(it, wb, gb, wa, ga, std::true_type{});
    else slab(it, wa, ga, wb, gb, std::true_type{});
  }

  // ---- epilogue.  Lane l holds, for fragment (af, bf): row (l % 16), tokens 4 * (l / 16) + v.
  if (kv < km.k_keep) {
    // the kept columns kv .. k_keep-1 (fewer than 8: one word of one group per row), in fp32
#pragma unroll
    for (int bf = 0; bf < BF; ++bf) {
      const size_t wr = frag_row(bf);
      const uint32_t word = a.qweight[wr * words_per_row + (kv >> 3)];
      const size_t gi = wr * groups_per_row + (kv >> 7);
      const float sf = (float)__builtin_bit_cast(half_t, a.scales[gi]);
      const int z = a.zeros ? a.zeros[gi] : 8;
      for (int j = 0; kv + j < km.k_keep; ++j) {
        const int q = (int)((word >> (4 * j)) & 15u);
        const float w = (float)(half_t)((float)(q - z) * sf);   // the canonical fp16 weight
#pragma unroll
        for (int af = 0; af < AF; ++af)
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const int tok = m0 + af * 16 + 4 * ks + v;
            const float xv = (float)a.x[(size_t)(tok < a.M ? tok : a.M - 1) * a.ldx + kv + j];
            acc[af][bf][v] = __builtin_fmaf(xv, w, acc[af][bf][v]);
          }
      }
    }
  }
#pragma unroll
  for (int af = 0; af < AF; ++af)
#pragma unroll
    for (int bf = 0; bf < BF; ++bf) {
      const int rc = n0 + (wn * BF + bf) * 16 + n;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int tok = m0 + af * 16 + 4 * ks + v;
        if (tok < a.M && rc < km.n_keep) a.y[(size_t)tok * a.ldy + rc] = (half_t)acc[af][bf][v];
      }
    }
}

static hipError_t launch_prefill(const LinearArgs& a, hipStream_t stream) {
  constexpr int BM = 128, BN = 256;
  const size_t smem = (size_t)2 * BM * 128 * sizeof(half_t);
  auto kern = a.zeros ? w4_mfma_prefill_kernel<true> : w4_mfma_prefill_kernel<false>;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (e != hipSuccess) return e;
  dim3 grid((a.km.n_keep + BN - 1) / BN, (a.M + BM - 1) / BM);
  hipLaunchKernelGGL(kern, grid, dim3(512), smem, stream, a);
  return hipGetLastError();
}

hipError_t launch_w4_gemm(const LinearArgs& a, hipStream_t stream) {
  if (a.bf16) return launch_w4_gemm_bf16(a, stream);
  return launch_gemm_fmt<false>(a, stream, launch_prefill);
}

}  // namespace uniql
