// W4A16 GEMM on MFMA for M >= 2 tokens: y[M][n_keep] = x[M][k_keep] * W'^T.
//
// "Direct-B" design: the packed weights never pass through LDS.  With
// v_mfma_f32_16x16x32_f16 the weight operand of lane l is 8 consecutive input columns of
// output row (l % 16) in k-slot (l / 16), which is exactly one 32-bit word of packed codes, so a
// wave fetches its 16 rows x 128 columns (one quantisation group per row) with ONE 128-bit load
// per lane (word t of the load feeds MFMA t of the group) and dequantises in registers to the
// canonical fp16 weights.  Only the activations go through LDS: the block stages a slab of x
// (its tokens x the columns of the current step) at *stored* column positions, zeros where
// pruned, pre-permuted inside every 8-column block to the (0,4,1,5,2,6,3,7) order the unpack
// produces, double-buffered so that the next slab is fetched while the current one is used.
//
// A wave owns BF fragments of 16 rows and AF fragments of 16 tokens (AF*BF accumulators of 4
// VGPRs); a dequantised weight fragment is reused by AF MFMAs, an activation fragment by BF.
// Small M (decode batches) is HBM-bound: AF = 1 and the K range is split over KS waves of the
// block (reduced through LDS at the end) to get enough waves; large M (prefill) is MFMA-bound:
// AF = 8, BF = 4, KS = 1.
#define UNIQL_ANDOR_PLAIN   // and-or as plain C here: the scheduler must be able to classify it as VALU
#include "common.h"
#include <type_traits>

namespace uniql {

struct WTile {
  uint4 w;
};

// AF token fragments, BF row fragments per wave, WN waves along rows, KS waves along K,
// S2 groups per wave and iteration (the slab holds KS * S2 groups: fewer, longer iterations hide
// the latency of fetching the next slab), PW iterations of weight loads kept in flight.
template <int AF, int BF, int WN, int KS, int S2, int PW, int XM>
__global__ __launch_bounds__(WN * KS * 64) void w4_mfma_kernel(LinearArgs a) {
  // activation staging mode: 0 = element by element through the column map, 1 = column prefix,
  // 2 = column segments whose stride is a multiple of 8 (128-bit loads in both)
  constexpr bool XVEC = XM == 1, XSEG = XM == 2;
  constexpr int NT = WN * KS * 64;
  constexpr int BM = 16 * AF;               // tokens per block
  constexpr int BN = WN * BF * 16;          // rows per block
  constexpr int SC = KS * S2 * 128;         // columns per slab (S2 groups per K-split wave)
  constexpr int NCH = SC / 8;               // 8-column chunks per slab
  constexpr int UNITS = BM * NCH;           // 16-byte units per slab
  static_assert(UNITS % NT == 0, "slab must divide evenly over the threads");
  constexpr int UPT = UNITS / NT;           // units per thread

  extern __shared__ __align__(16) unsigned char smem[];
  // Slab layout [2][NCH][BM] of 16-byte units (8 columns of one token).  The 16 lanes that read one
  // activation fragment (16 tokens, one chunk) touch one aligned 256-byte window, which is what
  // ds_read_b128 needs to run at the full LDS rate on this target (a padded token-major slab reads
  // at half rate).  Inside its window token j sits at slot j ^ swz(chunk), swz = (k-slot | step << 2)
  // of the chunk, so that the 16 lanes that WRITE 16 consecutive chunks of one token also hit 16
  // different bank groups; measured, both patterns are conflict-free.
  uint4* xs = reinterpret_cast<uint4*>(smem);
  // Scales and zero points of the slab's groups ride along: [2][BN][KS * S2] words (scale bits |
  // zero << 16).  A load whose lanes touch 16 different rows costs the memory pipeline about 4
  // clocks per row whatever its width, so instead of every wave fetching the two values of its 16
  // rows per group, one thread per (row, group) of the block fetches them with the slab, adjacent
  // lanes reading adjacent groups of a row.
  constexpr int NG = KS * S2;                // groups per slab
  static_assert(BN * NG <= NT, "one thread per (row, group) of a slab");
  uint32_t* szs = reinterpret_cast<uint32_t*>(smem + (size_t)2 * UNITS * sizeof(uint4));

  const KeepMap& km = a.km;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wn = wave % WN, wk = wave / WN;
  const int n = lane & 15, ks = lane >> 4;
  const int n0 = blockIdx.x * BN, m0 = blockIdx.y * BM;
  const int words_per_row = a.K_total >> 3, groups_per_row = a.K_total / kGroup;
  const int ngroups = (km.k_span + kGroup - 1) / kGroup;
  const int nit = (ngroups + KS * S2 - 1) / (KS * S2);
  const int nit_pw = (nit + PW - 1) / PW * PW;   // loop trip count; extra iterations multiply zeros

  // stored row of each of this lane's weight fragments (clamped: every address stays valid)
  size_t wrow[BF];
#pragma unroll
  for (int bf = 0; bf < BF; ++bf) {
    int rc = n0 + (wn * BF + bf) * 16 + n;
    rc = rc < km.n_keep ? rc : km.n_keep - 1;
    wrow[bf] = (size_t)stored_row(km, rc);
  }
  // group s2 of iteration it for this wave: slab-local group s2 * KS + wk
  auto load_w = [&](int it, WTile (&t)[S2][BF]) {
#pragma unroll
    for (int s2 = 0; s2 < S2; ++s2) {
      int g = (it * S2 + s2) * KS + wk;
      g = g < ngroups ? g : ngroups - 1;   // past the end: a valid, redundant load (x is zero there)
#pragma unroll
      for (int bf = 0; bf < BF; ++bf)
        t[s2][bf].w = *reinterpret_cast<const uint4*>(a.qweight + wrow[bf] * words_per_row + g * 16 + ks * 4);
    }
  };
  // this thread's (row, group) of the scale / zero staging, if it has one
  const bool sz_owner = tid < BN * NG;
  size_t sz_row;
  {
    int rc = n0 + tid / NG;
    rc = rc < km.n_keep ? rc : km.n_keep - 1;
    sz_row = (size_t)stored_row(km, rc) * groups_per_row;
  }
  auto fetch_sz = [&](int it, uint32_t& sbits, uint32_t& z) {
    int g = it * NG + tid % NG;
    g = g < ngroups ? g : ngroups - 1;
    sbits = a.scales[sz_row + g];
    z = a.zeros ? a.zeros[sz_row + g] : 8u;   // no zero points: the symmetric scheme, z = 8
  };

  // x slab staging: unit u of a slab = token (u / NCH), 8-column chunk (u % NCH).
  // fetch_x only issues loads (unconditional, on clamped addresses) and records which halves are
  // real; store_x, one iteration later, masks, permutes and writes them to LDS.  Nothing touches
  // the loaded registers in between, so the wave never waits for x at the point of issue.
  // XVEC: whole 8-column blocks below kv come from one 128-bit load; the up to 7 kept columns at
  // and after kv are added in the epilogue.  XSEG: a block lies in one segment and its kept columns
  // are its first nk, contiguous in x: one 128-bit load and a per-half mask (only the block that
  // holds a row's last kept columns, fewer than 8 of them, is read element by element).
  // Otherwise: eight element loads through the column map.
  auto unit_token = [](int u) { return u / NCH; };
  auto unit_chunk = [](int u) { return u % NCH; };
  auto swz = [](int chunk) { return ((chunk >> 2) & 3) | ((chunk & 3) << 2); };
  const int kv = km.k_keep & ~7;
  const uint16_t* xbits = reinterpret_cast<const uint16_t*>(a.x);
  struct XRegs {
    uint4 v[XM != 0 ? UPT : 1];
    uint32_t e[XM != 0 ? 1 : UPT][8];
    uint32_t ok[UPT];   // XVEC: all-ones / zero word mask; otherwise bit j = half j is real
  };
  auto fetch_x = [&](int it, XRegs& xr) {
#pragma unroll
    for (int i = 0; i < UPT; ++i) {
      const int u = tid + i * NT;
      const int tk = unit_token(u), cb = unit_chunk(u);
      const int k0 = it * SC + cb * 8;
      const int tok = m0 + tk;
      const bool tok_ok = tok < a.M;
      const size_t xoff = (size_t)(tok_ok ? tok : a.M - 1) * a.ldx;
      if constexpr (XVEC) {
        const bool full = k0 + 8 <= kv;
        xr.v[i] = load_u4_unaligned(a.x + xoff + (full ? k0 : 0));
        xr.ok[i] = (full && tok_ok) ? 0xffffffffu : 0u;
      } else if constexpr (XSEG) {
        const int seg = k0 / km.cs_stride, off = k0 - seg * km.cs_stride;
        int nk = km.cs_keep - off;                       // kept columns at the start of this block
        nk = nk < 0 ? 0 : (nk > 8 ? 8 : nk);
        nk = k0 < km.k_span ? nk : 0;
        const int c = seg * km.cs_keep + off;            // compact column of the block's first column
        const bool vec = nk > 0 && c + 8 <= km.k_keep;   // the 16 bytes at c lie inside the token row
        xr.v[i] = load_u4_unaligned(a.x + xoff + (vec ? c : 0));
        xr.ok[i] = tok_ok ? (1u << nk) - 1u : 0u;
        if (nk > 0 && !vec) {   // the row's last kept columns, fewer than 8 left
          uint32_t h[8];
#pragma unroll
          for (int j = 0; j < 8; ++j) h[j] = j < nk ? (uint32_t)xbits[xoff + c + j] : 0u;
          xr.v[i] = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
        }
      } else {
        xr.ok[i] = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int k = k0 + j;
          const int kc = k < km.k_span ? compact_col(km, k) : -1;
          xr.e[i][j] = xbits[xoff + (kc >= 0 ? kc : 0)];
          xr.ok[i] |= (kc >= 0 && tok_ok) ? (1u << j) : 0u;
        }
      }
    }
  };
  auto store_x = [&](int buf, const XRegs& xr) {
#pragma unroll
    for (int i = 0; i < UPT; ++i) {
      const int u = tid + i * NT;
      const int tk = unit_token(u), cb = unit_chunk(u);
      uint32_t e[8];
      if constexpr (XVEC) {
        const uint4 r = xr.v[i];
        const uint32_t m = xr.ok[i];
        e[0] = r.x & 0xffffu & m; e[1] = (r.x >> 16) & m; e[2] = r.y & 0xffffu & m; e[3] = (r.y >> 16) & m;
        e[4] = r.z & 0xffffu & m; e[5] = (r.z >> 16) & m; e[6] = r.w & 0xffffu & m; e[7] = (r.w >> 16) & m;
      } else if constexpr (XSEG) {
        const uint4 r = xr.v[i];
        const uint32_t full[8] = {r.x & 0xffffu, r.x >> 16, r.y & 0xffffu, r.y >> 16,
                                  r.z & 0xffffu, r.z >> 16, r.w & 0xffffu, r.w >> 16};
#pragma unroll
        for (int j = 0; j < 8; ++j) e[j] = full[j] & (uint32_t)((int32_t)(xr.ok[i] << (31 - j)) >> 31);
      } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) e[j] = (xr.ok[i] >> j) & 1u ? xr.e[i][j] : 0u;
      }
      xs[(buf * NCH + cb) * BM + (tk ^ swz(cb))] =
          make_uint4(e[0] | (e[4] << 16), e[1] | (e[5] << 16), e[2] | (e[6] << 16), e[3] | (e[7] << 16));
    }
  };

  float4_t acc[AF][BF];
#pragma unroll
  for (int af = 0; af < AF; ++af)
#pragma unroll
    for (int bf = 0; bf < BF; ++bf) acc[af][bf] = float4_t{0.f, 0.f, 0.f, 0.f};

  const Magic mg = make_magic();
  WTile ring[PW][S2][BF];
  XRegs xr;
  uint32_t sz_s = 0, sz_z = 0;
#pragma unroll
  for (int p = 0; p < PW; ++p) load_w(p, ring[p]);
  fetch_x(0, xr);
  if (sz_owner) fetch_sz(0, sz_s, sz_z);
  store_x(0, xr);
  if (sz_owner) szs[tid] = sz_s | (sz_z << 16);
  __syncthreads();

  for (int it0 = 0; it0 < nit_pw; it0 += PW) {
#pragma unroll
    for (int p = 0; p < PW; ++p) {
      const int it = it0 + p;
      const int buf = it & 1;
      // this slab's scales and zero points, read before anything else so that the LDS latency is
      // covered by issuing the loads below
      uint32_t szv[S2][BF];
#pragma unroll
      for (int s2 = 0; s2 < S2; ++s2)
#pragma unroll
        for (int bf = 0; bf < BF; ++bf) szv[s2][bf] = szs[(buf * BN + (wn * BF + bf) * 16 + n) * NG + s2 * KS + wk];
      // fetch the next slab into registers while this one is consumed
      if (it + 1 < nit_pw) fetch_x(it + 1, xr);
      if (sz_owner) fetch_sz(it + 1, sz_s, sz_z);

      // Word t of a lane's 128-bit load feeds MFMA t of the group.  Dequantising word t of every
      // row fragment right before its MFMAs keeps only BF operand fragments live and lets the
      // VALU work of step t+1 issue while the matrix pipe is busy with step t.
#pragma unroll
      for (int s2 = 0; s2 < S2; ++s2) {
        GroupQ gq[BF];
        uint32_t wv[BF][4];
#pragma unroll
        for (int bf = 0; bf < BF; ++bf) {
          const WTile& wt = ring[p][s2][bf];
          gq[bf] = make_groupq(szv[s2][bf] & 0xffffu, szv[s2][bf] >> 16);
          wv[bf][0] = wt.w.x; wv[bf][1] = wt.w.y; wv[bf][2] = wt.w.z; wv[bf][3] = wt.w.w;
        }
        const uint4* xb = xs + (buf * NCH + (s2 * KS + wk) * 16 + ks * 4) * BM;
        // Two-stage pipeline over the group's four MFMA steps: while step t multiplies, the
        // activation fragments of step t+1 are read from LDS and its weights dequantised.
        uint4 av[2][AF], bfrag[2][BF];
        auto stage = [&](int t, uint4 (&ao)[AF], uint4 (&bo)[BF]) {
#pragma unroll
          for (int af = 0; af < AF; ++af) ao[af] = xb[t * BM + af * 16 + (n ^ (ks | (t << 2)))];
#pragma unroll
          for (int bf = 0; bf < BF; ++bf) {
            half2_t d[4];
            dequant_word(wv[bf][t], gq[bf], mg, d);
            bo[bf] = make_uint4(as_u32(d[0]), as_u32(d[1]), as_u32(d[2]), as_u32(d[3]));
          }
        };
        stage(0, av[0], bfrag[0]);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          if (t < 3) stage(t + 1, av[(t + 1) & 1], bfrag[(t + 1) & 1]);
#pragma unroll
          for (int af = 0; af < AF; ++af)
#pragma unroll
            for (int bf = 0; bf < BF; ++bf)
              acc[af][bf] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, av[t & 1][af]),
                                                                  __builtin_bit_cast(half8_t, bfrag[t & 1][bf]),
                                                                  acc[af][bf], 0, 0, 0);
        }
      }
      load_w(it + PW, ring[p]);   // refill the ring slot (clamped past the end)
      if (it + 1 < nit_pw) store_x(buf ^ 1, xr);
      if (sz_owner) szs[(buf ^ 1) * BN * NG + tid] = sz_s | (sz_z << 16);
      __syncthreads();
    }
  }

  // ---- epilogue.  Lane l holds, for fragment (af, bf): row (l % 16), tokens 4 * (l / 16) + v.
  if constexpr (KS > 1) {
    float* red = reinterpret_cast<float*>(smem);   // [KS][WN][AF][BF][4][64], reuses the slab space
    constexpr int PER_WAVE = AF * BF * 4 * 64;
    float* mine = red + (size_t)(wk * WN + wn) * PER_WAVE;
#pragma unroll
    for (int af = 0; af < AF; ++af)
#pragma unroll
      for (int bf = 0; bf < BF; ++bf)
#pragma unroll
        for (int v = 0; v < 4; ++v) mine[((af * BF + bf) * 4 + v) * 64 + lane] = acc[af][bf][v];
    __syncthreads();
    if (wk != 0) return;
#pragma unroll
    for (int k2 = 1; k2 < KS; ++k2) {
      const float* other = red + (size_t)(k2 * WN + wn) * PER_WAVE;
#pragma unroll
      for (int af = 0; af < AF; ++af)
#pragma unroll
        for (int bf = 0; bf < BF; ++bf)
#pragma unroll
          for (int v = 0; v < 4; ++v) acc[af][bf][v] += other[((af * BF + bf) * 4 + v) * 64 + lane];
    }
  }
  if constexpr (XVEC) {
    // the kept columns kv .. k_keep-1 (fewer than 8: one word of one group per row), in fp32
    if (kv < km.k_keep) {
#pragma unroll
      for (int bf = 0; bf < BF; ++bf) {
        const uint32_t word = a.qweight[wrow[bf] * words_per_row + (kv >> 3)];
        const size_t gi = wrow[bf] * groups_per_row + (kv >> 7);
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

template <int AF, int BF, int WN, int KS, int S2, int PW, int XVEC>
static hipError_t launch_cfg(const LinearArgs& a, hipStream_t stream) {
  constexpr int BM = 16 * AF, BN = WN * BF * 16, SC = KS * S2 * 128;
  size_t smem = (size_t)2 * BM * SC * sizeof(half_t) + (size_t)2 * BN * KS * S2 * sizeof(uint32_t);
  const size_t red = KS > 1 ? (size_t)KS * WN * AF * BF * 4 * 64 * sizeof(float) : 0;
  if (red > smem) smem = red;
  auto kern = w4_mfma_kernel<AF, BF, WN, KS, S2, PW, XVEC>;
  if (smem > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
  }
  dim3 grid((a.km.n_keep + BN - 1) / BN, (a.M + BM - 1) / BM);
  hipLaunchKernelGGL(kern, grid, dim3(WN * KS * 64), smem, stream, a);
  return hipGetLastError();
}

template <int XVEC>
static hipError_t launch_m(const LinearArgs& a, hipStream_t stream) {
  // Decode batches (M <= 32) are bound by the weight stream: 16 rows per wave and the K range
  // split over the block's 8 waves, four ways when there are many row tiles, eight ways otherwise.
  const int row_tiles = (a.km.n_keep + 15) / 16;
  if (a.M <= 16) return row_tiles >= 600 ? launch_cfg<1, 1, 2, 4, 2, 2, XVEC>(a, stream) : launch_cfg<1, 1, 1, 8, 1, 2, XVEC>(a, stream);
  if (a.M <= 32) return row_tiles >= 600 ? launch_cfg<2, 1, 2, 4, 1, 4, XVEC>(a, stream) : launch_cfg<2, 1, 1, 8, 1, 2, XVEC>(a, stream);
  if (a.M <= 64) return launch_cfg<4, 2, 4, 1, 1, 2, XVEC>(a, stream);
  // Prefill: the largest tile that still gives the chip about a block per CU.
  auto blocks = [&](int bm, int bn) { return (long long)((a.km.n_keep + bn - 1) / bn) * ((a.M + bm - 1) / bm); };
  constexpr long long kEnough = 192;
  if (blocks(128, 256) >= kEnough) {
    // the prefill kernel addresses weights and one block's activations with 32-bit offsets
    // and fetches scales eight groups at a time
    const bool small_offsets = (unsigned long long)a.N_total * (unsigned long long)a.K_total / 2 < (1ull << 32) &&
                               128ull * (unsigned long long)a.ldx * 2 < (1ull << 32);
    if (XVEC == 1 && small_offsets && a.km.k_keep >= 128 && a.K_total >= 8 * kGroup) return launch_prefill(a, stream);
    return launch_cfg<8, 4, 4, 1, 1, 1, XVEC>(a, stream);
  }
  if (blocks(64, 256) >= kEnough) return launch_cfg<4, 2, 8, 1, 1, 2, XVEC>(a, stream);
  if (blocks(64, 128) >= kEnough) return launch_cfg<4, 2, 4, 2, 2, 1, XVEC>(a, stream);   // K split over two waves
  return launch_cfg<4, 1, 4, 2, 1, 2, XVEC>(a, stream);
}

hipError_t launch_w4_gemm(const LinearArgs& a, hipStream_t stream) {
  // 128-bit x loads: a column prefix (global loads of any size may start on any 2-byte boundary on
  // this target, so odd leading dimensions such as k_keep = 12185 qualify), or column segments
  // whose stride is a multiple of 8 and that keep at least 8 columns each
  if (a.km.cs_stride == 0) return a.km.k_keep >= 8 ? launch_m<1>(a, stream) : launch_m<0>(a, stream);
  if (a.km.cs_stride % 8 == 0 && a.km.cs_keep >= 8) return launch_m<2>(a, stream);
  return launch_m<0>(a, stream);
}

}  // namespace uniql
