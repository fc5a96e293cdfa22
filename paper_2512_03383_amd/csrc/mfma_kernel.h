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
// AF = 8, BF = 2, eight waves side by side over 256 rows, KS = 1, two groups per slab.
#pragma once
#define UNIQL_ANDOR_PLAIN   // and-or as plain C here: the scheduler must be able to classify it as VALU
#include "common.h"
#include "smallm_kernel.h"
#include "prefill_kernel.h"
#include <type_traits>

namespace uniql {

struct WTile {
  uint4 w;
};

// AF token fragments, BF row fragments per wave, WN waves along rows, KS waves along K,
// S2 groups per wave and iteration (the slab holds KS * S2 groups: fewer, longer iterations hide
// the latency of fetching the next slab), PW iterations of weight loads kept in flight.
// BF16: scales, x and y are bfloat16; the weights are rounded to bfloat16 and the MFMA is the bf16 one.
template <int AF, int BF, int WN, int KS, int S2, int PW, int XM, bool BF16>
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
  // Block -> tile.  Consecutive blocks of a launch go to the eight dies (XCDs) in turn, each with an L2 of its own, so
  // block b runs on die b % 8.  Blocks are renumbered so that a die's blocks are consecutive tiles of a walk that
  // takes kTokTilesPerPass token tiles at a time and, inside that, row tile by row tile: the 32 blocks a die runs at
  // once then cover 8 row tiles x 4 token tiles and share their weight rows and activation slabs through that die's
  // L2 (with the launch order, a token tile's activations were fetched once per die: 857 MB of L2 misses for the
  // 159 MB of the 4096-token down projection).
  int rt = blockIdx.x, tt = blockIdx.y;
  if (gridDim.y > 1) {
    constexpr int kDies = 8, kTokTilesPerPass = 4;
    const int nrt = gridDim.x, ntt = gridDim.y, nb = nrt * ntt;
    const int bid = blockIdx.y * nrt + blockIdx.x;
    const int die = bid % kDies, j = bid / kDies;
    const int L = die * (nb / kDies) + min(die, nb % kDies) + j;   // blocks of die 0, then of die 1, ...
    const int full = (ntt / kTokTilesPerPass) * kTokTilesPerPass;  // token tiles in whole passes
    const int in_full = nrt * full;
    if (L < in_full) {
      const int pass = L / (nrt * kTokTilesPerPass), r = L - pass * (nrt * kTokTilesPerPass);
      rt = r / kTokTilesPerPass;
      tt = pass * kTokTilesPerPass + (r - rt * kTokTilesPerPass);
    } else {
      const int w = ntt - full, r = L - in_full;                   // the last, narrower pass
      rt = r / w;
      tt = full + (r - rt * w);
    }
  }
  const int n0 = rt * BN, m0 = tt * BM;
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
  // registers -> LDS: the unit's 8 halves in the pair order of the unpack, (0,4) (1,5) (2,6) (3,7): with 128-bit loads
  // a mask per loaded word, then one byte permute per output word
  auto store_x = [&](int buf, const XRegs& xr) {
#pragma unroll
    for (int i = 0; i < UPT; ++i) {
      const int u = tid + i * NT;
      const int tk = unit_token(u), cb = unit_chunk(u);
      uint4 o;
      if constexpr (XVEC || XSEG) {
        uint4 r = xr.v[i];
        if constexpr (XVEC) {
          const uint32_t m = xr.ok[i];
          r.x &= m; r.y &= m; r.z &= m; r.w &= m;
        } else {
          // kept columns are the unit's first nk: a mask per 32-bit word (halves 2 w and 2 w + 1)
          const uint32_t ok = xr.ok[i];
          r.x &= (ok & 1u ? 0xffffu : 0u) | (ok & 2u ? 0xffff0000u : 0u);
          r.y &= (ok & 4u ? 0xffffu : 0u) | (ok & 8u ? 0xffff0000u : 0u);
          r.z &= (ok & 16u ? 0xffffu : 0u) | (ok & 32u ? 0xffff0000u : 0u);
          r.w &= (ok & 64u ? 0xffffu : 0u) | (ok & 128u ? 0xffff0000u : 0u);
        }
        o = make_uint4(__builtin_amdgcn_perm(r.z, r.x, 0x05040100u), __builtin_amdgcn_perm(r.z, r.x, 0x07060302u),
                       __builtin_amdgcn_perm(r.w, r.y, 0x05040100u), __builtin_amdgcn_perm(r.w, r.y, 0x07060302u));
      } else {
        uint32_t e[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) e[j] = (xr.ok[i] >> j) & 1u ? xr.e[i][j] : 0u;
        o = make_uint4(e[0] | (e[4] << 16), e[1] | (e[5] << 16), e[2] | (e[6] << 16), e[3] | (e[7] << 16));
      }
      xs[(buf * NCH + cb) * BM + (tk ^ swz(cb))] = o;
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
        typename GroupOf<BF16>::type gq[BF];
        uint32_t wv[BF][4];
#pragma unroll
        for (int bf = 0; bf < BF; ++bf) {
          const WTile& wt = ring[p][s2][bf];
          gq[bf] = make_group<BF16>(szv[s2][bf] & 0xffffu, szv[s2][bf] >> 16);
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
          for (int bf = 0; bf < BF; ++bf) bo[bf] = dequant_word4<BF16>(wv[bf][t], gq[bf], mg);
        };
        stage(0, av[0], bfrag[0]);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          if (t < 3) stage(t + 1, av[(t + 1) & 1], bfrag[(t + 1) & 1]);
#pragma unroll
          for (int af = 0; af < AF; ++af)
#pragma unroll
            for (int bf = 0; bf < BF; ++bf)
              acc[af][bf] = mfma_16x16x32<BF16>(av[t & 1][af], bfrag[t & 1][bf], acc[af][bf]);
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
        const float sf = in16<BF16>(__builtin_bit_cast(half_t, a.scales[gi]));
        const int z = a.zeros ? a.zeros[gi] : 8;
        for (int j = 0; kv + j < km.k_keep; ++j) {
          const int q = (int)((word >> (4 * j)) & 15u);
          const float w = in16<BF16>(out16<BF16>((float)(q - z) * sf));   // the canonical 16-bit weight
#pragma unroll
          for (int af = 0; af < AF; ++af)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
              const int tok = m0 + af * 16 + 4 * ks + v;
              const float xv = in16<BF16>(a.x[(size_t)(tok < a.M ? tok : a.M - 1) * a.ldx + kv + j]);
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
        if (tok < a.M && rc < km.n_keep) a.y[(size_t)tok * a.ldy + rc] = out16<BF16>(acc[af][bf][v]);
      }
    }
}


template <bool BF16, int AF, int BF, int WN, int KS, int S2, int PW, int XVEC>
static hipError_t launch_cfg(const LinearArgs& a, hipStream_t stream) {
  constexpr int BM = 16 * AF, BN = WN * BF * 16, SC = KS * S2 * 128;
  size_t smem = (size_t)2 * BM * SC * sizeof(half_t) + (size_t)2 * BN * KS * S2 * sizeof(uint32_t);
  const size_t red = KS > 1 ? (size_t)KS * WN * AF * BF * 4 * 64 * sizeof(float) : 0;
  if (red > smem) smem = red;
  auto kern = w4_mfma_kernel<AF, BF, WN, KS, S2, PW, XVEC, BF16>;
  if (smem > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
  }
  dim3 grid((a.km.n_keep + BN - 1) / BN, (a.M + BM - 1) / BM);
  hipLaunchKernelGGL(kern, grid, dim3(WN * KS * 64), smem, stream, a);
  return hipGetLastError();
}

template <int XVEC, bool BF16>
static hipError_t launch_m(const LinearArgs& a, hipStream_t stream) {
  // Decode batches (M <= 32) are bound by the weight stream and have a kernel of their own (smallm_kernel.h), except
  // tall matrices at more than 8 tokens: there this kernel's slab, staged once for 64 rows, costs less than every wave
  // staging its own activations (14336-row gate at 16 / 32 tokens, weights from HBM: 12.3 / 15.3 us here, 14.1 / 19.5 us
  // there; 3584-row down: 16.4 / 27.3 us here, 15.9 / 21.6 us there; up to 8 tokens the other kernel wins or ties
  // everywhere; with the activations staged once per block -- column prefixes of at most 32 groups, up to 16 tokens --
  // the other kernel takes the tall matrices at 9..16 tokens too: 18944-row gate at 16 tokens 11.6 against 12.7 us).  What that kernel does not take falls through to this one: 16 rows per wave and the K range split over
  // the block's 8 waves, four ways when there are many row tiles, eight ways otherwise.
  const int row_tiles = (a.km.n_keep + 15) / 16;
  if (smallm_takes(a, XVEC == 1)) return smallm_dispatch<XVEC, BF16>(a, stream);
  // (many row tiles: 32 rows per wave, so that an activation fragment read from LDS serves two weight fragments,
  // 64 rows per block; few: 16 rows per block, two groups per wave and slab, which halves the number of barriers)
  if (a.M <= 16) return row_tiles >= 600 ? launch_cfg<BF16, 1, 2, 2, 4, 1, 2, XVEC>(a, stream) : launch_cfg<BF16, 1, 1, 1, 8, 2, 1, XVEC>(a, stream);
  // 17..32 tokens: tall matrices 32 rows per wave and 64 per block with two groups per wave and slab (Qwen gate at 32
  // tokens 17.0 -> 14.5 us); short ones 16 rows per block, K over eight waves
  if (a.M <= 32) return row_tiles >= 600 ? launch_cfg<BF16, 2, 2, 2, 4, 2, 1, XVEC>(a, stream) : launch_cfg<BF16, 2, 1, 1, 8, 1, 2, XVEC>(a, stream);
  // 33..64 tokens: K over four waves in either case, or a matrix of a few thousand rows leaves most of the chip idle
  // (64 x 128 tiles without a K split: Qwen down 122 us, gate 33 us; now 50 us and 21 us)
  if (a.M <= 64) return row_tiles >= 600 ? launch_cfg<BF16, 4, 2, 2, 4, 1, 2, XVEC>(a, stream) : launch_cfg<BF16, 4, 1, 2, 4, 1, 2, XVEC>(a, stream);
  // Prefill: the largest tile that still gives the chip about a block per CU.
  auto blocks = [&](int bm, int bn) { return (long long)((a.km.n_keep + bn - 1) / bn) * ((a.M + bm - 1) / bm); };
  constexpr long long kEnough = 192;
  // 128 x 256: eight waves side by side over rows, 8 x 2 fragments each, two groups per wave and slab (a block barrier per
  // 256 columns) and two slabs of weight loads in flight
  // (bfloat16: with the longer unpack two slabs of weight loads in flight do not fit 256 registers; one does)
  // 256 x 256 on a persistent grid (prefill_kernel.h), where its tiles fill the chip in fewer, longer rounds than
  // twice as many 128 x 256 tiles would: a round of it takes about 1.8 rounds of those
  // (gate / up at 4096 tokens 412 against 472 us in the same process, down 389 against 477, gate / up at 1000 tokens 131 against 164)
  if constexpr (XVEC == 1) {
    if (prefill_serves(a) && blocks(256, 256) >= kEnough) {
      const long long cus = prefill_grid_limit();
      const long long rounds_big = (blocks(256, 256) + cus - 1) / cus, rounds_std = (blocks(128, 256) + cus - 1) / cus;
      if (rounds_big * 18 < rounds_std * 10) return launch_prefill_cfg<BF16, 16, 2, 8, 1, 1, 8, 2, 1>(a, stream);
    }
  }
  if (blocks(128, 256) >= kEnough) {
    if constexpr (BF16) return launch_cfg<BF16, 8, 2, 8, 1, 2, 1, XVEC>(a, stream);
    else return launch_cfg<BF16, 8, 2, 8, 1, 2, 2, XVEC>(a, stream);
  }
  if (blocks(64, 256) >= kEnough) return launch_cfg<BF16, 4, 2, 8, 1, 2, 2, XVEC>(a, stream);
  if (blocks(64, 128) >= kEnough) return launch_cfg<BF16, 4, 2, 4, 2, 2, 1, XVEC>(a, stream);   // K split over two waves
  // few tiles whatever the shape (e.g. 4096 rows at 128 or 256 tokens): 32 tokens x 128 rows, K over two waves
  // (down_proj at 256 tokens: 61 us against 77 us with 64 x 64 tiles)
  return launch_cfg<BF16, 2, 2, 4, 2, 2, 1, XVEC>(a, stream);
}

// the staging mode of the activations, then the tile shape
template <bool BF16>
static hipError_t launch_gemm_fmt(const LinearArgs& a, hipStream_t stream) {
  // 128-bit x loads: a column prefix (global loads of any size may start on any 2-byte boundary on
  // this target, so odd leading dimensions such as k_keep = 12185 qualify), or column segments
  // whose stride is a multiple of 8 and that keep at least 8 columns each
  if (a.km.cs_stride == 0) return a.km.k_keep >= 8 ? launch_m<1, BF16>(a, stream) : launch_m<0, BF16>(a, stream);
  if (a.km.cs_stride % 8 == 0 && a.km.cs_keep >= 8) return launch_m<2, BF16>(a, stream);
  return launch_m<0, BF16>(a, stream);
}

}  // namespace uniql
