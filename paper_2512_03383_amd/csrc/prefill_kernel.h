// W4A16 GEMM on MFMA for prompts (thousands of tokens) whose kept columns are a prefix of the row: 256 tokens x 256
// rows per block on a persistent grid.
//
// Same "direct-B" scheme as w4_mfma_kernel (mfma_kernel.h): a lane's 128-bit load of packed codes is the weight
// operand of four consecutive v_mfma_f32_16x16x32 steps after a register unpack, only the activations pass through
// LDS (slab layout, swizzle and pair order as there).  What differs is how much the vector ALU has to do per matrix
// instruction.  A SIMD does not hide vector instructions behind a running matrix instruction: with V of them per
// matrix instruction the pair takes max(17.5, 12 + 4 V) clocks.  The general kernel runs at V = 2.97 (1.6 of unpack,
// the rest address arithmetic and masking of the activation staging).  Here
//  - a wave owns 16 token fragments x 2 row fragments (256 tokens x 32 rows; eight waves side by side over 256 rows),
//    so an unpacked weight fragment feeds 16 matrix instructions instead of 8: 0.8 of unpack per matrix instruction;
//  - activations and weights are fetched through buffer resources: one VGPR offset per thread that never changes,
//    the per-unit and per-iteration parts are scalar, rows past the last token return zeros by the range check; the
//    LDS address of a thread's units differs by a constant, so the writes carry immediate offsets;
//  - beside the 128 accumulator registers there is room for two sets of eight activation fragments (a step runs in
//    two phases; the fragments of the next phase are read from LDS while the current phase multiplies) because the
//    staging registers hold only a quarter of a slab's units at a time and one slab of weight loads is in flight;
//    the only branch-free way found to drop the column mask of the staging from the common path (two loops under a
//    uniform branch) cost 8 to 19 % and is not used;
//  - the matrix instruction takes the weights as its first operand, so a lane ends up with four consecutive output
//    rows of one token and stores them with one 8-byte store;
//  - the grid is persistent (see the kernel).
// The sums are formed in the same order as in w4_mfma_kernel: the outputs are bit-identical.
#pragma once
#include "common.h"

namespace uniql {

// AF token fragments and BF row fragments of 16 per wave, WN waves side by side over rows, S2 groups of 128 columns
// per slab (one block barrier per slab), PW slabs of weight loads in flight.  AH token fragments are read from LDS
// per phase of a step, into a second set of registers while the current phase multiplies when ADB is set; the staging
// registers hold UPP units at a time.
//
// The grid is persistent: about one block per compute unit (the slabs take most of its LDS), each walking over tiles.
// A block that ended with its tile would leave its compute unit idle from the first load of the next block until
// that block's first slab is in LDS, and again while the last stores drain (together an eighth of the time at
// 4096 columns); here the first loads of the next tile are issued before the output of the current one is
// converted and stored.
template <int AF, int BF, int WN, int S2, int PW, bool BF16, int AH = (AF > 8 ? 8 : AF), int UPP = 8, int ADB = 1>
__global__ __launch_bounds__(WN * 64) void w4_prefill_kernel(LinearArgs a, int nrt, int ntt) {
  constexpr int NT = WN * 64;
  constexpr int BM = 16 * AF, BN = WN * BF * 16;
  constexpr int SC = S2 * 128, NCH = SC / 8;     // columns and 8-column chunks per slab
  constexpr int UNITS = BM * NCH;                // 16-byte units (8 columns of one token) per slab
  constexpr int UPT = UNITS / NT;                // units per thread
  constexpr int TSTEP = NT / NCH;                // tokens between a thread's consecutive units
  static_assert(UNITS % NT == 0 && NT % NCH == 0 && TSTEP % 16 == 0, "unit u = tid + i * NT: same chunk, token + i * TSTEP");
  constexpr int NPH = AF / AH;                   // phases per step
  static_assert(AF % AH == 0, "phases split the token fragments evenly");
  constexpr int XP = UPT > UPP ? UPT / UPP : 1;  // the staging registers are filled and drained in XP parts of UPP units
  constexpr int UPQ = UPT / XP;
  static_assert(UPT % XP == 0 && BN * S2 <= NT, "one thread per (row, group) of a slab");
  static_assert(XP == 1 || (S2 * 4 * NPH) % XP == 0, "parts change at phase boundaries");

  extern __shared__ __align__(16) unsigned char smem[];
  uint4* xs = reinterpret_cast<uint4*>(smem);                                               // [2][NCH][BM]
  uint32_t* szs = reinterpret_cast<uint32_t*>(smem + (size_t)2 * UNITS * sizeof(uint4));    // [2][BN][S2]: scale | zero << 16

  const KeepMap& km = a.km;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wn = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 15, ks = lane >> 4;
  const int words_per_row = a.K_total >> 3, groups_per_row = a.K_total / kGroup;
  const int ngroups = (km.k_span + kGroup - 1) / kGroup;
  const int nit = (ngroups + S2 - 1) / S2;
  const int nit_pw = (nit + PW - 1) / PW * PW;   // loop trip count; the extra iterations multiply zeros
  const int kv = km.k_keep & ~7;                 // whole 8-column blocks of kept columns; the rest is added in the epilogue
  const int ldx = (int)a.ldx;

  // Tiles of this block.  Consecutive blocks of a launch go to the eight dies (XCDs) in turn, each with an L2 of its
  // own, so block b runs on die b % 8.  The tiles are numbered along a walk that takes kTokTilesPerPass token tiles
  // at a time and, inside that, row tile by row tile; a die owns a contiguous stretch of the walk and its blocks take
  // consecutive tiles of it round by round, so that the tiles a die works on at any time share their weight rows and
  // activation slabs through that die's L2.
  constexpr int kDies = 8, kTokTilesPerPass = 4;
  const int nb = nrt * ntt;
  int q, q_step, q_end, L0;
  if (gridDim.x % kDies == 0) {
    const int die = blockIdx.x % kDies;
    q = blockIdx.x / kDies, q_step = gridDim.x / kDies;
    q_end = nb / kDies + (die < nb % kDies ? 1 : 0);
    L0 = die * (nb / kDies) + min(die, nb % kDies);
  } else {
    q = blockIdx.x, q_step = gridDim.x, q_end = nb, L0 = 0;
  }
  if (q >= q_end) return;
  auto tile_of = [&](int qq, int& rt, int& tt) {
    const int L = L0 + qq;
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
  };

  typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
  constexpr uint32_t kRsrcWord3 = 0x00020000u;
  const __amdgpu_buffer_rsrc_t rw =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(a.qweight), 0, a.N_total * words_per_row * 4, kRsrcWord3);

  // ---- what depends on the tile
  int n0, m0;
  __amdgpu_buffer_rsrc_t rx;   // the activations of the tile's tokens: rows past the last token lie beyond it and read as zero
  int woff[BF];                // byte offset of each of this lane's weight fragments (row clamped: every address stays valid)
  size_t sz_row;               // this thread's row of the scale / zero staging
  auto set_tile = [&](int qq) {
    int rt, tt;
    tile_of(qq, rt, tt);
    n0 = rt * BN, m0 = tt * BM;
    const int rows_here = a.M - m0 < BM ? a.M - m0 : BM;
    rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<half_t*>(a.x + (size_t)m0 * a.ldx), 0,
                                           ((rows_here - 1) * ldx + km.k_keep) * 2, kRsrcWord3);
#pragma unroll
    for (int bf = 0; bf < BF; ++bf) {
      int rc = n0 + (wn * BF + bf) * 16 + n;
      rc = rc < km.n_keep ? rc : km.n_keep - 1;
      woff[bf] = (stored_row(km, rc) * words_per_row + ks * 4) * 4;
    }
    int rc = n0 + tid / S2;
    rc = rc < km.n_keep ? rc : km.n_keep - 1;
    sz_row = (size_t)stored_row(km, rc) * groups_per_row;
  };
  auto load_w = [&](int it, u32x4_t (&t)[S2][BF]) {
#pragma unroll
    for (int s2 = 0; s2 < S2; ++s2) {
      int g = it * S2 + s2;
      g = g < ngroups ? g : ngroups - 1;   // past the end: a valid, redundant load (x is zero there)
#pragma unroll
      for (int bf = 0; bf < BF; ++bf) t[s2][bf] = __builtin_amdgcn_raw_buffer_load_b128(rw, woff[bf], g * 64, 0);
    }
  };
  const bool sz_owner = tid < BN * S2;   // one thread per (row, group) of a slab
  auto fetch_sz = [&](int it, uint32_t& sbits, uint32_t& z) {
    int g = it * S2 + tid % S2;
    g = g < ngroups ? g : ngroups - 1;
    sbits = a.scales[sz_row + g];
    z = a.zeros ? a.zeros[sz_row + g] : 8u;   // no zero points: the symmetric scheme, z = 8
  };

  // x staging.  Unit i of this thread: token tk0 + i * TSTEP, chunk cb of the slab.
  const int tk0 = tid / NCH, cb = tid % NCH;
  const int xoff0 = (tk0 * ldx + cb * 8) * 2;                       // bytes, inside the tile's resource
  const int swz_cb = ((cb >> 2) & 3) | ((cb & 3) << 2);
  uint4* const xdst = xs + cb * BM + (tk0 ^ swz_cb);                // + i * TSTEP + buf * UNITS
  u32x4_t xr[UPQ];
  auto fetch_x = [&](int it, int part) {
#pragma unroll
    for (int j = 0; j < UPQ; ++j) {
      const int i = part * UPQ + j;
      xr[j] = __builtin_amdgcn_raw_buffer_load_b128(rx, xoff0 + (i * TSTEP * ldx + it * SC) * 2, 0, 0);
    }
  };
  // registers -> LDS in the pair order of the unpack, (0,4) (1,5) (2,6) (3,7): one byte permute per output word.
  // Only the slab with the last kept columns has chunks to clear (those not wholly below kv).
  auto store_x = [&](int it, int part) {
    const int buf = it & 1;
    const int nfull = (kv - it * SC) >> 3;          // chunks of this slab that lie wholly below kv (may be negative)
    const bool clear = nfull < NCH;                 // uniform
    const uint32_t m = (!clear || cb < nfull) ? 0xffffffffu : 0u;
#pragma unroll
    for (int j = 0; j < UPQ; ++j) {
      const int i = part * UPQ + j;
      u32x4_t r = xr[j];
      if (clear) { r.x &= m; r.y &= m; r.z &= m; r.w &= m; }
      xdst[buf * UNITS + i * TSTEP] =
          make_uint4(__builtin_amdgcn_perm(r.z, r.x, 0x05040100u), __builtin_amdgcn_perm(r.z, r.x, 0x07060302u),
                     __builtin_amdgcn_perm(r.w, r.y, 0x05040100u), __builtin_amdgcn_perm(r.w, r.y, 0x07060302u));
    }
  };

  const Magic mg = make_magic();
  u32x4_t ring[PW][S2][BF];
  uint32_t sz_s = 0, sz_z = 0;
  // the first loads of a tile: PW slabs of weights, the scales / zero points and the first part of the activations of slab 0
  auto first_loads = [&]() {
#pragma unroll
    for (int p = 0; p < PW; ++p) load_w(p, ring[p]);
    if (sz_owner) fetch_sz(0, sz_s, sz_z);
    fetch_x(0, 0);
  };
  set_tile(q);
  first_loads();

  for (;;) {
    // slab 0 to LDS (every wave is past the last read of the previous tile: its main loop ends with a barrier)
    store_x(0, 0);
#pragma unroll
    for (int part = 1; part < XP; ++part) {
      fetch_x(0, part);
      store_x(0, part);
    }
    if (sz_owner) szs[tid] = sz_s | (sz_z << 16);
    __syncthreads();

    float4_t acc[AF][BF];
#pragma unroll
    for (int af = 0; af < AF; ++af)
#pragma unroll
      for (int bf = 0; bf < BF; ++bf) acc[af][bf] = float4_t{0.f, 0.f, 0.f, 0.f};

    for (int it0 = 0; it0 < nit_pw; it0 += PW) {
#pragma unroll
      for (int p = 0; p < PW; ++p) {
        const int it = it0 + p;
        const int buf = it & 1;
        uint32_t szv[S2][BF];
#pragma unroll
        for (int s2 = 0; s2 < S2; ++s2)
#pragma unroll
          for (int bf = 0; bf < BF; ++bf) szv[s2][bf] = szs[(buf * BN + (wn * BF + bf) * 16 + n) * S2 + s2];
        // the next slab travels to registers while this one is multiplied (past the last slab: offsets beyond kv, cleared)
        fetch_x(it + 1, 0);
        if (sz_owner) fetch_sz(it + 1, sz_s, sz_z);

#pragma unroll
        for (int s2 = 0; s2 < S2; ++s2) {
          typename GroupOf<BF16>::type gq[BF];
          uint32_t wv[BF][4];
#pragma unroll
          for (int bf = 0; bf < BF; ++bf) {
            const u32x4_t w = ring[p][s2][bf];
            gq[bf] = make_group<BF16>(szv[s2][bf] & 0xffffu, szv[s2][bf] >> 16);
            wv[bf][0] = w.x; wv[bf][1] = w.y; wv[bf][2] = w.z; wv[bf][3] = w.w;
          }
          const uint4* xb = xs + (buf * NCH + s2 * 16 + ks * 4) * BM;
          // A step (one word of every weight fragment, 32 columns) runs in NPH phases of AH token fragments.  While a
          // phase multiplies, the activation fragments of the next phase are read from LDS and a share of the next
          // step's weight words is unpacked.
          uint4 av[ADB ? 2 : 1][AH], wf[2][BF];
          auto read_a = [&](int ph, uint4 (&ao)[AH]) {
            const int t = ph / NPH, h = ph % NPH;
#pragma unroll
            for (int j = 0; j < AH; ++j) ao[j] = xb[t * BM + (h * AH + j) * 16 + (n ^ (ks | (t << 2)))];
          };
          read_a(0, av[0]);
#pragma unroll
          for (int bf = 0; bf < BF; ++bf) wf[0][bf] = dequant_word4<BF16>(wv[bf][0], gq[bf], mg);
#pragma unroll
          for (int ph = 0; ph < 4 * NPH; ++ph) {
            const int t = ph / NPH, h = ph % NPH;
            if (!ADB && ph > 0) read_a(ph, av[0]);
            if (ph + 1 < 4 * NPH) {
              if (ADB) read_a(ph + 1, av[(ph + 1) & 1]);
              if (t < 3) {
#pragma unroll
                for (int bf = (h * BF + NPH - 1) / NPH; bf < ((h + 1) * BF + NPH - 1) / NPH; ++bf)
                  wf[(t + 1) & 1][bf] = dequant_word4<BF16>(wv[bf][t + 1], gq[bf], mg);
              }
            }
#pragma unroll
            for (int j = 0; j < AH; ++j)
#pragma unroll
              for (int bf = 0; bf < BF; ++bf)
                acc[h * AH + j][bf] = mfma_16x16x32<BF16>(wf[t & 1][bf], av[ADB ? (ph & 1) : 0][j], acc[h * AH + j][bf]);
            __builtin_amdgcn_sched_barrier(0);   // phases stay in program order: the registers are sized for that
            if constexpr (XP > 1) {   // the staging registers change over to their next part at even distances
              constexpr int kEvery = S2 * 4 * NPH / XP;
              const int done = s2 * 4 * NPH + ph + 1;
              if (done % kEvery == 0 && done / kEvery < XP) {
                store_x(it + 1, done / kEvery - 1);
                fetch_x(it + 1, done / kEvery);
              }
            }
          }
        }
        load_w(it + PW, ring[p]);   // refill the ring slot (clamped past the end)
        store_x(it + 1, XP - 1);
        if (sz_owner) szs[((it + 1) & 1) * BN * S2 + tid] = sz_s | (sz_z << 16);
        __syncthreads();
      }
    }

    // ---- the next tile's first loads, then this tile's output
    const int en0 = n0, em0 = m0;
    q += q_step;
    const bool more = q < q_end;
    if (more) {
      set_tile(q);
      first_loads();
    }

    // Lane l holds, for fragment (af, bf): token (l % 16), rows 4 * (l / 16) + v.
    if (kv < km.k_keep) {
      // the kept columns kv .. k_keep-1 (fewer than 8: one word of one group per row), in fp32
      for (int j = 0; kv + j < km.k_keep; ++j) {
        float xv[AF];
#pragma unroll
        for (int af = 0; af < AF; ++af) {
          const int tok = em0 + af * 16 + n;
          xv[af] = in16<BF16>(a.x[(size_t)(tok < a.M ? tok : a.M - 1) * a.ldx + kv + j]);
        }
#pragma unroll
        for (int bf = 0; bf < BF; ++bf)
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            int rc = en0 + (wn * BF + bf) * 16 + 4 * ks + v;
            rc = rc < km.n_keep ? rc : km.n_keep - 1;
            const size_t row = (size_t)stored_row(km, rc);
            const uint32_t word = a.qweight[row * words_per_row + (kv >> 3)];
            const size_t gi = row * groups_per_row + (kv >> 7);
            const float sf = in16<BF16>(__builtin_bit_cast(half_t, a.scales[gi]));
            const int z = a.zeros ? a.zeros[gi] : 8;
            const int qv = (int)((word >> (4 * j)) & 15u);
            const float w = in16<BF16>(out16<BF16>((float)(qv - z) * sf));   // the canonical 16-bit weight
#pragma unroll
            for (int af = 0; af < AF; ++af) acc[af][bf][v] = __builtin_fmaf(xv[af], w, acc[af][bf][v]);
          }
      }
    }
    typedef uint32_t u32x2_u2 __attribute__((ext_vector_type(2), aligned(2)));
#pragma unroll
    for (int af = 0; af < AF; ++af) {
      const int tok = em0 + af * 16 + n;
      if (tok >= a.M) continue;
      half_t* yrow = a.y + (size_t)tok * a.ldy;
#pragma unroll
      for (int bf = 0; bf < BF; ++bf) {
        const int rc = en0 + (wn * BF + bf) * 16 + 4 * ks;
        half_t o[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) o[v] = out16<BF16>(acc[af][bf][v]);
        if (rc + 4 <= km.n_keep) {
          u32x2_u2 pk;
          pk.x = (uint32_t)__builtin_bit_cast(uint16_t, o[0]) | ((uint32_t)__builtin_bit_cast(uint16_t, o[1]) << 16);
          pk.y = (uint32_t)__builtin_bit_cast(uint16_t, o[2]) | ((uint32_t)__builtin_bit_cast(uint16_t, o[3]) << 16);
          *reinterpret_cast<u32x2_u2*>(yrow + rc) = pk;
        } else {
#pragma unroll
          for (int v = 0; v < 4; ++v)
            if (rc + v < km.n_keep) yrow[rc + v] = o[v];
        }
      }
    }
    if (!more) break;
  }
}

// Whether w4_prefill_kernel's 32-bit byte offsets reach everything: the whole packed matrix, and a block's rows of x.
static inline bool prefill_serves(const LinearArgs& a) {
  return a.km.cs_stride == 0 && a.km.k_keep >= 8 && (long long)a.N_total * (a.K_total / 2) < (1ll << 31) &&
         a.ldx * 256 * 2 + (long long)a.K_total * 2 + 8192 < (1ll << 31);
}

// Number of compute units of the current device (the size of the persistent grid), looked up once per device.
static inline int prefill_grid_limit() {
  static int cus[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  if (cus[dev] == 0) {
    int v = 0;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) v = 256;
    cus[dev] = v;
  }
  return cus[dev];
}

template <bool BF16, int AF, int BF, int WN, int S2, int PW, int AH = (AF > 8 ? 8 : AF), int UPP = 8, int ADB = 1>
static hipError_t launch_prefill_cfg(const LinearArgs& a, hipStream_t stream) {
  constexpr int BM = 16 * AF, BN = WN * BF * 16, SC = S2 * 128;
  const size_t smem = (size_t)2 * BM * SC * sizeof(half_t) + (size_t)2 * BN * S2 * sizeof(uint32_t);
  auto kern = w4_prefill_kernel<AF, BF, WN, S2, PW, BF16, AH, UPP, ADB>;
  if (smem > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
  }
  const int nrt = (a.km.n_keep + BN - 1) / BN, ntt = (a.M + BM - 1) / BM;
  int blocks = prefill_grid_limit();
  if ((long long)nrt * ntt < blocks) blocks = nrt * ntt;
  if (blocks >= 8) blocks -= blocks % 8;   // whole octets of blocks: the die-aware walk
  hipLaunchKernelGGL(kern, dim3(blocks), dim3(WN * 64), smem, stream, a, nrt, ntt);
  return hipGetLastError();
}

}  // namespace uniql
