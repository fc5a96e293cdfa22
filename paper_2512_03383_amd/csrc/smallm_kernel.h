// W4A16 GEMM for decode batches (2 .. 32 tokens): y[M][n_keep] = x[M][k_keep] * W'^T, bound by the weight stream.
//
// The weight operand is the "direct-B" one of mfma_kernel.h: lane l of a wave holds, for output row l % 16, the 32
// columns of k-slot l / 16 of one quantisation group -- one 128-bit load per lane and group, word t of which feeds
// matrix instruction t of the group; the codes never pass through LDS.  What differs is how the work is cut and how
// the activations travel:
//
//  * A wave owns 16 rows and a contiguous range of groups (the K range is split over KS = 1, 2, 4 or 8 waves of
//    the block, the other 8 / KS waves take further row tiles), chosen on the host so that the launch has about as
//    many waves as the chip holds.  It keeps eight weight loads in flight as a ring: every group consumed re-issues
//    its slot with the group eight further on.  Scales and zero points come eight groups at a time (one 128-bit and
//    one 64-bit load per lane), one batch ahead.
//  * Every wave stages the activations of ITS groups itself, into its own two LDS buffers: 16 (or 32) tokens x 128
//    columns per group, fetched two groups ahead with contiguous 128-bit loads, masked, permuted to the unpack order
//    and written at swizzled token slots (the layout of mfma_kernel.h).  Nothing in the loop is shared between waves,
//    so the loop has no block barrier: the only one stands before the K-split partial sums are added, in a fixed
//    order, by the wave that owns the row tile.
//
// Loads return in issue order, so the first two activation tiles are requested before the first weight and every
// later one between weight loads.
#pragma once
#include "common.h"

namespace uniql {

constexpr int kSmWaves = 8;
constexpr int kSmThreads = kSmWaves * kWave;
constexpr int kSmRing = 8;   // weight tiles in flight per wave = groups per batch of scales
constexpr int kSmPreGroups = 32;   // groups of a row the pre-staged activation image holds

struct SmallMShape {
  int ks;    // waves along K
  int gpw;   // groups per wave
};

// AF: 16-token fragments (1 or 2); XT: tokens staged per group (>= M; 4, 8, 16 or 32); XM: how the activations are
// fetched (0 = element by element through the column map, 1 = column prefix, 2 = column segments whose stride is a
// multiple of 8), as in mfma_kernel.h
// (block: the block's index within its linear -- blockIdx.x when the launch serves one linear)
//
// PRE (column prefixes of at most 32 groups, up to 16 tokens): the block stages the activations of ALL its groups once,
// before the loop -- every thread fetches its share with 128-bit loads issued ahead of the first weight loads, one
// block barrier -- and the loop only reads them.  The per-wave staging above costs as much as the unpack and the
// matrix instructions together, and with two to four waves per SIMD nothing hides it.
//
// GLU (with PRE): the block serves the gate and the up matrix of a gated MLP (Eq. 1) on the same activations -- waves
// with an even index along the rows take the gate rows of a row tile, their odd neighbours the up rows of the same tile
// -- and after the K-split sums the up wave hands its fp32 sums to the gate wave through LDS, which stores
// h = SiLU(g) * u rounded once.
template <int AF, int XT, int XM, bool BF16, bool PRE, bool GLU = false>
__device__ __forceinline__ void smallm_body(const LinearArgs& a_first, const SmallMShape sh, const int block,
                                            const LinearArgs* a_up = nullptr) {
  constexpr bool XVEC = XM == 1, XSEG = XM == 2;
  static_assert(!PRE || (XM == 1 && AF == 1 && XT <= 16), "the pre-staged image: a column prefix, one token fragment");
  static_assert(!GLU || PRE, "gate and up share the block's image of the activations");
  constexpr int D = kSmRing;
  constexpr int BM = 16 * AF;                 // token slots of a staged tile
  constexpr int UPL = XT * 16 / kWave;        // 16-byte units (8 columns of one token) per lane and group
  static_assert(XT * 16 % kWave == 0 && XT <= BM, "whole units per lane");
  constexpr int TILE_UNITS = 16 * BM;         // [16 chunks][BM token slots]

  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int KS = sh.ks, WN = kSmWaves / KS;
  const int wn = wave % WN, wk = wave / WN;
  const int n = lane & 15, ks = lane >> 4;
  const bool is_up = GLU && (wn & 1) != 0;            // wave-uniform
  const LinearArgs& a = is_up ? *a_up : a_first;
  const KeepMap& km = a.km;
  // PRE: one image for the block, [group][16 chunks][XT token slots]; else this wave's two tiles
  uint4* xs = reinterpret_cast<uint4*>(smem) + (PRE ? 0 : (size_t)wave * 2 * TILE_UNITS);
  float* red = reinterpret_cast<float*>(smem + (PRE ? (size_t)kSmPreGroups * 16 * XT : (size_t)kSmWaves * 2 * TILE_UNITS) * sizeof(uint4));   // [8][AF * 4][64]

  const int words_per_row = a.K_total >> 3, groups_per_row = a.K_total / kGroup;
  const int ngroups = (km.k_span + kGroup - 1) / kGroup;
  const int g0 = wk * sh.gpw;
  int ng = ngroups - g0;                      // groups of this wave
  ng = ng < 0 ? 0 : (ng > sh.gpw ? sh.gpw : ng);

  // Every load of the loop goes through a buffer resource, and a load that has nothing to fetch (a group past the
  // wave's last one, a token past M, a pruned block of columns) carries an offset beyond the resource: the hardware
  // returns zeros for it without touching memory.  The loop body is therefore free of branches, which is what lets
  // the compiler count the loads in flight exactly instead of draining them at every join.
  constexpr uint32_t kRsrcWord3 = 0x00020000u;
  constexpr int kNone = (int)0x80000000u;     // as an unsigned offset: beyond every resource (smallm_serves bounds their sizes)
  const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(a.qweight), 0, a.N_total * words_per_row * 4, kRsrcWord3);
  const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(a.scales), 0, a.N_total * groups_per_row * 2, kRsrcWord3);
  const __amdgpu_buffer_rsrc_t rz = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(a.zeros), 0, a.zeros ? a.N_total * groups_per_row : 0, kRsrcWord3);
  const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<half_t*>(a.x), 0, (int)(((long long)(a.M - 1) * a.ldx + km.k_keep) * 2), kRsrcWord3);

  // stored row of this lane's weight fragment (clamped: a lane past the last row re-reads it and stores nothing)
  const int rc = (GLU ? (block * WN + wn) >> 1 : block * WN + wn) * 16 + n;
  const int wrow = stored_row(km, rc < km.n_keep ? rc : km.n_keep - 1);
  typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
  typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
  const int w0 = (wrow * words_per_row + ks * 4 + g0 * 16) * 4;   // bytes
  auto load_w = [&](int i) { return __builtin_amdgcn_raw_buffer_load_b128(rw, i < ng ? w0 + i * 64 : kNone, 0, 0); };

  // scales / zero points of groups g0 + 8 b .. + 7 of the lane's row: one 128-bit and one 64-bit load.  A load whose
  // last 32-bit word lies partly past the end of the array comes back with that word zeroed, valid bytes included, so
  // the window never leaves the row: a batch that would run past the row's last group starts `back` groups earlier
  // (a row has at least 8 groups) and its values are shifted down by as much when the batch becomes current.  `back`
  // is the same for the whole wave.
  struct SZ { u32x4_t s; u32x2_t z; int back; };
  const bool has_z = a.zeros != nullptr;
  auto load_sz = [&](int b) {
    SZ r;
    const int start = g0 + 8 * b;
    int back = start + 8 - groups_per_row;
    back = back < 0 ? 0 : (back > 7 ? 7 : back);   // (7: a batch wholly past the row, never used)
    const int e0 = wrow * groups_per_row + (start < groups_per_row ? start : groups_per_row - 1) - back;
    r.s = __builtin_amdgcn_raw_buffer_load_b128(rs, 2 * e0, 0, 0);
    r.z = __builtin_amdgcn_raw_buffer_load_b64(rz, e0, 0, 0);
    r.back = back;
    return r;
  };
  auto shift_sz = [](const SZ& r) {
    SZ o;
    const unsigned __int128 sv = ((unsigned __int128)r.s.w << 96 | (unsigned __int128)r.s.z << 64 |
                                  (unsigned __int128)r.s.y << 32 | (unsigned __int128)r.s.x) >> (16 * r.back);
    o.s = u32x4_t{(uint32_t)sv, (uint32_t)(sv >> 32), (uint32_t)(sv >> 64), (uint32_t)(sv >> 96)};
    const uint64_t zv = (((uint64_t)r.z.y << 32) | r.z.x) >> (8 * r.back);
    o.z = u32x2_t{(uint32_t)zv, (uint32_t)(zv >> 32)};
    o.back = 0;
    return o;
  };

  // ---- activations.  Unit j of a lane: token (lane + 64 j) / 16, 8-column chunk (lane + 64 j) % 16 of the group.
  auto swz = [](int chunk) { return ((chunk >> 2) & 3) | ((chunk & 3) << 2); };
  const int kv = km.k_keep & ~7;
  struct XRegs {
    u32x4_t v[XM != 0 ? UPL : 1];
    uint32_t e[XM != 0 ? 1 : UPL][8];
    uint32_t ok[XSEG ? UPL : 1];   // XSEG: bit q = half q of the unit is a kept column
  };
  auto fetch_x = [&](int i, XRegs& xr) {
#pragma unroll
    for (int j = 0; j < UPL; ++j) {
      const int u = lane + 64 * j;
      const int tok = u >> 4, cb = u & 15;
      const int k0 = (g0 + i) * kGroup + cb * 8;
      const bool there = tok < a.M && i < ng;
      const int xoff = tok * (int)a.ldx;
      if constexpr (XVEC) {
        // whole 8-column blocks below kv; the up to 7 kept columns from kv on are added in the epilogue
        xr.v[j] = __builtin_amdgcn_raw_buffer_load_b128(rx, there && k0 + 8 <= kv ? 2 * (xoff + k0) : kNone, 0, 0);
      } else if constexpr (XSEG) {
        // a block lies in one segment and its kept columns are its first nk, contiguous in x
        const int seg = k0 / km.cs_stride, off = k0 - seg * km.cs_stride;
        int nk = km.cs_keep - off;
        nk = nk < 0 ? 0 : (nk > 8 ? 8 : nk);
        nk = k0 < km.k_span ? nk : 0;
        const int c = seg * km.cs_keep + off;            // compact column of the block's first column
        // (the 16 bytes at c may run past the token's row into the next one, or past x, where they read as zero: the mask drops them)
        xr.v[j] = __builtin_amdgcn_raw_buffer_load_b128(rx, there && nk > 0 ? 2 * (xoff + c) : kNone, 0, 0);
        xr.ok[j] = (1u << nk) - 1u;
      } else {
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          const int k = k0 + q;
          const int kc = k < km.k_span ? compact_col(km, k) : -1;
          xr.e[j][q] = __builtin_amdgcn_raw_buffer_load_b16(rx, there && kc >= 0 ? 2 * (xoff + kc) : kNone, 0, 0);
        }
      }
    }
  };
  // registers -> LDS: the unit's 8 halves in the pair order of the unpack, (0,4) (1,5) (2,6) (3,7).  With 128-bit
  // loads that is one byte permute per output word (pruned units already arrived as zeros).
  auto store_x = [&](int buf, const XRegs& xr) {
#pragma unroll
    for (int j = 0; j < UPL; ++j) {
      const int u = lane + 64 * j;
      const int tok = u >> 4, cb = u & 15;
      uint4 o;
      if constexpr (XM != 0) {
        u32x4_t r = xr.v[j];
        if constexpr (XSEG) {
          // kept columns are the unit's first nk: a mask per 32-bit word (halves 2 w and 2 w + 1)
          const uint32_t ok = xr.ok[j];
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            const uint32_t m = ((ok >> (2 * w)) & 1u ? 0xffffu : 0u) | ((ok >> (2 * w + 1)) & 1u ? 0xffff0000u : 0u);
            r[w] &= m;
          }
        }
        o = make_uint4(__builtin_amdgcn_perm(r.z, r.x, 0x05040100u), __builtin_amdgcn_perm(r.z, r.x, 0x07060302u),
                       __builtin_amdgcn_perm(r.w, r.y, 0x05040100u), __builtin_amdgcn_perm(r.w, r.y, 0x07060302u));
      } else {
        const uint32_t (&e)[8] = xr.e[j];
        o = make_uint4((e[0] & 0xffffu) | (e[4] << 16), (e[1] & 0xffffu) | (e[5] << 16),
                       (e[2] & 0xffffu) | (e[6] << 16), (e[3] & 0xffffu) | (e[7] << 16));
      }
      xs[(buf * 16 + cb) * BM + (tok ^ swz(cb))] = o;
    }
  };

  float4_t acc[AF];
#pragma unroll
  for (int af = 0; af < AF; ++af) acc[af] = float4_t{0.f, 0.f, 0.f, 0.f};
  const Magic mg = make_magic();

  // ---- prologue: two activation tiles, the first batch of scales, eight weight tiles.  LDS holds the tiles of
  // groups i and i + 1, the registers the one of group i + 2 on its way.
  XRegs xr;
  u32x4_t ring[D];
  SZ sz_cur, sz_nxt;
  if constexpr (PRE) {
    // unit u of the image: token u / (16 G), chunk-of-row u % (16 G) (G = groups of the row's kept span): consecutive
    // lanes fetch consecutive 16 bytes of one token.  XT units per thread cover 32 groups; all are requested before
    // the weights, so they arrive first.
    const int chunks = ngroups * 16;
    u32x4_t pre[XT];
#pragma unroll
    for (int j = 0; j < XT; ++j) {
      const int u = tid + kSmThreads * j;
      const int tok = u / chunks, gc = u - tok * chunks;
      const bool there = tok < a.M && tok < XT && gc * 8 + 8 <= kv;
      pre[j] = __builtin_amdgcn_raw_buffer_load_b128(rx, there ? 2 * (tok * (int)a.ldx + gc * 8) : kNone, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    sz_cur = load_sz(0);
    sz_nxt = sz_cur;
#pragma unroll
    for (int p = 0; p < D; ++p) ring[p] = load_w(p);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < XT; ++j) {
      const int u = tid + kSmThreads * j;
      const int tok = u / chunks, gc = u - tok * chunks;
      const u32x4_t r = pre[j];
      if (tok < XT)
        xs[gc * XT + tok] = make_uint4(__builtin_amdgcn_perm(r.z, r.x, 0x05040100u), __builtin_amdgcn_perm(r.z, r.x, 0x07060302u),
                                       __builtin_amdgcn_perm(r.w, r.y, 0x05040100u), __builtin_amdgcn_perm(r.w, r.y, 0x07060302u));
    }
    __syncthreads();
  } else {
    fetch_x(0, xr);
    __builtin_amdgcn_sched_barrier(0);
    XRegs x1;
    fetch_x(1, x1);
    sz_cur = load_sz(0);
    sz_nxt = sz_cur;
#pragma unroll
    for (int p = 0; p < D; ++p) ring[p] = load_w(p);
    __builtin_amdgcn_sched_barrier(0);
    store_x(0, xr);
    xr = x1;
    __builtin_amdgcn_sched_barrier(0);
  }

  // the walk over the wave's groups; it leaves through the first group past the last one.  The scheduling barriers
  // keep every load where it is written (the scheduler would otherwise sink a load to its first use to save registers).
  [&]() {
    for (int i0 = 0;; i0 += D) {
      if (i0 >= ng) return;
      sz_cur = shift_sz(sz_cur);
#pragma unroll
      for (int p = 0; p < D; ++p) {
        const int i = i0 + p;
        if (i >= ng) return;
        const int buf = p & 1;
        if constexpr (!PRE) {
          store_x(buf ^ 1, xr);      // group i + 1
          fetch_x(i + 2, xr);
        }
        __builtin_amdgcn_sched_barrier(0);
        const uint32_t sv[4] = {sz_cur.s.x, sz_cur.s.y, sz_cur.s.z, sz_cur.s.w};
        const uint32_t zv[2] = {sz_cur.z.x, sz_cur.z.y};
        const uint32_t sbits = (sv[p >> 1] >> (16 * (p & 1))) & 0xffffu;
        const uint32_t z = has_z ? (zv[p >> 2] >> (8 * (p & 3))) & 0xffu : 8u;   // no zero points: the symmetric scheme, z = 8
        const typename GroupOf<BF16>::type gq = make_group<BF16>(sbits, z);
        const uint32_t wv[4] = {ring[p].x, ring[p].y, ring[p].z, ring[p].w};
        // PRE: chunk ks * 4 + t of group g0 + i, token slot n (lanes past the staged tokens re-read a staged one: their
        // rows of the product are never stored)
        const uint4* xb = PRE ? xs + ((g0 + i) * 16 + ks * 4) * XT + (n & (XT - 1)) : xs + (buf * 16 + ks * 4) * BM;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const uint4 b = dequant_word4<BF16>(wv[t], gq, mg);
          if constexpr (PRE) {
            acc[0] = mfma_16x16x32<BF16>(xb[t * XT], b, acc[0]);
          } else {
#pragma unroll
            for (int af = 0; af < AF; ++af)
              acc[af] = mfma_16x16x32<BF16>(xb[t * BM + af * 16 + (n ^ (ks | (t << 2)))], b, acc[af]);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
        ring[p] = load_w(i + D);
        if (p == D - 3) sz_nxt = load_sz(i0 / D + 1);   // the next batch of scales, late so that it is live for three groups only
        __builtin_amdgcn_sched_barrier(0);
      }
      sz_cur = sz_nxt;
    }
  }();

  // ---- K-split partial sums, added in a fixed order by the wave that owns the row tile.
  // Lane l holds, for fragment af: row (l % 16), tokens 16 af + 4 (l / 16) + v.
  if (KS > 1) {
    float* mine = red + (size_t)wave * AF * 4 * 64;
#pragma unroll
    for (int af = 0; af < AF; ++af)
#pragma unroll
      for (int v = 0; v < 4; ++v) mine[(af * 4 + v) * 64 + lane] = acc[af][v];
    __syncthreads();
    if constexpr (!GLU) {
      if (wk != 0) return;
    }
    for (int k2 = 1; k2 < KS && wk == 0; ++k2) {
      const float* other = red + (size_t)(k2 * WN + wn) * AF * 4 * 64;
#pragma unroll
      for (int af = 0; af < AF; ++af)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[af][v] += other[(af * 4 + v) * 64 + lane];
    }
  }
  const bool owner = wk == 0;   // (GLU keeps every wave to the last barrier)
  if constexpr (XVEC) {
    // the kept columns kv .. k_keep-1 (fewer than 8: one word of one group per row), in fp32
    if (kv < km.k_keep && owner) {
      const uint32_t word = a.qweight[(size_t)wrow * words_per_row + (kv >> 3)];
      const size_t gi = (size_t)wrow * groups_per_row + (kv >> 7);
      const float sf = in16<BF16>(__builtin_bit_cast(half_t, a.scales[gi]));
      const int z = a.zeros ? a.zeros[gi] : 8;
      for (int j = 0; kv + j < km.k_keep; ++j) {
        const int q = (int)((word >> (4 * j)) & 15u);
        const float w = in16<BF16>(out16<BF16>((float)(q - z) * sf));   // the canonical 16-bit weight
#pragma unroll
        for (int af = 0; af < AF; ++af)
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const int tok = af * 16 + 4 * ks + v;
            const float xv = in16<BF16>(a.x[(size_t)(tok < a.M ? tok : a.M - 1) * a.ldx + kv + j]);
            acc[af][v] = __builtin_fmaf(xv, w, acc[af][v]);
          }
      }
    }
  }
  if constexpr (GLU) {
    // the up wave's region of the partial-sum buffer is its own (the K-split sums above read the regions of the waves
    // further along K only): u through it to the gate wave next door
    float* mine = red + (size_t)wave * 4 * 64;
    if (owner && is_up) {
#pragma unroll
      for (int v = 0; v < 4; ++v) mine[v * 64 + lane] = acc[0][v];
    }
    __syncthreads();
    if (owner && !is_up) {
      const float* theirs = red + (size_t)(wave + 1) * 4 * 64;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int tok = 4 * ks + v;
        const float g = acc[0][v], u = theirs[v * 64 + lane];
        if (tok < a.M && rc < km.n_keep)
          a.y[(size_t)tok * a.ldy + rc] = out16<BF16>(g * u * __builtin_amdgcn_rcpf(1.0f + __expf(-g)));
      }
    }
    return;
  }
#pragma unroll
  for (int af = 0; af < AF; ++af)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int tok = af * 16 + 4 * ks + v;
      if (tok < a.M && rc < km.n_keep) a.y[(size_t)tok * a.ldy + rc] = out16<BF16>(acc[af][v]);
    }
}

// the gated MLP's hidden vectors of a decode batch: gate and up in one launch, h = SiLU(g) * u
template <int XT, bool BF16, int OCC>
__global__ __launch_bounds__(kSmThreads, OCC) void w4_smallm_glu_kernel(LinearArgs gate, LinearArgs up, SmallMShape sh) {
  smallm_body<1, XT, 1, BF16, true, true>(gate, sh, (int)blockIdx.x, &up);
}

template <int AF, int XT, int XM, bool BF16, int OCC, bool PRE>
__global__ __launch_bounds__(kSmThreads, OCC) void w4_smallm_kernel(LinearArgs a, SmallMShape sh) {
  smallm_body<AF, XT, XM, BF16, PRE>(a, sh, (int)blockIdx.x);
}

// Up to four linears with the same token count in one launch (q, k, v or gate, up of a decode batch: a launch of this
// size is bound by its latency, not by its bytes).  Every block does exactly what it does in a launch of its own
// linear, so the results are the same bits.
struct SmallMBatch {
  LinearArgs p[kMaxBatch];
  SmallMShape sh[kMaxBatch];
  int first_block[kMaxBatch];
  int n;
};
template <int AF, int XT, int XM, bool BF16, int OCC, bool PRE>
__global__ __launch_bounds__(kSmThreads, OCC) void w4_smallm_batch_kernel(SmallMBatch b) {
  int pi = 0;
#pragma unroll
  for (int i = 1; i < kMaxBatch; ++i) pi += (i < b.n && (int)blockIdx.x >= b.first_block[i]) ? 1 : 0;
  // by value: the member's fields come from the argument buffer in a few wide scalar loads up front
  const LinearArgs a = b.p[pi];
  const SmallMShape sh = b.sh[pi];
  smallm_body<AF, XT, XM, BF16, PRE>(a, sh, (int)blockIdx.x - b.first_block[pi]);
}

// K split and groups per wave: the fewest waves along K that give the launch at least 1280 waves (five per compute
// unit; measured on 888 row tiles x 28 groups at 8 tokens: 16.0 / 11.1 / 11.5 / 13.4 us with K over 1 / 2 / 4 / 8
// waves), with at least four groups per wave
static inline SmallMShape smallm_shape(const LinearArgs& a) {
  const int row_tiles = (a.km.n_keep + 15) / 16;
  const int ngroups = (a.km.k_span + kGroup - 1) / kGroup;
  int ks = 1;
  while (ks < kSmWaves && row_tiles * ks < 1280 && (ngroups + 2 * ks - 1) / (2 * ks) >= 4) ks *= 2;
  return SmallMShape{ks, (ngroups + ks - 1) / ks};
}

// (waves per SIMD the compiler may count on: four with up to 8 staged tokens, which leaves 128 registers and lets two
// blocks share a compute unit; with 16 tokens that budget spills and measured 15.5 against 12.4 us)
// LDS of a block: the waves' private tiles, or the block's image of the activations, and the K-split partial sums
template <int AF, int XT, bool PRE>
static constexpr size_t smallm_lds() {
  return (PRE ? (size_t)kSmPreGroups * 16 * XT : (size_t)kSmWaves * 2 * 16 * 16 * AF) * sizeof(uint4) +
         (size_t)kSmWaves * AF * 4 * 64 * sizeof(float);
}

template <int AF, int XT, int XM, bool BF16, bool PRE = false, int OCC = ((XT <= 8 && XM != 0) ? 4 : 2)>
static hipError_t smallm_launch(const LinearArgs& a, hipStream_t stream) {
  const SmallMShape sh = smallm_shape(a);
  const int wn = kSmWaves / sh.ks;
  const int row_tiles = (a.km.n_keep + 15) / 16;
  constexpr size_t smem = smallm_lds<AF, XT, PRE>();
  auto kern = w4_smallm_kernel<AF, XT, XM, BF16, OCC, PRE>;
  if (smem > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(kern, dim3((row_tiles + wn - 1) / wn), dim3(kSmThreads), smem, stream, a, sh);
  return hipGetLastError();
}

// 2 .. 32 tokens, rows of at least 8 groups; the kernel addresses the arrays and x with signed 32-bit byte offsets
static inline bool smallm_serves(const LinearArgs& a) {
  const long long lim = 1ll << 31;
  return a.M >= 2 && a.M <= 32 && a.K_total >= 8 * kGroup && (long long)a.N_total * a.K_total / 2 < lim &&
         ((long long)(a.M - 1) * a.ldx + a.km.k_keep) * 2 < lim;
}

// the pre-staged image serves: a column prefix (the caller's XM = 1) of at most 32 groups, up to 16 tokens
static inline bool smallm_pre(const LinearArgs& a) {
  return a.M <= 16 && (a.km.k_span + kGroup - 1) / kGroup <= kSmPreGroups && smallm_shape(a).ks <= 2;
}

// which linears this kernel takes (prefix: the activations are a column prefix of at least 8 columns): up to 8 tokens
// all it serves; beyond that the short matrices, and the tall ones when their activations can be staged once per block
static inline bool smallm_takes(const LinearArgs& a, bool prefix) {
  const int row_tiles = (a.km.n_keep + 15) / 16;
  return smallm_serves(a) && (a.M <= 8 || row_tiles < 600 || (prefix && smallm_pre(a)));
}

template <int XM, bool BF16>
static hipError_t smallm_dispatch(const LinearArgs& a, hipStream_t stream) {
  // column segments: a unit that holds a segment's last kept columns is read as 16 bytes that may run past the end of
  // x; with an odd number of kept columns per segment the last valid element would share a 32-bit word with bytes
  // past the end and come back as zero, so such rules go element by element
  if constexpr (XM == 2) {
    if (a.km.cs_keep % 2 != 0) return smallm_dispatch<0, BF16>(a, stream);
  }
  if constexpr (XM == 1) {
    if (smallm_pre(a)) {
      if (a.M <= 4) return smallm_launch<1, 4, 1, BF16, true>(a, stream);
      if (a.M <= 8) return smallm_launch<1, 8, 1, BF16, true>(a, stream);
      return smallm_launch<1, 16, 1, BF16, true>(a, stream);
    }
  }
  if (a.M <= 4) return smallm_launch<1, 4, XM, BF16>(a, stream);
  if (a.M <= 8) return smallm_launch<1, 8, XM, BF16>(a, stream);
  if (a.M <= 16) return smallm_launch<1, 16, XM, BF16>(a, stream);
  return smallm_launch<2, 32, XM, BF16>(a, stream);
}

template <int AF, int XT, bool BF16, bool PRE = false, int OCC = (XT <= 8 ? 4 : 2)>
static hipError_t smallm_launch_batch(const LinearArgs* a, int n, hipStream_t stream) {
  constexpr size_t smem = smallm_lds<AF, XT, PRE>();
  auto kern = w4_smallm_batch_kernel<AF, XT, 1, BF16, OCC, PRE>;
  if (smem > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
  }
  SmallMBatch b;
  b.n = n;
  int blocks = 0;
  for (int i = 0; i < kMaxBatch; ++i) {
    b.p[i] = a[i < n ? i : 0];
    b.sh[i] = smallm_shape(b.p[i]);
    b.first_block[i] = blocks;
    if (i >= n) continue;
    const int wn = kSmWaves / b.sh[i].ks;
    blocks += ((a[i].km.n_keep + 15) / 16 + wn - 1) / wn;
  }
  hipLaunchKernelGGL(kern, dim3(blocks), dim3(kSmThreads), smem, stream, b);
  return hipGetLastError();
}

// n (2..4) linears of one decode batch in one launch: column prefixes of at least 8 columns, the same token count and
// format (the caller checks), each one a linear that smallm_dispatch<1> would take.  *done = false: not such a set,
// nothing was launched.
template <bool BF16>
static hipError_t smallm_batch(const LinearArgs* a, int n, hipStream_t stream, bool* done) {
  *done = false;
  for (int i = 0; i < n; ++i) {
    if (a[i].km.cs_stride != 0 || a[i].km.k_keep < 8 || a[i].M != a[0].M || !smallm_takes(a[i], true)) return hipSuccess;
  }
  *done = true;
  const int M = a[0].M;
  bool pre = true;
  for (int i = 0; i < n; ++i) pre = pre && smallm_pre(a[i]);
  if (pre) {
    if (M <= 4) return smallm_launch_batch<1, 4, BF16, true>(a, n, stream);
    if (M <= 8) return smallm_launch_batch<1, 8, BF16, true>(a, n, stream);
    return smallm_launch_batch<1, 16, BF16, true>(a, n, stream);
  }
  if (M <= 4) return smallm_launch_batch<1, 4, BF16>(a, n, stream);
  if (M <= 8) return smallm_launch_batch<1, 8, BF16>(a, n, stream);
  if (M <= 16) return smallm_launch_batch<1, 16, BF16>(a, n, stream);
  return smallm_launch_batch<2, 32, BF16>(a, n, stream);
}

template <int XT, bool BF16, int OCC = (XT <= 8 ? 4 : 2)>
static hipError_t smallm_launch_glu(const LinearArgs* p, hipStream_t stream) {
  const SmallMShape sh = smallm_shape(p[0]);
  const int wn = kSmWaves / sh.ks;                 // (at least 4: the K range goes over at most two waves)
  const int row_tiles = (p[0].km.n_keep + 15) / 16;
  constexpr size_t smem = smallm_lds<1, XT, true>();
  auto kern = w4_smallm_glu_kernel<XT, BF16, OCC>;
  if (smem > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(kern, dim3((2 * row_tiles + wn - 1) / wn), dim3(kSmThreads), smem, stream, p[0], p[1], sh);
  return hipGetLastError();
}

// gate (p[0]) and up (p[1]) of a decode batch with h = SiLU(g) * u in one launch: 2..16 tokens, the same kept rows in
// number and the same column prefix (the caller checks), tall matrices whose activations fit the block's image.
// *done = false: not such a pair, nothing was launched.
template <bool BF16>
static hipError_t smallm_glu(const LinearArgs* p, hipStream_t stream, bool* done) {
  *done = false;
  for (int i = 0; i < 2; ++i)
    if (p[i].km.cs_stride != 0 || p[i].km.k_keep < 8 || !smallm_serves(p[i]) || !smallm_pre(p[i])) return hipSuccess;
  *done = true;
  if (p[0].M <= 4) return smallm_launch_glu<4, BF16>(p, stream);
  if (p[0].M <= 8) return smallm_launch_glu<8, BF16>(p, stream);
  return smallm_launch_glu<16, BF16>(p, stream);
}

}  // namespace uniql
