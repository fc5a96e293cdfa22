// Streaming W4A16 GEMV, one token per launch (decode).
//
// The op is bound by the HBM stream of packed nibbles, so the kernel is built
// around that stream: a wave reads a kept row in contiguous 1 KB pieces (64
// lanes x 128-bit), i.e. every lane owns 32 consecutive input columns that lie
// in one quantisation group.  Pruned rows are never touched (row truncation
// saves their bytes); pruned columns are handled by staging the activations
// once per block into LDS at their *stored* column positions with zeros in the
// pruned slots, so the weight stream needs no per-element masking.
//
// Per 32-bit word (8 weights): 1 shift + 4 and-or build exact fp16 codes, 4
// packed subtracts and 4 packed multiplies give the canonical fp16 weights
// RN16((q - z) s); the word's 8-element dot product with the lane's activations is
// taken from the diagonal of one matrix instruction (see consume below), fp32.
//
// The kernel is fully unrolled over the row's 2048-column chunks (template NCH):
// a wave's tiles (row, chunk) are loaded a few tiles ahead (DW in the kernel) and consumed in issue
// order, each as soon as it has arrived, so the arithmetic overlaps the stream
// instead of starting after the last byte.
#pragma once
#include "common.h"

namespace uniql {
namespace gemv {

constexpr int kGemvThreads = 512;
constexpr int kGemvWaves = kGemvThreads / kWave;
constexpr int kChunk = kWave * 32;   // stored columns one wave covers with one 128-bit load per lane

__device__ __forceinline__ float dpp_xor_reduce(float v) {
  // butterfly within each row of 16 lanes with DPP, then across rows through the LDS crossbar
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true));  // row_half_mirror
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, true));  // row_mirror
  v += __shfl_xor(v, 16);
  v += __shfl_xor(v, 32);
  return v;
}

struct Tile {
  uint4 w;          // 32 packed codes
  uint32_t sbits;   // fp16 scale bits of the lane's group
  uint32_t z;       // zero point of the lane's group
};

// LDS slot of the 8 stored columns k0..k0+7, k0 = c*2048 + l*32 + t*8: [c][t][l], 16 bytes,
// halves ordered (k0,k0+4,k0+1,k0+5,k0+2,k0+6,k0+3,k0+7): dword p pairs with the dequantised
// pair (w_p, w_{p+4}), and a wave reads one t-plane of a chunk with consecutive addresses.
__device__ __forceinline__ int unit_k0(int u) { return (u >> 8) * kChunk + ((u >> 2) & 63) * 32 + (u & 3) * 8; }
__device__ __forceinline__ int unit_slot(int u) { return ((u >> 8) * 4 + (u & 3)) * 64 + ((u >> 2) & 63); }

__device__ __forceinline__ uint4 pack_unit(const half_t v[8]) {
  half2_t p0 = {v[0], v[4]}, p1 = {v[1], v[5]}, p2 = {v[2], v[6]}, p3 = {v[3], v[7]};
  return make_uint4(as_u32(p0), as_u32(p1), as_u32(p2), as_u32(p3));
}

// Branch-free map of a stored column to its compact column.  A column prefix is the
// one-segment case: stride 2^30, keep k_keep.
struct ColMap {
  int stride, keep;
};
__device__ __forceinline__ ColMap make_colmap(const KeepMap& km) {
  ColMap c;
  c.stride = km.cs_stride ? km.cs_stride : (1 << 30);
  c.keep = km.cs_stride ? km.cs_keep : km.k_keep;
  return c;
}

// R rows per wave.  XVEC: the kept columns are a prefix, or segments of a stride that is a multiple of 8, so x is
// fetched with 128-bit loads; otherwise element by element through the column map (segment
// strides are at least 8, so a unit of 8 columns wraps at most once).  NCH: chunks per row,
// compile-time, 1..8 (NCH = 0: run-time chunk count for rows longer than 8 chunks).
// The launch carries up to kMaxBatch independent linears (same R / XVEC / NCH, e.g. q, k and v
// of one layer, or gate and up): problem i owns the blocks [first_block[i], first_block[i+1]).
// EPI = 1 (R = 1 only): problems with batch.rf.heads[i] > 0 get the rotary embedding of their output as
// an epilogue.  Their blocks own four kept pairs instead of eight consecutive rows: waves 0..3 compute
// the first-half rows of the pairs, waves 4..7 the second-half rows, the two fp32 sums of a pair meet
// in LDS and are rotated before the one rounding to fp16.  The pair's sin / cos are formed while the
// weight stream is in flight, with the arithmetic of the stand-alone RoPE kernel.
// EPI = 2: the launch holds exactly two problems, gate and up of a gated MLP (Eq. 1), over the same x.
// Waves 0..3 of a block compute R gate rows each, waves 4..7 the up rows of the same indices; the
// sums meet in LDS and h = SiLU(gate) * up is written to the first problem's y.
// ZP = false: the members have no zero points (every z = 8, Eq. 3's symmetric scheme) and none is loaded.
// BF16: scales, x and y are bfloat16 and so are the dequantised weights (fp32 arithmetic, one rounding, bf16 MFMA).
template <int R, bool XVEC, int NCH, int EPI, bool ZP, bool BF16>
__global__ __launch_bounds__(kGemvThreads) void w4_gemv_kernel(GemvBatch batch, int m, int nchunk_rt) {
  constexpr bool ROPE = EPI == 1, GLU = EPI == 2;
  static_assert(!ROPE || R == 1, "the rotary epilogue pairs single-row waves");
  extern __shared__ __align__(16) unsigned char smem[];
  uint4* xs = reinterpret_cast<uint4*>(smem);   // [nchunk][4][64] units of 8 halves

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  int pi = 0;
  if (GLU) {
    pi = wave >> 2;   // wave-uniform: gate for the lower four waves, up for the upper four
  } else {
#pragma unroll
    for (int i = 1; i < kMaxBatch; ++i) pi += (i < batch.n && (int)blockIdx.x >= batch.first_block[i]) ? 1 : 0;
  }
  // by value: the member's fields are fetched from the argument buffer in a few wide scalar loads up
  // front, not one dependent load at a time where each is first used
  const LinearArgs a = batch.p[pi];
  const int block_id = (int)blockIdx.x - batch.first_block[GLU ? 0 : pi];
  const KeepMap km = a.km;
  const int nchunk = NCH > 0 ? NCH : nchunk_rt;
  const int rg = GLU ? block_id * 4 + (wave & 3) : block_id * kGemvWaves + wave;   // row group of this wave
  const int k_span32 = (km.k_span + 31) & ~31;
  const int words_per_row = a.K_total >> 3;
  const int groups_per_row = a.K_total / kGroup;
  const half_t* xrow = a.x + (size_t)m * a.ldx;

  // stored rows of this wave (clamped so that every address is valid)
  int srow[R];
  const int rope_heads = ROPE ? batch.rf.heads[pi] : 0;   // block-uniform
  int rope_row = 0, rope_j = 0, rope_pos = 0;
  bool rope_ok = false;
  if (ROPE && rope_heads > 0) {
    const int hk = batch.rf.D_keep >> 1;
    const int p = block_id * 4 + (wave & 3);              // kept pair of this wave, over all heads
    rope_ok = p < rope_heads * hk;
    const int pc = rope_ok ? p : rope_heads * hk - 1;
    const int head = pc / hk, i = pc - head * hk;
    rope_row = head * batch.rf.D_keep + i + (wave >> 2) * hk;
    srow[0] = stored_row(km, rope_row);
    // original pair index and position: issued first, consumed after the activations are staged
    rope_j = batch.rf.kept_idx[(size_t)(head / (rope_heads / batch.rf.H_tab)) * hk + i];
    rope_pos = batch.rf.positions[0];
  } else {
    // R consecutive compact rows: one division for the first, the others step through their zone.
    // Zones in compact order: first family of segments [0, rs_segrows), second family
    // [rs_segrows, rs_segrows + rs2_segrows), whole-kept tail; a prefix is one contiguous zone.
    int rc = rg * R;
    rc = rc < km.n_keep ? rc : km.n_keep - 1;
    const int z1 = km.rs_segrows, z2 = km.rs_segrows + km.rs2_segrows;   // compact starts of the second family and the tail
    int off = 0, len = 1 << 30, gap = 0;   // position in the segment, kept rows per segment, stored rows skipped at its end
    if (km.rs_stride == 0) {
      srow[0] = rc;
    } else if (rc < z1) {
      const int seg = rc / km.rs_keep;
      off = rc - seg * km.rs_keep;
      srow[0] = seg * km.rs_stride + off;
      len = km.rs_keep;
      gap = km.rs_stride - km.rs_keep;
    } else if (rc < z2) {
      const int t = rc - z1;
      const int seg = t / km.rs2_keep;
      off = t - seg * km.rs2_keep;
      srow[0] = km.rs_limit + seg * km.rs2_stride + off;
      len = km.rs2_keep;
      gap = km.rs2_stride - km.rs2_keep;
    } else {
      srow[0] = km.rs2_limit + (rc - z2);
    }
#pragma unroll
    for (int r = 1; r < R; ++r) {
      if (rc + 1 >= km.n_keep) {            // past the last kept row: repeat it
        srow[r] = srow[r - 1];
        continue;
      }
      rc += 1;
      if (km.rs_stride != 0 && rc == z2) {          // enters the whole-kept tail (also when there is no second family)
        srow[r] = km.rs2_limit;
        off = 0;
        len = 1 << 30;
        gap = 0;
      } else if (km.rs_stride != 0 && rc == z1) {   // enters the second family
        srow[r] = km.rs_limit;
        off = 0;
        len = km.rs2_keep;
        gap = km.rs2_stride - km.rs2_keep;
      } else if (off + 1 == len) {                  // next segment of the same family
        srow[r] = srow[r - 1] + 1 + gap;
        off = 0;
      } else {
        srow[r] = srow[r - 1] + 1;
        off += 1;
      }
    }
  }

  // Scales and zero points of ALL of the wave's tiles, fetched up front by two wide loads (one dword
  // = two scales or four zero points per lane, rows contiguous) instead of two narrow loads per
  // tile: the memory side sees a fifth fewer requests.  A tile's lanes later pick their group's
  // value out of the holding lane with ds_bpermute.  Needs rows of a multiple of four groups and a
  // compile-time tile count; otherwise (NCH = 0) every tile loads its own pair.
  constexpr int TILES = NCH > 0 ? NCH * R : 1;
  constexpr int NS = (TILES * 8 + 63) / 64, NZ = (TILES * 4 + 63) / 64;
  constexpr bool presz = NCH > 0 && R < 4;   // (the host sends rows of any other group count to the NCH = 0 kernel)
  uint32_t sreg[NS], zreg[NZ];
  auto row_of_tile = [&](int tile) {   // stored row of tile id r * NCH + c, tile varies per lane
    const int r = tile / (NCH > 0 ? NCH : 1);
    int sr = srow[0];
#pragma unroll
    for (int rr = 1; rr < R; ++rr) sr = r == rr ? srow[rr] : sr;
    return (size_t)sr * groups_per_row;
  };
  auto load_sz = [&]() {
#pragma unroll
    for (int i = 0; i < NS; ++i) {
      const int flat = i * 64 + lane;
      const int tile = flat / 8 < TILES ? flat / 8 : TILES - 1;
      int d = (tile % (NCH > 0 ? NCH : 1)) * 8 + (flat & 7);          // dword of the row's scales
      d = d < (groups_per_row >> 1) ? d : (groups_per_row >> 1) - 1;
      sreg[i] = load_u32_unaligned(a.scales + row_of_tile(tile) + 2 * d);
    }
#pragma unroll
    for (int i = 0; i < NZ; ++i) {
      const int flat = i * 64 + lane;
      const int tile = flat / 4 < TILES ? flat / 4 : TILES - 1;
      int d = (tile % (NCH > 0 ? NCH : 1)) * 4 + (flat & 3);          // dword of the row's zero points
      d = d < (groups_per_row >> 2) ? d : (groups_per_row >> 2) - 1;
      zreg[i] = ZP ? load_u32_unaligned(a.zeros + row_of_tile(tile) + 4 * d) : 0x08080808u;
    }
  };
  // lane constants of the pick: the lane's group inside a chunk is lane / 4
  const int pick_s = (lane >> 3) * 4, pick_z = (lane >> 4) * 4;                      // byte index of the holding lane
  const uint32_t sel_s = (lane >> 2) & 1 ? 0x03020302u : 0x01000100u;               // (s, s) from the low / high half
  const uint32_t sel_z = 0x0c000c00u | (((lane >> 2) & 3) * 0x00010001u);           // (z, z) from byte lane/4 % 4
  // the pick is issued one tile ahead (pick_tile) and turned into group constants when the tile is consumed
  struct Picked { uint32_t vs, vz; };
  auto pick_tile = [&](int tile) {   // tile = r * NCH + c, compile-time after unrolling
    Picked p;
    p.vs = (uint32_t)__builtin_amdgcn_ds_bpermute(pick_s + (tile % 8) * 32, (int)sreg[tile / 8 < NS ? tile / 8 : 0]);
    p.vz = (uint32_t)__builtin_amdgcn_ds_bpermute(pick_z + (tile % 16) * 16, (int)zreg[tile / 16 < NZ ? tile / 16 : 0]);
    return p;
  };
  typedef typename GroupOf<BF16>::type Group;
  auto groupq_of = [&](const Picked& p) {
    const uint32_t zp = __builtin_amdgcn_perm(0u, p.vz, sel_z);
    const uint32_t ss = __builtin_amdgcn_perm(0u, p.vs, sel_s);
    if constexpr (BF16) {
      return make_groupqb(ss & 0xffffu, zp & 0xffu);
    } else {
      GroupQ g;
      g.zlo = as_half2(zp | 0x64006400u);
      g.zhi = as_half2((zp << 4) | 0x54005400u);
      g.s2 = as_half2(ss);
      return g;
    }
  };

  // Row bases, once per wave (wave-uniform, so they live in scalar registers): a tile's addresses are
  // then base + a per-lane offset that depends on the chunk only.
  const uint32_t* qrow[R];
  const uint16_t* srow_s[R];
  const uint8_t* srow_z[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    qrow[r] = a.qweight + (size_t)srow[r] * words_per_row;
    srow_s[r] = a.scales + (size_t)srow[r] * groups_per_row;
    srow_z[r] = ZP ? a.zeros + (size_t)srow[r] * groups_per_row : nullptr;
  }
  // one tile = the lane's 32 columns of one row in chunk c (16 B of codes + scale + zero).
  // Lanes past the last kept column re-read the row start: their x slots hold zeros, so
  // whatever they fetch contributes nothing and no select has to wait on the loads.
  auto load_tile = [&](int c, int r, Tile& t) {
    const int kb = c * kChunk + lane * 32;
    const int kbc = kb < k_span32 ? kb : 0;
    t.w = *reinterpret_cast<const uint4*>(qrow[r] + (kbc >> 3));
    if (presz) {
      t.sbits = 0;
      t.z = 0;
    } else {
      t.sbits = srow_s[r][kbc >> 7];
      if constexpr (ZP) t.z = srow_z[r][kbc >> 7];
      else t.z = 8u;
    }
  };
  const Magic mg = make_magic();
  // The 8-element dot products of a word run on the matrix pipe, beside the VALU that dequantises:
  // with A = the lane's x values and B = its weights, v_mfma_f32_16x16x32_f16 forms D[i][n] =
  // sum over the four lanes {n, n+16, n+32, n+48} of dot(x of lane i + 16 ks, w of lane n + 16 ks);
  // its diagonal D[n][n] is the partial sum wanted, the rest is ignored.  Lane l holds D[4 (l / 16) + v][l % 16]
  // in register v, so the diagonal sits in lanes 5 m + 16 (m / 4) .. (one of every four), register l % 4.
  auto consume = [&](const Tile& t, const uint4 (&xr)[4], float4_t& acc, const Picked& pk) {
    const Group g = presz ? groupq_of(pk) : make_group<BF16>(t.sbits, t.z);
    const uint32_t wv[4] = {t.w.x, t.w.y, t.w.z, t.w.w};
#pragma unroll
    for (int q = 0; q < 4; ++q) acc = mfma_16x16x32<BF16>(xr[q], dequant_word4<BF16>(wv[q], g, mg), acc);
  };

  float4_t acc[R];
#pragma unroll
  for (int r = 0; r < R; ++r) acc[r] = float4_t{0.f, 0.f, 0.f, 0.f};
  // the lane's diagonal element of an accumulator (zero in the lanes that hold none), summed over the wave
  const bool on_diag = (lane >> 4) == ((lane & 15) >> 2);
  auto row_sum = [&](const float4_t& c) {
    const int v = lane & 3;
    float d = v == 0 ? c[0] : (v == 1 ? c[1] : (v == 2 ? c[2] : c[3]));
    return dpp_xor_reduce(on_diag ? d : 0.f);
  };
  float rope_sn = 0.f, rope_cs = 1.f;

  const ColMap cm = make_colmap(km);
  // XVEC: a unit of 8 stored columns starting at k0 lies in one segment (the stride is a multiple of 8, or
  // there is one segment: the prefix); pos = compact position of its first column, nk = how many of its
  // columns are kept, counted from the first (<= 0: none, >= 8: all)
  auto unit_map = [&](int k0, int& pos, int& nk) {
    if (km.cs_stride == 0) {
      pos = k0;
      nk = km.k_keep - k0;
    } else {
      const int seg = k0 / km.cs_stride, off0 = k0 - seg * km.cs_stride;
      pos = seg * km.cs_keep + off0;
      nk = k0 < km.k_span ? km.cs_keep - off0 : 0;
    }
  };
  // kept columns of the last, partly kept unit of a segment (8: the kept width is a multiple of 8)
  const int seg_keep = km.cs_stride ? km.cs_keep : km.k_keep;
  const int nk_tail = seg_keep - ((seg_keep - 1) & ~7);
  const int units = nchunk * 256;

  if constexpr (NCH > 0) {
    // ---- phase 1: issue the x loads.  Memory returns in issue order, so x (an L2 hit) goes
    // first and never queues behind the HBM stream; it is consumed only after the first weight
    // loads have been issued.  Every load is unconditional on a clamped, valid address.
    constexpr int XI = (NCH * 256 + kGemvThreads - 1) / kGemvThreads;   // x units per thread
    uint4 rawv[XVEC ? XI : 1];             // XVEC: 8 halves per unit, kept as opaque dwords
    uint32_t rawe[XVEC ? 1 : XI][8];       // element path: one zero-extended half per register
    uint32_t okmask[XI];                   // element path, bit j: element j of the unit is a kept column
    uint32_t tailv[8];                     // XVEC: the up to 7 kept columns at and after kv
    const uint16_t* xbits = reinterpret_cast<const uint16_t*>(xrow);
#pragma unroll
    for (int i = 0; i < XI; ++i) {
      const int uraw = tid + i * kGemvThreads;
      const int k0 = unit_k0(uraw < NCH * 256 ? uraw : NCH * 256 - 1);   // past the end: a redundant, valid load
      okmask[i] = 0;
      if constexpr (XVEC) {
        int pos, nk;
        unit_map(k0, pos, nk);
        // a unit wholly inside x is fetched where it lies (a partly kept unit of an inner segment reads on
        // into the next segment's values, masked later); anything else fetches a valid, unused address
        const int pc = (nk > 0 && pos + 8 <= km.k_keep) ? pos : km.k_keep - 8;   // the host selects XVEC only when k_keep >= 8
        rawv[i] = load_u4_unaligned(xrow + pc);
      } else {
        const int seg0 = k0 / cm.stride, off0 = k0 - seg0 * cm.stride;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          int seg = seg0, off = off0 + j;
          if (off >= cm.stride) { off -= cm.stride; seg += 1; }
          const bool ok = off < cm.keep && k0 + j < km.k_span;
          rawe[i][j] = xbits[ok ? seg * cm.keep + off : 0];
          okmask[i] |= ok ? (1u << j) : 0u;
        }
      }
    }
    if constexpr (XVEC) {
#pragma unroll
      for (int j = 0; j < 8; ++j) tailv[j] = 0;
      if (nk_tail < 8) {   // uniform: only a kept width that is not a multiple of 8 has a tail
#pragma unroll
        for (int j = 0; j < 8; ++j) tailv[j] = xbits[km.k_keep - nk_tail + (j < nk_tail ? j : 0)];
      }
    }

    // ---- phase 2: start the weight stream.  Tile t = (chunk t / R, row t % R).
    __builtin_amdgcn_sched_barrier(0);
    constexpr int T = NCH * R;
    constexpr int DW = R >= 2 ? 2 : 4;   // tiles in flight: few per wave when a wave owns several rows (many waves), more for one-row waves
    constexpr int D = T < DW ? T : DW;
    Tile ring[D];
    if (presz) load_sz();   // after x (memory returns in issue order), before the tiles that need them
#pragma unroll
    for (int t = 0; t < D; ++t) load_tile(t / R, t % R, ring[t]);
    __builtin_amdgcn_sched_barrier(0);

    // ---- phase 3: x registers -> LDS (zeros for pruned columns), in the pair order of the slot
#pragma unroll
    for (int i = 0; i < XI; ++i) {
      const int u = tid + i * kGemvThreads;
      const int k0 = unit_k0(u);
      uint32_t e[8];
      if constexpr (XVEC) {
        // the unit's first nk columns are kept (8 or more: all of it; none: pruned); the partly kept unit
        // that ends x takes the tail values, any other its own load
        const uint4 r = rawv[i];
        const uint32_t full[8] = {r.x & 0xffffu, r.x >> 16, r.y & 0xffffu, r.y >> 16,
                                  r.z & 0xffffu, r.z >> 16, r.w & 0xffffu, r.w >> 16};
        int pos, nk;
        unit_map(k0, pos, nk);
        const bool tail = nk < 8 && pos + nk == km.k_keep;
#pragma unroll
        for (int j = 0; j < 8; ++j) e[j] = j < nk ? (tail ? tailv[j] : full[j]) : 0u;
      } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) e[j] = (okmask[i] >> j) & 1u ? rawe[i][j] : 0u;
      }
      if (u < NCH * 256)
        xs[unit_slot(u)] = make_uint4(e[0] | (e[4] << 16), e[1] | (e[5] << 16), e[2] | (e[6] << 16), e[3] | (e[7] << 16));
    }
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
    if (ROPE && rope_heads > 0) {
      // sin / cos of pos * theta^(-2j/D): fp64 angle in revolutions, its fraction to the hardware sin / cos
      // theta^(-2j/D) = base^j by binary powering (a dozen fp64 multiplies, error of a few ulp) instead
      // of a library exp2
      double inv_freq = 1.0, bpow = batch.rf.base;
      for (int e = rope_j; e != 0; e >>= 1) {
        inv_freq = e & 1 ? inv_freq * bpow : inv_freq;
        bpow *= bpow;
      }
      const double rev = (double)rope_pos * inv_freq * 0.15915494309189534561;
      const float rr = (float)(rev - rint(rev));
      rope_sn = __builtin_amdgcn_sinf(rr);
      rope_cs = __builtin_amdgcn_cosf(rr);
    }

    // ---- phase 4: consume tiles in issue order, re-issuing D tiles ahead
    uint4 xr[4];
    Picked pk = {0, 0}, pk_next = {0, 0};
    if (presz) pk_next = pick_tile(0);   // tile t = (chunk t / R, row t % R) has id r * NCH + c
#pragma unroll
    for (int t = 0; t < T; ++t) {
      const int c = t / R, r = t % R;
      pk = pk_next;
      if (presz && t + 1 < T) pk_next = pick_tile(((t + 1) % R) * NCH + (t + 1) / R);
      if (r == 0) {
#pragma unroll
        for (int q = 0; q < 4; ++q) xr[q] = xs[(c * 4 + q) * 64 + lane];
      }
      // Order fence: the tile's registers and the accumulator of the previous tile pass through
      // an empty asm, so this tile's unpacking cannot be hoisted above the previous tile's
      // arithmetic (which would make the wave wait for loads that were issued later).
      Tile& tl = ring[t % D];
      asm volatile("" : "+v"(tl.w.x), "+v"(tl.w.y), "+v"(tl.w.z), "+v"(tl.w.w), "+v"(tl.sbits), "+v"(tl.z),
                        "+v"(acc[(t + R - 1) % R][0]));
      consume(tl, xr, acc[r], pk);
      if (t + D < T) load_tile((t + D) / R, (t + D) % R, tl);
    }
  } else {
    // ---- long rows: run-time chunk count, plain staging loop and a two-deep register pipeline
    for (int u = tid; u < units; u += kGemvThreads) {
      const int k0 = unit_k0(u);
      half_t v[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int k = k0 + j;
        const int kc = k < k_span32 ? compact_col(km, k) : -1;
        const half_t val = xrow[kc >= 0 ? kc : 0];
        v[j] = kc >= 0 ? val : (half_t)0;
      }
      xs[unit_slot(u)] = pack_unit(v);
    }
    Tile cur[R], nxt[R];
#pragma unroll
    for (int r = 0; r < R; ++r) load_tile(0, r, cur[r]);
    __syncthreads();
    for (int c = 0; c < nchunk; ++c) {
      if (c + 1 < nchunk) {
#pragma unroll
        for (int r = 0; r < R; ++r) load_tile(c + 1, r, nxt[r]);
      }
      uint4 xr[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) xr[q] = xs[(c * 4 + q) * 64 + lane];
#pragma unroll
      for (int r = 0; r < R; ++r) consume(cur[r], xr, acc[r], Picked{0, 0});
#pragma unroll
      for (int r = 0; r < R; ++r) cur[r] = nxt[r];
    }
  }

  if (ROPE && rope_heads > 0) {
    __shared__ float pair_sum[kGemvWaves];
    const float v = row_sum(acc[0]);
    if (lane == 0) pair_sum[wave] = v;
    __syncthreads();
    const float x1 = pair_sum[wave & 3], x2 = pair_sum[(wave & 3) + 4];
    const float out = wave < 4 ? x1 * rope_cs - x2 * rope_sn : x2 * rope_cs + x1 * rope_sn;
    if (lane == 0 && rope_ok) a.y[(size_t)m * a.ldy + rope_row] = out16<BF16>(out);
    return;
  }
  if (GLU) {
    __shared__ float glu_sum[kGemvWaves][R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const float v = row_sum(acc[r]);
      if (lane == 0) glu_sum[wave][r] = v;
    }
    __syncthreads();
    if (wave < 4 && lane < R) {
      const float g = glu_sum[wave][lane], u = glu_sum[wave + 4][lane];
      const int rc = rg * R + lane;
      // SiLU(g) * u; exp and the reciprocal are the hardware approximations (about 1 ulp of fp32)
      if (rc < km.n_keep) batch.p[0].y[(size_t)m * batch.p[0].ldy + rc] = out16<BF16>(g * u * __builtin_amdgcn_rcpf(1.0f + __expf(-g)));
    }
    return;
  }
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const float v = row_sum(acc[r]);
    const int rc = rg * R + r;
    if (lane == 0 && rc < km.n_keep) a.y[(size_t)m * a.ldy + rc] = out16<BF16>(v);
  }
}

template <int R>
static int blocks_for(const LinearArgs& a) {
  const int row_groups = (a.km.n_keep + R - 1) / R;
  return (row_groups + kGemvWaves - 1) / kGemvWaves;
}

template <bool ZP, bool BF16, int R, bool XVEC, int NCH, int EPI = 0>
static hipError_t launch_one(const LinearArgs* probs, int n, int m, int nchunk, hipStream_t stream, const RopeFuse* rf = nullptr) {
  const size_t smem = (size_t)nchunk * 4096;
  auto kern = w4_gemv_kernel<R, XVEC, NCH, EPI, ZP, BF16>;
  constexpr bool ROPE = EPI == 1, GLU = EPI == 2;
  if (smem > 160 * 1024) return hipErrorInvalidValue;
  if (smem > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
  }
  GemvBatch b;
  b.n = n;
  b.rf = RopeFuse{};
  if (rf) b.rf = *rf;
  int blocks = 0;
  for (int i = 0; i < kMaxBatch; ++i) {
    b.p[i] = probs[i < n ? i : 0];
    b.first_block[i] = blocks;
    if (i >= n) continue;
    // a rotated problem: four kept pairs per block; otherwise eight waves of R rows
    if (ROPE && b.rf.heads[i] > 0) blocks += (b.rf.heads[i] * (b.rf.D_keep / 2) + 3) / 4;
    else if (GLU) blocks += i == 0 ? (probs[0].km.n_keep + 4 * R - 1) / (4 * R) : 0;   // a block = 4 R gate rows + their up rows
    else blocks += blocks_for<R>(probs[i]);
  }
  hipLaunchKernelGGL(kern, dim3(blocks), dim3(kGemvThreads), smem, stream, b, m, nchunk);
  return hipGetLastError();
}

template <bool ZP, bool BF16, int R, bool XVEC>
static hipError_t launch_nch(const LinearArgs* probs, int n, int m, int nchunk, hipStream_t stream) {
  // the unrolled kernels fetch scales and zero points as dwords: rows of a multiple of four groups
  bool wide = true;
  for (int i = 0; i < n; ++i) wide = wide && (probs[i].K_total / kGroup) % 4 == 0;
  switch (wide ? nchunk : 0) {
    case 1: return launch_one<ZP, BF16, R, XVEC, 1>(probs, n, m, nchunk, stream);
    case 2: return launch_one<ZP, BF16, R, XVEC, 2>(probs, n, m, nchunk, stream);
    case 3: return launch_one<ZP, BF16, R, XVEC, 3>(probs, n, m, nchunk, stream);
    case 4: return launch_one<ZP, BF16, R, XVEC, 4>(probs, n, m, nchunk, stream);
    case 5: return launch_one<ZP, BF16, R, XVEC, 5>(probs, n, m, nchunk, stream);
    case 6: return launch_one<ZP, BF16, R, XVEC, 6>(probs, n, m, nchunk, stream);
    case 7: return launch_one<ZP, BF16, R, XVEC, 7>(probs, n, m, nchunk, stream);
    case 8: return launch_one<ZP, BF16, R, XVEC, 8>(probs, n, m, nchunk, stream);
    default: return launch_one<ZP, BF16, R, XVEC, 0>(probs, n, m, nchunk, stream);
  }
}

template <bool ZP, bool BF16, bool XVEC>
static hipError_t launch_rows(const LinearArgs* probs, int n, int r1, int m, int nchunk, hipStream_t stream) {
  if (r1 == 4) return launch_nch<ZP, BF16, 4, XVEC>(probs, n, m, nchunk, stream);
  if (r1 == 2) return launch_nch<ZP, BF16, 2, XVEC>(probs, n, m, nchunk, stream);
  return launch_nch<ZP, BF16, 1, XVEC>(probs, n, m, nchunk, stream);
}

static inline int nchunk_of(const LinearArgs& a) {
  const int k_span32 = (a.km.k_span + 31) & ~31;
  return (k_span32 + kChunk - 1) / kChunk;
}
static inline bool xvec_of(const LinearArgs& a, int) {
  // a column prefix is fetched with 128-bit loads whatever the alignment of x (global loads may
  // start on any 2-byte boundary on this target)
  // ... and so are column segments whose stride is a multiple of 8: a unit of 8 stored columns then lies in
  // one segment and its kept columns are contiguous in x
  // (with at least 8 kept columns per segment, so that a partly kept unit of an inner segment can read 16 bytes
  // without leaving x)
  return (a.km.cs_stride == 0 || (a.km.cs_stride % 8 == 0 && a.km.cs_keep >= 8)) && a.km.k_keep >= 8;
}

template <bool ZP, bool BF16>
static hipError_t gemv_one(const LinearArgs& a, hipStream_t stream) {
  // rows per wave: fewer when the matrix is small, so that every CU still gets several waves
  // (long rows already from 4096: one block per CU with two rows per wave gives steadier times than two blocks per CU
  // with one, which measured anything from 0.7 us faster to 1 us slower from one run to the next)
  const int r1 = a.km.n_keep >= 16384 ? 4 : ((a.km.n_keep >= 6144 || (a.km.n_keep >= 4096 && nchunk_of(a) >= 4)) ? 2 : 1);
  for (int m = 0; m < a.M; ++m) {
    hipError_t e = xvec_of(a, m) ? launch_rows<ZP, BF16, true>(&a, 1, r1, m, nchunk_of(a), stream)
                                 : launch_rows<ZP, BF16, false>(&a, 1, r1, m, nchunk_of(a), stream);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

// n single-token linears in one launch when they can share a kernel instantiation (same chunk
// count and x access mode); otherwise one launch each.
template <bool ZP, bool BF16>
static hipError_t gemv_batch(const LinearArgs* probs, int n, hipStream_t stream) {
  bool same = n <= kMaxBatch;
  long long rows = 0;
  for (int i = 0; i < n; ++i) {
    same = same && probs[i].M == 1 && nchunk_of(probs[i]) == nchunk_of(probs[0]) && xvec_of(probs[i], 0) == xvec_of(probs[0], 0);
    rows += probs[i].km.n_keep;
  }
  if (!same) {
    for (int i = 0; i < n; ++i) {
      hipError_t e = gemv_one<ZP, BF16>(probs[i], stream);
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  }
  const int r1 = rows >= 16384 ? 4 : (rows >= 6144 ? 2 : 1);
  return xvec_of(probs[0], 0) ? launch_rows<ZP, BF16, true>(probs, n, r1, 0, nchunk_of(probs[0]), stream)
                              : launch_rows<ZP, BF16, false>(probs, n, r1, 0, nchunk_of(probs[0]), stream);
}

template <bool ZP, bool BF16, bool XVEC>
static hipError_t launch_rope_nch(const LinearArgs* probs, int nchunk, hipStream_t stream, const RopeFuse& rf) {
  switch (nchunk) {
    case 1: return launch_one<ZP, BF16, 1, XVEC, 1, 1>(probs, 3, 0, nchunk, stream, &rf);
    case 2: return launch_one<ZP, BF16, 1, XVEC, 2, 1>(probs, 3, 0, nchunk, stream, &rf);
    case 3: return launch_one<ZP, BF16, 1, XVEC, 3, 1>(probs, 3, 0, nchunk, stream, &rf);
    case 4: return launch_one<ZP, BF16, 1, XVEC, 4, 1>(probs, 3, 0, nchunk, stream, &rf);
    case 5: return launch_one<ZP, BF16, 1, XVEC, 5, 1>(probs, 3, 0, nchunk, stream, &rf);
    case 6: return launch_one<ZP, BF16, 1, XVEC, 6, 1>(probs, 3, 0, nchunk, stream, &rf);
    case 7: return launch_one<ZP, BF16, 1, XVEC, 7, 1>(probs, 3, 0, nchunk, stream, &rf);
    default: return launch_one<ZP, BF16, 1, XVEC, 8, 1>(probs, 3, 0, nchunk, stream, &rf);
  }
}

template <bool ZP, bool BF16, int R, bool XVEC>
static hipError_t launch_glu_nch(const LinearArgs* probs, int nchunk, hipStream_t stream) {
  switch (nchunk) {
    case 1: return launch_one<ZP, BF16, R, XVEC, 1, 2>(probs, 2, 0, nchunk, stream);
    case 2: return launch_one<ZP, BF16, R, XVEC, 2, 2>(probs, 2, 0, nchunk, stream);
    case 3: return launch_one<ZP, BF16, R, XVEC, 3, 2>(probs, 2, 0, nchunk, stream);
    case 4: return launch_one<ZP, BF16, R, XVEC, 4, 2>(probs, 2, 0, nchunk, stream);
    case 5: return launch_one<ZP, BF16, R, XVEC, 5, 2>(probs, 2, 0, nchunk, stream);
    case 6: return launch_one<ZP, BF16, R, XVEC, 6, 2>(probs, 2, 0, nchunk, stream);
    case 7: return launch_one<ZP, BF16, R, XVEC, 7, 2>(probs, 2, 0, nchunk, stream);
    default: return launch_one<ZP, BF16, R, XVEC, 8, 2>(probs, 2, 0, nchunk, stream);
  }
}

// gate and up of one token with h = SiLU(gate) * up as epilogue, written to probs[0].y; *fused = false
// (nothing launched) when the shapes do not allow it
template <bool ZP, bool BF16>
static hipError_t gate_up_silu(const LinearArgs* probs, hipStream_t stream, bool* fused) {
  bool ok = probs[0].M == 1 && probs[1].M == 1 && nchunk_of(probs[0]) == nchunk_of(probs[1]) &&
            xvec_of(probs[0], 0) == xvec_of(probs[1], 0) && nchunk_of(probs[0]) >= 1 && nchunk_of(probs[0]) <= 8 &&
            (probs[0].K_total / kGroup) % 4 == 0 && (probs[1].K_total / kGroup) % 4 == 0;
  *fused = ok;
  if (!ok) return hipSuccess;
  const int rows = 2 * probs[0].km.n_keep, nch = nchunk_of(probs[0]);
  const bool xv = xvec_of(probs[0], 0);
  if (rows >= 16384) return xv ? launch_glu_nch<ZP, BF16, 4, true>(probs, nch, stream) : launch_glu_nch<ZP, BF16, 4, false>(probs, nch, stream);
  if (rows >= 6144) return xv ? launch_glu_nch<ZP, BF16, 2, true>(probs, nch, stream) : launch_glu_nch<ZP, BF16, 2, false>(probs, nch, stream);
  return xv ? launch_glu_nch<ZP, BF16, 1, true>(probs, nch, stream) : launch_glu_nch<ZP, BF16, 1, false>(probs, nch, stream);
}

template <bool ZP, bool BF16>
static hipError_t qkv_rope(const LinearArgs* probs, const RopeFuse& rf, hipStream_t stream, bool* fused) {
  // one launch needs the three problems to share a kernel instantiation: one token, the same
  // compile-time chunk count and x access mode, rows of a multiple of four groups
  bool ok = true;
  for (int i = 0; i < 3; ++i)
    ok = ok && probs[i].M == 1 && nchunk_of(probs[i]) == nchunk_of(probs[0]) && xvec_of(probs[i], 0) == xvec_of(probs[0], 0) &&
         (probs[i].K_total / kGroup) % 4 == 0;
  ok = ok && nchunk_of(probs[0]) >= 1 && nchunk_of(probs[0]) <= 8;
  *fused = ok;
  if (!ok) return hipSuccess;
  return xvec_of(probs[0], 0) ? launch_rope_nch<ZP, BF16, true>(probs, nchunk_of(probs[0]), stream, rf)
                              : launch_rope_nch<ZP, BF16, false>(probs, nchunk_of(probs[0]), stream, rf);
}

}  // namespace gemv
}  // namespace uniql
