// Streaming W4A16 GEMV, one token per launch (decode).
//
// The op is bound by the HBM stream of packed nibbles, so the kernel is built
// around that stream: a wave reads a kept row in wave-wide 128-bit loads ("tiles"), every lane 32 consecutive input
// columns that lie in one quantisation group.  Pruned rows are never touched (row truncation
// saves their bytes); pruned columns are handled by staging the activations
// once per block into LDS at their *stored* column positions with zeros in the
// pruned slots, so the weight stream needs no per-element masking.
//
// Column layout of a wave (shared with the persistent kernel of gemv_stream_kernel.h, so that a row's result has the
// same bits whichever kernel serves it).  A row of NCH tiles: lanes 4g..4g+3 (a quad) own the NCH ADJACENT groups
// g * NCH .. g * NCH + NCH - 1, and tile c is group g * NCH + c of every quad.  A quad reads 64 contiguous bytes per tile
// (one request of the address unit, like a contiguous load), the NCH tiles of a row together read the row
// contiguously, and the NCH scales of a lane are adjacent in memory, as are its zero points: a ROW needs one scale load
// and one zero-point load, not one of each per tile.
//
// Per 32-bit word (8 weights): 1 shift + 4 and-or build exact fp16 codes, 4
// packed subtracts and 4 packed multiplies give the canonical fp16 weights
// RN16((q - z) s); the word's 8-element dot product with the lane's activations is
// taken from the diagonal of one matrix instruction (see consume below), fp32.
//
// The kernel is fully unrolled over the row's tiles (template NCH):
// a wave's tiles (row, tile) are loaded a few tiles ahead (DW in the kernel) and consumed in issue
// order, each as soon as it has arrived, so the arithmetic overlaps the stream
// instead of starting after the last byte.
#pragma once
#include "common.h"

namespace uniql {
namespace gemv {

constexpr int kGemvThreads = 512;
constexpr int kGemvWaves = kGemvThreads / kWave;
constexpr int kChunk = kWave * 32;   // stored columns one wave covers with one 128-bit load per lane

typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x3_t __attribute__((ext_vector_type(3)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

// tiles per row: the groups that hold kept columns (stored columns [0, k_span)), sixteen quads
static inline int row_tiles(int k_span) { return ((k_span + kGroup - 1) / kGroup + 15) / 16; }
// A quad's NCH groups must not straddle the end of a row (its scales are fetched as one run): the row's group count is
// a multiple of NCH, or the sixteen quads end inside the row.
static inline bool whole_quads(int K_total, int nch) {
  const int gpr = K_total / kGroup;
  return gpr % nch == 0 || 16 * nch <= gpr;
}

// Sum of the 16 diagonal elements of an MFMA accumulator (lane l holds D[4 (l / 16) + v][l % 16] in register v, so
// the diagonal sits in quad r of row r, register = lane % 4), valid in lane 63.  Four DPP moves / adds gather a quad's
// four diagonal registers into every lane of the quad, one select keeps the quads that are on the diagonal, two mirrors
// add up a row of 16 lanes, the two row broadcasts add up the rows: 9 VALU instructions, no LDS crossbar.
#define UNIQL_DPP_MOV(src, ctrl, rmask, bmask) \
  __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, (src)), (ctrl), (rmask), (bmask), true))
__device__ __forceinline__ float diag_sum_to_lane63(const float4_t& a, bool on_diag) {
  // (the elements are copied to scalars first: a bit cast applied to a vector element directly reads element 0
  // with this compiler)
  const float a0 = a[0], a1 = a[1], a2 = a[2], a3 = a[3];
  float t = UNIQL_DPP_MOV(a0, 0x00, 0xF, 0xF);    // quad_perm [0,0,0,0]
  t += UNIQL_DPP_MOV(a1, 0x55, 0xF, 0xF);         // quad_perm [1,1,1,1]
  t += UNIQL_DPP_MOV(a2, 0xAA, 0xF, 0xF);         // quad_perm [2,2,2,2]
  t += UNIQL_DPP_MOV(a3, 0xFF, 0xF, 0xF);         // quad_perm [3,3,3,3]
  t = on_diag ? t : 0.f;
  t += UNIQL_DPP_MOV(t, 0x141, 0xF, 0xF);         // row_half_mirror
  t += UNIQL_DPP_MOV(t, 0x140, 0xF, 0xF);         // row_mirror
  // the row broadcasts add in place (rows outside the row mask keep their value), one instruction each; the
  // s_nop is the wait a DPP instruction needs after the instruction that wrote its operand
  asm volatile("s_nop 1\n\tv_add_f32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\ts_nop 1\n\t"
               "v_add_f32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf" : "+v"(t));
  return t;
}
// Two accumulators at once, the same arithmetic: the two chains alternate instruction by instruction, which fills the
// two wait states a DPP instruction needs after the instruction that wrote one of its operands.
__device__ __forceinline__ void diag_sums_to_lane63(const float4_t& a, const float4_t& b, bool on_diag, float& sa, float& sb) {
  const float a0 = a[0], a1 = a[1], a2 = a[2], a3 = a[3], b0 = b[0], b1 = b[1], b2 = b[2], b3 = b[3];
  float t = UNIQL_DPP_MOV(a0, 0x00, 0xF, 0xF), u = UNIQL_DPP_MOV(b0, 0x00, 0xF, 0xF);
  t += UNIQL_DPP_MOV(a1, 0x55, 0xF, 0xF); u += UNIQL_DPP_MOV(b1, 0x55, 0xF, 0xF);
  t += UNIQL_DPP_MOV(a2, 0xAA, 0xF, 0xF); u += UNIQL_DPP_MOV(b2, 0xAA, 0xF, 0xF);
  t += UNIQL_DPP_MOV(a3, 0xFF, 0xF, 0xF); u += UNIQL_DPP_MOV(b3, 0xFF, 0xF, 0xF);
  t = on_diag ? t : 0.f; u = on_diag ? u : 0.f;
  t += UNIQL_DPP_MOV(t, 0x141, 0xF, 0xF); u += UNIQL_DPP_MOV(u, 0x141, 0xF, 0xF);
  t += UNIQL_DPP_MOV(t, 0x140, 0xF, 0xF); u += UNIQL_DPP_MOV(u, 0x140, 0xF, 0xF);
  asm volatile("s_nop 0\n\tv_add_f32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
               "v_add_f32_dpp %1, %1, %1 row_bcast:15 row_mask:0xa bank_mask:0xf\n\ts_nop 0\n\t"
               "v_add_f32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"
               "v_add_f32_dpp %1, %1, %1 row_bcast:31 row_mask:0xc bank_mask:0xf" : "+v"(t), "+v"(u));
  sa = t;
  sb = u;
}

struct Tile {
  uint4 w;          // 32 packed codes
  uint32_t sbits;   // fp16 scale bits of the lane's group (rows of a run-time tile count only)
  uint32_t z;       // zero point of the lane's group     (rows of a run-time tile count only)
};

// A lane's scales (fp16 bits) and zero points (bytes) of one row: NCH adjacent groups.
template <int NCH> struct RowQ {
  uint32_t s[(2 * NCH + 3) / 4], z[(NCH + 3) / 4];
};
// Exactly NB bytes (NB <= 16) at p, in pieces of 16 / 12 / 8 / 4 / 2 / 1 bytes, packed little-endian into out[].
// Nothing beyond the NB bytes is read, so the last row of an array is safe; p may have any alignment (the target
// loads unaligned).
template <int NB>
__device__ __forceinline__ void load_bytes(const uint8_t* p, uint32_t (&out)[(NB + 3) / 4]) {
  typedef uint32_t u32x4_u1 __attribute__((ext_vector_type(4), aligned(1)));
  typedef uint32_t u32x3_u1 __attribute__((ext_vector_type(3), aligned(1)));
  typedef uint32_t u32x2_u1 __attribute__((ext_vector_type(2), aligned(1)));
  typedef uint16_t u16_u1 __attribute__((aligned(1)));
  constexpr int W = NB / 4;   // whole dwords
  if constexpr (W == 4) {
    const u32x4_u1 v = *reinterpret_cast<const u32x4_u1*>(p);
    out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
  } else if constexpr (W == 3) {
    const u32x3_u1 v = *reinterpret_cast<const u32x3_u1*>(p);
    out[0] = v.x; out[1] = v.y; out[2] = v.z;
  } else if constexpr (W == 2) {
    const u32x2_u1 v = *reinterpret_cast<const u32x2_u1*>(p);
    out[0] = v.x; out[1] = v.y;
  } else if constexpr (W == 1) {
    out[0] = load_u32_unaligned(p);
  }
  constexpr int R = NB - 4 * W;   // 0..3 bytes left
  if constexpr (R == 1) {
    out[W] = p[4 * W];
  } else if constexpr (R == 2) {
    out[W] = *reinterpret_cast<const u16_u1*>(p + 4 * W);
  } else if constexpr (R == 3) {
    const uint32_t lo = *reinterpret_cast<const u16_u1*>(p + 4 * W);
    const uint32_t hi = p[4 * W + 2];
    out[W] = lo | (hi << 16);
  }
}
// the same through a buffer resource (lane offset voff + scalar offset soff)
template <int NB>
__device__ __forceinline__ void load_bytes(__amdgpu_buffer_rsrc_t r, int voff, int soff, uint32_t (&out)[(NB + 3) / 4]) {
  constexpr int W = NB / 4;
  if constexpr (W == 4) {
    const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0);
    out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
  } else if constexpr (W == 3) {
    const u32x3_t v = __builtin_amdgcn_raw_buffer_load_b96(r, voff, soff, 0);
    out[0] = v.x; out[1] = v.y; out[2] = v.z;
  } else if constexpr (W == 2) {
    const u32x2_t v = __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, 0);
    out[0] = v.x; out[1] = v.y;
  } else if constexpr (W == 1) {
    out[0] = __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0);
  }
  constexpr int R = NB - 4 * W;
  if constexpr (R == 1) {
    out[W] = __builtin_amdgcn_raw_buffer_load_b8(r, voff + 4 * W, soff, 0);
  } else if constexpr (R == 2) {
    out[W] = __builtin_amdgcn_raw_buffer_load_b16(r, voff + 4 * W, soff, 0);
  } else if constexpr (R == 3) {
    const uint32_t lo = __builtin_amdgcn_raw_buffer_load_b16(r, voff + 4 * W, soff, 0);
    const uint32_t hi = __builtin_amdgcn_raw_buffer_load_b8(r, voff + 4 * W + 2, soff, 0);
    out[W] = lo | (hi << 16);
  }
}
// group constants of tile c of a row (c is a compile-time constant after unrolling)
template <bool ZP, bool BF16, int NCH>
__device__ __forceinline__ typename GroupOf<BF16>::type group_of(const RowQ<NCH>& r, int c) {
  const half_t sc = as_half2(r.s[c >> 1])[c & 1];
  const half2_t sv = {sc, sc};   // (the compiler folds the splat into op_sel of the packed multiply)
  const uint32_t ss = as_u32(sv);
  const uint32_t zz = ZP ? __builtin_amdgcn_perm(0u, r.z[c >> 2], 0x0c000c00u | ((c & 3) * 0x00010001u)) : 0x00080008u;   // (z, z)
  if constexpr (BF16) {
    return make_groupqb(ss & 0xffffu, zz & 0xffu);
  } else {
    GroupQ g;
    g.zlo = as_half2(zz | 0x64006400u);
    g.zhi = as_half2((zz << 4) | 0x54005400u);
    g.s2 = as_half2(ss);
    return g;
  }
}

// Unit u = the 8 stored columns [8u, 8u + 8).  Its LDS slot in the image [tile][word][lane] of a row of nch tiles,
// halves ordered (k0,k0+4,k0+1,k0+5,k0+2,k0+6,k0+3,k0+7): dword p pairs with the dequantised
// pair (w_p, w_{p+4}), and a wave reads one word-plane of a tile with consecutive addresses.
__device__ __forceinline__ int unit_slot(int u, int nch) {
  const int G = u >> 4, qd = G / nch, c = G - qd * nch;   // group of the unit, its quad and tile
  return (c * 4 + (u & 3)) * 64 + qd * 4 + ((u >> 2) & 3);
}
// stored column where lane `lane` starts in tile c
__device__ __forceinline__ int tile_k0(int lane, int c, int nch) { return ((lane >> 2) * nch + c) * kGroup + (lane & 3) * 32; }

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
// weight stream is in flight: the angle in fp64 and in revolutions like the stand-alone RoPE kernel's, but
// theta^(-2j/D) as base^j by binary powering (a dozen fp64 multiplies) where that kernel calls exp2.
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

  // Scales and zero points: a lane's NCH groups of a row are adjacent (see the layout above), so every row costs one
  // scale load and one zero-point load, issued with the row's first tile.  Rows of a run-time tile count (NCH = 0) load
  // the pair of every tile instead.
  constexpr int NCQ = NCH > 0 ? NCH : 1;
  typedef typename GroupOf<BF16>::type Group;
  const int quad = lane >> 2;
  // first group of the lane; a quad past the row's groups reads the row start (its columns are pruned by definition).
  // The host sends only rows whose quads do not straddle the row's end to the kernels with NCH > 0.
  const int goff = (quad + 1) * NCQ <= groups_per_row ? quad * NCQ : 0;
  RowQ<NCQ> rowq[R];
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
  // one tile = the lane's 32 columns of one row in tile c (16 B of codes; + scale + zero for NCH = 0).
  // Lanes past the last kept column re-read the row start: their x slots hold zeros, so
  // whatever they fetch contributes nothing and no select has to wait on the loads.
  auto load_tile = [&](int c, int r, Tile& t) {
    const int kb = tile_k0(lane, c, nchunk);
    const int kbc = kb < k_span32 ? kb : 0;
    t.w = *reinterpret_cast<const uint4*>(qrow[r] + (kbc >> 3));
    if constexpr (NCH > 0) {
      t.sbits = 0;
      t.z = 0;
    } else {
      t.sbits = srow_s[r][kbc >> 7];
      if constexpr (ZP) t.z = srow_z[r][kbc >> 7];
      else t.z = 8u;
    }
  };
  auto load_rowq = [&](int r) {
    if constexpr (NCH > 0) {
      load_bytes<2 * NCQ>(reinterpret_cast<const uint8_t*>(srow_s[r] + goff), rowq[r].s);
      if constexpr (ZP) load_bytes<NCQ>(srow_z[r] + goff, rowq[r].z);
    }
  };
  const Magic mg = make_magic();
  // The 8-element dot products of a word run on the matrix pipe, beside the VALU that dequantises:
  // with A = the lane's x values and B = its weights, v_mfma_f32_16x16x32_f16 forms D[i][n] =
  // sum over the four lanes {n, n+16, n+32, n+48} of dot(x of lane i + 16 ks, w of lane n + 16 ks);
  // its diagonal D[n][n] is the partial sum wanted, the rest is ignored.  Lane l holds D[4 (l / 16) + v][l % 16]
  // in register v, so the diagonal sits in lanes 5 m + 16 (m / 4) .. (one of every four), register l % 4.
  auto consume = [&](const Tile& t, const uint4 (&xr)[4], float4_t& acc, const Group& g) {
    const uint32_t wv[4] = {t.w.x, t.w.y, t.w.z, t.w.w};
#pragma unroll
    for (int q = 0; q < 4; ++q) acc = mfma_16x16x32<BF16>(xr[q], dequant_word4<BF16>(wv[q], g, mg), acc);
  };

  float4_t acc[R];
#pragma unroll
  for (int r = 0; r < R; ++r) acc[r] = float4_t{0.f, 0.f, 0.f, 0.f};
  // the sum of an accumulator's diagonal over the wave, valid in lane 63
  const bool on_diag = (lane >> 4) == ((lane & 15) >> 2);
  auto row_sum = [&](const float4_t& c) { return diag_sum_to_lane63(c, on_diag); };
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
      const int k0 = 8 * (uraw < NCH * 256 ? uraw : NCH * 256 - 1);   // past the end: a redundant, valid load
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
#pragma unroll
    for (int r = 0; r < R; ++r) load_rowq(r);   // after x (memory returns in issue order), before the tiles that need them
#pragma unroll
    for (int t = 0; t < D; ++t) load_tile(t / R, t % R, ring[t]);
    __builtin_amdgcn_sched_barrier(0);

    // ---- phase 3: x registers -> LDS (zeros for pruned columns), in the pair order of the slot
#pragma unroll
    for (int i = 0; i < XI; ++i) {
      const int u = tid + i * kGemvThreads;
      const int k0 = 8 * u;
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
        xs[unit_slot(u, NCH)] = make_uint4(e[0] | (e[4] << 16), e[1] | (e[5] << 16), e[2] | (e[6] << 16), e[3] | (e[7] << 16));
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
#pragma unroll
    for (int t = 0; t < T; ++t) {
      const int c = t / R, r = t % R;
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
      consume(tl, xr, acc[r], group_of<ZP, BF16, NCQ>(rowq[r], c));
      if (t + D < T) load_tile((t + D) / R, (t + D) % R, tl);
    }
  } else {
    // ---- long rows: run-time chunk count, plain staging loop and a two-deep register pipeline
    for (int u = tid; u < units; u += kGemvThreads) {
      const int k0 = 8 * u;
      half_t v[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int k = k0 + j;
        const int kc = k < k_span32 ? compact_col(km, k) : -1;
        const half_t val = xrow[kc >= 0 ? kc : 0];
        v[j] = kc >= 0 ? val : (half_t)0;
      }
      xs[unit_slot(u, nchunk)] = pack_unit(v);
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
      for (int r = 0; r < R; ++r) consume(cur[r], xr, acc[r], make_group<BF16>(cur[r].sbits, cur[r].z));
#pragma unroll
      for (int r = 0; r < R; ++r) cur[r] = nxt[r];
    }
  }

  if (ROPE && rope_heads > 0) {
    __shared__ float pair_sum[kGemvWaves];
    const float v = row_sum(acc[0]);
    if (lane == 63) pair_sum[wave] = v;
    __syncthreads();
    const float x1 = pair_sum[wave & 3], x2 = pair_sum[(wave & 3) + 4];
    const float out = wave < 4 ? x1 * rope_cs - x2 * rope_sn : x2 * rope_cs + x1 * rope_sn;
    if (lane == 63 && rope_ok) a.y[(size_t)m * a.ldy + rope_row] = out16<BF16>(out);
    return;
  }
  if (GLU) {
    __shared__ float glu_sum[kGemvWaves][R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const float v = row_sum(acc[r]);
      if (lane == 63) glu_sum[wave][r] = v;
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
    if (lane == 63 && rc < km.n_keep) a.y[(size_t)m * a.ldy + rc] = out16<BF16>(v);
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
  // the unrolled kernels fetch a quad's scales and zero points as one run: no quad may straddle the end of a row
  bool wide = true;
  for (int i = 0; i < n; ++i) wide = wide && whole_quads(probs[i].K_total, nchunk);
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

static inline int nchunk_of(const LinearArgs& a) { return row_tiles(a.km.k_span); }
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
            whole_quads(probs[0].K_total, nchunk_of(probs[0])) && whole_quads(probs[1].K_total, nchunk_of(probs[0]));
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
         whole_quads(probs[i].K_total, nchunk_of(probs[0]));
  ok = ok && nchunk_of(probs[0]) >= 1 && nchunk_of(probs[0]) <= 8;
  *fused = ok;
  if (!ok) return hipSuccess;
  return xvec_of(probs[0], 0) ? launch_rope_nch<ZP, BF16, true>(probs, nchunk_of(probs[0]), stream, rf)
                              : launch_rope_nch<ZP, BF16, false>(probs, nchunk_of(probs[0]), stream, rf);
}

}  // namespace gemv
}  // namespace uniql
