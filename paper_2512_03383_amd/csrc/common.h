// Internal declarations shared by the HIP translation units of libuniql.
// Nothing here is part of the C ABI (see include/uniql.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace uniql {

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float float2_t __attribute__((ext_vector_type(2)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef float float16_t __attribute__((ext_vector_type(16)));

constexpr int kGroup = 128;    // quantisation group along the input dimension
constexpr int kWave = 64;      // wavefront width on CDNA

// Normalised keep descriptor, computed on the host from uniql_keep_t.
struct KeepMap {
  int n_keep;       // compact output rows
  int k_keep;       // compact input columns
  int rs_stride;    // 0 = row prefix
  int rs_keep;
  int rs_limit;
  int rs_segrows;   // compact rows that come from the (first) segmented part
  int rs2_stride;   // second family of segments, stored rows [rs_limit, rs2_limit); 0 = none
  int rs2_keep;
  int rs2_limit;    // rows from here on are kept whole (= rs_limit without a second family)
  int rs2_segrows;  // compact rows that come from the second family
  int cs_stride;    // 0 = column prefix
  int cs_keep;
  int k_span;       // stored columns [0, k_span) contain every kept column
};

// Everything a linear kernel needs, passed by value.
struct LinearArgs {
  const uint32_t* qweight;
  const uint16_t* scales;
  const uint8_t* zeros;
  const half_t* x;    // 16-bit elements: fp16, or bfloat16 when bf16 is set
  half_t* y;
  long long ldx, ldy;
  int N_total, K_total, M;
  int bf16;           // scales, x and y are bfloat16 (the weights are then rounded to bfloat16 as well)
  int il_heads;       // > 0: the row's words are stored head-interleaved over this many heads (uniql_w4_t.col_interleave)
  int bits;           // width of a code: 4, or 8 (w8.hip serves those), or 3 / 6 (wbits.hip)
  KeepMap km;
};

// Several independent linears served by one GEMV launch.
constexpr int kMaxBatch = 4;
// Rotary epilogue of a fused q / k / v launch: problem i is rotated when heads[i] > 0; its compact
// output is [heads[i]][D_keep] and kept pair p of a head is (y[p], y[p + D_keep / 2]).
struct RopeFuse {
  const int32_t* positions;       // device, [1]: the token's position
  const int32_t* kept_idx;        // device, [H_tab][D_keep / 2]
  int H_tab, D_keep;
  double base;                    // theta^(-2 / D_full): inv_freq_j = base^j
  int heads[kMaxBatch];
};
struct GemvBatch {
  LinearArgs p[kMaxBatch];
  int first_block[kMaxBatch];
  int n;
  RopeFuse rf;
};

// compact output row -> stored row
__device__ __forceinline__ int stored_row(const KeepMap& km, int rc) {
  if (km.rs_stride == 0) return rc;
  if (rc < km.rs_segrows) {
    int seg = rc / km.rs_keep;
    return seg * km.rs_stride + (rc - seg * km.rs_keep);
  }
  rc -= km.rs_segrows;
  if (rc < km.rs2_segrows) {
    int seg = rc / km.rs2_keep;
    return km.rs_limit + seg * km.rs2_stride + (rc - seg * km.rs2_keep);
  }
  return km.rs2_limit + (rc - km.rs2_segrows);
}

// stored column -> compact column, or -1 when the column is pruned
__device__ __forceinline__ int compact_col(const KeepMap& km, int k) {
  if (km.cs_stride == 0) return k < km.k_keep ? k : -1;
  int seg = k / km.cs_stride;
  int off = k - seg * km.cs_stride;
  return off < km.cs_keep ? seg * km.cs_keep + off : -1;
}

// 128-bit global load from an address that is only 2-byte aligned (one global_load_dwordx4: the
// target allows unaligned vector loads from global memory).
__device__ __forceinline__ uint4 load_u4_unaligned(const half_t* p) {
  typedef uint32_t u32x4_u2 __attribute__((ext_vector_type(4), aligned(2)));
  u32x4_u2 v = *reinterpret_cast<const u32x4_u2*>(p);
  return make_uint4(v.x, v.y, v.z, v.w);
}

// A load that sees what other compute units of the chip have written during the same launch (after the writer's
// release and this reader's acquire at agent scope): relaxed atomic loads at agent scope, which bypass the caches that
// are not coherent across the chip's dies.  8-byte aligned address.
__device__ __forceinline__ uint4 load_u4_coherent(const half_t* p) {
  const uint64_t* q = reinterpret_cast<const uint64_t*>(p);
  const uint64_t lo = __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  const uint64_t hi = __hip_atomic_load(q + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return make_uint4((uint32_t)lo, (uint32_t)(lo >> 32), (uint32_t)hi, (uint32_t)(hi >> 32));
}

__device__ __forceinline__ uint32_t load_u32_unaligned(const void* p) {
  typedef uint32_t u32_u1 __attribute__((aligned(1)));
  return *reinterpret_cast<const u32_u1*>(p);
}

// ---- int4 -> fp16 ---------------------------------------------------------
// A 32-bit word holds codes q0..q7.  OR-ing a masked word with an fp16 exponent
// pattern yields exact fp16 numbers without any conversion instruction:
//   (w      & 0x000F000F) | 0x64006400 = (1024 + q0, 1024 + q4)
//   (w      & 0x00F000F0) | 0x54005400 = (  64 + q1,   64 + q5)   (ulp of 64 is 1/16)
//   (w >> 8 & 0x000F000F) | 0x64006400 = (1024 + q2, 1024 + q6)
//   (w >> 8 & 0x00F000F0) | 0x54005400 = (  64 + q3,   64 + q7)
// Subtracting (1024 + z) resp. (64 + z) is exact in fp16 and the following fp16
// multiply by s rounds (q - z) * s once, to nearest even: the canonical weight.
struct GroupQ {   // per (row, group) constants, as packed halves
  half2_t zlo;    // (1024 + z, 1024 + z)
  half2_t zhi;    // (  64 + z,   64 + z)
  half2_t s2;     // (s, s)
};

__device__ __forceinline__ half2_t as_half2(uint32_t u) { return __builtin_bit_cast(half2_t, u); }
__device__ __forceinline__ uint32_t as_u32(half2_t h) { return __builtin_bit_cast(uint32_t, h); }

__device__ __forceinline__ GroupQ make_groupq(uint32_t scale_bits, uint32_t z) {
  GroupQ g;
  uint32_t zz = z | (z << 16);
  g.zlo = as_half2(zz | 0x64006400u);
  g.zhi = as_half2((zz << 4) | 0x54005400u);
  g.s2 = as_half2(scale_bits | (scale_bits << 16));
  return g;
}

// (a & mask) | orv in one VALU instruction.  The compiler splits this into v_and + v_or when
// both constants are literals (a VOP3 encoding cannot carry two of them on this target), so the
// mask is pinned to an SGPR and the exponent pattern to a VGPR.
__device__ __forceinline__ uint32_t and_or(uint32_t a, uint32_t mask, uint32_t orv) {
  asm("" : "+s"(mask));
  return (a & mask) | orv;   // selected as one v_and_or_b32 (written as inline asm it costs a wait state before every use)
}

// The two exponent patterns, materialised once per thread in VGPRs.
struct Magic {
  uint32_t m1024, m64;
};
__device__ __forceinline__ Magic make_magic() {
  Magic m = {0x64006400u, 0x54005400u};
  asm volatile("" : "+v"(m.m1024), "+v"(m.m64));   // keep them in registers, not re-materialised as literals
  return m;
}

// Dequantise one word into four half2: d[0]=(w0,w4) d[1]=(w1,w5) d[2]=(w2,w6) d[3]=(w3,w7).
__device__ __forceinline__ void dequant_word(uint32_t w, const GroupQ& g, const Magic& mg, half2_t d[4]) {
  uint32_t w8 = w >> 8;
  half2_t h0 = as_half2(and_or(w, 0x000F000Fu, mg.m1024));
  half2_t h1 = as_half2(and_or(w, 0x00F000F0u, mg.m64));
  half2_t h2 = as_half2(and_or(w8, 0x000F000Fu, mg.m1024));
  half2_t h3 = as_half2(and_or(w8, 0x00F000F0u, mg.m64));
  d[0] = (h0 - g.zlo) * g.s2;
  d[1] = (h1 - g.zhi) * g.s2;
  d[2] = (h2 - g.zlo) * g.s2;
  d[3] = (h3 - g.zhi) * g.s2;
}

// ---- int4 -> bfloat16 ------------------------------------------------------
// There is no packed bfloat16 arithmetic on this target, so the weight is formed in fp32 and rounded
// once by the packed conversion instruction (nearest even): q as a float from its byte (the even and
// the odd codes of a word are two masked words of four bytes each), then q * s - z * s in one fma.
// Both products are exact (4 x 8 significant bits) and so is their difference, (q - z) * s.
struct GroupQB {
  float s;      // scale
  float nzs;    // -(z * s)
};

__device__ __forceinline__ GroupQB make_groupqb(uint32_t scale_bits, uint32_t z) {
  GroupQB g;
  g.s = __builtin_bit_cast(float, scale_bits << 16);
  g.nzs = -((float)z * g.s);
  return g;
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  float2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));   // v_cvt_pk_bf16_f32
}

__device__ __forceinline__ float byte_f32(uint32_t v, int b) { return (float)((v >> (8 * b)) & 0xffu); }   // v_cvt_f32_ubyte<b>

// The four dwords of a dequantised word, as pairs (w0,w4) (w1,w5) (w2,w6) (w3,w7) like dequant_word.
// SIGNED_ZERO: a zero weight gets the sign of (q - z) * s (subtract first, then multiply: one more
// instruction per weight); without it a zero weight is +0, which no sum can tell apart.
template <bool SIGNED_ZERO>
__device__ __forceinline__ uint4 dequant_word_bf16(uint32_t w, const GroupQB& g, float zf) {
  uint32_t lo = w & 0x0F0F0F0Fu, hi = (w >> 4) & 0x0F0F0F0Fu;   // bytes q0 q2 q4 q6 / q1 q3 q5 q7
  asm("" : "+v"(lo), "+v"(hi));   // keep the two masked words: the byte conversions below read them in place
  float f[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const float qf = byte_f32(j & 1 ? hi : lo, j >> 1);
    f[j] = SIGNED_ZERO ? (qf - zf) * g.s : __builtin_fmaf(qf, g.s, g.nzs);
  }
  return make_uint4(pack_bf16(f[0], f[4]), pack_bf16(f[1], f[5]), pack_bf16(f[2], f[6]), pack_bf16(f[3], f[7]));
}

// ---- the two formats behind one set of names (BF16 = false: fp16) -------------
template <bool BF16> struct GroupOf { typedef GroupQ type; };
template <> struct GroupOf<true> { typedef GroupQB type; };

template <bool BF16>
__device__ __forceinline__ typename GroupOf<BF16>::type make_group(uint32_t scale_bits, uint32_t z) {
  if constexpr (BF16) return make_groupqb(scale_bits, z);
  else return make_groupq(scale_bits, z);
}

// the MFMA weight operand of one word (8 weights in the pair order above)
template <bool BF16>
__device__ __forceinline__ uint4 dequant_word4(uint32_t w, const typename GroupOf<BF16>::type& g, const Magic& mg) {
  if constexpr (BF16) {
    return dequant_word_bf16<false>(w, g, 0.f);
  } else {
    half2_t d[4];
    dequant_word(w, g, mg, d);
    return make_uint4(as_u32(d[0]), as_u32(d[1]), as_u32(d[2]), as_u32(d[3]));
  }
}

template <bool BF16>
__device__ __forceinline__ float4_t mfma_16x16x32(const uint4& a, const uint4& b, float4_t c) {
  if constexpr (BF16) return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
  else return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, a), __builtin_bit_cast(half8_t, b), c, 0, 0, 0);
}

// fp32 -> the 16-bit output element (nearest even), in the 16-bit container type of the pointers
template <bool BF16>
__device__ __forceinline__ half_t out16(float v) {
  if constexpr (BF16) return __builtin_bit_cast(half_t, (__bf16)v);
  else return (half_t)v;
}

// 16-bit element -> fp32
template <bool BF16>
__device__ __forceinline__ float in16(half_t v) {
  if constexpr (BF16) return __builtin_bit_cast(float, (uint32_t)__builtin_bit_cast(uint16_t, v) << 16);
  else return (float)v;
}

// host-side launchers (one per translation unit)
hipError_t launch_w4_gemv(const LinearArgs& a, hipStream_t stream);
hipError_t launch_w4_gemv_batch(const LinearArgs* probs, int n, hipStream_t stream);
// q, k, v of one token with the rotation of q and k fused into the launch; *fused = false (and nothing
// launched) when the shapes do not allow it
hipError_t launch_w4_qkv_rope(const LinearArgs* probs, const RopeFuse& rf, hipStream_t stream, bool* fused);
// gate and up of one token (probs[0], probs[1], same x) with h = SiLU(gate) * up written to probs[0].y
hipError_t launch_w4_gate_up_silu(const LinearArgs* probs, hipStream_t stream, bool* fused);
// the same four for matrices without zero points, and for bfloat16 with and without zero points (a
// translation unit each)
hipError_t launch_w4_gemv_sym(const LinearArgs& a, hipStream_t stream);
hipError_t launch_w4_gemv_batch_sym(const LinearArgs* probs, int n, hipStream_t stream);
hipError_t launch_w4_qkv_rope_sym(const LinearArgs* probs, const RopeFuse& rf, hipStream_t stream, bool* fused);
hipError_t launch_w4_gate_up_silu_sym(const LinearArgs* probs, hipStream_t stream, bool* fused);
hipError_t launch_w4_gemv_bf16(const LinearArgs& a, hipStream_t stream);
hipError_t launch_w4_gemv_batch_bf16(const LinearArgs* probs, int n, hipStream_t stream);
hipError_t launch_w4_qkv_rope_bf16(const LinearArgs* probs, const RopeFuse& rf, hipStream_t stream, bool* fused);
hipError_t launch_w4_gate_up_silu_bf16(const LinearArgs* probs, hipStream_t stream, bool* fused);
hipError_t launch_w4_gemv_bf16_sym(const LinearArgs& a, hipStream_t stream);
hipError_t launch_w4_gemv_batch_bf16_sym(const LinearArgs* probs, int n, hipStream_t stream);
hipError_t launch_w4_qkv_rope_bf16_sym(const LinearArgs* probs, const RopeFuse& rf, hipStream_t stream, bool* fused);
hipError_t launch_w4_gate_up_silu_bf16_sym(const LinearArgs* probs, hipStream_t stream, bool* fused);
// persistent streaming GEMV for tall row-prefix x column-prefix matrices; *done = false (nothing launched)
// when the shape is not one it serves
hipError_t launch_w4_gemv_stream(const LinearArgs& a, hipStream_t stream, bool* done);
hipError_t launch_w4_gate_up_stream(const LinearArgs* probs, hipStream_t stream, bool* done);
hipError_t launch_w4_gate_up_stream_probe(const LinearArgs* probs, hipStream_t stream, bool* done);
hipError_t launch_w4_gemv_stream_bf16(const LinearArgs& a, hipStream_t stream, bool* done);
// q, k, v of one token with the rotation of q and k as one walk of the streaming kernel; *done = false (nothing
// launched) when the shapes are not ones it serves
hipError_t launch_w4_qkv_rope_stream(const LinearArgs* probs, const RopeFuse& rf, hipStream_t stream, bool* done);
hipError_t launch_w4_qkv_rope_stream_bf16(const LinearArgs* probs, const RopeFuse& rf, hipStream_t stream, bool* done);
hipError_t launch_w4_gate_up_stream_bf16(const LinearArgs* probs, hipStream_t stream, bool* done);
// gate, up, down of one token in one persistent launch (probs[0..2]); the hidden vector (probs[0].y = probs[2].x) lies in
// `scratch` behind the launch's control and arrival words (see mlp_stream_kernel.h)
hipError_t launch_w4_mlp_fused(const LinearArgs* probs, void* scratch, hipStream_t stream, bool* done);
hipError_t launch_w4_mlp_fused_bf16(const LinearArgs* probs, void* scratch, hipStream_t stream, bool* done);
hipError_t launch_w4_gemm(const LinearArgs& a, hipStream_t stream);
hipError_t launch_w4_gemm_bf16(const LinearArgs& a, hipStream_t stream);
// n (2..4) linears of one decode batch in one launch where the decode-batch kernel takes them all (*done says whether)
hipError_t launch_w4_gemm_batch(const LinearArgs* a, int n, hipStream_t stream, bool* done);
hipError_t launch_w4_gemm_batch_bf16(const LinearArgs* a, int n, hipStream_t stream, bool* done);
// gate (p[0]) and up (p[1]) of a decode batch (2..16 tokens) with h = SiLU(g) * u in one launch (*done says whether)
hipError_t launch_w4_gate_up_silu_batch(const LinearArgs* p, hipStream_t stream, bool* done);
hipError_t launch_w4_gate_up_silu_batch_bf16(const LinearArgs* p, hipStream_t stream, bool* done);
hipError_t launch_w4_dequant(const LinearArgs& a, hipStream_t stream);
// codes of 8 bits: the dequantised matrix, and the linear for any number of tokens
hipError_t launch_w8_dequant(const LinearArgs& a, hipStream_t stream);
hipError_t launch_w8_linear(const LinearArgs& a, hipStream_t stream);
// codes of 3 and 6 bits (a.bits), packed as a bit stream: the same two operations
hipError_t launch_wb_dequant(const LinearArgs& a, hipStream_t stream);
hipError_t launch_wb_linear(const LinearArgs& a, hipStream_t stream);
hipError_t launch_w4_embedding(const uint32_t* qweight, const uint16_t* scales, const uint8_t* zeros, int K_total,
                               const int32_t* ids, int n, half_t* out, long long ld, int bf16, hipStream_t stream);

// Compact copy of the kept channels of a quantised matrix (host fills it from the repack plan).
struct RepackArgs {
  const uint32_t* qweight;
  const uint16_t* scales;
  const uint8_t* zeros;
  uint32_t* out_qweight;
  uint16_t* out_scales;
  uint8_t* out_zeros;
  int K_total, K_out;
  int gps_src, gps_out;   // groups per column segment in the source / carried to the output (gps_out = 0: all groups stay)
  KeepMap km;             // rows only
};
hipError_t launch_w4_repack(const RepackArgs& a, hipStream_t stream);
// the words of every row from [heads][words per head] to [words per head][heads]
hipError_t launch_w4_interleave(const uint32_t* qweight, uint32_t* out, int N_total, int K_total, int heads, bool inverse,
                                hipStream_t stream);

struct RopeArgs {
  half_t* q;
  half_t* k;
  const int32_t* positions;
  const int32_t* kept_idx;
  int T, Hq, Hkv, H_tab, D_full, D_keep;
  double theta;
  int bf16;   // q and k are bfloat16
};
hipError_t launch_pruned_rope(const RopeArgs& a, hipStream_t stream);
hipError_t launch_stream_read(const void* src, long long bytes, uint32_t* out, hipStream_t stream);

}  // namespace uniql
