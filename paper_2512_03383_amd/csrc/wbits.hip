// Codes of 3 and 6 bits (Eq. 3 with N = 3, 6; Sec. 3.4 and App. C name 8, 6, 4 and 3 bits as the widths the method
// covers): the dequantised matrix and the linear y = x W'^T.  A row's codes are one little-endian bit stream over its
// 32-bit words: code k sits in bits [N k, N k + N) of the stream, so some codes run over a word boundary.  Zero points
// are 0..2^N - 1 (NULL: 2^(N-1)).  The weight is the 16-bit float nearest (ties to even) to (q - z) * s, as for 4-bit
// codes.
//
// The linear is a streaming kernel bound by the byte stream of the weights, with the launch shape of the 8-bit one: a
// block stages its token's activations in LDS, a wave walks rows, a lane takes units of three words (96 bits = 32 codes
// of 3 bits or 16 codes of 6 bits; groups of 128 columns are whole units).  Inside a unit of C codes, code p and code
// p + C/2 lie 48 bits apart, i.e. at the same offset of two 16-bit half-words, so one merged register
// (low half from one word, high half from another) shifted by a constant and masked gives the pair
// (1024 + q_p, 1024 + q_{p + C/2}) as exact fp16 numbers; three merged registers cover every pair whose low code lies
// inside a half-word, the two pairs per unit whose codes run over a half-word boundary take two funnel shifts and a
// merge of their own.  The subtraction of 1024 + z is exact, the fp16 multiply by s rounds once, and the pair meets
// (x_p, x_{p + C/2}) in one two-element dot product with fp32 accumulation (the activations are staged in that order,
// 16 bytes = four pairs per piece, piece-major so that the 64 lanes of a wave read consecutive pieces).  bfloat16: the
// weight is formed in fp32 (q s - z s, exact) and rounded by the packed conversion.  One launch serves one token per
// block row (grid.y = tokens): batches re-read the weights through L2.
#include "common.h"

namespace uniql {

constexpr int kWbThreads = 512;

template <int BITS, bool BF16>
__global__ __launch_bounds__(kWbThreads) void wb_dequant_kernel(LinearArgs a) {
  const long long total = (long long)a.km.n_keep * a.km.k_keep;
  const size_t words_per_row = (size_t)a.K_total * BITS / 32;
  const int groups_per_row = a.K_total / kGroup;
  for (long long i = (long long)blockIdx.x * kWbThreads + threadIdx.x; i < total; i += (long long)gridDim.x * kWbThreads) {
    const int rc = (int)(i / a.km.k_keep), kc = (int)(i - (long long)rc * a.km.k_keep);
    const int r = stored_row(a.km, rc);
    int k = kc;
    if (a.km.cs_stride != 0) {
      const int seg = kc / a.km.cs_keep;
      k = seg * a.km.cs_stride + (kc - seg * a.km.cs_keep);
    }
    const uint32_t* row = a.qweight + (size_t)r * words_per_row;
    const int pos = BITS * k, w = pos >> 5, o = pos & 31;
    uint32_t bits = row[w] >> o;
    if (o + BITS > 32) bits |= row[w + 1] << (32 - o);   // the code's upper part: the next word of the same row
    const int q = (int)(bits & ((1u << BITS) - 1u));
    const size_t g = (size_t)r * groups_per_row + k / kGroup;
    const int z = a.zeros ? a.zeros[g] : 1 << (BITS - 1);
    const float s = in16<BF16>(__builtin_bit_cast(half_t, a.scales[g]));
    a.y[i] = out16<BF16>((float)(q - z) * s);   // the product is exact in fp32 (7 x 11 bits): one rounding
  }
}

// Sum over the 64 lanes of a wave, valid in lane 63, in a fixed order: two quad permutes, the two mirrors of a row of 16
// lanes and the two row broadcasts.
#define UNIQL_WB_DPP(v, ctrl) __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, (v)), (ctrl), 0xF, 0xF, true))
__device__ __forceinline__ float wb_wave_sum_to_lane63(float t) {
  t += UNIQL_WB_DPP(t, 0xB1);    // quad_perm [1,0,3,2]
  t += UNIQL_WB_DPP(t, 0x4E);    // quad_perm [2,3,0,1]
  t += UNIQL_WB_DPP(t, 0x141);   // row_half_mirror
  t += UNIQL_WB_DPP(t, 0x140);   // row_mirror
  // the row broadcasts add in place; the s_nop is the wait a DPP instruction needs after the write of its operand
  asm volatile("s_nop 1\n\tv_add_f32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\ts_nop 1\n\t"
               "v_add_f32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf" : "+v"(t));
  return t;
}

typedef uint32_t u32x3_a4 __attribute__((ext_vector_type(3), aligned(4)));

// low 16 bits of lo, high 16 bits of hi
__device__ __forceinline__ uint32_t merge_halves(uint32_t lo, uint32_t hi) { return __builtin_amdgcn_perm(hi, lo, 0x07060100u); }

// The C/2 pairs of a unit (three words of the stream) as registers holding code p in bits 0.. and code p + C/2 in
// bits 16.., OR-ed into the fp16 exponent pattern of 1024 (upper bits of both halves cleared by the mask).
template <int BITS>
__device__ __forceinline__ void unit_pairs(uint32_t w0, uint32_t w1, uint32_t w2, uint32_t m1024, uint32_t (&out)[48 / BITS]) {
  constexpr uint32_t kMask = ((1u << BITS) - 1u) * 0x00010001u;
  const uint32_t merged[3] = {merge_halves(w0, w1),                       // stream bits 0..15 | 48..63
                              __builtin_amdgcn_alignbit(w2, w0, 16),      // 16..31 | 64..79
                              merge_halves(w1, w2)};                      // 32..47 | 80..95
#pragma unroll
  for (int p = 0; p < 48 / BITS; ++p) {
    const int s = BITS * p, h = s >> 4, o = s & 15;
    uint32_t src;
    if (o + BITS <= 16) {
      src = o == 0 ? merged[h] : merged[h] >> o;
    } else {
      // the low code runs over a half-word boundary (s < 32 for both widths): 32-bit windows of the stream at s and s + 32
      src = merge_halves(__builtin_amdgcn_alignbit(w1, w0, s & 31), __builtin_amdgcn_alignbit(w2, w1, s & 31));
    }
    out[p] = and_or(src, kMask, m1024);
  }
}

template <int BITS, bool BF16>
__global__ __launch_bounds__(kWbThreads) void wb_gemv_kernel(LinearArgs a) {
  constexpr int C = 96 / BITS;       // codes per unit: 32 or 16
  constexpr int P = C / 8;           // 16-byte pieces of staged activations per unit: four pairs each
  constexpr int U = 2;               // units per lane and item
  constexpr int UG = kGroup / C;     // units per group
  static_assert(BITS == 3 || BITS == 6, "units of three words hold 32 codes of 3 bits or 16 codes of 6 bits");
  extern __shared__ __align__(16) unsigned char smem[];
  uint16_t* xs = reinterpret_cast<uint16_t*>(smem);   // [P][nunits] pieces of 8 elements
  const KeepMap& km = a.km;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int m = blockIdx.y;
  const int nunits = (km.k_span + C - 1) / C;
  const uint16_t* xrow = reinterpret_cast<const uint16_t*>(a.x) + (size_t)m * a.ldx;

  const size_t words_per_row = (size_t)a.K_total * BITS / 32;
  const int groups_per_row = a.K_total / kGroup;
  const int waves = kWbThreads / 64;
  // A wave walks rows; an item is one step of a row: U units per lane, whose loads are issued together (units past the
  // row's end re-read the last one and are multiplied by a zero scale).  The loads of the item three further on are
  // issued before the current one is multiplied, and those of the first three items before the activations are staged.
  // The loop body has no branch: zero points of a matrix that has none are read through an empty buffer resource (they
  // come back as zero and are replaced), and the output goes through a buffer store whose offset lies beyond the
  // resource except in lane 63 at the end of a row.
  struct Item {
    u32x3_a4 wq[U];
    uint32_t sb[U], zb[U];
  };
  constexpr uint32_t kRsrcWord3 = 0x00020000u;
  constexpr int kNone = (int)0x80000000u;
  const bool has_z = a.zeros != nullptr;
  const uint32_t zmask = has_z ? 0xffu : 0u, zdef = has_z ? 0u : (1u << (BITS - 1));
  const long long nsz = (long long)a.N_total * groups_per_row;             // (launch_wb_linear bounds it)
  const __amdgpu_buffer_rsrc_t rz = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(a.zeros), 0, has_z ? (int)nsz : 0, kRsrcWord3);
  const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(a.y + (size_t)m * a.ldy, 0, km.n_keep * 2, kRsrcWord3);
  const int steps = (nunits + U * 64 - 1) / (U * 64);
  const int stride = gridDim.x * waves;
  auto issue = [&](int rc, int step, Item& it) {
    const int r = stored_row(km, rc < km.n_keep ? rc : km.n_keep - 1);   // past the last row: a valid, unused load
    const uint32_t* wrow = a.qweight + (size_t)r * words_per_row;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int c = min(step * (U * 64) + lane + 64 * u, nunits - 1);
      it.wq[u] = *reinterpret_cast<const u32x3_a4*>(wrow + 3 * c);
      const int g = r * groups_per_row + c / UG;
      it.sb[u] = a.scales[g];
      it.zb[u] = __builtin_amdgcn_raw_buffer_load_b8(rz, g, 0, 0);
    }
  };
  int rc = blockIdx.x * waves + wave, step = 0;
  int irc = rc, istep = 0;
  auto advance = [&](int& r, int& st) {
    if (++st == steps) { st = 0; r += stride; }
  };
  Item it0, it1, it2, it3;
  issue(irc, istep, it0);
  advance(irc, istep);
  issue(irc, istep, it1);
  advance(irc, istep);
  issue(irc, istep, it2);
  advance(irc, istep);
  __builtin_amdgcn_sched_barrier(0);

  // staged order: piece j of unit c (at [j][c]) holds the pairs 4j .. 4j+3, pair p = (column p, column p + C/2) of the unit
  if (km.cs_stride == 0) {
    // a column prefix: a thread takes 8 columns of the lower half of a unit and the 8 columns C/2 further on (128-bit
    // loads; the 8 columns with the last kept ones by element), and writes the two pieces they interleave to
    const int kv = km.k_keep & ~7;
    auto load8 = [&](int k0) {
      uint4 v = make_uint4(0u, 0u, 0u, 0u);
      if (k0 + 8 <= kv) {
        v = load_u4_unaligned(a.x + (size_t)m * a.ldx + k0);
      } else if (k0 < km.k_keep) {
        uint32_t e[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) e[j] = k0 + j < km.k_keep ? (uint32_t)xrow[k0 + j] : 0u;
        v = make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16));
      }
      return v;
    };
    constexpr int TPU = C / 16;   // threads per unit
    for (int t = tid; t < nunits * TPU; t += kWbThreads) {
      const int c = t / TPU, sub = t - c * TPU;
      const uint4 lo = load8(c * C + 8 * sub), hi = load8(c * C + C / 2 + 8 * sub);
      const uint4 p0 = make_uint4(__builtin_amdgcn_perm(hi.x, lo.x, 0x05040100u), __builtin_amdgcn_perm(hi.x, lo.x, 0x07060302u),
                                  __builtin_amdgcn_perm(hi.y, lo.y, 0x05040100u), __builtin_amdgcn_perm(hi.y, lo.y, 0x07060302u));
      const uint4 p1 = make_uint4(__builtin_amdgcn_perm(hi.z, lo.z, 0x05040100u), __builtin_amdgcn_perm(hi.z, lo.z, 0x07060302u),
                                  __builtin_amdgcn_perm(hi.w, lo.w, 0x05040100u), __builtin_amdgcn_perm(hi.w, lo.w, 0x07060302u));
      *reinterpret_cast<uint4*>(xs + ((size_t)(2 * sub) * nunits + c) * 8) = p0;
      *reinterpret_cast<uint4*>(xs + ((size_t)(2 * sub + 1) * nunits + c) * 8) = p1;
    }
  } else {
    for (int k = tid; k < nunits * C; k += kWbThreads) {
      const int kc = k < km.k_span ? compact_col(km, k) : -1;
      const int c = k / C, j = k - c * C;
      const int hi = j >= C / 2 ? 1 : 0, p = j - hi * (C / 2);
      xs[((size_t)(p >> 2) * nunits + c) * 8 + 2 * (p & 3) + hi] = kc >= 0 ? xrow[kc] : (uint16_t)0;
    }
  }
  __syncthreads();

  float acc = 0.f;
  const Magic mg = make_magic();
  auto process = [&](const Item& cur, Item& refill) {
    issue(irc, istep, refill);
    advance(irc, istep);
    __builtin_amdgcn_sched_barrier(0);   // the loads stay ahead of the arithmetic
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int cu = step * (U * 64) + lane + 64 * u;
      const int c = min(cu, nunits - 1);
      const uint32_t sbits = cu < nunits ? cur.sb[u] : 0u;   // a unit past the row's end adds zeros
      const uint32_t z = (cur.zb[u] & zmask) | zdef;
      uint32_t pr[C / 2];
      unit_pairs<BITS>(cur.wq[u].x, cur.wq[u].y, cur.wq[u].z, mg.m1024, pr);
      uint32_t xv[C / 2];
#pragma unroll
      for (int j = 0; j < P; ++j) {
        const uint4 x4 = *reinterpret_cast<const uint4*>(xs + ((size_t)j * nunits + c) * 8);
        xv[4 * j] = x4.x; xv[4 * j + 1] = x4.y; xv[4 * j + 2] = x4.z; xv[4 * j + 3] = x4.w;
      }
      if constexpr (!BF16) {
        const half2_t zz = as_half2(0x64006400u | z | (z << 16));      // (1024 + z, 1024 + z)
        const half2_t s2 = as_half2(sbits | (sbits << 16));
#pragma unroll
        for (int p = 0; p < C / 2; ++p) {
          const half2_t wv = (as_half2(pr[p]) - zz) * s2;               // the canonical weights of columns p, p + C/2
          acc = __builtin_amdgcn_fdot2(wv, as_half2(xv[p]), acc, false);
        }
      } else {
        const float sc = __builtin_bit_cast(float, sbits << 16);
        const float nzs = -((float)z * sc);
#pragma unroll
        for (int p = 0; p < C / 2; ++p) {
          const float wl = __builtin_fmaf(byte_f32(pr[p], 0), sc, nzs), wh = __builtin_fmaf(byte_f32(pr[p], 2), sc, nzs);   // exact: (q - z) s
          const uint32_t pw = pack_bf16(wl, wh);                        // the canonical bfloat16 weights
          acc = __builtin_fmaf(__builtin_bit_cast(float, xv[p] << 16), __builtin_bit_cast(float, pw << 16), acc);
          acc = __builtin_fmaf(__builtin_bit_cast(float, xv[p] & 0xffff0000u), __builtin_bit_cast(float, pw & 0xffff0000u), acc);
        }
      }
    }
    // the wave's sum, in a fixed order; it is stored at the end of a row only
    const float tot = wb_wave_sum_to_lane63(acc);
    const bool row_end = step == steps - 1;
    __builtin_amdgcn_raw_buffer_store_b16(__builtin_bit_cast(uint16_t, out16<BF16>(tot)), ry, row_end && lane == 63 ? 2 * rc : kNone, 0, 0);
    acc = row_end ? 0.f : acc;
    advance(rc, step);
  };
  for (;;) {
    if (rc >= km.n_keep) break;
    process(it0, it3);
    if (rc >= km.n_keep) break;
    process(it1, it0);
    if (rc >= km.n_keep) break;
    process(it2, it1);
    if (rc >= km.n_keep) break;
    process(it3, it2);
  }
}

template <int BITS>
static hipError_t dequant_bits(const LinearArgs& a, hipStream_t stream) {
  const long long total = (long long)a.km.n_keep * a.km.k_keep;
  long long blocks = (total + kWbThreads - 1) / kWbThreads;
  if (blocks > 8192) blocks = 8192;
  if (a.bf16) hipLaunchKernelGGL((wb_dequant_kernel<BITS, true>), dim3((unsigned)blocks), dim3(kWbThreads), 0, stream, a);
  else hipLaunchKernelGGL((wb_dequant_kernel<BITS, false>), dim3((unsigned)blocks), dim3(kWbThreads), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_wb_dequant(const LinearArgs& a, hipStream_t stream) {
  return a.bits == 3 ? dequant_bits<3>(a, stream) : dequant_bits<6>(a, stream);
}

template <int BITS>
static hipError_t linear_bits(const LinearArgs& a, hipStream_t stream) {
  constexpr int C = 96 / BITS;
  const int nunits = (a.km.k_span + C - 1) / C;
  const size_t smem = (size_t)nunits * C * 2;
  if (smem > 64 * 1024 || a.M > 65535) return hipErrorInvalidValue;
  if ((long long)a.N_total * (a.K_total / kGroup) > 0x7fffffffLL) return hipErrorInvalidValue;   // group indices are 32-bit
  const int waves = kWbThreads / 64;
  int bx = (a.km.n_keep + waves - 1) / waves;
  if (bx > 256) bx = 256;   // a block of eight waves per compute unit, each stages the activations once; waves walk the rows
                            // (3-bit gate / down shapes 10.7 / 11.1 us; 512 blocks 10.9 / 12.2, 384 blocks 12.1 / 13.9)
  if (a.bf16) hipLaunchKernelGGL((wb_gemv_kernel<BITS, true>), dim3(bx, a.M), dim3(kWbThreads), smem, stream, a);
  else hipLaunchKernelGGL((wb_gemv_kernel<BITS, false>), dim3(bx, a.M), dim3(kWbThreads), smem, stream, a);
  return hipGetLastError();
}

// hipErrorInvalidValue: rows whose kept span does not fit the LDS image of the activations (more than 32768 columns)
hipError_t launch_wb_linear(const LinearArgs& a, hipStream_t stream) {
  return a.bits == 3 ? linear_bits<3>(a, stream) : linear_bits<6>(a, stream);
}

}  // namespace uniql
