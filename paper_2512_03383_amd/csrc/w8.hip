// Codes of 8 bits (Eq. 3 with N = 8; Sec. 3.4 and App. C name 8, 6, 4 and 3 bits as the widths the method covers):
// the dequantised matrix and the linear y = x W'^T.  qweight holds four codes per 32-bit word, byte j of word w of a
// row = input column 4 w + j; zero points are 0..255 (NULL: 128).  The weight is the 16-bit float nearest (ties to
// even) to (q - z) * s, as for 4-bit codes.
//
// The linear is a plain streaming kernel, bound by the byte stream of the weights: a block stages its token's
// activations in LDS at stored column positions (zeros where pruned), a wave walks rows, a lane takes 16 codes per
// 128-bit load.  fp16: (w & 0x00FF00FF) | 0x64006400 is the pair (1024 + q0, 1024 + q2) as exact fp16 numbers, the
// subtraction of 1024 + z is exact and the fp16 multiply by s rounds once; the pair meets (x0, x2) in one
// two-element dot product with fp32 accumulation (the activations are staged in that order).  bfloat16: the weight is
// formed in fp32 (q s - z s, exact) and rounded by the packed conversion.  One launch serves one token per block row
// (grid.y = tokens): batches re-read the weights through L2, which is what an occasional 8-bit layer needs, not a
// prefill kernel.
#include "common.h"

namespace uniql {

constexpr int kW8Threads = 512;

// compact column -> stored column
__device__ __forceinline__ int stored_col(const KeepMap& km, int kc) {
  if (km.cs_stride == 0) return kc;
  const int seg = kc / km.cs_keep;
  return seg * km.cs_stride + (kc - seg * km.cs_keep);
}

template <bool BF16>
__global__ __launch_bounds__(kW8Threads) void w8_dequant_kernel(LinearArgs a) {
  const long long total = (long long)a.km.n_keep * a.km.k_keep;
  const uint8_t* codes = reinterpret_cast<const uint8_t*>(a.qweight);
  const int groups_per_row = a.K_total / kGroup;
  for (long long i = (long long)blockIdx.x * kW8Threads + threadIdx.x; i < total; i += (long long)gridDim.x * kW8Threads) {
    const int rc = (int)(i / a.km.k_keep), kc = (int)(i - (long long)rc * a.km.k_keep);
    const int r = stored_row(a.km, rc), k = stored_col(a.km, kc);
    const int q = codes[(size_t)r * a.K_total + k];
    const size_t g = (size_t)r * groups_per_row + k / kGroup;
    const int z = a.zeros ? a.zeros[g] : 128;
    const float s = in16<BF16>(__builtin_bit_cast(half_t, a.scales[g]));
    a.y[i] = out16<BF16>((float)(q - z) * s);   // the product is exact in fp32 (9 x 11 bits): one rounding
  }
}

// Sum over the 64 lanes of a wave, valid in lane 63, in a fixed order: two quad permutes, the two mirrors of a row of 16
// lanes and the two row broadcasts -- six DPP additions, no LDS crossbar.
#define UNIQL_W8_DPP(v, ctrl) __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, (v)), (ctrl), 0xF, 0xF, true))
__device__ __forceinline__ float wave_sum_to_lane63(float t) {
  t += UNIQL_W8_DPP(t, 0xB1);    // quad_perm [1,0,3,2]
  t += UNIQL_W8_DPP(t, 0x4E);    // quad_perm [2,3,0,1]
  t += UNIQL_W8_DPP(t, 0x141);   // row_half_mirror
  t += UNIQL_W8_DPP(t, 0x140);   // row_mirror
  // the row broadcasts add in place (rows outside the row mask keep their value); the s_nop is the wait a DPP
  // instruction needs after the instruction that wrote its operand
  asm volatile("s_nop 1\n\tv_add_f32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\ts_nop 1\n\t"
               "v_add_f32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf" : "+v"(t));
  return t;
}

template <bool BF16>
__global__ __launch_bounds__(kW8Threads) void w8_gemv_kernel(LinearArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  uint16_t* xs = reinterpret_cast<uint16_t*>(smem);   // [16 * nchunks] at stored column positions
  const KeepMap& km = a.km;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int m = blockIdx.y;
  const int nchunks = (km.k_span + 15) >> 4;          // 16 codes (one 128-bit load) per chunk
  const uint16_t* xrow = reinterpret_cast<const uint16_t*>(a.x) + (size_t)m * a.ldx;

  const uint8_t* codes = reinterpret_cast<const uint8_t*>(a.qweight);
  const int groups_per_row = a.K_total / kGroup;
  const int waves = kW8Threads / 64;
  // A wave walks rows; an item is one step of a row: four chunks per lane, whose loads are issued together (chunks
  // past the row's end re-read the last one and are multiplied by a zero scale).  The loads of the next item are
  // two items further on are issued before the current one is multiplied, and those of the first two items before the
  // activations are staged, so a wave always has two steps in flight.  The loop body has no branch: zero points of a matrix that has none are read
  // through an empty buffer resource (they come back as zero and are replaced), and the output goes through a buffer
  // store whose offset lies beyond the resource except in lane 63 at the end of a row -- with a branch around a load or
  // store the compiler drains every load at the join.
  struct Item {
    uint4 wq[4];
    uint32_t sb[4], zb[4];
  };
  constexpr uint32_t kRsrcWord3 = 0x00020000u;
  constexpr int kNone = (int)0x80000000u;
  const bool has_z = a.zeros != nullptr;
  const uint32_t zmask = has_z ? 0xffu : 0u, zdef = has_z ? 0u : 128u;   // (arithmetic, not a branch per chunk)
  const long long nsz = (long long)a.N_total * groups_per_row;             // (launch_w8_linear bounds it)
  const __amdgpu_buffer_rsrc_t rz = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(a.zeros), 0, has_z ? (int)nsz : 0, kRsrcWord3);
  const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(a.y + (size_t)m * a.ldy, 0, km.n_keep * 2, kRsrcWord3);
  const int steps = (nchunks + 4 * 64 - 1) / (4 * 64);
  const int stride = gridDim.x * waves;
  auto issue = [&](int rc, int step, Item& it) {
    const int r = stored_row(km, rc < km.n_keep ? rc : km.n_keep - 1);   // past the last row: a valid, unused load
    const uint8_t* wrow = codes + (size_t)r * a.K_total;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int c = min(step * 256 + lane + 64 * u, nchunks - 1);
      it.wq[u] = *reinterpret_cast<const uint4*>(wrow + 16 * c);
      const int g = r * groups_per_row + (c >> 3);
      it.sb[u] = a.scales[g];
      it.zb[u] = __builtin_amdgcn_raw_buffer_load_b8(rz, g, 0, 0);
    }
  };
  // (rc, step): the item being multiplied; (irc, istep): the item whose loads are issued next, two items further on
  int rc = blockIdx.x * waves + wave, step = 0;
  int irc = rc, istep = 0;
  auto advance = [&](int& r, int& st) {
    if (++st == steps) { st = 0; r += stride; }
  };
  Item it0, it1, it2;
  issue(irc, istep, it0);
  advance(irc, istep);
  issue(irc, istep, it1);
  advance(irc, istep);
  __builtin_amdgcn_sched_barrier(0);

  // fp16: inside every aligned four columns the order is (0, 2, 1, 3), the pair order of the byte unpack
  if (km.cs_stride == 0) {
    // a column prefix: units of 8 columns with one 128-bit load each, the unit with the last kept columns by element
    const int kv = km.k_keep & ~7;
    for (int u = tid; u < nchunks * 2; u += kW8Threads) {
      const int k0 = 8 * u;
      uint4 v = make_uint4(0u, 0u, 0u, 0u);
      if (k0 + 8 <= kv) {
        v = load_u4_unaligned(a.x + (size_t)m * a.ldx + k0);
      } else if (k0 < km.k_keep) {
        uint32_t e[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) e[j] = k0 + j < km.k_keep ? (uint32_t)xrow[k0 + j] : 0u;
        v = make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16));
      }
      if constexpr (!BF16)
        v = make_uint4(__builtin_amdgcn_perm(v.y, v.x, 0x05040100u), __builtin_amdgcn_perm(v.y, v.x, 0x07060302u),
                       __builtin_amdgcn_perm(v.w, v.z, 0x05040100u), __builtin_amdgcn_perm(v.w, v.z, 0x07060302u));
      *reinterpret_cast<uint4*>(xs + k0) = v;
    }
  } else {
    for (int k = tid; k < nchunks * 16; k += kW8Threads) {
      const int kc = k < km.k_span ? compact_col(km, k) : -1;
      const int pos = BF16 ? k : ((k & ~3) | ((k & 1) << 1) | ((k >> 1) & 1));
      xs[pos] = kc >= 0 ? xrow[kc] : (uint16_t)0;
    }
  }
  __syncthreads();

  float acc = 0.f;
  const Magic mg = make_magic();
  // one item: the loads of the item two further on go out first, into the registers the previous item has left
  auto process = [&](const Item& cur, Item& refill) {
    issue(irc, istep, refill);
    advance(irc, istep);
    __builtin_amdgcn_sched_barrier(0);   // the loads stay ahead of the arithmetic
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int cu = step * 256 + lane + 64 * u;
      const int c = min(cu, nchunks - 1);
      const uint4 w = cur.wq[u];
      const uint32_t sbits = cu < nchunks ? cur.sb[u] : 0u;   // a chunk past the row's end adds zeros
      const uint32_t z = (cur.zb[u] & zmask) | zdef;          // no zero points: every zero point is 128
      const uint4 x0 = *reinterpret_cast<const uint4*>(xs + 16 * c), x1 = *reinterpret_cast<const uint4*>(xs + 16 * c + 8);
      const uint32_t wv[4] = {w.x, w.y, w.z, w.w};
      const uint32_t xv[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
      if constexpr (!BF16) {
        const half2_t zz = as_half2(0x64006400u | z | (z << 16));      // (1024 + z, 1024 + z)
        const half2_t s2 = as_half2(sbits | (sbits << 16));
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const half2_t even = (as_half2(and_or(wv[i], 0x00FF00FFu, mg.m1024)) - zz) * s2;         // columns 4i, 4i + 2
          const half2_t odd = (as_half2(and_or(wv[i] >> 8, 0x00FF00FFu, mg.m1024)) - zz) * s2;     // columns 4i + 1, 4i + 3
          acc = __builtin_amdgcn_fdot2(even, as_half2(xv[2 * i]), acc, false);
          acc = __builtin_amdgcn_fdot2(odd, as_half2(xv[2 * i + 1]), acc, false);
        }
      } else {
        const float sc = __builtin_bit_cast(float, sbits << 16);
        const float nzs = -((float)z * sc);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float wf[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) wf[j] = __builtin_fmaf(byte_f32(wv[i], j), sc, nzs);   // exact: (q - z) s
          const uint32_t p01 = pack_bf16(wf[0], wf[1]), p23 = pack_bf16(wf[2], wf[3]);      // the canonical bfloat16 weights
          const uint32_t xa = xv[2 * i], xb = xv[2 * i + 1];
          acc = __builtin_fmaf(__builtin_bit_cast(float, xa << 16), __builtin_bit_cast(float, p01 << 16), acc);
          acc = __builtin_fmaf(__builtin_bit_cast(float, xa & 0xffff0000u), __builtin_bit_cast(float, p01 & 0xffff0000u), acc);
          acc = __builtin_fmaf(__builtin_bit_cast(float, xb << 16), __builtin_bit_cast(float, p23 << 16), acc);
          acc = __builtin_fmaf(__builtin_bit_cast(float, xb & 0xffff0000u), __builtin_bit_cast(float, p23 & 0xffff0000u), acc);
        }
      }
    }
    // the wave's sum, in a fixed order; it is stored at the end of a row only
    const float tot = wave_sum_to_lane63(acc);
    const bool row_end = step == steps - 1;
    __builtin_amdgcn_raw_buffer_store_b16(__builtin_bit_cast(uint16_t, out16<BF16>(tot)), ry, row_end && lane == 63 ? 2 * rc : kNone, 0, 0);
    acc = row_end ? 0.f : acc;
    advance(rc, step);
  };
  for (;;) {
    if (rc >= km.n_keep) break;
    process(it0, it2);
    if (rc >= km.n_keep) break;
    process(it1, it0);
    if (rc >= km.n_keep) break;
    process(it2, it1);
  }
}

hipError_t launch_w8_dequant(const LinearArgs& a, hipStream_t stream) {
  const long long total = (long long)a.km.n_keep * a.km.k_keep;
  long long blocks = (total + kW8Threads - 1) / kW8Threads;
  if (blocks > 8192) blocks = 8192;
  if (a.bf16) hipLaunchKernelGGL(w8_dequant_kernel<true>, dim3((unsigned)blocks), dim3(kW8Threads), 0, stream, a);
  else hipLaunchKernelGGL(w8_dequant_kernel<false>, dim3((unsigned)blocks), dim3(kW8Threads), 0, stream, a);
  return hipGetLastError();
}

// hipErrorInvalidValue: rows whose kept span does not fit the LDS image of the activations (more than 32768 columns)
hipError_t launch_w8_linear(const LinearArgs& a, hipStream_t stream) {
  const int nchunks = (a.km.k_span + 15) >> 4;
  const size_t smem = (size_t)nchunks * 32;
  if (smem > 64 * 1024 || a.M > 65535) return hipErrorInvalidValue;
  const int waves = kW8Threads / 64;
  int bx = (a.km.n_keep + waves - 1) / waves;
  if (bx > 256) bx = 256;   // a block of eight waves per compute unit, each stages the activations once; waves walk the rows
                            // (gate / down shapes: 13.7 / 13.9 us; 512 blocks of four waves 13.5 / 14.5, 384 blocks of eight 15.1 / 16.9)
  if (a.bf16) hipLaunchKernelGGL(w8_gemv_kernel<true>, dim3(bx, a.M), dim3(kW8Threads), smem, stream, a);
  else hipLaunchKernelGGL(w8_gemv_kernel<false>, dim3(bx, a.M), dim3(kW8Threads), smem, stream, a);
  return hipGetLastError();
}

}  // namespace uniql
