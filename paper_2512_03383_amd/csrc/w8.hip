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

constexpr int kW8Threads = 256;

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

template <bool BF16>
__global__ __launch_bounds__(kW8Threads) void w8_gemv_kernel(LinearArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  uint16_t* xs = reinterpret_cast<uint16_t*>(smem);   // [16 * nchunks] at stored column positions
  const KeepMap& km = a.km;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int m = blockIdx.y;
  const int nchunks = (km.k_span + 15) >> 4;          // 16 codes (one 128-bit load) per chunk
  const uint16_t* xrow = reinterpret_cast<const uint16_t*>(a.x) + (size_t)m * a.ldx;
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

  const uint8_t* codes = reinterpret_cast<const uint8_t*>(a.qweight);
  const int groups_per_row = a.K_total / kGroup;
  const int waves = kW8Threads / 64;
  for (int rc = blockIdx.x * waves + wave; rc < km.n_keep; rc += gridDim.x * waves) {
    const size_t r = (size_t)stored_row(km, rc);
    const uint8_t* wrow = codes + r * a.K_total;
    float acc = 0.f;
    // four chunks per lane and step: their loads are issued together (chunks past the row's end re-read the last
    // one and are not added)
    for (int c0 = lane; c0 < nchunks; c0 += 4 * 64) {
      uint4 wq[4];
      uint32_t sb[4], zb[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int c = min(c0 + 64 * u, nchunks - 1);
        wq[u] = *reinterpret_cast<const uint4*>(wrow + 16 * c);
        const size_t g = r * groups_per_row + (c >> 3);
        sb[u] = a.scales[g];
        zb[u] = a.zeros ? a.zeros[g] : 128u;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int c = c0 + 64 * u;
        if (c < nchunks) {
          const uint4 w = wq[u];
          const uint32_t sbits = sb[u], z = zb[u];
          const uint4 x0 = *reinterpret_cast<const uint4*>(xs + 16 * c), x1 = *reinterpret_cast<const uint4*>(xs + 16 * c + 8);
          const uint32_t wv[4] = {w.x, w.y, w.z, w.w};
          const uint32_t xv[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
          if constexpr (!BF16) {
            const half2_t zz = as_half2(0x64006400u | z | (z << 16));      // (1024 + z, 1024 + z)
            const half2_t s2 = as_half2(sbits | (sbits << 16));
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const half2_t even = (as_half2((wv[i] & 0x00FF00FFu) | 0x64006400u) - zz) * s2;          // columns 4i, 4i + 2
              const half2_t odd = (as_half2(((wv[i] >> 8) & 0x00FF00FFu) | 0x64006400u) - zz) * s2;    // columns 4i + 1, 4i + 3
              acc = __builtin_amdgcn_fdot2(even, as_half2(xv[2 * i]), acc, false);
              acc = __builtin_amdgcn_fdot2(odd, as_half2(xv[2 * i + 1]), acc, false);
            }
          } else {
            const float s = __builtin_bit_cast(float, sbits << 16);
            const float nzs = -((float)z * s);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              float wf[4];
#pragma unroll
              for (int j = 0; j < 4; ++j) wf[j] = __builtin_fmaf(byte_f32(wv[i], j), s, nzs);   // exact: (q - z) s
              const uint32_t p01 = pack_bf16(wf[0], wf[1]), p23 = pack_bf16(wf[2], wf[3]);      // the canonical bfloat16 weights
              const uint32_t xa = xv[2 * i], xb = xv[2 * i + 1];
              acc = __builtin_fmaf(__builtin_bit_cast(float, xa << 16), __builtin_bit_cast(float, p01 << 16), acc);
              acc = __builtin_fmaf(__builtin_bit_cast(float, xa & 0xffff0000u), __builtin_bit_cast(float, p01 & 0xffff0000u), acc);
              acc = __builtin_fmaf(__builtin_bit_cast(float, xb << 16), __builtin_bit_cast(float, p23 << 16), acc);
              acc = __builtin_fmaf(__builtin_bit_cast(float, xb & 0xffff0000u), __builtin_bit_cast(float, p23 & 0xffff0000u), acc);
            }
          }
        }
      }
    }
    // the wave's sum, in a fixed order
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (lane == 0) a.y[(size_t)m * a.ldy + rc] = out16<BF16>(acc);
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
  if (bx > 512) bx = 512;   // two blocks per compute unit, each stages the activations once; waves walk the rows
  if (a.bf16) hipLaunchKernelGGL(w8_gemv_kernel<true>, dim3(bx, a.M), dim3(kW8Threads), smem, stream, a);
  else hipLaunchKernelGGL(w8_gemv_kernel<false>, dim3(bx, a.M), dim3(kW8Threads), smem, stream, a);
  return hipGetLastError();
}

}  // namespace uniql
