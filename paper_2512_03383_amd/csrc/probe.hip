// Read-stream probe: the bandwidth ceiling the GEMV is measured against.
// Each wave reads 8 KB (eight 1 KB wave-wide 128-bit loads in flight), xors the
// words together and writes one word per wave, so the compiler cannot drop the loads.
#include "common.h"

namespace uniql {

__global__ __launch_bounds__(256) void stream_read_kernel(const uint4* __restrict__ src, long long n16,
                                                          uint32_t* __restrict__ out) {
  const long long wave = ((long long)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int lane = threadIdx.x & 63;
  const long long base = wave * 512 + lane;   // 512 uint4 = 8 KB per wave
  uint4 v[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const long long idx = base + i * 64;
    v[i] = idx < n16 ? src[idx] : make_uint4(0, 0, 0, 0);
  }
  uint32_t x = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i) x ^= v[i].x ^ v[i].y ^ v[i].z ^ v[i].w;
  for (int o = 32; o > 0; o >>= 1) x ^= __shfl_xor(x, o);
  if (lane == 0 && base < n16) out[wave] = x;
}

hipError_t launch_stream_read(const void* src, long long bytes, uint32_t* out, hipStream_t stream) {
  const long long n16 = bytes / 16;
  const long long waves = (n16 + 511) / 512;
  const long long blocks = (waves + 3) / 4;
  if (blocks < 1) return hipSuccess;
  hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)blocks), dim3(256), 0, stream,
                     (const uint4*)src, n16, out);
  return hipGetLastError();
}

}  // namespace uniql
