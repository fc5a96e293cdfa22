// The gated MLP of one token in ONE persistent launch (Eq. 1): y = W_down (SiLU(W_gate x) * (W_up x)).
//
// Two walks of gemv_stream_kernel.h back to back on the same grid: gate + up with the activation as epilogue writes
// the hidden vector h (16-bit, like every activation of the path) to scratch memory, down reads it.  Every row of
// W_down needs all of h, so the second walk cannot start its arithmetic before the whole grid has finished the first.
// A wave that has finished its gate / up rows issues the first tiles of its first down row and only then waits, so the
// stream of W_down is already running when the last block arrives.
//
// How the grid meets.  A word per block in scratch memory holds the tag (serial number) of the last launch whose first
// walk the block has finished: a block stores it once all of its waves have seen their stores to h acknowledged, one
// wave per block polls all words with one load per lane.  h is written through to memory and read with loads that
// bypass the L2s (a cache write-back / invalidation walks a whole 4 MB L2; issued by every wave it took tens of
// microseconds).  The serial number lives in the scratch memory itself, so that a captured launch can be replayed:
// every block reads it at its start, block 0 stores the incremented value at its end.  The wait is bounded
// (`wait_ticks`): a block that does not see every word in time records the tag in the give-up word and skips its down
// rows; every wave still runs to its end.  The grid is one block per CU and must be resident as a whole, which it is
// on an otherwise idle device; launches that share the scratch memory must not overlap.
//
// What it buys: one launch instead of two for the host, and the first down tiles in flight during the meeting.  On the
// device it is no faster than the two launches (20.9 against 21.0 us on the Llama-3-8B shapes at 15 %): the meeting is a
// chain of three trips across the chip (h acknowledged, arrival words seen, h fetched), as long as the launch it
// replaces.  Tried and not adopted: h as 64-bit words that carry the tag, so that readers poll the data itself and
// nobody waits for acknowledgements -- 27 us, the readers' first look usually comes too early and every retry re-reads
// the vector.
#pragma once
#include "gemv_stream_kernel.h"

namespace uniql {
namespace gemv {

// scratch layout: control words (word 0: serial number of the last finished launch; word 2: tag of the last launch in
// which a block gave up), an arrival word per block from byte 256 on, then h from kMlpHeaderBytes on
constexpr int kMlpHeaderBytes = 4352;   // 256 bytes of control words, 4096 of arrival words (up to 1024 blocks)

struct MlpArgs {
  StreamArgs gu;        // gate + up over x; gu.y = h
  StreamArgs dn;        // down over dn.x = h; dn.y = y
  uint32_t* ctrl;
};

template <int NCH1, int NCH2, bool ZP, bool BF16>
__global__ __launch_bounds__(kStreamThreads) void w4_mlp_stream_kernel(MlpArgs m) {
  extern __shared__ __align__(16) unsigned char smem[];   // the larger of the two activation images
  __shared__ int next_body;
  uint4* xs = reinterpret_cast<uint4*>(smem);
  // this launch's tag: one more than the last finished launch's (nobody changes the word while this launch runs)
  const uint32_t tag = __hip_atomic_load(m.ctrl, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1u;
  stream_phase<NCH1, 2, ZP, BF16, false, false, false, true>(m.gu, xs, &next_body, tag);
  // every wave waits for the acknowledgements of its own stores to h (written through: acknowledged from memory), and
  // only then meets the others; then the block says that it has arrived.  The wait is spelled out: a release fence
  // at workgroup scope orders the stores for the waves of this block only and does not wait for them, and the waiting
  // that the compiler puts before thread 0's store below covers the stores of that one wave.
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __syncthreads();
  if (threadIdx.x == 0) __hip_atomic_store(m.dn.arrived + blockIdx.x, tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  stream_phase<NCH2, 1, ZP, BF16, false, false, true, false>(m.dn, xs, &next_body, tag);
  // block 0 records the launch as done: every block of the next launch (which starts after this one has ended) then
  // derives the next tag.  One writer, no read-modify-write.
  if (blockIdx.x == 0 && threadIdx.x == 0) __hip_atomic_store(m.ctrl, tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int NCH1, int NCH2, bool ZP, bool BF16>
static hipError_t mlp_launch(const MlpArgs& m, int blocks, hipStream_t stream) {
  const size_t smem = (size_t)(NCH1 > NCH2 ? NCH1 : NCH2) * 4096;
  hipLaunchKernelGGL((w4_mlp_stream_kernel<NCH1, NCH2, ZP, BF16>), dim3(blocks), dim3(kStreamThreads), smem, stream, m);
  return hipGetLastError();
}

template <int NCH1, bool ZP, bool BF16>
static hipError_t mlp_nch2(const MlpArgs& m, int nch2, int blocks, hipStream_t stream) {
  switch (nch2) {
    case 1: return mlp_launch<NCH1, 1, ZP, BF16>(m, blocks, stream);
    case 2: return mlp_launch<NCH1, 2, ZP, BF16>(m, blocks, stream);
    case 3: return mlp_launch<NCH1, 3, ZP, BF16>(m, blocks, stream);
    case 4: return mlp_launch<NCH1, 4, ZP, BF16>(m, blocks, stream);
    case 5: return mlp_launch<NCH1, 5, ZP, BF16>(m, blocks, stream);
    case 6: return mlp_launch<NCH1, 6, ZP, BF16>(m, blocks, stream);
    case 7: return mlp_launch<NCH1, 7, ZP, BF16>(m, blocks, stream);
    case 8: return mlp_launch<NCH1, 8, ZP, BF16>(m, blocks, stream);
    default: return hipErrorInvalidValue;
  }
}

// probs: gate, up (over x, writing h = probs[0].y in scratch), down (over h).  *done = false (nothing launched) when
// the shapes are not ones the fused launch serves: the caller then runs the two launches one after the other.
template <bool BF16>
static hipError_t mlp_fused(const LinearArgs* p, void* scratch, hipStream_t stream, bool* done) {
  // the shapes of the two walks: gate + up as in stream_gate_up (rows of two tiles here), down as in stream_one
  const bool gu_ok = stream_shape(p[0], 2) && stream_shape(p[1], 2) && p[0].km.n_keep >= kStreamMinRows / 2 &&
                     p[0].km.n_keep == p[1].km.n_keep && p[0].km.k_keep == p[1].km.k_keep && p[0].K_total == p[1].K_total &&
                     p[0].x == p[1].x && p[0].N_total == p[1].N_total && p[0].km.rs_stride == 0 && p[1].km.rs_stride == 0 &&
                     row_tiles(p[0].km.k_keep) == 2;
  const bool zp = p[0].zeros != nullptr;
  const bool same = (p[1].zeros != nullptr) == zp && (p[2].zeros != nullptr) == zp && p[0].bf16 == p[1].bf16 && p[1].bf16 == p[2].bf16;
  const bool dn_ok = stream_shape(p[2], 8) && p[2].km.rs_stride == 0 && p[2].km.n_keep >= kStreamMinRowsShort &&
                     p[2].km.k_keep == p[0].km.n_keep;
  *done = gu_ok && dn_ok && same;
  if (!*done) return hipSuccess;
  int dev = 0, cus = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) return e;
  if (cus < 1 || cus > 1024) return hipErrorInvalidValue;
  MlpArgs m;
  m.gu = stream_args(p[0]);
  m.gu.qweight[1] = p[1].qweight;
  m.gu.scales[1] = p[1].scales;
  m.gu.zeros[1] = p[1].zeros;
  m.dn = stream_args(p[2]);
  m.ctrl = reinterpret_cast<uint32_t*>(scratch);
  m.gu.gave_up = m.dn.gave_up = m.ctrl + 2;
  m.gu.arrived = m.dn.arrived = m.ctrl + 64;
  m.gu.wait_ticks = m.dn.wait_ticks = 20000000ull;   // 0.2 s
  const int nch2 = row_tiles(p[2].km.k_keep);
  return zp ? mlp_nch2<2, true, BF16>(m, nch2, cus, stream) : mlp_nch2<2, false, BF16>(m, nch2, cus, stream);
}

}  // namespace gemv
}  // namespace uniql
