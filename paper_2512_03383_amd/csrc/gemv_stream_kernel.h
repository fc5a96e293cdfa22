// Persistent streaming GEMV for tall matrices (one token): any row rule x column prefix, at least a row
// or two per wave of the whole chip -- gate / up / output-head / in_proj shaped linears.
//
// The launch fills the chip once (one or two blocks per CU) and every wave walks its own rows,
// row r of the wave being compact row wave_id + r * total_waves, so that at any moment the chip reads
// one contiguous window of the matrix and every CU ends up with the same number of rows whatever
// the pruning rate.  The activations are staged once per block (LDS, stored column positions, zeros
// where pruned) and, for rows of at most two 2048-column chunks, held in registers for the whole walk:
// after the one barrier behind the staging a wave runs alone -- no LDS traffic, no barrier.
// A wave keeps D tiles (1 KB of codes + scale + zero point each) in flight: the loop body consumes D
// tiles in issue order and re-issues each slot, as soon as it is free, with the same tile of the next
// body.  Arithmetic per tile is that of gemv_kernel.h (13 VALU per word in fp16, 23 in bfloat16, dot products on the matrix
// pipe's diagonal).
//
// NM = 2 is the gated MLP (Eq. 1): a wave streams row r of W_gate and of W_up side by side and writes
// h[r] = SiLU(gate) * up itself, so gate and up never meet through memory or LDS.
#pragma once
#include "gemv_kernel.h"
#include <atomic>

namespace uniql {
namespace gemv {

constexpr int kStreamThreads = 512;
constexpr int kStreamWaves = kStreamThreads / kWave;

struct StreamArgs {
  const uint32_t* qweight[2];
  const uint16_t* scales[2];
  const uint8_t* zeros[2];
  const half_t* x;
  half_t* y;
  int n_keep, k_keep, K_total;
  int N_total;           // stored rows (extent of the buffer resources)
  KeepMap km;            // row map (rows only; the kept columns are a prefix)
};

template <int NCH, int NM, bool ZP, bool BF16>
__global__ __launch_bounds__(kStreamThreads) void w4_gemv_stream_kernel(StreamArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  uint4* xs = reinterpret_cast<uint4*>(smem);   // [NCH][4][64] units of 8 halves
  constexpr int TPR = NM * NCH;                           // tiles per row (pair)
  constexpr int RB = TPR >= 4 ? 1 : 4 / TPR;              // rows per loop body
  constexpr int D = RB * TPR;                             // tiles per body = tiles in flight
  constexpr bool XREG = NCH <= 2;                         // activations live in registers

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int gw = (int)blockIdx.x * kStreamWaves + wave;           // this wave among all waves
  const int total_waves = (int)gridDim.x * kStreamWaves;
  const int words_per_row = a.K_total >> 3, groups_per_row = a.K_total / kGroup;
  const int k_span32 = (a.k_keep + 31) & ~31;

  // ---- x loads first (memory returns in issue order; x is an L2 hit)
  constexpr int XI = (NCH * 256 + kStreamThreads - 1) / kStreamThreads;
  const int kv = a.k_keep & ~7;
  const uint16_t* xbits = reinterpret_cast<const uint16_t*>(a.x);
  uint4 rawv[XI];
  uint32_t tailv[8];
#pragma unroll
  for (int i = 0; i < XI; ++i) {
    const int uraw = tid + i * kStreamThreads;
    const int k0 = unit_k0(uraw < NCH * 256 ? uraw : NCH * 256 - 1);
    const int k0c = k0 + 8 <= kv ? k0 : kv - 8;     // the host sends k_keep >= 8 only
    rawv[i] = load_u4_unaligned(a.x + k0c);
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) tailv[j] = 0;
  if (kv < a.k_keep) {
#pragma unroll
    for (int j = 0; j < 8; ++j) tailv[j] = xbits[kv + j < a.k_keep ? kv + j : a.k_keep - 1];
  }

  // ---- the wave's rows and the first body of tiles
  // lane offsets of a tile inside its row, per chunk: lanes past the last kept column re-read the row
  // start (their x is zero)
  uint32_t woff[NCH], goff[NCH];   // byte offset of the lane's codes, index of its group
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int kb = c * kChunk + lane * 32;
    const int kbc = kb < k_span32 ? kb : 0;
    woff[c] = (uint32_t)kbc >> 1;
    goff[c] = (uint32_t)kbc >> 7;
  }
  // Buffer resources over the kept rows of each array (base, byte count): a tile's address is then
  // resource + scalar row offset + 32-bit lane offset, and no per-lane 64-bit pointer exists.
  constexpr int kRsrcWord3 = 0x00020000;   // raw 32-bit data format of this target's buffer resource
  __amdgpu_buffer_rsrc_t rq[NM], rs[NM], rz[NM];
#pragma unroll
  for (int m = 0; m < NM; ++m) {
    rq[m] = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(a.qweight[m]), 0, a.N_total * words_per_row * 4, kRsrcWord3);
    rs[m] = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(a.scales[m]), 0, a.N_total * groups_per_row * 2, kRsrcWord3);
    if constexpr (ZP)
      rz[m] = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(a.zeros[m]), 0, a.N_total * groups_per_row, kRsrcWord3);
  }
  typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
  auto load_tile = [&](int rc, int m, int c, Tile& t) {   // rc: compact row, clamped by the caller
    const int sr = a.km.rs_stride ? stored_row(a.km, rc) : rc;              // uniform: scalar arithmetic
    const int row_q = sr * words_per_row * 4, row_g = sr * groups_per_row;   // scalar byte offsets of the row
    const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(rq[m], (int)woff[c], row_q, 0);
    t.w = make_uint4(v.x, v.y, v.z, v.w);
    t.sbits = __builtin_amdgcn_raw_buffer_load_b16(rs[m], (int)(2u * goff[c]), 2 * row_g, 0);
    if constexpr (ZP) t.z = __builtin_amdgcn_raw_buffer_load_b8(rz[m], (int)goff[c], row_g, 0);
    else t.z = 8u;
  };
  // slot s of a body: row s / TPR of the body, then chunk-major with the matrices of a chunk adjacent
  auto slot_row = [](int s) { return s / TPR; };
  auto slot_chunk = [](int s) { return (s % TPR) / NM; };
  auto slot_mat = [](int s) { return s % NM; };
  const int last = a.n_keep - 1;
  auto row_of = [&](int body, int rr) { return gw + (body * RB + rr) * total_waves; };   // may exceed n_keep

  Tile ring[D];
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int s = 0; s < D; ++s) {
    const int rc = row_of(0, slot_row(s));
    load_tile(rc < last ? rc : last, slot_mat(s), slot_chunk(s), ring[s]);
  }
  __builtin_amdgcn_sched_barrier(0);

  // ---- x registers -> LDS in the pair order of the slot, zeros for pruned columns
#pragma unroll
  for (int i = 0; i < XI; ++i) {
    const int u = tid + i * kStreamThreads;
    const int k0 = unit_k0(u);
    const uint4 r = rawv[i];
    const uint32_t full[8] = {r.x & 0xffffu, r.x >> 16, r.y & 0xffffu, r.y >> 16,
                              r.z & 0xffffu, r.z >> 16, r.w & 0xffffu, r.w >> 16};
    const bool whole = k0 + 8 <= kv, tail = k0 == kv;
    uint32_t e[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) e[j] = whole ? full[j] : ((tail && kv + j < a.k_keep) ? tailv[j] : 0u);
    if (u < NCH * 256)
      xs[unit_slot(u)] = make_uint4(e[0] | (e[4] << 16), e[1] | (e[5] << 16), e[2] | (e[6] << 16), e[3] | (e[7] << 16));
  }
  __builtin_amdgcn_sched_barrier(0);
  __syncthreads();

  uint4 xr[XREG ? NCH : 1][4];
  if constexpr (XREG) {
#pragma unroll
    for (int c = 0; c < NCH; ++c)
#pragma unroll
      for (int q = 0; q < 4; ++q) xr[c][q] = xs[(c * 4 + q) * 64 + lane];
  }

  const Magic mg = make_magic();
  const bool on_diag = (lane >> 4) == ((lane & 15) >> 2);
  auto row_sum = [&](const float4_t& c) {
    const int v = lane & 3;
    float d = v == 0 ? c[0] : (v == 1 ? c[1] : (v == 2 ? c[2] : c[3]));
    return dpp_xor_reduce(on_diag ? d : 0.f);
  };
  auto consume = [&](const Tile& t, const uint4 (&xf)[4], float4_t& acc) {
    const typename GroupOf<BF16>::type g = make_group<BF16>(t.sbits, t.z);
    const uint32_t wv[4] = {t.w.x, t.w.y, t.w.z, t.w.w};
#pragma unroll
    for (int q = 0; q < 4; ++q) acc = mfma_16x16x32<BF16>(xf[q], dequant_word4<BF16>(wv[q], g, mg), acc);
  };

  // rows of this wave: gw, gw + total_waves, ...; bodies of RB rows
  const int my_rows = gw < a.n_keep ? (a.n_keep - gw + total_waves - 1) / total_waves : 0;
  const int bodies = (my_rows + RB - 1) / RB;
  float4_t acc[RB][NM];
#pragma unroll
  for (int rr = 0; rr < RB; ++rr)
#pragma unroll
    for (int m = 0; m < NM; ++m) acc[rr][m] = float4_t{0.f, 0.f, 0.f, 0.f};
  for (int body = 0; body < bodies; ++body) {
#pragma unroll
    for (int rr = 0; rr < RB; ++rr) {
      // rows of a body past the wave's last one (only in its last body) are skipped as a whole
      if (rr > 0 && body * RB + rr >= my_rows) break;
#pragma unroll
      for (int t = 0; t < TPR; ++t) {
        const int s = rr * TPR + t, c = slot_chunk(s), m = slot_mat(s);
        if (c == 0) acc[rr][m] = float4_t{0.f, 0.f, 0.f, 0.f};
        Tile& tl = ring[s];
        // order fence: this tile's unpacking may not be hoisted above the previous tile's arithmetic
        const int ps = (s + D - 1) % D;   // the tile consumed just before this one (compile-time after unrolling)
        asm volatile("" : "+v"(tl.w.x), "+v"(tl.w.y), "+v"(tl.w.z), "+v"(tl.w.w), "+v"(tl.sbits), "+v"(tl.z),
                          "+v"(acc[ps / TPR][ps % NM][0]));
        if constexpr (XREG) {
          consume(tl, xr[c], acc[rr][m]);
        } else {
          uint4 xf[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) xf[q] = xs[(c * 4 + q) * 64 + lane];
          consume(tl, xf, acc[rr][m]);
        }
        // the slot is free: the same tile of the next body (a valid row even when that body does not exist)
        const int rn = row_of(body + 1, rr);
        load_tile(rn < last ? rn : last, m, c, tl);
      }
      const int rc = row_of(body, rr);
      if constexpr (NM == 1) {
        const float v = row_sum(acc[rr][0]);
        if (lane == 0) a.y[rc] = out16<BF16>(v);
      } else {
        const float g = row_sum(acc[rr][0]), u = row_sum(acc[rr][1]);
        // SiLU(g) * u; exp and the reciprocal are the hardware approximations (about 1 ulp of fp32)
        if (lane == 0) a.y[rc] = out16<BF16>(g * u * __builtin_amdgcn_rcpf(1.0f + __expf(-g)));
      }
    }
  }
}

// blocks per CU that the kernel's register use allows, times the CU count: the persistent grid
template <int NCH, int NM, bool ZP, bool BF16>
static hipError_t stream_launch(const StreamArgs& a, hipStream_t stream) {
  auto kern = w4_gemv_stream_kernel<NCH, NM, ZP, BF16>;
  const size_t smem = (size_t)NCH * 4096;
  // CU count and blocks per CU of this instantiation, per device ordinal: one word each (count | blocks << 16),
  // written once, so that host threads that race on the first call all read a complete pair
  static std::atomic<uint32_t> cached[64];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const bool slot = dev >= 0 && dev < 64;
  uint32_t packed = slot ? cached[dev].load(std::memory_order_acquire) : 0u;
  if (packed == 0) {
    int cus = 0, per_cu = 0;
    e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void*>(kern), kStreamThreads, smem);
    if (e != hipSuccess) return e;
    e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return e;
    if (per_cu < 1) per_cu = 1;
    if (cus < 1 || cus > 0xffff || per_cu > 0xffff) return hipErrorInvalidValue;
    packed = (uint32_t)cus | ((uint32_t)per_cu << 16);
    if (slot) cached[dev].store(packed, std::memory_order_release);
  }
  const int cus = (int)(packed & 0xffffu), per_cu = (int)(packed >> 16);
  // One block (8 waves, four tiles in flight each) per CU measured fastest up to the size of a gated MLP
  // (more waves only add start-up work); an output-head sized stream needs two to keep enough loads in flight.
  const long long bytes = (long long)NM * a.n_keep * (a.k_keep / 2);
  const int want = bytes >= 100000000ll ? 2 : 1;
  const int cap = cus * (want < per_cu ? want : per_cu);
  int blocks = (a.n_keep + kStreamWaves - 1) / kStreamWaves;
  if (blocks > cap) blocks = cap;
  hipLaunchKernelGGL(kern, dim3(blocks), dim3(kStreamThreads), smem, stream, a);
  return hipGetLastError();
}

template <int NM, bool ZP, bool BF16>
static hipError_t stream_nch(const StreamArgs& a, int nchunk, hipStream_t stream) {
  switch (nchunk) {
    case 1: return stream_launch<1, NM, ZP, BF16>(a, stream);
    case 2: return stream_launch<2, NM, ZP, BF16>(a, stream);
    case 3: return stream_launch<3, NM, ZP, BF16>(a, stream);
    case 4: return stream_launch<4, NM, ZP, BF16>(a, stream);
    default: break;
  }
  if constexpr (NM == 1) {
    switch (nchunk) {
      case 5: return stream_launch<5, 1, ZP, BF16>(a, stream);
      case 6: return stream_launch<6, 1, ZP, BF16>(a, stream);
      case 7: return stream_launch<7, 1, ZP, BF16>(a, stream);
      case 8: return stream_launch<8, 1, ZP, BF16>(a, stream);
      default: break;
    }
  }
  return hipErrorInvalidValue;
}

// Rows below which the kernels of gemv_kernel.h are used: the walk pays off once every wave of the
// persistent grid has more than a row or two.  Rows of up to four chunks (short tile rings, activations in
// registers or few LDS reads) already gain from one row per wave.
constexpr int kStreamMinRows = 8192;
constexpr int kStreamMinRowsShort = 2048;
constexpr int kStreamMinRowsLong = 4096;    // row prefix with rows of more than four chunks (down_proj)

static inline bool stream_shape(const LinearArgs& a, int max_chunks) {
  const KeepMap& km = a.km;
  const int nch = ((km.k_keep + 31) / 32 * 32 + kChunk - 1) / kChunk;
  // row offsets inside the buffer resources are signed 32-bit byte counts
  const bool fits = (long long)a.N_total * (a.K_total / 2) < (1ll << 31);
  return a.M == 1 && km.cs_stride == 0 && km.k_keep >= 8 && nch <= max_chunks && fits;
}

// One linear: *done = false (nothing launched) when the shape is not one this kernel serves.
template <bool BF16>
static hipError_t stream_one(const LinearArgs& a, hipStream_t stream, bool* done) {
  const int nchunks = ((a.km.k_keep + 31) / 32 * 32 + kChunk - 1) / kChunk;
  // (segmented row rules, one division per row, only from the higher threshold: q_proj sized launches measured slower)
  const int min_rows = a.km.rs_stride != 0 ? kStreamMinRows : (nchunks <= 4 ? kStreamMinRowsShort : kStreamMinRowsLong);
  *done = stream_shape(a, 8) && a.km.n_keep >= min_rows;
  if (!*done) return hipSuccess;
  StreamArgs s;
  s.qweight[0] = s.qweight[1] = a.qweight;
  s.scales[0] = s.scales[1] = a.scales;
  s.zeros[0] = s.zeros[1] = a.zeros;
  s.x = a.x;
  s.y = a.y;
  s.n_keep = a.km.n_keep;
  s.k_keep = a.km.k_keep;
  s.K_total = a.K_total;
  s.N_total = a.N_total;
  s.km = a.km;
  const int nch = ((a.km.k_keep + 31) / 32 * 32 + kChunk - 1) / kChunk;
  return a.zeros ? stream_nch<1, true, BF16>(s, nch, stream) : stream_nch<1, false, BF16>(s, nch, stream);
}

// gate and up of one token with h = SiLU(gate) * up written to probs[0].y
template <bool BF16>
static hipError_t stream_gate_up(const LinearArgs* p, hipStream_t stream, bool* done) {
  *done = stream_shape(p[0], 4) && stream_shape(p[1], 4) && p[0].km.n_keep >= kStreamMinRows / 2 &&
          p[0].km.n_keep == p[1].km.n_keep && p[0].km.k_keep == p[1].km.k_keep && p[0].K_total == p[1].K_total &&
          p[0].x == p[1].x && p[0].bf16 == p[1].bf16 && (p[0].zeros != nullptr) == (p[1].zeros != nullptr) && p[0].N_total == p[1].N_total &&
          p[0].km.rs_stride == p[1].km.rs_stride && p[0].km.rs_keep == p[1].km.rs_keep && p[0].km.rs_limit == p[1].km.rs_limit &&
          p[0].km.rs2_stride == p[1].km.rs2_stride && p[0].km.rs2_keep == p[1].km.rs2_keep && p[0].km.rs2_limit == p[1].km.rs2_limit;
  if (!*done) return hipSuccess;
  StreamArgs s;
  for (int m = 0; m < 2; ++m) {
    s.qweight[m] = p[m].qweight;
    s.scales[m] = p[m].scales;
    s.zeros[m] = p[m].zeros;
  }
  s.x = p[0].x;
  s.y = p[0].y;
  s.n_keep = p[0].km.n_keep;
  s.k_keep = p[0].km.k_keep;
  s.K_total = p[0].K_total;
  s.N_total = p[0].N_total;
  s.km = p[0].km;
  const int nch = ((s.k_keep + 31) / 32 * 32 + kChunk - 1) / kChunk;
  return p[0].zeros ? stream_nch<2, true, BF16>(s, nch, stream) : stream_nch<2, false, BF16>(s, nch, stream);
}

}  // namespace gemv
}  // namespace uniql
