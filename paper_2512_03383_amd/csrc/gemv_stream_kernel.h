// Persistent streaming GEMV for tall matrices (one token): any row rule x column prefix -- gate / up / down /
// output-head / in_proj shaped linears.
//
// The launch fills the chip once (one block per CU) and every wave WALKS rows: a block's bodies (a body = the rows one
// loop iteration serves, normally one row, or one row of W_gate and of W_up) are spread over the matrix with a stride of
// the whole grid, so that at any moment the chip reads one contiguous window of the matrix and every CU ends up with the
// same number of rows whatever the pruning rate.  Inside a block the bodies are handed out by a counter in LDS: the two
// waves that share a SIMD do not advance at the same pace (the issue arbiter prefers the older one), and a fixed split
// left the younger four waves of every block 2 us behind the older four.
//
// Column layout of a wave.  A row is covered by NCH wave-wide 128-bit loads ("tiles").  Lanes 4g..4g+3 (a quad) own NCH
// ADJACENT quantisation groups, g * NCH .. g * NCH + NCH - 1, and tile c of the row is group g * NCH + c of every quad: a
// quad reads 64 contiguous bytes per tile (one request of the address unit, like a contiguous load) and the NCH tiles of
// a row together read the row contiguously.  What this buys: the NCH scales of a lane are adjacent in memory, and so are
// its zero points, so a ROW needs one scale load and one zero-point load instead of one of each per TILE (with a
// contiguous kilobyte per tile a lane's groups lie 16 apart; the small loads were the largest single cost of the body).
//
// The activations are staged once per block (LDS image [tile][word][lane], zeros where pruned) and, for short rows, held
// in registers for the whole walk.  A wave keeps one body of tiles in flight as a ring: the loop consumes them in issue
// order and re-issues each slot, as soon as it is free, with the same tile of the wave's next body; the scales and zero
// points of that body are issued at the top.  A wave's last body re-issues nothing.  Arithmetic per 32-bit word: 13 VALU
// in fp16 (23 in bfloat16) for the canonical weights RN16((q - z) s), the 8-element dot product on the diagonal of one
// matrix instruction.  The kernel is bound by instruction issue as much as by the stream (every instruction of a body,
// scalar ones included, costs a SIMD about 4.5 clocks), so the body is kept short: no LDS crossbar in the wave
// reduction, scales applied through op_sel instead of a splat, the row rule a template parameter.
//
// NM = 2 is the gated MLP (Eq. 1): a wave streams row r of W_gate and of W_up side by side and writes
// h[r] = SiLU(gate) * up itself, so gate and up never meet through memory or LDS.
#pragma once
#include "gemv_kernel.h"
#include <atomic>
#include <type_traits>

namespace uniql {
namespace gemv {

constexpr int kStreamThreads = 512;
constexpr int kStreamWaves = kStreamThreads / kWave;

struct StreamArgs {
  const uint32_t* qweight[3];
  const uint16_t* scales[3];
  const uint8_t* zeros[3];
  const half_t* x;
  half_t* y;
  // a launch may serve several tokens, one per grid row (blockIdx.y): token t reads x + t * tok_x and writes
  // y + t * tok_y (elements); the weights of the later tokens come from the caches
  long long tok_x, tok_y;
  int tokens;
  int n_keep, k_keep, K_total;
  int N_total;           // stored rows (extent of the buffer resources)
  KeepMap km;            // row map (rows only; the kept columns are a prefix)
  // the fused gated MLP only (mlp_stream_kernel.h): a word per block of the grid, in which a block stores the launch's
  // tag once its outputs have reached memory; the word a walk records a give-up in; the bound of its wait in 100 MHz
  // ticks
  uint32_t* arrived;
  uint32_t* gave_up;
  unsigned long long wait_ticks;
  // head-interleaved words (HI): the row's words are stored as [dims / 8][heads], il_heads heads of 128 dims, of which
  // the leading d_keep are kept; x is compact [heads][d_keep]
  int il_heads, d_keep;
  // column segments (CS): every cs_units * 8 stored columns keep their leading d_keep; the stored columns up to the last
  // kept one are [0, k_span); x is compact [segments][d_keep]
  int cs_units, k_span;
  // q, k, v of one token with the rotation of q and k (QKV): three matrices over one x, outputs y3[].  A body is one
  // pair of rows (p, p + hk) of a head, hk = D_keep / 2; bodies [0, pair_end[0]) are q's, [pair_end[0], pair_end[1])
  // k's, the rest v's (pairs of a head's rows like the others, not rotated); n_keep = 2 * all pairs.  Head h of matrix
  // i starts at stored row h * head_stride[i] and row p + hk of the head lies pair_off[i] stored rows behind row p;
  // n_total3[i] = the matrix's stored rows.  hk_magic = ceil(2^32 / hk).
  // The row of the kept-index table that head h of q or k uses: h / (heads per table row), by hpt_magic[].
  half_t* y3[3];
  int pair_end[2];
  int hk;
  unsigned long long hk_magic;
  int head_stride[3];
  int pair_off[3];   // stored rows between the two rows of a pair
  int n_total3[3];
  unsigned long long hpt_magic[2];   // ceil(2^32 / heads per table row) of q and k
  const int32_t* positions;
  const int32_t* kept_idx;
  int H_tab;
  double base;   // theta^(-2 / D_full): inv_freq_j = base^j
};

// PROBE: the kernel's loads alone, folded into one word per row -- the read-stream ceiling of exactly this launch
// shape (what the arithmetic is measured against), not a linear.
//
// The walk is a device function so that a launch may run several of them back to back (the fused gated MLP of
// mlp_stream_kernel.h runs gate + up, then down).  YTHROUGH: the outputs are written through to memory (stores at
// agent scope) for a later walk of the same launch.  XWAIT: the activations are such outputs: the walk issues its first
// tiles, then waits until every block of the grid has stored this launch's tag in a.arrived (for at most a.wait_ticks)
// and fetches the activations with loads that bypass the caches that are not coherent across the chip's dies; a.x
// is then 16-byte aligned and padded to whole units of 8.  A block that gives up records the tag in a.gave_up and ends
// its walk there (every wave still runs to its end).  The function returns false in that case.
//
// HI: the matrix stores its words head-interleaved (uniql_w4_t.col_interleave: word (d / 8) * H + h holds dims
// 8 (d / 8) .. + 7 of head h; a head is one quantisation group of 128 dims), so that pruning the trailing dims of
// every head -- o_proj's per-head column segments -- leaves a PREFIX of the row's words: the pruned bytes are never
// fetched.  Tiles are contiguous kilobytes here: lane l of every tile holds the four words of heads 4l % H .. + 3 at
// dims 8 ((256 c + 4 l) / H) .., so the lane's four scales and zero points are adjacent, the same for all tiles of a
// row (H divides 256), and every word has its own group constants, formed once per row.
//
// QKV: three matrices of equal row length over one x (a.qweight[0..2]), q and k rotated (Sec. 3.4 fused rotary
// embedding of the pruned head dimension).  A body is the pair of rows (p, p + D_keep / 2) of one head, so both halves
// of a rotation pair end up in the same wave: lane 63 rotates them with the sin / cos of the pair, which the block
// puts into LDS once ([table row][pair], then one identity entry for v), and writes both outputs.  The loads of a
// body go through the resources of that body's matrix; they are switched when a wave's next body lies in another
// matrix (bodies are handed out in rising order, so at most twice per wave).
template <int NCH, int NM, bool ZP, bool BF16, bool SEG, bool PROBE, bool XWAIT = false, bool YTHROUGH = false, bool HI = false, bool QKV = false,
          bool CS = false>
__device__ __forceinline__ bool stream_phase(const StreamArgs& a, uint4* xs /* LDS, [NCH][4][64] units of 8 halves */,
                                             int* next_body_p /* LDS */, uint32_t tag = 0) {
  constexpr int TPR = NM * NCH;                                  // tiles per row (pair)
  constexpr int RB = QKV ? 2 : (TPR >= 4 ? 1 : 4 / TPR);         // rows per loop body
  static_assert(!QKV || (NM == 1 && !SEG && !PROBE && !XWAIT && !YTHROUGH && !HI && !CS), "the fused q / k / v walk is a mode of its own");
  static_assert(!CS || (NM == 1 && !PROBE && !XWAIT && !HI), "column segments: one matrix, plain words");
  constexpr int D = RB * TPR;                                    // tiles per body = tiles in flight
  constexpr bool XREG = NCH <= 2;                                // activations live in registers

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int total_waves = (int)gridDim.x * kStreamWaves;
  const int words_per_row = a.K_total >> 3, groups_per_row = a.K_total / kGroup;
  const int k_span32 = ((CS ? a.k_span : a.k_keep) + 31) & ~31;

  // ---- x loads first (memory returns in issue order; x is an L2 hit).  Unit u = stored columns [8u, 8u + 8).
  constexpr int XI = (NCH * 256 + kStreamThreads - 1) / kStreamThreads;
  const int kv = a.k_keep & ~7;
  // (HI: a launch may serve several tokens, one per grid row)
  const half_t* const ax = HI ? a.x + (long long)blockIdx.y * a.tok_x : a.x;
  half_t* const ay = HI ? a.y + (long long)blockIdx.y * a.tok_y : a.y;
  const uint16_t* xbits = reinterpret_cast<const uint16_t*>(ax);
  uint4 rawv[XI];
  uint32_t tailv[8];
  uint32_t elv[(HI || CS) ? XI : 1][8];   // HI, CS: the kept dims of a unit that is only partly kept, one per register
  auto load_x = [&]() {
    if constexpr (HI || CS) {
#pragma unroll
      for (int i = 0; i < XI; ++i) {
        // HI: word u of the row is head u % H, dims 8 (u / H) ..; CS: unit u is segment u / cs_units, columns
        // 8 (u % cs_units) .. of it (nothing past the row's last kept column)
        const int u = tid + i * kStreamThreads;
        int dblk, head;
        if constexpr (HI) { dblk = u / a.il_heads; head = u - dblk * a.il_heads; }
        else { head = u / a.cs_units; dblk = u - head * a.cs_units; }
        int nk = a.d_keep - 8 * dblk;                     // kept dims of the unit, counted from its first
        if constexpr (CS) nk = 8 * u < a.k_span ? nk : 0;
        const int base = head * a.d_keep + 8 * dblk;
        rawv[i] = load_u4_unaligned(ax + (nk >= 8 ? base : 0));
#pragma unroll
        for (int j = 0; j < 8; ++j) elv[i][j] = 0;
        if (nk > 0 && nk < 8) {
#pragma unroll
          for (int j = 0; j < 8; ++j) elv[i][j] = j < nk ? (uint32_t)xbits[base + j] : 0u;
        }
      }
      return;
    }
#pragma unroll
    for (int i = 0; i < XI; ++i) {
      const int k0 = 8 * (tid + i * kStreamThreads);
      const int k0c = k0 + 8 <= kv ? k0 : kv - 8;     // the host sends k_keep >= 8 only
      rawv[i] = load_u4_unaligned(ax + k0c);
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) tailv[j] = 0;
    if (kv < a.k_keep) {
#pragma unroll
      for (int j = 0; j < 8; ++j) tailv[j] = xbits[kv + j < a.k_keep ? kv + j : a.k_keep - 1];
    }
  };
  // XWAIT: wait for every block's arrival word (one wave polls, a load per lane and 64 blocks), then fetch the units
  auto wait_x = [&](int* verdict /* LDS */) {
    if (tid < kWave) {
      const unsigned long long t0 = wall_clock64();
      bool all = false;
      for (int polls = 0;; ++polls) {
        bool mine = true;
        for (int b = tid; b < (int)gridDim.x; b += kWave)
          mine = mine && __hip_atomic_load(a.arrived + b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == tag;
        all = __builtin_amdgcn_ballot_w64(mine) == ~0ull;
        if (all) break;
        if ((polls & 63) == 63 && wall_clock64() - t0 >= a.wait_ticks) break;   // the wait is bounded
        __builtin_amdgcn_s_sleep(8);   // about a quarter of a microsecond between polls
      }
      if (tid == 0) {
        *verdict = all ? 1 : 0;
        if (!all) __hip_atomic_store(a.gave_up, tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    __syncthreads();
    if (*verdict == 0) return false;
#pragma unroll
    for (int i = 0; i < XI; ++i) {
      const int k0 = 8 * (tid + i * kStreamThreads);
      rawv[i] = load_u4_coherent(ax + (k0 < a.k_keep ? k0 : 0));   // the unit with the last kept columns is read whole
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) tailv[j] = 0;
    return true;
  };
  if constexpr (!XWAIT) load_x();
  // QKV: the position and this thread's entry of the kept-pair table (at most one per thread), requested with x
  int rot_j = 0, rot_pos = 0;
  if constexpr (QKV) {
    rot_j = a.kept_idx[tid < a.H_tab * a.hk ? tid : 0];
    rot_pos = a.positions[0];
  }

  // ---- lane offsets inside a row.  Lanes whose columns lie past the last kept one re-read the row start: their
  // activations are zero, so what they fetch does not matter.
  const int quad = lane >> 2;
  uint32_t woff[NCH];
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    if constexpr (HI) {
      const int w0 = c * 256 + 4 * lane;   // the lane's first word; its four words are of one block of 8 dims
      woff[c] = w0 < ((a.d_keep + 7) >> 3) * a.il_heads ? (uint32_t)w0 * 4u : 0u;
    } else {
      const int kb = tile_k0(lane, c, NCH);
      woff[c] = kb < k_span32 ? (uint32_t)kb >> 1 : 0u;
    }
  }
  // first group of the lane (a quad past the row's groups reads the row start).  A quad may own groups past the row's
  // last one when 16 NCH exceeds the groups of a row: their columns are pruned by definition, what is read for them
  // (the next row's values; nothing past the arrays, which the resources bound) is multiplied by zero.
  const int goff = HI ? (4 * lane) % a.il_heads : (quad * NCH < groups_per_row ? quad * NCH : 0);
  // Buffer resources over the arrays: an address is resource + scalar row offset + 32-bit lane offset.
  constexpr int kRsrcWord3 = 0x00020000;   // raw 32-bit data format of this target's buffer resource
  __amdgpu_buffer_rsrc_t rq[NM], rs[NM], rz[NM];
#pragma unroll
  for (int m = 0; m < NM; ++m) {
    const int rows = QKV ? a.n_total3[m] : a.N_total;
    rq[m] = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(a.qweight[m]), 0, rows * words_per_row * 4, kRsrcWord3);
    rs[m] = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(a.scales[m]), 0, rows * groups_per_row * 2, kRsrcWord3);
    if constexpr (ZP)
      rz[m] = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(a.zeros[m]), 0, rows * groups_per_row, kRsrcWord3);
  }
  // QKV: loads are issued through the resources of the matrix of the body being fetched, rebuilt from that matrix's
  // pointers when the matrix changes (a select between ready-made resources ends up in vector registers, and every
  // load through such a resource becomes a loop over its distinct values)
  int issue_mid = 0;
  auto use_matrix = [&](int mid) {
    if constexpr (QKV) {
      if (mid != issue_mid) {
        const int rows = mid == 1 ? a.n_total3[1] : a.n_total3[2];   // (bodies come in rising order: never back to q)
        const uint32_t* qp = mid == 1 ? a.qweight[1] : a.qweight[2];
        const uint16_t* sp = mid == 1 ? a.scales[1] : a.scales[2];
        rq[0] = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(qp), 0, rows * words_per_row * 4, kRsrcWord3);
        rs[0] = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(sp), 0, rows * groups_per_row * 2, kRsrcWord3);
        if constexpr (ZP) {
          const uint8_t* zp = mid == 1 ? a.zeros[1] : a.zeros[2];
          rz[0] = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(zp), 0, rows * groups_per_row, kRsrcWord3);
        }
        issue_mid = mid;
      }
    }
  };
  // QKV: pair -> matrix, head, pair of the head.  What the mapping needs of the arguments is pinned in scalar registers
  // (left to itself the compiler indexes the argument block with the matrix number: a chain of dependent scalar
  // loads per body).
  struct PairLoc { int mid, head, p; };
  auto locate = [&](int pair) {
    PairLoc l;
    l.mid = __builtin_amdgcn_readfirstlane((pair >= a.pair_end[0] ? 1 : 0) + (pair >= a.pair_end[1] ? 1 : 0));
    const int lp = pair - (l.mid == 0 ? 0 : (l.mid == 1 ? a.pair_end[0] : a.pair_end[1]));
    l.head = (int)(((unsigned long long)(uint32_t)lp * a.hk_magic) >> 32);
    l.p = lp - l.head * a.hk;
    return l;
  };
  struct RowOff { int q, g; };   // scalar byte / element offsets of a row inside the arrays (once per row)
  auto row_off = [&](int rc) {   // rc: compact row, clamped by the caller
    const int sr = SEG ? stored_row(a.km, rc) : rc;   // SEG = false: the kept rows are a prefix
    return RowOff{sr * words_per_row * 4, sr * groups_per_row};
  };
  constexpr int NGQ = HI ? 4 : NCH;   // groups of a lane per row
  typedef RowQ<NGQ> RowQn;   // a lane's scales (fp16 bits) and zero points (bytes) of one row
  auto load_rowq = [&](const RowOff& ro, int m, RowQn& r) {
    load_bytes<2 * NGQ>(rs[m], 2 * goff, 2 * ro.g, r.s);
    if constexpr (ZP) load_bytes<NGQ>(rz[m], goff, ro.g, r.z);
  };
  auto load_codes = [&](const RowOff& ro, int m, int c) {
    return __builtin_amdgcn_raw_buffer_load_b128(rq[m], (int)woff[c], ro.q, 0);
  };
  // slot s of a body: row s / TPR of the body, then tile-major with the matrices of a tile adjacent
  auto slot_tile = [](int s) { return (s % TPR) / NM; };
  auto slot_mat = [](int s) { return s % NM; };
  const int last = a.n_keep - 1;
  // Bodies of a block: body j is RB adjacent rows, (block * 8 + j % 8) * RB + (j / 8) * RB * total_waves onwards (may
  // exceed n_keep: bodies are valid up to some j and invalid from there on).  Wave w starts on body w; every further
  // body is handed out by a counter in LDS to whichever wave of the block asks first.  The two waves that share a SIMD do
  // not advance at the same pace (the issue arbiter prefers the older wave: with a fixed split the younger four waves of
  // every block finished 2.3 us after the older four), so the faster ones simply take more bodies.
  const int blk8 = (int)blockIdx.x * kStreamWaves;
  auto row_of = [&](int j, int rr) { return (blk8 + (j & 7)) * RB + rr + (j >> 3) * RB * total_waves; };
  int& next_body = *next_body_p;

  u32x4_t ring[D];
  RowQn cur[RB][NM], nxt[RB][NM];
  PairLoc cur_loc = {0, 0, 0}, nxt_loc = {0, 0, 0};   // QKV: where the body in hand and the next one lie
  // the RB rows of body j as offsets into the arrays (QKV: through the resources of the body's matrix, which become current)
  auto body_offsets = [&](int j, RowOff (&ro)[RB], PairLoc& loc) {
    if constexpr (QKV) {
      const int pair = min(row_of(j, 0), last) >> 1;
      loc = locate(pair);
      use_matrix(loc.mid);
      const int sr = loc.head * (loc.mid == 0 ? a.head_stride[0] : (loc.mid == 1 ? a.head_stride[1] : a.head_stride[2])) + loc.p;
      const int sr2 = sr + (loc.mid == 0 ? a.pair_off[0] : (loc.mid == 1 ? a.pair_off[1] : a.pair_off[2]));
      ro[0] = RowOff{sr * words_per_row * 4, sr * groups_per_row};
      ro[1] = RowOff{sr2 * words_per_row * 4, sr2 * groups_per_row};
    } else {
#pragma unroll
      for (int rr = 0; rr < RB; ++rr) {
        const int rc = row_of(j, rr);   // the first row of a body that is fetched exists; its other rows may not
        ro[rr] = row_off(rc < last ? rc : last);
      }
    }
  };
  __builtin_amdgcn_sched_barrier(0);
  {
    RowOff ro0[RB];
    body_offsets(wave, ro0, cur_loc);
#pragma unroll
    for (int rr = 0; rr < RB; ++rr) {
#pragma unroll
      for (int m = 0; m < NM; ++m) load_rowq(ro0[rr], m, cur[rr][m]);
#pragma unroll
      for (int t = 0; t < TPR; ++t) ring[rr * TPR + t] = load_codes(ro0[rr], slot_mat(t), slot_tile(t));
    }
  }
  __builtin_amdgcn_sched_barrier(0);
  if constexpr (XWAIT) {
    if (!wait_x(next_body_p)) return false;   // (the body counter is free until it is set below, behind a barrier)
    __syncthreads();
  }
  if (tid == 0) next_body = kStreamWaves;   // visible after the barrier behind the staging

  // ---- x registers -> LDS image [tile][word][lane] in the pair order of the unpack, zeros for pruned columns
#pragma unroll
  for (int i = 0; i < XI; ++i) {
    const int u = tid + i * kStreamThreads;
    const int k0 = 8 * u;
    const uint4 r = rawv[i];
    const uint32_t full[8] = {r.x & 0xffffu, r.x >> 16, r.y & 0xffffu, r.y >> 16,
                              r.z & 0xffffu, r.z >> 16, r.w & 0xffffu, r.w >> 16};
    const bool whole = k0 + 8 <= kv, tail = k0 == kv;
    uint32_t e[8];
    if constexpr (HI || CS) {
      int nk = a.d_keep - 8 * (HI ? u / a.il_heads : u % a.cs_units);
      if constexpr (CS) nk = 8 * u < a.k_span ? nk : 0;
#pragma unroll
      for (int j = 0; j < 8; ++j) e[j] = nk >= 8 ? full[j] : elv[i][j];   // (elv is zero where nothing is kept)
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) e[j] = whole ? full[j] : ((tail && kv + j < a.k_keep) ? (XWAIT ? full[j] : tailv[j]) : 0u);
    }
    if (u < NCH * 256)
      xs[HI ? ((u >> 8) * 4 + (u & 3)) * 64 + ((u >> 2) & 63) : unit_slot(u, NCH)] =
          make_uint4(e[0] | (e[4] << 16), e[1] | (e[5] << 16), e[2] | (e[6] << 16), e[3] | (e[7] << 16));
  }
  // QKV: sin / cos of pos * theta^(-2j/D) for every (table row, kept pair), then the identity for v.  The angle is
  // formed in fp64, in revolutions (theta^(-2j/D) = base^j by binary powering), and its fraction goes to the hardware
  // sin / cos.
  float2_t* rot = reinterpret_cast<float2_t*>(xs + NCH * 256);
  if constexpr (QKV) {
    const int n_tab = a.H_tab * a.hk;
    if (tid <= n_tab) {
      float sn = 0.f, cs = 1.f;
      if (tid < n_tab) {
        double inv_freq = 1.0, bpow = a.base;
        for (int e = rot_j; e != 0; e >>= 1) {
          inv_freq = e & 1 ? inv_freq * bpow : inv_freq;
          bpow *= bpow;
        }
        const double rev = (double)rot_pos * inv_freq * 0.15915494309189534561;
        const float rr = (float)(rev - rint(rev));
        sn = __builtin_amdgcn_sinf(rr);
        cs = __builtin_amdgcn_cosf(rr);
      }
      rot[tid] = float2_t{sn, cs};
    }
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
  auto store_y = [&](int rc, half_t v) {
    if constexpr (YTHROUGH)
      __hip_atomic_store(reinterpret_cast<uint16_t*>(ay + rc), __builtin_bit_cast(uint16_t, v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else
      ay[rc] = v;
  };
  const bool on_diag = (lane >> 4) == ((lane & 15) >> 2);
  typedef typename GroupOf<BF16>::type Group;
  auto consume = [&](const u32x4_t& w, const Group (&gq)[HI ? 4 : 1], const uint4 (&xf)[4], float4_t& acc) {
    const uint32_t wv[4] = {w.x, w.y, w.z, w.w};
    const Group& g = gq[0];
    if constexpr (PROBE) {
      uint32_t fold = w.x ^ w.y ^ w.z ^ w.w;
      if constexpr (BF16) fold ^= __builtin_bit_cast(uint32_t, g.s) ^ __builtin_bit_cast(uint32_t, g.nzs);
      else fold ^= as_u32(g.s2) ^ as_u32(g.zlo);
      acc[0] += __builtin_bit_cast(float, fold & 0x3fffffffu);
      return;
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) acc = mfma_16x16x32<BF16>(xf[q], dequant_word4<BF16>(wv[q], gq[HI ? q : 0], mg), acc);
  };

  float4_t acc[RB][NM];
#pragma unroll
  for (int rr = 0; rr < RB; ++rr)
#pragma unroll
    for (int m = 0; m < NM; ++m) acc[rr][m] = float4_t{0.f, 0.f, 0.f, 0.f};

  // One body: RB rows.  RELOAD: every slot is re-issued, as soon as it has been consumed, with the same tile of the
  // next body (all bodies but the wave's last, which therefore issues no load that nobody consumes).
  auto run_body = [&](int body, int body_next, auto reload_tag) {
    constexpr bool RELOAD = decltype(reload_tag)::value;
    RowOff nro[RB];
    if constexpr (RELOAD) {
      body_offsets(body_next, nro, nxt_loc);
#pragma unroll
      for (int rr = 0; rr < RB; ++rr) {
#pragma unroll
        for (int m = 0; m < NM; ++m) load_rowq(nro[rr], m, nxt[rr][m]);
      }
    }
#pragma unroll
    for (int rr = 0; rr < RB; ++rr) {
      // rows of a body past the wave's last one (only in its last body) are skipped as a whole
      if (rr > 0 && row_of(body, rr) > last) break;
#pragma unroll
      for (int t = 0; t < TPR; ++t) {
        const int s = rr * TPR + t, c = slot_tile(s), m = slot_mat(s);
        if (c == 0) acc[rr][m] = float4_t{0.f, 0.f, 0.f, 0.f};
        // order fence: this tile's unpacking may not be hoisted above the previous tile's arithmetic.  The codes pass
        // as ONE 128-bit operand, so that they keep their register tuple across the loop's back edge (copies of
        // loaded registers there would wait for every load in flight).
        const int ps = (s + D - 1) % D;   // the tile consumed just before this one (compile-time after unrolling)
        asm volatile("" : "+v"(ring[s]), "+v"(acc[ps / TPR][ps % NM]));
        Group g[HI ? 4 : 1];
        if constexpr (HI) {
#pragma unroll
          for (int q = 0; q < 4; ++q) g[q] = group_of<ZP, BF16, 4>(cur[rr][m], q);   // (the same for every tile of the row)
        } else {
          g[0] = group_of<ZP, BF16, NCH>(cur[rr][m], c);
        }
        if constexpr (XREG) {
          consume(ring[s], g, xr[c], acc[rr][m]);
        } else {
          uint4 xf[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) xf[q] = xs[(c * 4 + q) * 64 + lane];
          consume(ring[s], g, xf, acc[rr][m]);
        }
        if constexpr (RELOAD) ring[s] = load_codes(nro[rr], m, c);
      }
      const int rc = row_of(body, rr);
      if constexpr (QKV) {
        // both rows of the pair are summed and rotated below
      } else if constexpr (NM == 1) {
        const float v = diag_sum_to_lane63(acc[rr][0], on_diag);
        if (lane == 63) store_y(rc, out16<BF16>(v));
      } else {
        float g, u;
        diag_sums_to_lane63(acc[rr][0], acc[rr][1], on_diag, g, u);
        // SiLU(g) * u; exp and the reciprocal are the hardware approximations (about 1 ulp of fp32)
        if (lane == 63) store_y(rc, out16<BF16>(g * u * __builtin_amdgcn_rcpf(1.0f + __expf(-g))));
      }
    }
    if constexpr (QKV) {
      float x1, x2;
      diag_sums_to_lane63(acc[0][0], acc[1][0], on_diag, x1, x2);
      // q and k: the entry of (the head's table row, the pair); v: the identity behind the table
      const int mid = cur_loc.mid;
      const int tab_row = (int)(((unsigned long long)(uint32_t)cur_loc.head * (mid == 0 ? a.hpt_magic[0] : a.hpt_magic[1])) >> 32);
      const float2_t sc = rot[mid == 2 ? a.H_tab * a.hk : tab_row * a.hk + cur_loc.p];
      half_t* y = (mid == 0 ? a.y3[0] : (mid == 1 ? a.y3[1] : a.y3[2])) + cur_loc.head * (2 * a.hk) + cur_loc.p;
      if (lane == 63) {
        y[0] = out16<BF16>(x1 * sc.y - x2 * sc.x);
        y[a.hk] = out16<BF16>(x2 * sc.y + x1 * sc.x);
      }
      if constexpr (RELOAD) cur_loc = nxt_loc;
    }
    if constexpr (RELOAD) {
#pragma unroll
      for (int rr = 0; rr < RB; ++rr)
#pragma unroll
        for (int m = 0; m < NM; ++m) cur[rr][m] = nxt[rr][m];
    }
  };
  auto grab = [&]() {   // one counter increment per wave
    int v = 0;
    if (lane == 0) v = __hip_atomic_fetch_add(&next_body, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    return __builtin_amdgcn_readfirstlane(v);
  };
  int cur_body = wave;
  if (row_of(cur_body, 0) <= last) {
    int nb = grab();
    while (true) {
      // the body after the next is asked for now and looked at in the next round (the counter's latency hides behind a body)
      const int nnb = grab();
      if (row_of(nb, 0) > last) break;
      run_body(cur_body, nb, std::true_type{});
      cur_body = nb;
      nb = nnb;
    }
    run_body(cur_body, 0, std::false_type{});
  }
  return true;
}


template <int NCH, int NM, bool ZP, bool BF16, bool SEG, bool PROBE = false, bool HI = false, bool QKV = false, bool CS = false>
__global__ __launch_bounds__(kStreamThreads) void w4_gemv_stream_kernel(StreamArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ int next_body;
  stream_phase<NCH, NM, ZP, BF16, SEG, PROBE, false, false, HI, QKV, CS>(a, reinterpret_cast<uint4*>(smem), &next_body);
}

template <int NCH, int NM, bool ZP, bool BF16, bool SEG, bool PROBE, bool HI = false, bool QKV = false, bool CS = false>
static hipError_t stream_launch(const StreamArgs& a, hipStream_t stream) {
  auto kern = w4_gemv_stream_kernel<NCH, NM, ZP, BF16, SEG, PROBE, HI, QKV, CS>;
  // the image of x, then (QKV) the sin / cos table and its identity entry
  const size_t smem = (size_t)NCH * 4096 + (QKV ? ((size_t)a.H_tab * a.hk + 1) * sizeof(float2_t) : 0);
  // CU count per device ordinal, read once (host threads that race on the first call all store the same value)
  static std::atomic<int> cached[64];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const bool slot = dev >= 0 && dev < 64;
  int cus = slot ? cached[dev].load(std::memory_order_acquire) : 0;
  if (cus == 0) {
    e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return e;
    if (cus < 1) return hipErrorInvalidValue;
    if (slot) cached[dev].store(cus, std::memory_order_release);
  }
  // One block (8 waves, one body of tiles in flight each) per CU: more waves or deeper rings measured slower at every
  // size tried (the kernel is bound by instruction issue, and more loads in flight only queue).
  constexpr int TPR = NM * NCH, RB = QKV ? 2 : (TPR >= 4 ? 1 : 4 / TPR);
  int blocks = (a.n_keep + kStreamWaves * RB - 1) / (kStreamWaves * RB);
  // (QKV, a few thousand pairs in all: one, two or three blocks per compute unit measured the same, 6.7 us for 11.1 MB)
  // (down_proj, two rows per wave: two blocks per compute unit 8.6 against 8.2 us)
  if (blocks > cus) blocks = cus;
  hipLaunchKernelGGL(kern, dim3(blocks, a.tokens), dim3(kStreamThreads), smem, stream, a);
  return hipGetLastError();
}

template <int NM, bool ZP, bool BF16, bool SEG, bool PROBE, bool CS = false>
static hipError_t stream_nch(const StreamArgs& a, int nch, hipStream_t stream) {
  switch (nch) {
    case 1: return stream_launch<1, NM, ZP, BF16, SEG, PROBE, false, false, CS>(a, stream);
    case 2: return stream_launch<2, NM, ZP, BF16, SEG, PROBE, false, false, CS>(a, stream);
    case 3: return stream_launch<3, NM, ZP, BF16, SEG, PROBE, false, false, CS>(a, stream);
    case 4: return stream_launch<4, NM, ZP, BF16, SEG, PROBE, false, false, CS>(a, stream);
    default: break;
  }
  if constexpr (NM == 1) {
    switch (nch) {
      case 5: return stream_launch<5, 1, ZP, BF16, SEG, PROBE, false, false, CS>(a, stream);
      case 6: return stream_launch<6, 1, ZP, BF16, SEG, PROBE, false, false, CS>(a, stream);
      case 7: return stream_launch<7, 1, ZP, BF16, SEG, PROBE, false, false, CS>(a, stream);
      case 8: return stream_launch<8, 1, ZP, BF16, SEG, PROBE, false, false, CS>(a, stream);
      default: break;
    }
  }
  return hipErrorInvalidValue;
}

// Rows below which the kernels of gemv_kernel.h are used: the walk pays off once every wave of the
// persistent grid has more than a row or two.  Rows of up to four tiles (short tile rings, activations in
// registers or few LDS reads) already gain from one row per wave.
// (one-token launches, weights from HBM, this walk against the block kernel: 3584 rows of seven tiles 9.1 against
// 10.1 us; segmented row rules, one division per row, 3072 rows x 3584 columns 4.2 against 4.5 us and 3482 x 4096 4.7
// against 5.0 us)
constexpr int kStreamMinRows = 8192;        // fused launches are measured from half of this
constexpr int kStreamMinRowsShort = 2048;
constexpr int kStreamMinRowsLong = 2048;    // row prefix with rows of more than four tiles (down_proj)
constexpr int kStreamMinRowsSeg = 2048;     // segmented row rules (q_proj's heads)
constexpr int kStreamMinPairs = 1024;       // fused q / k / v: row pairs of the three matrices together

static inline bool stream_shape(const LinearArgs& a, int max_tiles) {
  const KeepMap& km = a.km;
  const int nch = row_tiles(km.k_keep);
  // row offsets inside the buffer resources are signed 32-bit byte counts
  const bool fits = (long long)a.N_total * (a.K_total / 2) < (1ll << 31);
  return a.M == 1 && a.il_heads == 0 && km.cs_stride == 0 && km.k_keep >= 8 && nch <= max_tiles && fits && whole_quads(a.K_total, nch);
}

// The same for column segments whose stride is a whole number of 8-column units (o_proj on head-major words, the SSM
// output projection): the activations are staged segment by segment, everything else is the walk over a row prefix.
static inline bool stream_shape_cs(const LinearArgs& a, int max_tiles) {
  const KeepMap& km = a.km;
  const int nch = row_tiles(km.k_span);
  const bool fits = (long long)a.N_total * (a.K_total / 2) < (1ll << 31);
  return a.M == 1 && a.il_heads == 0 && km.cs_stride >= 8 && km.cs_stride % 8 == 0 && km.cs_keep >= 1 && km.k_keep >= 8 &&
         km.rs_stride == 0 && nch <= max_tiles && fits && whole_quads(a.K_total, nch);
}

static inline StreamArgs stream_args(const LinearArgs& a) {
  StreamArgs s;
  s.qweight[0] = s.qweight[1] = a.qweight;
  s.scales[0] = s.scales[1] = a.scales;
  s.zeros[0] = s.zeros[1] = a.zeros;
  s.x = a.x;
  s.y = a.y;
  s.tok_x = s.tok_y = 0;
  s.tokens = 1;
  s.n_keep = a.km.n_keep;
  s.k_keep = a.km.k_keep;
  s.K_total = a.K_total;
  s.N_total = a.N_total;
  s.km = a.km;
  s.arrived = nullptr;
  s.gave_up = nullptr;
  s.wait_ticks = 0;
  s.il_heads = a.il_heads;
  s.d_keep = a.km.cs_stride ? a.km.cs_keep : kGroup;
  s.cs_units = a.km.cs_stride ? a.km.cs_stride / 8 : 1;
  s.k_span = a.km.k_span;
  s.qweight[2] = nullptr; s.scales[2] = nullptr; s.zeros[2] = nullptr;
  s.y3[0] = s.y3[1] = s.y3[2] = nullptr;
  s.pair_end[0] = s.pair_end[1] = 0;
  s.hk = 0; s.hk_magic = 0;
  for (int i = 0; i < 3; ++i) { s.head_stride[i] = 0; s.pair_off[i] = 0; s.n_total3[i] = 0; }
  s.hpt_magic[0] = s.hpt_magic[1] = 0;
  s.positions = nullptr; s.kept_idx = nullptr; s.H_tab = 0; s.base = 1.0;
  return s;
}

// A matrix with head-interleaved words (1..64 tokens, one per grid row: a decode batch re-reads the words through the
// caches): every shape this layout is defined for runs here, there is no other kernel for it.  hipErrorInvalidValue for the rest: more than four kilobytes of kept words per row, a head
// count that does not divide 256 or is not a multiple of four, heads of another width than a group, pruned rows,
// kept columns that are not the leading dims of every head.
template <bool BF16>
static hipError_t stream_interleaved(const LinearArgs& a, hipStream_t stream) {
  const int H = a.il_heads;
  const bool cols_ok = a.km.cs_stride == 0 ? a.km.k_keep == a.K_total : a.km.cs_stride == kGroup;
  const bool fits = (long long)a.N_total * (a.K_total / 2) < (1ll << 31);
  if (a.M < 1 || a.M > 64 || H < 4 || H % 4 || 256 % H || a.K_total != H * kGroup || a.km.rs_stride != 0 || !cols_ok || !fits)
    return hipErrorInvalidValue;
  StreamArgs s = stream_args(a);
  s.tokens = a.M;
  s.tok_x = a.ldx;
  s.tok_y = a.ldy;
  const int nch = (((s.d_keep + 7) >> 3) * H + 255) / 256;
  switch (nch) {
    case 1: return a.zeros ? stream_launch<1, 1, true, BF16, false, false, true>(s, stream) : stream_launch<1, 1, false, BF16, false, false, true>(s, stream);
    case 2: return a.zeros ? stream_launch<2, 1, true, BF16, false, false, true>(s, stream) : stream_launch<2, 1, false, BF16, false, false, true>(s, stream);
    case 3: return a.zeros ? stream_launch<3, 1, true, BF16, false, false, true>(s, stream) : stream_launch<3, 1, false, BF16, false, false, true>(s, stream);
    case 4: return a.zeros ? stream_launch<4, 1, true, BF16, false, false, true>(s, stream) : stream_launch<4, 1, false, BF16, false, false, true>(s, stream);
    default: return hipErrorInvalidValue;
  }
}

// One linear: *done = false (nothing launched) when the shape is not one this kernel serves.
template <bool BF16>
static hipError_t stream_one(const LinearArgs& a, hipStream_t stream, bool* done) {
  if (a.il_heads > 0) {
    *done = true;
    return stream_interleaved<BF16>(a, stream);
  }
  if (a.km.cs_stride != 0) {
    *done = stream_shape_cs(a, 8) && a.km.n_keep >= kStreamMinRowsShort;
    if (!*done) return hipSuccess;
    const StreamArgs s = stream_args(a);
    const int nch_cs = row_tiles(a.km.k_span);
    return a.zeros ? stream_nch<1, true, BF16, false, false, true>(s, nch_cs, stream) : stream_nch<1, false, BF16, false, false, true>(s, nch_cs, stream);
  }
  const int nch = row_tiles(a.km.k_keep);
  const int min_rows = a.km.rs_stride != 0 ? kStreamMinRowsSeg : (nch <= 4 ? kStreamMinRowsShort : kStreamMinRowsLong);
  *done = stream_shape(a, 8) && a.km.n_keep >= min_rows;
  if (!*done) return hipSuccess;
  const StreamArgs s = stream_args(a);
  if (a.km.rs_stride != 0)
    return a.zeros ? stream_nch<1, true, BF16, true, false>(s, nch, stream) : stream_nch<1, false, BF16, true, false>(s, nch, stream);
  return a.zeros ? stream_nch<1, true, BF16, false, false>(s, nch, stream) : stream_nch<1, false, BF16, false, false>(s, nch, stream);
}

// The loads of stream_one's launch without its arithmetic (y receives one folded word per row): the read-stream
// ceiling of the same launch shape.  *done = false when the shape is not one the kernel serves.
template <bool BF16>
static hipError_t stream_probe(const LinearArgs& a, hipStream_t stream, bool* done) {
  *done = stream_shape(a, 8) && a.km.rs_stride == 0 && a.zeros != nullptr;
  if (!*done) return hipSuccess;
  return stream_nch<1, true, BF16, false, true>(stream_args(a), row_tiles(a.km.k_keep), stream);
}

// gate and up of one token with h = SiLU(gate) * up written to probs[0].y (row prefix x column prefix)
template <bool BF16, bool PROBE = false>
static hipError_t stream_gate_up(const LinearArgs* p, hipStream_t stream, bool* done) {
  *done = stream_shape(p[0], 4) && stream_shape(p[1], 4) && p[0].km.n_keep >= kStreamMinRows / 2 &&
          p[0].km.n_keep == p[1].km.n_keep && p[0].km.k_keep == p[1].km.k_keep && p[0].K_total == p[1].K_total &&
          p[0].x == p[1].x && p[0].bf16 == p[1].bf16 && (p[0].zeros != nullptr) == (p[1].zeros != nullptr) && p[0].N_total == p[1].N_total &&
          p[0].km.rs_stride == 0 && p[1].km.rs_stride == 0;
  if (PROBE) *done = *done && p[0].zeros != nullptr;
  if (!*done) return hipSuccess;
  StreamArgs s = stream_args(p[0]);
  s.qweight[1] = p[1].qweight;
  s.scales[1] = p[1].scales;
  s.zeros[1] = p[1].zeros;
  const int nch = row_tiles(s.k_keep);
  if constexpr (PROBE) return stream_nch<2, true, BF16, false, true>(s, nch, stream);
  return p[0].zeros ? stream_nch<2, true, BF16, false, false>(s, nch, stream) : stream_nch<2, false, BF16, false, false>(s, nch, stream);
}

// q, k, v of one token with q and k rotated, as one walk (*done = false, nothing launched, when the shapes are not
// ones it serves): one x, kept columns a prefix, rows of at most four tiles, and in every matrix the kept rows are the
// leading D_keep rows of each head (a row prefix, or one family of row segments that keeps D_keep rows each) or the
// leading D_keep / 2 rows of either half of each head (segments of half a head).
template <bool BF16>
static hipError_t stream_qkv_rope(const LinearArgs* p, const RopeFuse& rf, hipStream_t stream, bool* done) {
  const int D = rf.D_keep, hk = D / 2;
  bool ok = hk >= 2 && (long long)rf.H_tab * hk < kStreamThreads;   // a table entry per thread, and the identity
  int stride[3] = {0, 0, 0}, poff[3] = {0, 0, 0};
  for (int i = 0; i < 3 && ok; ++i) {
    const KeepMap& km = p[i].km;
    ok = stream_shape(p[i], 4) && p[i].K_total == p[0].K_total && km.k_keep == p[0].km.k_keep && p[i].x == p[0].x &&
         p[i].bf16 == p[0].bf16 && (p[i].zeros != nullptr) == (p[0].zeros != nullptr) && km.n_keep % D == 0;
    const bool one_family = km.rs_segrows == km.n_keep && km.rs2_stride == 0;
    if (km.rs_stride == 0) { stride[i] = D; poff[i] = hk; }   // a row prefix: heads of D_keep stored rows
    else if (one_family && km.rs_keep == D) { stride[i] = km.rs_stride; poff[i] = hk; }   // the leading D_keep rows of every head
    else if (one_family && km.rs_keep == hk) { stride[i] = 2 * km.rs_stride; poff[i] = km.rs_stride; }   // the leading pairs of either half of every head
    else ok = false;
  }
  ok = ok && p[0].km.n_keep == rf.heads[0] * D && p[1].km.n_keep == rf.heads[1] * D;
  const int pairs = ok ? (p[0].km.n_keep + p[1].km.n_keep + p[2].km.n_keep) / 2 : 0;
  ok = ok && pairs >= kStreamMinPairs;
  *done = ok;
  if (!ok) return hipSuccess;
  StreamArgs s = stream_args(p[0]);
  for (int i = 0; i < 3; ++i) {
    s.qweight[i] = p[i].qweight;
    s.scales[i] = p[i].scales;
    s.zeros[i] = p[i].zeros;
    s.y3[i] = p[i].y;
    s.head_stride[i] = stride[i];
    s.pair_off[i] = poff[i];
    s.n_total3[i] = p[i].N_total;
  }
  s.pair_end[0] = p[0].km.n_keep / 2;
  s.pair_end[1] = s.pair_end[0] + p[1].km.n_keep / 2;
  s.n_keep = 2 * pairs;
  s.km = KeepMap{};
  s.hk = hk;
  s.hk_magic = ((1ull << 32) + hk - 1) / hk;
  for (int i = 0; i < 2; ++i) {
    const unsigned long long hpt = (unsigned long long)(rf.heads[i] / rf.H_tab);
    s.hpt_magic[i] = ((1ull << 32) + hpt - 1) / hpt;
  }
  s.positions = rf.positions;
  s.kept_idx = rf.kept_idx;
  s.H_tab = rf.H_tab;
  s.base = rf.base;
  const bool zp = p[0].zeros != nullptr;
  switch (row_tiles(s.k_keep)) {
    case 1: return zp ? stream_launch<1, 1, true, BF16, false, false, false, true>(s, stream) : stream_launch<1, 1, false, BF16, false, false, false, true>(s, stream);
    case 2: return zp ? stream_launch<2, 1, true, BF16, false, false, false, true>(s, stream) : stream_launch<2, 1, false, BF16, false, false, false, true>(s, stream);
    case 3: return zp ? stream_launch<3, 1, true, BF16, false, false, false, true>(s, stream) : stream_launch<3, 1, false, BF16, false, false, false, true>(s, stream);
    default: return zp ? stream_launch<4, 1, true, BF16, false, false, false, true>(s, stream) : stream_launch<4, 1, false, BF16, false, false, false, true>(s, stream);
  }
}

}  // namespace gemv
}  // namespace uniql
