// GATHER_M: SRead -> dense MFMA tile -> SWrite with m as the PIT-axis (paper Section 3.1, sparse kernel
// template; Table 1, MatMul axis m), for gfx950.  Used for whole-row micro-tiles: the valid token rows
// of a padded batch, and both matmuls of the mixture-of-experts FFN.
//
// One workgroup = 2 x 2 wavefronts computes a (64 WM) x (64 WN) tile of C; a wave owns (32 WM) x (32 WN)
// of it as WM x WN blocks of v_mfma_f32_32x32x16 (bf16 or f16 in, fp32 accumulate).
//
// SRead.  The tile's row numbers come from the index once (into LDS).  Per step of 32 along k, the
// operands travel global -> LDS directly (global_load_lds_dwordx4: 16 bytes per lane, no registers in
// between), into a ring of NST stages so that NST - 1 steps of loads are in flight while one is
// multiplied.  A direct load writes 1 KiB of LDS contiguously per wavefront but takes its 64 source
// addresses per lane, so the gather (which row) and the bank swizzle (which 16 bytes of the row) are
// both expressed by the choice of source address:
//   A tile [64 WM rows][32 k]   (K-minor, 64 B per row).  One load instruction = 16 listed rows x 64 B.
//                               16-byte chunk c of row r lies at slot c ^ ((r >> 2) & 3); operands are
//                               read with ds_read_b128 (8 consecutive k of one row per lane).
//   B tile [32 k][64 WN cols]   (K-major as stored, 128 WN B per k-row).  One load instruction =
//                               1 KiB of consecutive k-rows.  64-byte chunk q of k-row k lies at
//                               position q ^ (k & 3); operands are read with the transposing LDS read
//                               (ds_read_b64_tr_b16: in each group of 16 lanes, lane i receives column i
//                               of the four k-rows addressed by lanes 4 j .. 4 j + 3), two reads giving the 8
//                               consecutive k of one column that the MFMA wants.  Nothing is transposed
//                               by vector instructions and nothing is written to LDS from registers.
// Synchronisation: the loads are inline assembly, invisible to the compiler's counters; a wave waits
// for its own loads of a stage with an explicit s_waitcnt vmcnt(n) that leaves the younger stages in
// flight, then the workgroup meets at one barrier per stage, after which the stage that was read before
// the barrier may be overwritten by the loads of stage s + NST - 1.
//
// SWrite.  Every 32 x 32 block is computed transposed (operands swapped), so a lane holds one row of C
// and four consecutive columns per register quad: one row number (and gate) per lane, 16-byte stores to
// the row the index names (or to compact rows), optionally GELU + rounding to the input type.
#include "pit_gemm.hpp"
#include "pit_gemm_dev.hpp"
#include <climits>
#include <type_traits>

namespace pit {
namespace {

// Direct global -> LDS load of 16 bytes per lane: lane i's bytes land at lds_wave_base + 16 i.
// `base` and `lds_wave_base` are wave-uniform.
__device__ __forceinline__ void dma16(const char* base, uint32_t byte_off, uint32_t lds_wave_base) {
  const uint32_t m0v = __builtin_amdgcn_readfirstlane(lds_wave_base);
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :: "s"(m0v), "v"(byte_off), "s"(reinterpret_cast<uint64_t>(base)) : "memory", "m0");
}
__device__ __forceinline__ uint2 lds_tr(uint32_t addr) {
  return __builtin_bit_cast(uint2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((PIT_LDS v4i16_t*)(uintptr_t)addr));
}
// wait until at most n vector-memory operations of this wavefront are outstanding (gfx9 encoding:
// vmcnt in bits 3:0 and 15:14, expcnt 6:4 and lgkmcnt 11:8 left at "no wait"); LDS accesses that
// follow in program order stay behind it
#define PIT_WAIT_VMCNT(n) do { __builtin_amdgcn_s_waitcnt(((n) & 15) | (7 << 4) | (15 << 8) | (((n) >> 4) << 14)); \
                               asm volatile("" ::: "memory"); } while (0)
// workgroup barrier that waits for this wave's LDS operations only (not for vector-memory operations:
// the younger stages' loads stay in flight across it)
#define PIT_LDS_BARRIER() do { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); __builtin_amdgcn_s_barrier(); \
                               asm volatile("" ::: "memory"); } while (0)

// Zero the rows of C that an ascending list does not name, for the rows [r_begin, r_end): the share of one
// workgroup without a tile (all of these shares together cover [0, M)).  One 64-ary search finds the list
// position of the first row (three or four dependent loads for a list of thousands); from there the list is
// read 64 entries at a time: the entries below the end of a chunk of 64 rows mark its covered rows in a 64-bit
// mask, and as many entries as the mask has bits are consumed.  Wave w clears rows w, w + 4, ... of the chunk,
// 16 bytes per lane.
template <int ESIZE>
__device__ __forceinline__ void zero_unlisted_rows(const GemmArgs& g, int r_begin, int r_end, int wv, int lane) {
  const int n = g.seg_ptr[1] - g.seg_ptr[0];
  const int32_t* list = g.idx + g.seg_ptr[0];
  int lo = 0, hi = n;                      // smallest j with list[j] >= r_begin (n if none)
  while (lo < hi) {
    const int step = (hi - lo + 63) >> 6;
    const int p = lo + lane * step;
    const int v = p < hi ? list[p] : INT_MAX;
    const int k = __builtin_popcountll(__ballot(v < r_begin));   // the probes ascend: the first k are below
    if (k == 0) { hi = lo; break; }
    const int below = lo + (k - 1) * step;
    hi = min(hi, below + step);
    lo = below + 1;
  }
  const int64_t nbytes = (int64_t)g.N * ESIZE;
  for (int r0 = r_begin; r0 < r_end; r0 += 64) {
    const int v = lo + lane < n ? list[lo + lane] : INT_MAX;     // strictly ascending: entry j is >= r0 + j
    uint64_t m = (v < r0 + 64) ? (1ull << (v - r0)) : 0ull;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) m |= __shfl_xor(m, d);
    lo += __builtin_popcountll(m);
    for (int r = r0 + wv; r < min(r0 + 64, r_end); r += 4) {
      if ((m >> (r - r0)) & 1) continue;
      char* p = reinterpret_cast<char*>(g.C) + (int64_t)r * g.ldc * ESIZE;
      for (int64_t b = (int64_t)lane * 16; b < nbytes; b += 64 * 16)
        *reinterpret_cast<uint4*>(p + b) = make_uint4(0, 0, 0, 0);
    }
  }
}

// GM x GN = arrangement of the four waves over the tile (2 x 2 or 1 x 4); a wave owns WM x WN blocks of 32 x 32.
template <int WM, int WN, int NST, int GN> struct MTile {
  static constexpr int GM = 4 / GN;
  static constexpr int TMW = 32 * WM * GM, TNW = 32 * WN * GN, KS = 32;
  static constexpr int A_STAGE = TMW * KS * 2, B_STAGE = KS * TNW * 2, STAGE = A_STAGE + B_STAGE;
  static constexpr int LA = TMW / 64, LB = TNW / 64;   // load instructions per wave and stage: A, B
  static constexpr int LOADS = LA + LB;
  static_assert(GN == 2 || GN == 4, "wave arrangement");
  static_assert(TMW % 64 == 0, "rows of a tile");
  static_assert(TNW == 128 || TNW == 256, "the B swizzle assumes k-rows of 256 or 512 bytes");
  static_assert(NST >= 2 && NST <= 8 && (NST - 1) * LOADS < 64, "stages in flight must fit the 6-bit counter");
};

template <bool BF, int EPI, int CT, int WM, int WN, int NST, int GN>
__global__ void __launch_bounds__(256, 2)
k_gather_m_lds(const GemmArgs g) {
  using T = MTile<WM, WN, NST, GN>;
  constexpr int TMW = T::TMW, TNW = T::TNW, KS = T::KS, LA = T::LA, LB = T::LB;
  __shared__ __attribute__((aligned(1024))) char smem[NST * T::STAGE];
  __shared__ int s_rows_a[TMW];   // source row of A per tile row
  __shared__ int s_rows_c[TMW];   // destination row of C per tile row (-1 = skip)
  const uint32_t lds0 = (uint32_t)(uintptr_t)(PIT_LDS char*)smem;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wv / GN, wn = wv % GN;

  // ---------------------------------------------------------------- which tile is this workgroup?
  // Consecutive workgroup ids go to different XCDs (8, each with its own L2).  The row tiles that exist (their
  // number is known only here, from the segment lengths) are dealt out in contiguous shares and each XCD works
  // through its share in order, all its column tiles of a row tile back to back: they read the same gathered A
  // rows, and neighbouring row tiles of one segment (one expert) read the same B, through the same L2.  The grid
  // is sized for the worst case; workgroups beyond an XCD's share have no tile.
  const int tn = gridDim.x;
  const int lin = blockIdx.x + tn * blockIdx.y;
  const int xcd = lin & 7, slot = lin >> 3;
  const int row_in_share = slot / tn;
  int n0 = (slot % tn) * TNW;
  // One pass over the segment lengths gives the number of row tiles and, in the same registers, the segment and
  // position of this workgroup's tile (up to 64 segments: one load per lane; more: a second pass).  Every load
  // here is a round trip to memory on the critical path of the tile, so nothing is fetched twice.
  int seg = -1, tile_in_seg = 0, seg_begin = 0, seg_cnt = 0, total_tiles = 0;
  auto scan64 = [&](int s0, int& beg, int& cnt, int& nt) -> int {   // inclusive scan of the tile counts of 64 segments
    const int s = s0 + lane;
    beg = 0; cnt = 0;
    if (s < g.nseg) { beg = g.seg_ptr[s]; cnt = g.seg_ptr[s + 1] - beg; }
    nt = (cnt + TMW - 1) / TMW;
    int inc = nt;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int t = __shfl_up(inc, d);
      if (lane >= d) inc += t;
    }
    return inc;
  };
  auto locate = [&](int tile, int base, int inc, int nt, int beg, int cnt, int s0) {   // tile lies in this chunk
    const unsigned long long hit = __ballot(base + inc > tile);
    const int l = __builtin_ctzll(hit);
    seg = s0 + l;
    tile_in_seg = tile - (base + __shfl(inc, l) - __shfl(nt, l));
    seg_begin = __shfl(beg, l);
    seg_cnt = __shfl(cnt, l);
  };
  if (g.nseg <= 64) {
    int beg, cnt, nt;
    const int inc = scan64(0, beg, cnt, nt);
    total_tiles = __shfl(inc, 63);
    // The 8 XCDs form XR row groups x XC column groups (XC = g.xcd_cols, set by the launcher): an XCD works on
    // tn / XC column tiles of a contiguous share of the row tiles.  XC = 1 (every segment has a B of its own): an
    // XCD runs all column tiles of a row tile back to back.  XC > 1 (one B for all row tiles): an XCD's slice of
    // B stays in its L2 for the whole launch and only A rows stream through.
    const int xcn = g.xcd_cols, xrn = 8 / xcn;
    const int xr = xcd % xrn, xc = xcd / xrn;
    const int share = (total_tiles + xrn - 1) / xrn;
    const int cpx = tn / xcn;                      // column tiles an XCD works on
    const int mine = share * cpx;                  // tile slots of an XCD
    // Slots of an XCD beyond its tiles have no work and come last in dispatch order, so they run beside the last,
    // partly filled round of tiles.  With zero_rest they clear the unlisted rows of C meanwhile, each an equal
    // share of the rows (their number grows with the number of unlisted rows: both are what the worst-case grid
    // has left over).  (Placed behind the first round of tiles instead, so that their stores drain under the
    // second round's loops: the padded-batch step 3 us slower with bf16 output, 2 us faster with fp32 output.)
    if (slot >= mine) {
      if (g.zero_rest) {
        const int idle = (int)(gridDim.x * gridDim.y / 8) - mine;
        const int d = (slot - mine) * 8 + xcd, per = (g.M + 8 * idle - 1) / (8 * idle);
        const int rb = min(g.M, d * per), re = min(g.M, rb + per);
        if (rb < re) zero_unlisted_rows<CT ? 2 : 4>(g, rb, re, wv, lane);
      }
      return;
    }
    const int tile = xr * share + slot / cpx;
    n0 = (xc * cpx + slot % cpx) * TNW;
    if (tile >= total_tiles) return;
    locate(tile, 0, inc, nt, beg, cnt, 0);
  } else {
    for (int s0 = 0; s0 < g.nseg; s0 += 64) {
      int beg, cnt, nt;
      total_tiles += __shfl(scan64(s0, beg, cnt, nt), 63);
    }
    const int share = (total_tiles + 7) >> 3;
    const int tile = xcd * share + row_in_share;
    if (row_in_share >= share || tile >= total_tiles) return;
    int base = 0;
    for (int s0 = 0; s0 < g.nseg; s0 += 64) {
      int beg, cnt, nt;
      const int inc = scan64(s0, beg, cnt, nt);
      const int total = __shfl(inc, 63);
      if (tile < base + total) { locate(tile, base, inc, nt, beg, cnt, s0); break; }
      base += total;
    }
    if (seg < 0) return;
  }
  seg = __builtin_amdgcn_readfirstlane(seg);
  const int list_begin = __builtin_amdgcn_readfirstlane(seg_begin + tile_in_seg * TMW);
  const int list_len = __builtin_amdgcn_readfirstlane(min(TMW, seg_cnt - tile_in_seg * TMW));

  const int nsteps = g.slab / KS;                  // the k extent is a multiple of 32 (checked on the host)

  // ---------------------------------------------------------------- loader: source offsets per lane
  const char* a_src = uniform_ptr(g.A);
  const char* b_src = uniform_ptr(reinterpret_cast<const char*>(g.B) + (int64_t)seg * g.b_seg_stride * 2);
  const uint32_t pitch_a = (uint32_t)(g.lda * 2), pitch_b = (uint32_t)(g.ldb * 2);
  // B: a k-row of the tile is SPR slots of 16 B; load instruction j brings k-rows RPI j .. RPI j + RPI - 1;
  // lane l -> k-row RPI j + l / SPR, slot s = l % SPR, which holds source chunk ((s >> 2) ^ (k & 3)) * 4 + s % 4
  constexpr int SPR = TNW / 8, RPI = 64 / SPR;
  uint32_t b_off[LB];
#pragma unroll
  for (int jj = 0; jj < LB; ++jj) {
    const int kk = RPI * (wv + 4 * jj) + lane / SPR;
    const int s = lane % SPR;
    const int q = (s >> 2) ^ (kk & 3);
    b_off[jj] = __umul24((uint32_t)kk, pitch_b) + (uint32_t)((n0 + q * 32 + (s & 3) * 8) * 2);
  }
  const uint32_t b_step = 32u * pitch_b;           // bytes between two stages of B
  // k_rot: the tile walks its k range starting at step k_rot and wrapping round (the order of the reduction is
  // free).  With a B of its own per segment (every expert's weights are read from memory, and all of them lie
  // at the same offsets modulo a large power of two), tiles that all stand at the same k ask the same few memory
  // channels at the same time; tiles of different segments or column tiles therefore start at different steps.
  // Tiles that share B (the row tiles of one segment and column tile) keep the same start and stay in step.
  // (Mixture-of-experts call: 162.4-162.8 against 164.0 us.)
  const int k_rot = __builtin_amdgcn_readfirstlane((g.k_stagger && nsteps > 1) ? (int)(((unsigned)(seg * tn + n0 / TNW) * 37u) % (unsigned)nsteps) : 0);
  auto rot = [&](int t) { const int tt = t + k_rot; return tt >= nsteps ? tt - nsteps : tt; };
  auto issue_b = [&](int t, int u) {                  // B rows of stage t into buffer u = t % NST
    const uint32_t buf = lds0 + (uint32_t)(u * T::STAGE + T::A_STAGE), kb = (uint32_t)rot(t) * b_step;
#pragma unroll
    for (int jj = 0; jj < LB; ++jj) dma16(b_src, b_off[jj] + kb, buf + (uint32_t)((wv + 4 * jj) * 1024));
  };
  // The B rows of the first stages do not depend on the row numbers: they are requested now, and the row
  // numbers (one more round trip: the index entries) are fetched while they travel.
#pragma unroll
  for (int t = 0; t < NST; ++t)
    if (t < nsteps) issue_b(t, t);

  for (int r = tid; r < TMW; r += 256) {
    // rows past the end of the list read the list's last row (a valid address); their results
    // are never stored
    const int p = list_begin + min(r, list_len - 1);
    const int v = (g.a_gather || g.c_scatter) ? g.idx[p] : 0;
    s_rows_a[r] = g.a_gather ? v : p;
    s_rows_c[r] = r < list_len ? (g.c_scatter ? v : list_begin + r) : -1;
  }
  __syncthreads();

  f32x16_t acc[WM][WN];
#pragma unroll
  for (int i = 0; i < WM; ++i)
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // A: load instruction j (this wave: j = wv + 4 jj) brings tile rows 16 j .. 16 j + 15; lane l -> row
  // 16 j + l / 4, slot l % 4, which holds source chunk (l % 4) ^ ((row >> 2) & 3)
  uint32_t a_off[LA];
#pragma unroll
  for (int jj = 0; jj < LA; ++jj) {
    const int r = 16 * (wv + 4 * jj) + (lane >> 2);
    const int c = (lane & 3) ^ ((r >> 2) & 3);
    a_off[jj] = __umul24((uint32_t)s_rows_a[r], pitch_a) + (uint32_t)(c * 16);
  }
  auto issue_a = [&](int t, int u) {
    const uint32_t buf = lds0 + (uint32_t)(u * T::STAGE), ka = (uint32_t)rot(t) * 64u;
#pragma unroll
    for (int jj = 0; jj < LA; ++jj) dma16(a_src, a_off[jj] + ka, buf + (uint32_t)((wv + 4 * jj) * 1024));
  };
  auto issue = [&](int t, int u) { issue_a(t, u); issue_b(t, u); };   // stage t into buffer u = t % NST

  // ---------------------------------------------------------------- operand reads: lane constants
  // A: row block i, k-substep ks -> row wm * 32 WM + 32 i + lane % 32, chunk 2 ks + lane / 32 (at slot chunk ^ xa,
  //    xa = (row >> 2) & 3: the row's other bits are multiples of 32)
  // B: column block j, k-substep ks -> k-rows 16 ks + 8 h + kq (+ 4), 64-byte chunk (wn WN + j) ^ kq
  // Every address is a per-lane constant plus a compile-time offset (stage, row block, substep).
  const int h = lane >> 5, xa = (lane >> 2) & 3, kq = (lane & 15) >> 2;
  uint32_t a_rd[2], b_rd[WN];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks)
    a_rd[ks] = lds0 + (uint32_t)((wm * 32 * WM + (lane & 31)) * 64 + (((2 * ks + h) ^ xa) << 4));
#pragma unroll
  for (int j = 0; j < WN; ++j)
    b_rd[j] = lds0 + (uint32_t)(T::A_STAGE + (8 * h + kq) * (TNW * 2) + ((lane >> 4) & 1) * 32 + (lane & 3) * 8 +
                                (((wn * WN + j) ^ kq) << 6));
  // row blocks of this wave that hold at least one listed row (a tile at the end of a segment, or a segment
  // with few rows -- an expert with few tokens -- leaves the others without work: no operand reads, no MFMAs)
  const int live_i = __builtin_amdgcn_readfirstlane(max(0, min(WM, (list_len - wm * 32 * WM + 31) >> 5)));

  struct Frags { u32x4_t a[WM], b[WN]; };
  // FULL (compile time): every row block of the wave is live -- no conditions at all, so that a run of stages
  // is one basic block and the compiler can place its LDS waits precisely and spread the reads among the MFMAs
  // (with branches in between it falls back to a full wait in front of every read).
  auto read_frags = [&](uint32_t so, int ks, Frags& f, auto full) {     // so = byte offset of the stage's buffer
    constexpr bool FULL = decltype(full)::value;
#pragma unroll
    for (int i = 0; i < WM; ++i)
      if (FULL || i < live_i) f.a[i] = lds_read_frag(a_rd[ks] + so + (uint32_t)(i * 2048));
    if (FULL || live_i > 0) {
#pragma unroll
      for (int j = 0; j < WN; ++j) {
        const uint32_t at = b_rd[j] + so + (uint32_t)(ks * 16 * (TNW * 2));
        const uint2 lo = lds_tr(at), hi = lds_tr(at + 4 * (TNW * 2));
        f.b[j] = u32x4_t{lo.x, lo.y, hi.x, hi.y};
      }
    }
  };
  auto mfmas = [&](const Frags& f, auto full) {
    constexpr bool FULL = decltype(full)::value;
#pragma unroll
    for (int i = 0; i < WM; ++i)
      if (FULL || i < live_i) {
#pragma unroll
        for (int j = 0; j < WN; ++j)
          // operands swapped: the accumulator holds the 32 x 32 block transposed (lane = row of C,
          // registers = columns, four consecutive ones at a time), which is what the stores below want
          acc[i][j] = mfma32<BF>(f.b[j], f.a[i], acc[i][j]);
      }
  };

  // wait until this wave's loads of a stage have landed while `younger` later stages stay in flight
  auto wait_stage = [&](int younger) {
    if constexpr (NST >= 8) { if (younger >= 7) { PIT_WAIT_VMCNT(7 * T::LOADS); return; } }
    if constexpr (NST >= 7) { if (younger == 6) { PIT_WAIT_VMCNT(6 * T::LOADS); return; } }
    if constexpr (NST >= 6) { if (younger == 5) { PIT_WAIT_VMCNT(5 * T::LOADS); return; } }
    if constexpr (NST >= 5) { if (younger == 4) { PIT_WAIT_VMCNT(4 * T::LOADS); return; } }
    if constexpr (NST >= 4) { if (younger == 3) { PIT_WAIT_VMCNT(3 * T::LOADS); return; } }
    if constexpr (NST >= 3) { if (younger == 2) { PIT_WAIT_VMCNT(2 * T::LOADS); return; } }
    if (younger == 1) { PIT_WAIT_VMCNT(1 * T::LOADS); return; }
    PIT_WAIT_VMCNT(0);
  };

  // Pipeline.  Stage s is multiplied in two halves (k-substeps 0 and 1).  Between them the wave waits for its
  // loads of stage s + 1 and the workgroup meets at a barrier: after it every wave holds stage s in registers,
  // so buffer s % NST takes the loads of stage s + NST, and stage s + 1 has landed for everyone, so the
  // operands of its first half are requested before the MFMAs of the second half of stage s -- every LDS read
  // has a group of MFMAs to hide behind, and NST - 1 stages of loads are in flight.
  // The steady state (stages whose stage s + NST exists) runs NST stages per trip without a branch; the last
  // stages run through the general form.
  auto pipeline = [&](auto full) {
    // (the B rows of these stages are under way since before the row numbers were fetched; a full wait here:
    // the A rows of the first NST stages were requested together and land together)
#pragma unroll
    for (int t = 0; t < NST; ++t)
      if (t < nsteps) issue_a(t, t);
    PIT_WAIT_VMCNT(0);
    PIT_LDS_BARRIER();
    Frags f0, f1;
    read_frags(0u, 0, f0, full);
    int s0 = 0;
    for (; s0 + 2 * NST - 1 < nsteps; s0 += NST) {
#pragma unroll
      for (int u = 0; u < NST; ++u) {
        read_frags((uint32_t)(u * T::STAGE), 1, f1, full);
        mfmas(f0, full);
        PIT_WAIT_VMCNT((NST - 2) * T::LOADS);
        PIT_LDS_BARRIER();
        issue(s0 + u + NST, u);
        read_frags((uint32_t)(((u + 1) % NST) * T::STAGE), 0, f0, full);
        mfmas(f1, full);
      }
    }
    for (int s = s0; s < nsteps; ++s) {          // s0 is a multiple of NST: buffers continue at 0
      const int u = s - s0 < NST ? s - s0 : s - s0 - NST;
      read_frags((uint32_t)(u * T::STAGE), 1, f1, full);
      mfmas(f0, full);
      if (s + 1 < nsteps) {
        wait_stage(min(NST - 2, nsteps - 2 - s));
        PIT_LDS_BARRIER();
        if (s + NST < nsteps) issue(s + NST, u);
        read_frags((uint32_t)((u + 1 == NST ? 0 : u + 1) * T::STAGE), 0, f0, full);
      }
      mfmas(f1, full);
    }
  };
  if (nsteps > 0) {
    if (live_i == WM) pipeline(std::true_type{});
    else pipeline(std::false_type{});
  }

  // ---------------------------------------------------------------- SWrite
  // A lane holds one row of a 32 x 32 block, four columns per register quad; stored from there, one instruction
  // would touch 32 rows with 32 bytes each -- 32 partial-line requests per instruction (the padded-batch product
  // took 114 us that way, 99 us with whole lines).  So the wave's
  // 32 x (32 WN) row blocks go through LDS (the ring is free now; each wave has a region of its own): written as
  // the accumulators hold them, read back row-contiguous, and stored with 16 bytes per lane so that consecutive
  // lanes fill whole 128-byte lines of the destination row.
  constexpr int WCOLS = 32 * WN;                 // columns of the wave's tile
  constexpr int PITCH = WCOLS + 4;               // floats per row in LDS: rows 16 bytes apart in the banks
  static_assert(4 * 32 * PITCH * 4 <= NST * T::STAGE, "the four waves' row blocks must fit the ring");
  __syncthreads();                               // every wave has read its last operands from the ring
  float* cw = reinterpret_cast<float*>(smem) + wv * (32 * PITCH);
  const int ql = lane & 31, hh = lane >> 5;
#pragma unroll
  for (int i = 0; i < WM; ++i) {
    const int rb = wm * 32 * WM + i * 32;        // first tile row of this row block
    if (i >= live_i) break;                      // (uniform) no listed row in this block or the following ones
    {
      const int crow = s_rows_c[rb + ql];
      float scale = 1.f;
      if constexpr (EPI == EPI_STORE) { if (g.gate && crow >= 0) scale = g.gate[crow]; }
#pragma unroll
      for (int j = 0; j < WN; ++j)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          float v[4];
#pragma unroll
          for (int x = 0; x < 4; ++x) {
            v[x] = acc[i][j][4 * gq + x];
            if constexpr (EPI == EPI_GELU) v[x] = gelu_erf_fast(v[x]);
            if constexpr (EPI == EPI_STORE) v[x] *= scale;
          }
          *reinterpret_cast<float4*>(cw + ql * PITCH + j * 32 + 8 * gq + 4 * hh) = make_float4(v[0], v[1], v[2], v[3]);
        }
    }
    __builtin_amdgcn_wave_barrier();
    if constexpr (CT == 0) {
      constexpr int LPR = WCOLS / 4, RPI = 64 / LPR;        // lanes per row, rows per store instruction
      const int rr = lane / LPR, c4 = (lane % LPR) * 4;
#pragma unroll
      for (int t = 0; t < 32 / RPI; ++t) {
        const int row = t * RPI + rr;
        const int64_t crow = s_rows_c[rb + row];
        const float4 v = *reinterpret_cast<const float4*>(cw + row * PITCH + c4);
        if (crow >= 0) *reinterpret_cast<float4*>(reinterpret_cast<float*>(g.C) + crow * g.ldc + n0 + wn * WCOLS + c4) = v;
      }
    } else {
      constexpr int LPR = WCOLS / 8, RPI = 64 / LPR;
      const int rr = lane / LPR, c8 = (lane % LPR) * 8;
#pragma unroll
      for (int t = 0; t < 32 / RPI; ++t) {
        const int row = t * RPI + rr;
        const int64_t crow = s_rows_c[rb + row];
        const float4 a = *reinterpret_cast<const float4*>(cw + row * PITCH + c8);
        const float4 b = *reinterpret_cast<const float4*>(cw + row * PITCH + c8 + 4);
        uint4 pk;
        pk.x = pack2_in<BF>(a.x, a.y);
        pk.y = pack2_in<BF>(a.z, a.w);
        pk.z = pack2_in<BF>(b.x, b.y);
        pk.w = pack2_in<BF>(b.z, b.w);
        if (crow >= 0) *reinterpret_cast<uint4*>(reinterpret_cast<uint16_t*>(g.C) + crow * g.ldc + n0 + wn * WCOLS + c8) = pk;
      }
    }
    __builtin_amdgcn_wave_barrier();             // the next row block reuses the region
  }
}

template <bool BF, int EPI, int CT, int WM, int WN, int NST, int GN = 2>
int launch_cfg(GemmArgs g, int64_t total_rows, hipStream_t st) {
  using T = MTile<WM, WN, NST, GN>;
  // One B for all row tiles: 2 row groups x 4 column groups of XCDs where the number of column tiles allows
  // (padded batch, 16 column tiles: 96 us per step with 8 x 1, 88-89 us with 4 x 2, 2 x 4 and 1 x 8).
  g.xcd_cols = 1;
  if (g.nseg == 1) {
    const int tn = g.N / T::TNW;
    g.xcd_cols = tn % 4 == 0 ? 4 : tn % 2 == 0 ? 2 : 1;
  }
  g.k_stagger = g.b_seg_stride != 0 ? 1 : 0;
  const int64_t max_tiles = total_rows / T::TMW + g.nseg;      // sum over segments of ceil(count / TMW)
  if (max_tiles > 65520) return PIT_ESHAPE;
  // (row tiles rounded up to a multiple of 8: every XCD then has room for its share of the tiles that exist;
  // with zero_rest one more row of workgroups per XCD, so that some are without a tile whatever the list holds)
  dim3 grid((unsigned)(g.N / T::TNW), (unsigned)(((max_tiles + 7) & ~(int64_t)7) + (g.zero_rest ? 8 : 0)));
  hipLaunchKernelGGL((k_gather_m_lds<BF, EPI, CT, WM, WN, NST, GN>), grid, dim3(256), 0, st, g);
  PIT_LAUNCH_CHECK();
  return PIT_OK;
}

// Tile shape by the shape of the product.  128 x 256 (a wave owns 64 x 128) where N allows: fewer bytes through
// LDS per MFMA and fewer workgroups' worth of set-up than 128 x 128.  (Measured on the padded-batch product,
// 8364 x 1024 x 4096: 128 x 128 with a ring of 3 or 4 stages 127 us, 256 x 128 117, 128 x 256 108-115; on the
// mixture-of-experts call 189-193, 230 (rows of small experts are padded to 256) and 177 us.  Rings of 5 or 6 stages
// with one workgroup per compute unit: no gain on either.  256 x 256 with a wave owning 128 x 128 -- two thirds of the
// LDS bytes per MFMA, one workgroup per compute unit: 107 against 85 us and 214 against 163 us.)
template <bool BF, int EPI, int CT>
int launch_shape(const GemmArgs& g, int64_t total_rows, hipStream_t st) {
  // (a product too small to give every compute unit a 128 x 256 tile even in the worst case takes 128 x 128)
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) cus = 256;
  const int64_t wide_tiles = (total_rows / 128 + g.nseg) * (g.N / 256);
  if (g.N % 256 == 0 && wide_tiles >= cus) return launch_cfg<BF, EPI, CT, 2, 4, 3>(g, total_rows, st);
  return launch_cfg<BF, EPI, CT, 2, 2, 4>(g, total_rows, st);
}

template <bool BF>
int launch_bf(int epi, int ct, const GemmArgs& g, int64_t total_rows, hipStream_t st) {
  switch (epi) {
    case EPI_STORE: return ct ? launch_shape<BF, EPI_STORE, 1>(g, total_rows, st) : launch_shape<BF, EPI_STORE, 0>(g, total_rows, st);
    case EPI_GELU:  return ct ? launch_shape<BF, EPI_GELU, 1>(g, total_rows, st) : PIT_EINVAL;
    default: return PIT_EINVAL;
  }
}

}  // namespace

int launch_gather_m(bool bf, int epi, int c_is_in_type, const GemmArgs& g, int64_t total_rows, hipStream_t st) {
  if (total_rows <= 0 || g.N <= 0 || g.nseg <= 0) return PIT_OK;
  if (g.slab % 32 || g.N % 128) return PIT_ESHAPE;
  if (g.zero_rest && (g.nseg != 1 || !g.c_scatter)) return PIT_EINVAL;
  // the kernel addresses each operand with 32-bit byte offsets from a per-segment base and multiplies
  // row numbers by the row pitch in 24 bits
  if (g.lda * 2 >= (1ll << 24) || g.ldb * 2 >= (1ll << 24) || (int64_t)g.M >= (1ll << 24) || (int64_t)g.K >= (1ll << 24)) return PIT_ESHAPE;
  if ((int64_t)g.M * g.lda * 2 >= (1ll << 32) || (int64_t)g.K * g.ldb * 2 >= (1ll << 32)) return PIT_ESHAPE;
  return bf ? launch_bf<true>(epi, c_is_in_type, g, total_rows, st) : launch_bf<false>(epi, c_is_in_type, g, total_rows, st);
}

}  // namespace pit
