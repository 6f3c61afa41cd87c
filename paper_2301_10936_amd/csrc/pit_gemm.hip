// pit_sread_gemm: the SRead -> dense MFMA tile -> SWrite kernels (paper Section 3.1, sparse kernel
// template) for gfx950 with k as the PIT-axis, or m with micro-tiles along k, and the host-side
// validation and launch of all GEMM modes.  bf16 or f16 inputs, fp32 accumulation.
// There is one kernel per PIT-axis of MatMul (paper Table 1):
//
//   k_gather_k_direct  GATHER_K: A is K-major (At[k][m]); the tile's k-list comes from the index and
//             names the rows of At and of B to multiply.  Operands go global -> registers directly
//             and are transposed inside each lane; the waves of a workgroup split the k-list and
//             reduce their partial tiles through LDS at the end (details above the kernel).
//             Tiles of 128, 64 or 32 rows x 128 columns.
//   k_slab_strip  GATHER_M with several k-slabs per row (1 x mt micro-tiles of a row-major A): a strip
//             of C stays in LDS while the listed rows of every slab are added to it.
//   k_gather_m_lds (pit_gemm_m.hip)  GATHER_M with whole-row micro-tiles (padded batches, MoE): the
//             tile's row numbers come from the index once, operands are staged through LDS.
//
// SWrite.  GATHER_K writes the rows of its m-tile in place; k_slab_strip stores whole strips.
#include "pit_gemm.hpp"
#include "pit_gemm_dev.hpp"
#include <type_traits>
#include <algorithm>
#include <climits>

namespace pit {
namespace {

// ------------------------------------------------------------------------------------------------
// GATHER_K, register-direct: no LDS and no barrier inside the k loop.
//
// Both operands of GATHER_K are K-major (rows of At and of B), and an MFMA operand register holds
// 8 consecutive k of ONE column.  A lane that loads 16 bytes (8 columns) from each of 8 listed
// rows owns an 8 k x 8 column block, and transposing that block inside the lane (v_perm_b32, no
// cross-lane traffic) yields 8 operand registers, one per column.  With v_mfma_f32_16x16x32 (lane
// l: column l % 16, k-block l / 16) 16 lanes x 8 columns cover 128 columns, so a wavefront's 8
// loads of At give it the A operands of all 128 tile rows for 32 k, its 8 loads of B the B
// operands of all 128 tile columns, and 8 x 8 MFMAs consume them: MFMA (ja, jb) works on the
// strided row set {8r + ja} and column set {8c + jb}.  Each operand byte travels global -> register
// exactly once per workgroup and never through LDS.
// The four wavefronts split the tile's k-list in slabs of 32 entries (wave w takes slabs w, w+4, ..),
// each accumulating a full 128 x 128 partial tile in 256 accumulator registers; at the end the
// partial tiles are reduce-scattered through LDS (4 rounds of 48 KiB) and every wave stores a
// quarter of the tile, 512 contiguous bytes per row.  With more tiles than compute units a workgroup
// loops over tiles.
// The k loop is branch-free: list positions past the end are clamped to the last entry on load, the
// last slab of each wave is processed apart with the clamped rows zeroed.
// ------------------------------------------------------------------------------------------------
typedef float f32x4_t __attribute__((ext_vector_type(4)));

// acc += A * B with v_mfma_f32_16x16x32.  Written as inline assembly so that the accumulator is
// updated IN PLACE in an accumulation register: with all 256 of them live the register allocator
// otherwise gives the result a different register than the input and shuffles accumulators
// through vector registers between MFMAs.  The assembly is opaque to the compiler's hazard
// handling: callers must leave 64 other MFMAs (or PIT_MFMA_DRAIN) between an update of an
// accumulator and its next use.
template <bool BF>
__device__ __forceinline__ void mfma16_acc(const uint4& a, const uint4& b, f32x4_t& c) {
  const u32x4_t av = __builtin_bit_cast(u32x4_t, a), bv = __builtin_bit_cast(u32x4_t, b);
  if constexpr (BF) asm("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(av), "v"(bv));
  else              asm("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+a"(c) : "v"(av), "v"(bv));
}
// wait until the matrix pipe has written every accumulator (a 4-pass MFMA needs at most 10 idle
// issue slots before another kind of instruction may read its result)
#define PIT_MFMA_DRAIN() do { PIT_SCHED_FENCE(); asm volatile("s_nop 15\n\ts_nop 15" ::: "memory"); PIT_SCHED_FENCE(); } while (0)

constexpr int RED_SLOT_BYTES = 16 * 64 * 16;        // 16 accumulator quads x 64 lanes x 16 B
constexpr int RED_BUF_BYTES = 4 * RED_SLOT_BYTES;   // one slot per sending wave

// Round P of the reduction: the partial sums of tile rows {8r + ja : ja in {2P, 2P + 1}} go to wave
// P.  P is a compile-time constant so that every accumulator index is static.
template <int P>
__device__ __forceinline__ void red_send(const f32x4_t (&acc)[8][8], PIT_LDS char* buf, int wv, int lane) {
  PIT_LDS char* slot = buf + wv * RED_SLOT_BYTES + lane * 16;
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int jb = 0; jb < 8; ++jb) *(PIT_LDS f32x4_t*)(slot + (a * 8 + jb) * 1024) = acc[2 * P + a][jb];
}
// Wave P adds the three other waves' partial sums to its own.
template <int P>
__device__ __forceinline__ void red_recv(f32x4_t (&acc)[8][8], PIT_LDS char* buf, int lane) {
  // (all 16 reads of one sender are issued before the first addition: one LDS latency per sender
  // instead of one per read)
#pragma unroll
  for (int o = 1; o < 4; ++o) {
    PIT_LDS char* slot = buf + ((P + o) & 3) * RED_SLOT_BYTES + lane * 16;
    f32x4_t part[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) part[i] = *(PIT_LDS f32x4_t*)(slot + i * 1024);
    PIT_SCHED_FENCE();
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[2 * P + (i >> 3)][i & 7] += part[i];
    PIT_SCHED_FENCE();
  }
}
// Two-wave workgroups: half H of the tile = the row groups ja in {H * JA / 2 .. (H + 1) * JA / 2 - 1}
// (JA = row groups of the tile = tile rows / 16).
template <int JA> constexpr int red_half_bytes() { return 4 * JA * 64 * 16; }
template <int JA, int H>
__device__ __forceinline__ void red_send_half(const f32x4_t (&acc)[JA][8], PIT_LDS char* slot) {
#pragma unroll
  for (int i = 0; i < 4 * JA; ++i) *(PIT_LDS f32x4_t*)(slot + i * 1024) = acc[(JA / 2) * H + (i >> 3)][i & 7];
}
template <int JA, int H>
__device__ __forceinline__ void red_recv_half(f32x4_t (&acc)[JA][8], PIT_LDS char* slot) {
  constexpr int CH = 4 * JA < 16 ? 4 * JA : 16;     // reads issued together, ahead of their additions
#pragma unroll
  for (int a = 0; a < 4 * JA / CH; ++a) {
    f32x4_t part[CH];
#pragma unroll
    for (int i = 0; i < CH; ++i) part[i] = *(PIT_LDS f32x4_t*)(slot + (a * CH + i) * 1024);
    PIT_SCHED_FENCE();
#pragma unroll
    for (int i = 0; i < CH; ++i) acc[(JA / 2) * H + ((a * CH + i) >> 3)][(a * CH + i) & 7] += part[i];
    PIT_SCHED_FENCE();
  }
}
// Store the row groups ja in [J0, J0 + NJ) of the tile: rows JA * (4 * (lane / 16) + e) + ja; a lane holds 8
// consecutive columns of such a row (one per jb), so 16 lanes write 512 (fp32) or 256 contiguous bytes.
template <bool BF, int CT, int JA, int J0, int NJ>
__device__ __forceinline__ void red_store(const f32x4_t (&acc)[JA][8], const GemmArgs& g, int m_base, int n0, int lane) {
  const int q = lane & 15, kb = lane >> 4;
#pragma unroll
  for (int a = 0; a < NJ; ++a) {
    const int ja = J0 + a;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int64_t row = m_base + JA * (4 * kb + e) + ja;
      const int col = n0 + 8 * q;
      if constexpr (CT == 0) {
        // (streaming stores: the result is not read again by this kernel and should not displace the
        // operand panels from L2)
        typedef float f4_t __attribute__((ext_vector_type(4)));
        f4_t* d = reinterpret_cast<f4_t*>(reinterpret_cast<float*>(g.C) + row * g.ldc + col);
        __builtin_nontemporal_store(f4_t{acc[ja][0][e], acc[ja][1][e], acc[ja][2][e], acc[ja][3][e]}, d);
        __builtin_nontemporal_store(f4_t{acc[ja][4][e], acc[ja][5][e], acc[ja][6][e], acc[ja][7][e]}, d + 1);
      } else {
        uint32_t w[4];
#pragma unroll
        for (int x = 0; x < 4; ++x)
          w[x] = pack2_in<BF>(acc[ja][2 * x][e], acc[ja][2 * x + 1][e]);
        __builtin_nontemporal_store(u32x4_t{w[0], w[1], w[2], w[3]},
                                    reinterpret_cast<u32x4_t*>(reinterpret_cast<uint16_t*>(g.C) + row * g.ldc + col));
      }
    }
  }
}

// what a wave needs to know about one tile
struct DirectTile {
  int seg, n0, list_len, n_w;      // tile row (= index segment), first column, length of the k-list, this wave's slabs
  const char* list;                // the k-list
  uint32_t a_col, b_col;           // this lane's byte offsets into a row of At and of B
};

// NW = waves per workgroup that split the k-list: 4 (one workgroup fills a compute unit) or 2 (two
// workgroups, i.e. two tiles, share a compute unit at the same register cost, and the set-up, drain,
// reduction and stores of one tile run under the MFMA loop of the other; used when there are at
// least two tiles per compute unit).
// JA = row groups of the tile: the tile is 16 * JA rows high (128, 64 or 32 = the micro-tile height of the
// index), a lane loads JA consecutive m of each listed row of At (16, 8 or 4 bytes) and a slab takes JA x 8
// MFMAs.  Lower tiles follow a finer sparsity pattern (fewer all-zero micro-tiles are multiplied) and pay for
// it with more traffic of B per row of C; they always run as two-wave workgroups, several per compute unit.
template <bool BF, int CT, int NW, int JA>
__global__ void __launch_bounds__(64 * NW)
k_gather_k_direct(const GemmArgs g, const int tm_tiles) {
  static_assert(JA == 8 || (NW == 2 && (JA == 4 || JA == 2)), "tile heights: 128 (2 or 4 waves), 64 and 32 (2 waves)");
  constexpr int SK = 32;   // list entries per slab = k extent of one MFMA
  constexpr int TMJ = 16 * JA;   // tile rows
  constexpr int RED_HALF_BYTES = red_half_bytes<JA>();
  __shared__ __attribute__((aligned(16))) char s_red[NW == 4 ? 2 * RED_BUF_BYTES : 2 * RED_HALF_BYTES];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int q = lane & 15, kb = lane >> 4;
  const char* a_src = uniform_ptr(g.A);
  const char* b_src = uniform_ptr(g.B);
  const uint32_t pitch_a = (uint32_t)(g.lda * 2), pitch_b = (uint32_t)(g.ldb * 2);

  // The grid is one-dimensional and may hold fewer workgroups than there are tiles: a workgroup then
  // works through tiles lin = blockIdx.x, blockIdx.x + gridDim.x, ... (gridDim.x is a multiple of 8
  // in that case, so all of them belong to the same XCD).
  const int tn = g.N / TN, total = tn * tm_tiles;
  // Consecutive workgroup ids go to different XCDs (8, each with its own L2): renumber so that each
  // XCD works on a contiguous run of tiles, ordered in bands of 4 tile rows x all tile columns.
  const bool dense = g.idx == nullptr;
  auto tile_of = [&](int lin) -> DirectTile {
    const int x = lin & 7, qq = total >> 3, rr = total & 7;
    const int lp = x * qq + min(x, rr) + (lin >> 3);
    constexpr int GM = 4;
    const int band = lp / (GM * tn), within = lp - band * (GM * tn);
    const int rows = min(GM, tm_tiles - band * GM);
    DirectTile t;
    t.seg = band * GM + within % rows;
    t.n0 = (within / rows) * TN;
    // dense mode (no index): every tile's list is 0, 1, .., K - 1 and is never read from memory
    const int list_begin = dense ? 0 : g.seg_ptr[t.seg];
    t.list_len = dense ? g.K : g.seg_ptr[t.seg + 1] - list_begin;
    const int nslab = (t.list_len + SK - 1) / SK;
    t.n_w = nslab > wv ? (nslab - wv + NW - 1) / NW : 0;   // this wave's slabs: wv, wv + NW, ...
    t.list = uniform_ptr(g.idx + list_begin);
    t.a_col = (uint32_t)(t.seg * TMJ + JA * q) * 2u;
    t.b_col = (uint32_t)(t.n0 + 8 * q) * 2u;
    return t;
  };

  // lane l of a slab's list load holds entry (l % 32) of the slab
  auto load_list = [&](const DirectTile& T, int t) -> int {
    const int pos = min(SK * (wv + NW * t) + (lane & 31), T.list_len - 1);
    if (dense) return pos;
    typedef const int __attribute__((address_space(1))) * gint_t;
    return *(gint_t)(uintptr_t)(reinterpret_cast<uintptr_t>(T.list) + (uint32_t)pos * 4u);
  };
  // rows k(8 kb + i), i = 0..7, of At and of B
  auto issue = [&](const DirectTile& T, int kraw, ACols<JA> (&ra)[8], uint4 (&rb)[8]) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const uint32_t k = (uint32_t)__builtin_amdgcn_ds_bpermute((8 * kb + i) * 4, kraw);
      ra[i] = load_cols<JA>(a_src, __umul24(k, pitch_a) + T.a_col);
      rb[i] = load16(b_src, __umul24(k, pitch_b) + T.b_col);
    }
  };

  f32x4_t acc[JA][8];
#pragma unroll
  for (int i = 0; i < JA; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  // JA x 8 MFMAs on one slab (64 for the 128-row tile, which the description below is written for).  All B operands are transposed first; the A operand of column group
  // ja + 1 is transposed (4 v_perm_b32) in the shadow of the first MFMAs of group ja.  The order is
  // pinned: an MFMA must not read a register in the issue slot right after a vector instruction
  // wrote it, and the inline-assembly MFMAs are invisible to the compiler's hazard handling, so
  // every operand is produced at least four MFMAs (or the explicit s_nop) before its first use.
  // ISSUE: the loads of the slab two ahead (list entries in kraw) are issued from inside the MFMA
  // sequence as soon as their registers are free: the B rows during column groups 0..3 (rb is dead
  // once the B operands are transposed), the A rows during group 7 (ra is dead once the last A
  // operand is transposed).  Spreading them keeps 16 to 24 loads of a wave in flight; with 32 in
  // flight at once the load path of a CU runs at less than half its rate (measured).  (Lower tiles: the B
  // rows during the second half of every column group but the last, the A rows during the last group.)
  auto process_impl = [&](const DirectTile& T, ACols<JA> (&ra)[8], uint4 (&rb)[8], int kraw, auto issue_tag) {
    constexpr bool ISSUE = decltype(issue_tag)::value;
    uint4 bfr[8];
#pragma unroll
    for (int jb = 0; jb < 8; ++jb) bfr[jb] = transpose8x8_row(rb, jb);
    uint32_t af[4], afn[4] = {0, 0, 0, 0};
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) af[jj] = transpose_cols_dword<JA>(ra, 0, jj);
    uint32_t kk[8];
    if constexpr (ISSUE) {
#pragma unroll
      for (int i = 0; i < 8; ++i) kk[i] = (uint32_t)__builtin_amdgcn_ds_bpermute((8 * kb + i) * 4, kraw);
    }
    PIT_SCHED_FENCE();
    asm volatile("s_nop 7");
    PIT_SCHED_FENCE();
#pragma unroll
    for (int ja = 0; ja < JA; ++ja) {
#pragma unroll
      for (int jb = 0; jb < 8; ++jb) {
        mfma16_acc<BF>(make_uint4(af[0], af[1], af[2], af[3]), bfr[jb], acc[ja][jb]);
        if (ja < JA - 1 && jb < 4) afn[jb] = transpose_cols_dword<JA>(ra, ja + 1, jb);
        if constexpr (ISSUE) {
          if constexpr (JA >= 4) {
            if (ja < 4 && (jb == 4 || jb == 6)) {
              const int i = ja * 2 + ((jb - 4) >> 1);
              rb[i] = load16(b_src, __umul24(kk[i], pitch_b) + T.b_col);
            }
          } else {
            if (jb >= 4) {   // JA == 2: 8 loads in the second halves of the two column groups
              const int i = ja * 4 + (jb - 4);
              rb[i] = load16(b_src, __umul24(kk[i], pitch_b) + T.b_col);
            }
          }
          // (the A rows of the next-but-one slab may only replace ra once the last A operand of this
          // slab has been taken out of it: during the last column group)
          if (ja == JA - 1) ra[jb] = load_cols<JA>(a_src, __umul24(kk[jb], pitch_a) + T.a_col);
        }
        PIT_SCHED_FENCE();
      }
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) af[jj] = afn[jj];
    }
  };
  auto process = [&](const DirectTile& T, ACols<JA> (&ra)[8], uint4 (&rb)[8]) { process_impl(T, ra, rb, 0, std::false_type{}); };
  auto process_issue = [&](const DirectTile& T, ACols<JA> (&ra)[8], uint4 (&rb)[8], int kraw) { process_impl(T, ra, rb, kraw, std::true_type{}); };
  // local slab t with the rows of positions past the end of the list zeroed
  auto process_last = [&](const DirectTile& T, int t, ACols<JA> (&ra)[8], uint4 (&rb)[8]) {
    const int p0 = SK * (wv + NW * t) + 8 * kb;
#pragma unroll
    for (int i = 0; i < 8; ++i)
      if (p0 + i >= T.list_len) {
#pragma unroll
        for (int d = 0; d < JA / 2; ++d) ra[i].d[d] = 0u;
        rb[i] = make_uint4(0, 0, 0, 0);
      }
    process(T, ra, rb);
  };

  // With several tiles per workgroup the next tile's description and the list entries of its first
  // two slabs are fetched ahead of the current tile's reduction, so that only the row loads remain
  // between two tiles.
  ACols<JA> ra0[8], ra1[8];
  uint4 rb0[8], rb1[8];
  PIT_LDS char* red = (PIT_LDS char*)s_red;
  int lin = blockIdx.x;
  DirectTile T = tile_of(lin);
  int k0 = 0, k1 = 0;
  if (T.n_w > 0) { k0 = load_list(T, 0); k1 = load_list(T, 1); }
  for (;;) {
    if (T.n_w > 0) {
      // (the fences keep the list loads of slabs 2 and 3 ahead of the second slab's data loads: the
      // memory counter retires in order, so a list load issued last would make the loop wait for all)
      PIT_SCHED_FENCE();
      issue(T, k0, ra0, rb0); k0 = load_list(T, 2); PIT_SCHED_FENCE();
      issue(T, k1, ra1, rb1); k1 = load_list(T, 3); PIT_SCHED_FENCE();
      int t = 0;
      for (; t + 2 < T.n_w; t += 2) {
        process_issue(T, ra0, rb0, k0); k0 = load_list(T, t + 4); PIT_SCHED_FENCE();
        process_issue(T, ra1, rb1, k1); k1 = load_list(T, t + 5); PIT_SCHED_FENCE();
      }
      if (T.n_w - t == 2) {
        process(T, ra0, rb0);
#pragma unroll
        for (int i = 0; i < 8; ++i) { ra0[i] = ra1[i]; rb0[i] = rb1[i]; }
        ++t;
      }
      process_last(T, t, ra0, rb0);
      PIT_MFMA_DRAIN();
    }
    const int lin_next = lin + (int)gridDim.x;
    const bool more = lin_next < total;
    DirectTile Tn = T;
    if (more) {
      Tn = tile_of(lin_next);
      if (Tn.n_w > 0) { k0 = load_list(Tn, 0); k1 = load_list(Tn, 1); }
    }
    PIT_SCHED_FENCE();

    const int m_base = T.seg * TMJ;
    if constexpr (NW == 4) {
      // Reduction across the four waves, one quarter of the tile rows per round, double-buffered in
      // LDS: round P's partial sums are written before barrier P and read by wave P after it, while the
      // other waves already write round P + 1 into the other buffer.
      if (wv != 0) red_send<0>(acc, red, wv, lane);
      __syncthreads();
      if (wv == 0) { red_recv<0>(acc, red, lane); red_store<BF, CT, 8, 0, 2>(acc, g, m_base, T.n0, lane); }
      if (wv != 1) red_send<1>(acc, red + RED_BUF_BYTES, wv, lane);
      __syncthreads();
      if (wv == 1) { red_recv<1>(acc, red + RED_BUF_BYTES, lane); red_store<BF, CT, 8, 2, 2>(acc, g, m_base, T.n0, lane); }
      if (wv != 2) red_send<2>(acc, red, wv, lane);
      __syncthreads();
      if (wv == 2) { red_recv<2>(acc, red, lane); red_store<BF, CT, 8, 4, 2>(acc, g, m_base, T.n0, lane); }
      if (wv != 3) red_send<3>(acc, red + RED_BUF_BYTES, wv, lane);
      __syncthreads();
      if (wv == 3) { red_recv<3>(acc, red + RED_BUF_BYTES, lane); red_store<BF, CT, 8, 6, 2>(acc, g, m_base, T.n0, lane); }
    } else {
      // The two waves trade the halves of their partial tiles that the other one owns (wave 0: the
      // row groups ja < 4).  The first barrier keeps a wave from overwriting what the other still
      // reads for the previous tile.
      __syncthreads();
      if (wv == 0) red_send_half<JA, 1>(acc, red + lane * 16);
      else         red_send_half<JA, 0>(acc, red + RED_HALF_BYTES + lane * 16);
      __syncthreads();
      if (wv == 0) {
        red_recv_half<JA, 0>(acc, red + RED_HALF_BYTES + lane * 16);
        red_store<BF, CT, JA, 0, JA / 2>(acc, g, m_base, T.n0, lane);
      } else {
        red_recv_half<JA, 1>(acc, red + lane * 16);
        red_store<BF, CT, JA, JA / 2, JA / 2>(acc, g, m_base, T.n0, lane);
      }
    }
    if (!more) break;
    PIT_SCHED_FENCE();
    lin = lin_next;
    T = Tn;
#pragma unroll
    for (int i = 0; i < JA; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  }
}

// ------------------------------------------------------------------------------------------------
// GATHER_M with micro-tiles along k (several k-slabs per row: 1 x mt micro-tiles of a row-major A).
//
// The rows listed for slab s differ from those of slab s', so the partial products of the slabs
// have to meet in C.  Here C stays put: a workgroup owns a strip of R rows x W columns of C
// (R x W = 4096: 64 x 64, or 32 x 128) and walks ALL slabs; per slab it gathers the strip's listed
// rows (SRead along m inside the strip, in blocks of 16 rows), multiplies them with the slab's rows
// of B on v_mfma_f32_16x16x32, and adds the result to the strip held in LDS.  The four waves take
// the slabs round-robin, each with a strip of its own (no atomics, no races); at the end the four
// strips are added in a fixed order and the whole strip is stored, rows that nothing touched as
// zeros.  So the result does not depend on the order in which anything ran, and C needs no clearing
// beforehand.  B is read once per strip of rows, so its traffic falls with R; A is read once per
// strip of columns.
//   rows of a slab inside the strip: the slab's list is ascending, so they are one contiguous run
//   of it; a 64-ary search by the wave finds where the run starts, two 64-entry loads hold it.
//   A operand: 16 bytes (8 k) of a listed row per lane -- already the operand layout.
//   B operand: 8 k-rows x CW columns (CW = W / 16) per lane, transposed inside the lane.
//   strip in LDS: a lane moves the CW columns it holds of a row as 16-byte vectors and the 16
//   lanes of a row lie side by side; a spare row swallows the results of unused block rows.
// ------------------------------------------------------------------------------------------------
constexpr int SS_BATCH = 8;                          // slabs per wave whose row lookups are in flight together
static_assert(SS_BATCH == 8, "the lane layout of the list-bounds load assumes 8");
template <int CW> struct StripShape {
  static_assert(CW == 4 || CW == 8, "columns per lane");
  static constexpr int W = 16 * CW;                  // columns of C per workgroup
  static constexpr int R = 4096 / W;                 // rows of C per workgroup (at most 64: one lane per listed row)
  static constexpr int FLOATS = (R + 1) * W;         // one wave's strip, with the spare row
};

// CW 16-bit columns of one k-row, as loaded
template <int CW> struct BRow { uint32_t d[CW / 2]; };
template <int CW>
__device__ __forceinline__ BRow<CW> load_brow(const char* base, uint32_t byte_off) {
  BRow<CW> r;
  if constexpr (CW == 8) {
    const uint4 v = load16(base, byte_off);
    r.d[0] = v.x; r.d[1] = v.y; r.d[2] = v.z; r.d[3] = v.w;
  } else {
    typedef const u32x2_t __attribute__((address_space(1))) * gptr_t;
    const u32x2_t v = *(gptr_t)(uintptr_t)(reinterpret_cast<uintptr_t>(base) + byte_off);
    r.d[0] = v[0]; r.d[1] = v[1];
  }
  return r;
}
// 8 consecutive k of column x out of 8 k-rows (4 v_perm_b32)
template <int CW>
__device__ __forceinline__ uint4 bcolumn(const BRow<CW> (&r)[8], int x) {
  const uint32_t sel = (x & 1) ? 0x07060302u : 0x05040100u;
  uint32_t d[4];
#pragma unroll
  for (int jj = 0; jj < 4; ++jj) d[jj] = __builtin_amdgcn_perm(r[2 * jj + 1].d[x >> 1], r[2 * jj].d[x >> 1], sel);
  return make_uint4(d[0], d[1], d[2], d[3]);
}

template <bool BF>
__device__ __forceinline__ f32x4_t mfma16(const uint4& a, const uint4& b, const f32x4_t& c) {
  if constexpr (BF)
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
}

template <bool BF, int CW>
__global__ void __launch_bounds__(256, 2)
k_slab_strip(const GemmArgs g) {
  using SH = StripShape<CW>;
  constexpr int SS_RM = SH::R;
  __shared__ __attribute__((aligned(16))) float s_c[4][SH::FLOATS];
  __shared__ __attribute__((aligned(16))) int s_rows[4][SS_BATCH][64];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int q = lane & 15, kb = lane >> 4;
  const int n0 = blockIdx.x * SH::W;
  const int r0 = blockIdx.y * SS_RM;
  float* strip = s_c[wv];
  for (int i = lane * 4; i < SH::FLOATS; i += 256) *reinterpret_cast<f32x4_t*>(strip + i) = f32x4_t{0.f, 0.f, 0.f, 0.f};

  const char* a_src = uniform_ptr(g.A);
  const char* b_src = uniform_ptr(g.B);
  const uint32_t pitch_a = (uint32_t)(g.lda * 2), pitch_b = (uint32_t)(g.ldb * 2);
  const uint32_t b_lane = __umul24((uint32_t)(8 * kb), pitch_b) + (uint32_t)(n0 + CW * q) * 2u;
  const int ksteps = g.slab / 32;                   // items per block of a slab
  const int nsl = g.nseg > wv ? (g.nseg - wv + 3) >> 2 : 0;   // this wave's slabs: wv, wv + 4, ...

  for (int j0 = 0; j0 < nsl; j0 += SS_BATCH) {
    // ---- which rows of the strip does each slab of the batch list?  rowsel[j]: lane i < cnt[j]
    //      holds the i-th of them (ascending)
    int rowsel[SS_BATCH], cnt[SS_BATCH];
    int lo[SS_BATCH], hi[SS_BATCH], end[SS_BATCH];
    // one vector load brings the batch's list bounds: lane j the start of slab j's list, lane 8 + j its end
    // (slabs past the last: slab 0 stands in, so that nothing branches)
    const int pv = g.seg_ptr[(j0 + (lane & 7) < nsl ? wv + 4 * (j0 + (lane & 7)) : 0) + ((lane >> 3) & 1)];
#pragma unroll
    for (int j = 0; j < SS_BATCH; ++j) {
      const bool valid = j0 + j < nsl;                         // slabs past the end: empty
      lo[j] = valid ? __builtin_amdgcn_readlane(pv, j) : 0;
      end[j] = valid ? __builtin_amdgcn_readlane(pv, SS_BATCH + j) : 0;
      hi[j] = end[j];
    }
    // 64-ary search for p* = the first position whose entry is >= r0.  Invariant: lo <= p* <= hi, every
    // entry before lo is below r0, the entry at hi (if hi < end) is not.  All slabs of the batch advance
    // together, one round trip to memory per round.
    for (;;) {
      bool any_wide = false;
#pragma unroll
      for (int j = 0; j < SS_BATCH; ++j) any_wide |= hi[j] - lo[j] > 64;
      if (!any_wide) break;
      // every slab of the batch takes the round (it leaves a narrow range correct and no wider), so the code
      // is free of branches and the eight loads are in flight together; entry 0 exists because some list is wide
      int smp[SS_BATCH], step[SS_BATCH];
#pragma unroll
      for (int j = 0; j < SS_BATCH; ++j) {
        step[j] = (hi[j] - lo[j] + 63) / 64;
        const int pos = lo[j] + lane * step[j];
        const int v = g.idx[max(min(pos, hi[j] - 1), 0)];
        smp[j] = pos < hi[j] ? v : 0x7fffffff;
      }
#pragma unroll
      for (int j = 0; j < SS_BATCH; ++j) {
        const int c = __popcll(__ballot(smp[j] < r0));        // samples below the strip: a prefix
        const int hi_new = (c < 64 && lo[j] + c * step[j] < hi[j]) ? lo[j] + c * step[j] : hi[j];
        hi[j] = c == 0 ? lo[j] : hi_new;
        lo[j] = c == 0 ? lo[j] : lo[j] + (c - 1) * step[j] + 1;
      }
    }
    // the run of entries inside [r0, r0 + R) starts at most 64 positions after lo and is at most R <= 64 long
    int e0[SS_BATCH], e1[SS_BATCH];
#pragma unroll
    for (int j = 0; j < SS_BATCH; ++j) {
      const int p0 = lo[j] + lane, p1 = lo[j] + 64 + lane;
      e0[j] = p0 < end[j] ? g.idx[p0] : 0x7fffffff;
      e1[j] = p1 < end[j] ? g.idx[p1] : 0x7fffffff;
    }
#pragma unroll
    for (int j = 0; j < SS_BATCH; ++j) {
      const bool in0 = e0[j] >= r0 && e0[j] < r0 + SS_RM, in1 = e1[j] >= r0 && e1[j] < r0 + SS_RM;
      const unsigned long long b0 = __ballot(in0), b1 = __ballot(in1);
      const unsigned long long below = (1ull << lane) - 1ull;
      const int rank0 = __popcll(b0 & below), rank1 = __popcll(b0) + __popcll(b1 & below);
      // forward permutes: an in-range entry goes to the lane of its rank; the other lanes send a zero to a
      // lane that no entry of the same permute goes to (lane 63, which only a full first vector reaches, and
      // then every lane has an entry; for the second vector lane 0 when the ranks reach 63: the first vector
      // then holds rank 0, or the second is full)
      cnt[j] = __popcll(b0) + __popcll(b1);
      const int idle1 = cnt[j] == 64 ? 0 : 63;
      int got = 0;
      {
        const int a = __builtin_amdgcn_ds_permute((in0 ? rank0 : 63) * 4, in0 ? e0[j] + 1 : 0);
        const int b = __builtin_amdgcn_ds_permute((in1 ? rank1 : idle1) * 4, in1 ? e1[j] + 1 : 0);
        got = a | b;
      }
      rowsel[j] = got - 1;                              // -1 where no entry arrived
    }

    // ---- hand the row lists to the item loop through LDS (so that a slab can be picked at run time)
    uint32_t live = 0;
#pragma unroll
    for (int j = 0; j < SS_BATCH; ++j) {
      s_rows[wv][j][lane] = rowsel[j];
      live |= cnt[j] > 0 ? 1u << j : 0u;
    }
    if (live == 0) continue;

    // ---- one item = one 32-k step of one block (16 listed rows) of one live slab; the loads of item
    //      t + 1 are in flight while item t is computed.  (A later block of a slab reads the slab's
    //      rows of B again, from the L1 that the first block has just filled.)
    struct Item { uint32_t k0, a; int c[4]; int j, b, nblk, ks; };
    struct Regs { uint4 ra; BRow<CW> rb[8]; };
    auto setup = [&](int j, int b, Item& T) {
      const int* rs = s_rows[wv][j];
      const int first = rs[0];                                  // live slab: lane 0 holds a listed row
      const int r_a = rs[16 * b + q];
      T.j = j; T.b = b; T.ks = 0;
      T.nblk = (__popcll(__ballot(rs[lane] >= 0)) + 15) >> 4;   // blocks of 16 listed rows
      T.k0 = (uint32_t)((wv + 4 * (j0 + j)) * g.slab);
      T.a = __umul24((uint32_t)(r_a < 0 ? first : r_a), pitch_a) + 16u * (uint32_t)kb;   // unused block rows re-read a listed row
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int x = rs[16 * b + 4 * kb + e];
        // float offset of (row, q) in the strip; unused rows: the spare row
        T.c[e] = (((x < 0 ? SS_RM : x - r0) * (CW / 4)) * 16 + q) * 4;
      }
    };
    auto loads = [&](const Item& T, Regs& R) {
      const uint32_t k = T.k0 + 32u * (uint32_t)T.ks;
      R.ra = load16(a_src, T.a + 2u * k);
#pragma unroll
      for (int i = 0; i < 8; ++i) R.rb[i] = load_brow<CW>(b_src, b_lane + __umul24(k + (uint32_t)i, pitch_b));
    };
    f32x4_t acc[CW];
    // strip element (row, column CW q + x) lives at ((row * (CW / 4) + x / 4) * 16 + q) * 4 + x % 4: a lane
    // moves its columns of a row as 16-byte vectors, 16 lanes of a row side by side
    auto process = [&](const Item& T, const Regs& R) {
      if (T.ks == 0) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
          for (int h = 0; h < CW / 4; ++h) {
            const f32x4_t v = *reinterpret_cast<const f32x4_t*>(strip + T.c[e] + 64 * h);
#pragma unroll
            for (int x = 0; x < 4; ++x) acc[4 * h + x][e] = v[x];
          }
      }
#pragma unroll
      for (int x = 0; x < CW; ++x) acc[x] = mfma16<BF>(R.ra, bcolumn<CW>(R.rb, x), acc[x]);
      if (T.ks == ksteps - 1) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
          for (int h = 0; h < CW / 4; ++h)
            *reinterpret_cast<f32x4_t*>(strip + T.c[e] + 64 * h) =
                f32x4_t{acc[4 * h][e], acc[4 * h + 1][e], acc[4 * h + 2][e], acc[4 * h + 3][e]};
      }
    };
    // the item after T: the block's next k-step, else the slab's next block, else the next live slab.
    // After the last item the same item is named again: its loads are issued once more and dropped, so
    // that the loop holds no conditional load and every wait counts exactly the loads of the item after.
    auto copy_item = [&](const Item& T, Item& N) {
      N.k0 = T.k0; N.a = T.a; N.j = T.j; N.b = T.b; N.nblk = T.nblk; N.ks = T.ks;
#pragma unroll
      for (int e = 0; e < 4; ++e) N.c[e] = T.c[e];
    };
    auto advance = [&](const Item& T, Item& N) -> bool {
      if (T.ks + 1 < ksteps) { copy_item(T, N); N.ks = T.ks + 1; return true; }
      if (T.b + 1 < T.nblk) { setup(T.j, T.b + 1, N); return true; }
      if (live != 0) {
        const int j = __builtin_ctz(live);
        live &= live - 1;
        setup(j, 0, N);
        return true;
      }
      copy_item(T, N);
      return false;
    };
    Item T0, T1;
    Regs Ra, Rb;
    {
      const int j = __builtin_ctz(live);
      live &= live - 1;
      setup(j, 0, T0);
    }
    loads(T0, Ra);
    for (;;) {
      bool more = advance(T0, T1);
      loads(T1, Rb);
      process(T0, Ra);
      if (!more) break;
      more = advance(T1, T0);
      loads(T0, Ra);
      process(T1, Rb);
      if (!more) break;
    }
  }
  __syncthreads();
  // the four strips in a fixed order; thread (row, q) stores CW consecutive columns
  for (int i = tid; i < SS_RM * 16; i += 256) {
    const int row = i >> 4, qq = i & 15;
    if (r0 + row >= g.M) continue;
    float* d = reinterpret_cast<float*>(g.C) + (int64_t)(r0 + row) * g.ldc + n0 + CW * qq;
#pragma unroll
    for (int h = 0; h < CW / 4; ++h) {
      const int o = ((row * (CW / 4) + h) * 16 + qq) * 4;
      const f32x4_t v = ((*reinterpret_cast<const f32x4_t*>(&s_c[0][o]) + *reinterpret_cast<const f32x4_t*>(&s_c[1][o])) +
                         *reinterpret_cast<const f32x4_t*>(&s_c[2][o])) + *reinterpret_cast<const f32x4_t*>(&s_c[3][o]);
      *reinterpret_cast<float4*>(d + 4 * h) = make_float4(v[0], v[1], v[2], v[3]);
    }
  }
}

__global__ void __launch_bounds__(256) k_zero_rows(void* C, int64_t ld_bytes, int M, int64_t row_bytes) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= M) return;
  char* p = reinterpret_cast<char*>(C) + (int64_t)row * ld_bytes;
  for (int64_t b = (int64_t)(threadIdx.x & 63) * 16; b < row_bytes; b += 64 * 16)
    *reinterpret_cast<uint4*>(p + b) = make_uint4(0, 0, 0, 0);
}



}  // namespace

// compute units of the current device rounded down to a multiple of 8 (one share per XCD)
static int compute_units() {
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 256;
  if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 8) n = 256;
  return n & ~7;
}

template <bool BF, int CT>
static int launch_gather_k(const GemmArgs& g, int tm_tiles, hipStream_t st) {
  // one workgroup of the 128-row tile fits on a compute unit: with more tiles than compute units the workgroups loop
  const int total = (int)(g.N / TN) * tm_tiles, cus = compute_units();
  if (g.slab == 64 || g.slab == 32) {
    // lower tiles: two-wave workgroups; as many as the registers let a compute unit hold (64 rows: two,
    // 32 rows: four, i.e. two waves per SIMD)
    const int resident = (g.slab == 64 ? 2 : 4) * cus;
    const unsigned wgs = (unsigned)(total <= resident ? total : resident);
    if (g.slab == 64) hipLaunchKernelGGL((k_gather_k_direct<BF, CT, 2, 4>), dim3(wgs), dim3(128), 0, st, g, tm_tiles);
    else              hipLaunchKernelGGL((k_gather_k_direct<BF, CT, 2, 2>), dim3(wgs), dim3(128), 0, st, g, tm_tiles);
  } else if (total >= 2 * cus) {      // two workgroups of two waves per compute unit
    hipLaunchKernelGGL((k_gather_k_direct<BF, CT, 2, 8>), dim3((unsigned)(2 * cus)), dim3(128), 0, st, g, tm_tiles);
  } else {
    const unsigned wgs = (unsigned)(total <= cus ? total : cus);
    hipLaunchKernelGGL((k_gather_k_direct<BF, CT, 4, 8>), dim3(wgs), dim3(256), 0, st, g, tm_tiles);
  }
  PIT_LAUNCH_CHECK();
  return PIT_OK;
}

// GATHER_K: tm_tiles = number of row tiles = segments of the index
static int launch_sread_gemm_k(bool bf, int c_is_in_type, const GemmArgs& g, int tm_tiles, hipStream_t st) {
  if (tm_tiles <= 0 || g.N <= 0) return PIT_OK;
  // the kernel addresses each operand with 32-bit byte offsets from a uniform base and multiplies row
  // numbers by the row pitch in 24 bits
  if (g.lda * 2 >= (1ll << 24) || g.ldb * 2 >= (1ll << 24) || (int64_t)g.K >= (1ll << 24)) return PIT_ESHAPE;
  if ((int64_t)g.K * g.lda * 2 >= (1ll << 32) || (int64_t)g.K * g.ldb * 2 >= (1ll << 32)) return PIT_ESHAPE;
  if (bf) return c_is_in_type ? launch_gather_k<true, 1>(g, tm_tiles, st) : launch_gather_k<true, 0>(g, tm_tiles, st);
  return c_is_in_type ? launch_gather_k<false, 1>(g, tm_tiles, st) : launch_gather_k<false, 0>(g, tm_tiles, st);
}

int launch_zero_rows(void* C, int64_t ld_bytes, int M, int64_t row_bytes, hipStream_t st) {
  if (M <= 0 || row_bytes <= 0) return PIT_OK;
  hipLaunchKernelGGL(k_zero_rows, dim3((unsigned)ceil_div(M, 4)), dim3(256), 0, st, C, ld_bytes, M, row_bytes);
  PIT_LAUNCH_CHECK();
  return PIT_OK;
}

}  // namespace pit

using namespace pit;

extern "C" int pit_sread_gemm(int mode, const void* d_A, int64_t lda, const void* d_B, int64_t ldb,
                              void* d_C, int64_t ldc, int M, int N, int K, int in_dt, int c_dt,
                              const pit_index* ix, int mt, int zero_uncovered, pit_stream stream) {
  if (mode != PIT_GEMM_GATHER_M && mode != PIT_GEMM_GATHER_K && mode != PIT_GEMM_DENSE_K) return PIT_EINVAL;
  if (mode != PIT_GEMM_DENSE_K && (!ix || !ix->seg_ptr)) return PIT_EINVAL;
  if (in_dt != PIT_BF16 && in_dt != PIT_F16) return PIT_EINVAL;
  if (c_dt != PIT_F32 && c_dt != in_dt) return PIT_EINVAL;
  if (M < 0 || N < 0 || K < 0 || mt <= 0) return PIT_ESHAPE;
  if (N % TN) return PIT_ESHAPE;
  const int c_esize = c_dt == PIT_F32 ? 4 : 2;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  if (M == 0 || N == 0) return PIT_OK;
  if (!d_C || !aligned(d_C, 16) || ldc < N || (ldc * c_esize) % 16) return PIT_EINVAL;
  if (K > 0) {
    if (!d_A || !d_B || (mode != PIT_GEMM_DENSE_K && !ix->idx)) return PIT_EINVAL;
    if (!aligned(d_A, 16) || !aligned(d_B, 16) || lda % 8 || ldb % 8 || ldb < N) return PIT_EINVAL;
  }

  GemmArgs g = {};
  g.A = d_A; g.lda = lda; g.B = d_B; g.ldb = ldb; g.b_seg_stride = 0;
  g.C = d_C; g.ldc = ldc; g.gate = nullptr;
  g.M = M; g.N = N; g.K = K;
  if (mode == PIT_GEMM_DENSE_K) {
    // the dense kernel of Algorithm 1's fallback: the GATHER_K tile with identity addressing
    if ((mt != 128 && mt != 64 && mt != 32) || M % mt) return PIT_ESHAPE;
    if (K > 0 && lda < M) return PIT_EINVAL;
    g.seg_ptr = nullptr; g.idx = nullptr; g.nseg = M / mt; g.slab = mt;
    return launch_sread_gemm_k(in_dt == PIT_BF16, c_dt != PIT_F32, g, M / mt, st);
  }
  g.seg_ptr = ix->seg_ptr; g.idx = ix->idx; g.nseg = ix->nseg;

  if (mode == PIT_GEMM_GATHER_K) {
    if ((mt != 128 && mt != 64 && mt != 32) || M % mt) return PIT_ESHAPE;
    if (ix->nseg != M / mt) return PIT_ECAPACITY;
    if (K > 0 && lda < M) return PIT_EINVAL;
    g.slab = mt;       // GATHER_K: the tile height (= micro-tile height of the index)
    return launch_sread_gemm_k(in_dt == PIT_BF16, c_dt != PIT_F32, g, ix->nseg, st);
  }

  // GATHER_M
  if (K == 0) {  // empty product: C is zero wherever the call is asked to define it
    if (zero_uncovered || ix->nseg > 1) {
      return launch_zero_rows(d_C, ldc * c_esize, M, (int64_t)N * c_esize, st);
    }
    return PIT_OK;
  }
  if (mt % 32 || K % mt) return PIT_ESHAPE;
  if (ix->nseg != K / mt) return PIT_ECAPACITY;
  if (lda < K) return PIT_EINVAL;
  g.slab = mt; g.a_gather = 1; g.c_scatter = 1; g.slab_per_seg = 1;
  if (ix->nseg == 1) {
    // (rows the list does not name are cleared inside the product's launch, by its workgroups without a tile)
    g.zero_rest = zero_uncovered ? 1 : 0;
    return launch_gather_m(in_dt == PIT_BF16, EPI_STORE, c_dt != PIT_F32, g, M, st);
  }
  if (c_dt != PIT_F32) return PIT_EINVAL;
  // several k-slabs per row: C-stationary strips (every element of C is written, nothing to clear)
  if (g.lda * 2 >= (1ll << 24) || g.ldb * 2 >= (1ll << 24) || (int64_t)M >= (1ll << 24) || (int64_t)K >= (1ll << 24)) return PIT_ESHAPE;
  if ((int64_t)M * g.lda * 2 >= (1ll << 32) || (int64_t)K * g.ldb * 2 >= (1ll << 32)) return PIT_ESHAPE;
  // 32 x 128 strips.  (64 x 64 strips, CW = 4, halve the traffic of B and double that of A: measured 10-15 %
  // faster at 90-95 % sparsity of a 4096^3 product, 10-20 % slower at 50 % and at 99 %.)
  constexpr int CW = 8;
  const int64_t strips = ceil_div(M, StripShape<CW>::R);
  if (strips > 65535 || N % StripShape<CW>::W) return PIT_ESHAPE;
  dim3 grid((unsigned)(N / StripShape<CW>::W), (unsigned)strips);
  if (in_dt == PIT_BF16) hipLaunchKernelGGL((k_slab_strip<true, CW>), grid, dim3(256), 0, st, g);
  else                   hipLaunchKernelGGL((k_slab_strip<false, CW>), grid, dim3(256), 0, st, g);
  PIT_LAUNCH_CHECK();
  return PIT_OK;
}

// ------------------------------------------------------------------------------------------------
// Algorithm 1 end to end: select among the GATHER_K tile heights and the dense kernel, then run the winner.
// ------------------------------------------------------------------------------------------------
namespace pit {
namespace {
struct SelectWs { size_t seg_ptr_off, idx_off, build_off, total; };
// sized for the finest micro-tile (32): the most segments and the most entries
SelectWs select_layout(int M, int K) {
  SelectWs w;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o += (bytes + 255) & ~(size_t)255; return at; };
  const size_t nseg = (size_t)(M > 0 ? M : 0) / 32 + 1;
  w.seg_ptr_off = take((nseg + 1) * 4);
  w.idx_off = take((nseg * (size_t)(K > 0 ? K : 1)) * 4);
  size_t b = 0;
  for (int mt : {32, 64, 128}) b = std::max(b, pit_build_index_workspace(K, M - M % mt, 1, mt, 0, 0));
  w.build_off = take(b + 64);
  w.total = o;
  return w;
}
}  // namespace
}  // namespace pit

extern "C" size_t pit_select_and_run_gemm_workspace(int M, int K) {
  if (M < 0 || K < 0) return 0;
  return select_layout(M, K).total;
}

extern "C" int pit_select_and_run_gemm(const pit_kernel_candidate* cand, int ncand, const int64_t* num_tiles,
                                       const int64_t* grid_tiles, int nsamples,
                                       const void* d_At, int64_t lda, const void* d_B, int64_t ldb,
                                       void* d_C, int64_t ldc, int M, int N, int K, int in_dt, int c_dt,
                                       void* d_ws, size_t ws_bytes, int* chosen, pit_stream stream) {
  if (!cand || ncand <= 0) return PIT_EINVAL;
  for (int j = 0; j < ncand; ++j) {
    const int mt = cand[j].mt_cols;
    if (cand[j].mt_rows != 1 || (mt != 32 && mt != 64 && mt != 128)) return PIT_ESHAPE;
  }
  int best = 0;
  const int rc = pit_select_kernel(cand, ncand, num_tiles, grid_tiles, nsamples, nullptr, &best);
  if (rc != PIT_OK) return rc;
  if (chosen) *chosen = best;
  const int mt = cand[best].mt_cols;
  if (M < 0 || N < 0 || K < 0) return PIT_ESHAPE;
  if (M % mt) return PIT_ESHAPE;
  if (cand[best].dense)
    return pit_sread_gemm(PIT_GEMM_DENSE_K, d_At, lda, d_B, ldb, d_C, ldc, M, N, K, in_dt, c_dt, nullptr, mt, 0, stream);
  const SelectWs L = select_layout(M, K);
  if (!d_ws || !aligned(d_ws, 256)) return PIT_EINVAL;
  if (ws_bytes < L.total) return PIT_ECAPACITY;
  char* ws = reinterpret_cast<char*>(d_ws);
  pit_index ix;
  ix.seg_ptr = reinterpret_cast<int32_t*>(ws + L.seg_ptr_off);
  ix.idx = reinterpret_cast<int32_t*>(ws + L.idx_off);
  ix.bits = nullptr;
  ix.nseg = M / mt;
  ix.cap = (int32_t)std::min<int64_t>((int64_t)(M / mt) * K, INT32_MAX);
  if ((int64_t)(M / mt) * K > INT32_MAX) return PIT_ESHAPE;
  const int rb = pit_build_index(d_At, in_dt, K, M, lda, 1, mt, 0, &ix, ws + L.build_off, L.total - L.build_off, stream);
  if (rb != PIT_OK) return rb;
  return pit_sread_gemm(PIT_GEMM_GATHER_K, d_At, lda, d_B, ldb, d_C, ldc, M, N, K, in_dt, c_dt, &ix, mt, 0, stream);
}
