// pit_sread_gemm: the SRead -> dense MFMA tile -> SWrite kernel (paper Section 3.1, sparse kernel
// template) for gfx950, and its host-side validation and launch.
//
// One workgroup (256 threads = 4 wavefronts, 2 x 2) computes a 128 x 128 dense tile of C with
// v_mfma_f32_32x32x16 (bf16 or f16 inputs, fp32 accumulation), 64 k per step.
//
// SRead.  Two gathers, one per PIT-axis of MatMul (paper Table 1):
//   GATHER_K  A is K-major (At[k][m]); the tile's k-list comes from the index; a step loads the 64
//             listed rows of At (128 m = 256 B each) and the SAME rows of B.
//   GATHER_M  A is K-minor (A[m][k]); the tile's 128 row numbers come from the index once, the
//             k loop walks a contiguous k range; B rows are contiguous.
// Every operand tile is K-MINOR in LDS ([128 x][64 k], 128 B per row) and is read with
// ds_read_b128.  K-major sources (rows of At and of B) are transposed in registers on the way in:
// a thread loads an 8 k x 8 column block (8 x 16 B, one source row each), interleaves the 16-bit
// elements with v_perm_b32 and writes 8 tile rows of 16 B.
//
// Pipeline.  Global loads run D steps ahead in a register ring.  The steady-state loop is
// branch-free: all loads are unconditional (positions past the end of a list are clamped to its
// last entry and zeroed on the way into LDS, in the last step only).  Inside a step the LDS reads
// of k-substep s+1, the transposes and the LDS writes of the next tile are interleaved with the
// MFMAs of k-substep s, so the LDS pipe and the matrix pipe work at the same time although there
// is a single wavefront per SIMD.
// GATHER_K keeps a sliding window of the k-list in LDS (16 steps x 64 entries).  Every 4th step each
// thread fetches one entry 12 steps ahead and stores it 3 steps later, so no load in the loop
// depends on a load issued less than 3 steps before it.
//
// SWrite.  The epilogue stores accumulator rows to the row numbers held in LDS (identity or the
// index), optionally through fp32 atomics (several k-slabs accumulate into one C), a GELU + round
// to the input type (first MoE matmul) or a per-row gate (second MoE matmul).
#include "pit_gemm.hpp"
#include <cstdlib>

namespace pit {
namespace {

__device__ __forceinline__ void lds_write_b128(uint32_t addr, const uint4& v) {
  *(PIT_LDS u32x4_t*)(uintptr_t)addr = __builtin_bit_cast(u32x4_t, v);
}
__device__ __forceinline__ u32x4_t lds_read_frag(uint32_t addr) {
  return *(PIT_LDS u32x4_t*)(uintptr_t)addr;
}
template <bool BF>
__device__ __forceinline__ f32x16_t mfma32(const u32x4_t& a, const u32x4_t& b, const f32x16_t& c) {
  if constexpr (BF)
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __builtin_bit_cast(uint32_t, f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0;
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ uint16_t f32_to_f16_rne(float f) {
  return __builtin_bit_cast(uint16_t, (_Float16)f);
}
template <bool BF> __device__ __forceinline__ uint16_t f32_to_in(float f) {
  return BF ? f32_to_bf16_rne(f) : f32_to_f16_rne(f);
}
__device__ __forceinline__ float gelu_erf(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752f)); }

// Global loads are laid out so that 16 consecutive lanes read 256 contiguous bytes of one source
// row (the address unit merges 4 neighbouring lanes into one 64-byte request; lanes that jump
// between rows cost one request each, four times the address-unit time).
//
// LDS address of 16-byte chunk c (8 k) of tile row m, with a = m >> 4, h = (m >> 3) & 1, l = m & 7:
//   256-byte bank row = a * 8 + l,   128-byte half = h,   16-byte slot inside the half = c ^ l ^ a
// The LDS serves 16 lanes per clock and conflicts are decided by the position inside the
// 256-byte bank row.  All three access shapes put 16 lanes on 16 different positions:
//   operand read        16 consecutive rows (a fixed; h, l vary), one chunk
//   transposing write   rows 8*cg + x for 16 consecutive cg (l = x fixed; a, h vary), one chunk
//   straight write      rows m and m + 8 (h differs), all 8 chunks each
// (measured: XOR rotations keep ds_read_b128 at its full rate, additive rotations cost ~35 %)
__device__ __forceinline__ uint32_t tile_off(int m, int c) {
  const int a = m >> 4, h = (m >> 3) & 1, l = m & 7;
  return (uint32_t)((((a << 3) | l) << 8) | (h << 7) | (((c ^ l ^ a) & 7) << 4));
}

// One output row of the 8 x 8 transpose below: out_x = 8 consecutive k of column x (4 v_perm_b32).
__device__ __forceinline__ uint4 transpose8x8_row(const uint4 (&r)[8], int x) {
  const int i = x >> 1;
  const uint32_t sel = (x & 1) ? 0x07060302u : 0x05040100u;
  uint32_t d[4];
#pragma unroll
  for (int jj = 0; jj < 4; ++jj) {
    const uint32_t a = i == 0 ? r[2 * jj].x : i == 1 ? r[2 * jj].y : i == 2 ? r[2 * jj].z : r[2 * jj].w;
    const uint32_t b = i == 0 ? r[2 * jj + 1].x : i == 1 ? r[2 * jj + 1].y : i == 2 ? r[2 * jj + 1].z : r[2 * jj + 1].w;
    d[jj] = __builtin_amdgcn_perm(b, a, sel);
  }
  return make_uint4(d[0], d[1], d[2], d[3]);
}

// r[j] = 8 consecutive columns of k-row j (16-bit elements); out[x] = 8 consecutive k of column x
__device__ __forceinline__ void transpose8x8_b16(const uint4 (&r)[8], uint4 (&out)[8]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    uint32_t lo[4], hi[4];
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      const uint32_t a = i == 0 ? r[2 * jj].x : i == 1 ? r[2 * jj].y : i == 2 ? r[2 * jj].z : r[2 * jj].w;
      const uint32_t b = i == 0 ? r[2 * jj + 1].x : i == 1 ? r[2 * jj + 1].y : i == 2 ? r[2 * jj + 1].z : r[2 * jj + 1].w;
      lo[jj] = __builtin_amdgcn_perm(b, a, 0x05040100u);
      hi[jj] = __builtin_amdgcn_perm(b, a, 0x07060302u);
    }
    out[2 * i] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
    out[2 * i + 1] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
  }
}

__device__ __forceinline__ const char* uniform_ptr(const void* p) {
  const uint64_t v = reinterpret_cast<uint64_t>(p);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return reinterpret_cast<const char*>(((uint64_t)hi << 32) | lo);
}
// 16-byte load from global memory at a wave-uniform base plus a 32-bit per-lane byte offset.  The
// explicit global address space keeps the access a global_load (a flat load would tie up both
// memory counters and force full waits).
__device__ __forceinline__ uint4 load16(const char* base, uint32_t byte_off) {
  typedef const u32x4_t __attribute__((address_space(1))) * gptr_t;
  const u32x4_t v = *(gptr_t)(uintptr_t)(reinterpret_cast<uintptr_t>(base) + byte_off);
  return __builtin_bit_cast(uint4, v);
}

// nothing may be scheduled across this point
#define PIT_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

// GK = true: GATHER_K (A K-major), false: GATHER_M (A K-minor).  CT: 0 = fp32 C, 1 = C in the input type.
// D: depth of the register ring of global loads (2 or 4 steps).
template <bool BF, bool GK, int EPI, int CT, int D>
__global__ void __launch_bounds__(256)
k_sread_gemm(const GemmArgs g) {
  static_assert(D == 2 || D == 4, "ring depth must divide the unroll factor 4");
  __shared__ __attribute__((aligned(1024))) char smem[2 * STAGE_BYTES];
  __shared__ int s_rows_a[TM];   // GATHER_M: source row of A per tile row
  __shared__ int s_rows_c[TM];   // destination row of C per tile row (-1 = skip)
  constexpr int KRING = 16 * TK;
  __shared__ __attribute__((aligned(32))) int s_kidx[GK ? KRING : 4];
  const uint32_t lds0 = (uint32_t)(uintptr_t)(PIT_LDS char*)smem;
  const uint32_t kring = (uint32_t)(uintptr_t)(PIT_LDS char*)s_kidx;

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int wm = wv >> 1, wn = wv & 1;

  // ---------------------------------------------------------------- which tile is this workgroup?
  int tile_row, tile_col;
  if constexpr (GK) {
    // XCD-aware tile order.  Workgroups are handed to the 8 XCDs round-robin by linear id, and
    // each XCD has its own L2.  Renumber so that the workgroups of one XCD are consecutive, then
    // walk the tile grid in bands of 4 row tiles (row-fastest inside a band): an XCD's workgroups
    // then cover a compact block of tiles and share their A and B panels through that L2.
    const int tn = gridDim.x, tm = gridDim.y, total = tn * tm;
    const int lin = blockIdx.x + tn * blockIdx.y;
    const int x = lin & 7, q = total >> 3, r = total & 7;
    const int lp = x * q + min(x, r) + (lin >> 3);
    constexpr int GM = 4;
    const int band = lp / (GM * tn), within = lp - band * (GM * tn);
    const int rows = min(GM, tm - band * GM);
    tile_row = band * GM + within % rows;
    tile_col = within / rows;
  } else {
    tile_row = blockIdx.y;
    tile_col = blockIdx.x;
  }
  const int n0 = tile_col * TN;

  int seg, list_begin, list_len;   // GATHER_K: the k-list; GATHER_M: the row-list slice of this tile
  int k_begin = 0, k_len = 0;      // GATHER_M: contiguous k range
  if constexpr (GK) {
    seg = tile_row;
    list_begin = g.seg_ptr[seg];
    list_len = g.seg_ptr[seg + 1] - list_begin;
  } else {
    // linear row-tile number -> (segment, tile inside segment); every wave does the same search
    const int tile = tile_row;
    int acc = 0;
    seg = -1;
    int tile_in_seg = 0;
    for (int s0 = 0; s0 < g.nseg; s0 += 64) {
      const int s = s0 + lane;
      int cnt = 0;
      if (s < g.nseg) cnt = g.seg_ptr[s + 1] - g.seg_ptr[s];
      const int nt = (cnt + TM - 1) / TM;
      int inc = nt;
#pragma unroll
      for (int d = 1; d < 64; d <<= 1) {
        const int t = __shfl_up(inc, d);
        if (lane >= d) inc += t;
      }
      const int total = __shfl(inc, 63);
      if (tile < acc + total) {
        const unsigned long long hit = __ballot(acc + inc > tile);
        const int l = __builtin_ctzll(hit);
        seg = s0 + l;
        tile_in_seg = tile - (acc + __shfl(inc, l) - __shfl(nt, l));
        break;
      }
      acc += total;
    }
    if (seg < 0) return;
    const int sb = g.seg_ptr[seg];
    const int cnt = g.seg_ptr[seg + 1] - sb;
    list_begin = sb + tile_in_seg * TM;
    list_len = min(TM, cnt - tile_in_seg * TM);
    k_begin = g.slab_per_seg ? seg * g.slab : 0;
    k_len = g.slab;
    if (tid < TM) {
      // rows past the end of the list read the list's last row (a valid address); their results
      // are never stored
      const int v = g.idx[list_begin + min(tid, list_len - 1)];
      s_rows_a[tid] = g.a_gather ? v : list_begin + min(tid, list_len - 1);
      s_rows_c[tid] = tid < list_len ? (g.c_scatter ? v : list_begin + tid) : -1;
    }
    __syncthreads();
  }
  seg = __builtin_amdgcn_readfirstlane(seg);
  list_begin = __builtin_amdgcn_readfirstlane(list_begin);
  list_len = __builtin_amdgcn_readfirstlane(list_len);

  f32x16_t acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int len = GK ? list_len : k_len;          // extent of the k loop (list entries or slab width)
  const int nsteps = (len + TK - 1) / TK;
  const int tail = len % TK;                       // != 0: the last step is partial

  // ---- loader roles: threads 0..127 fill the A tile, threads 128..255 the B tile (wave-uniform)
  const bool is_b = __builtin_amdgcn_readfirstlane(tid >> 7) != 0;
  const int u = tid & 127;
  const int t_cg = u & 15, t_kg = u >> 4;                               // transposing role: 8 k x 8 columns
  const int s_chunk = u & 7, s_row = (((u >> 3) & 1) << 3) | (u >> 4);  // straight role (GATHER_M, A): rows r, r+8 per 16 lanes
  const bool transposing = GK || is_b;

  const char* a_bytes = reinterpret_cast<const char*>(g.A);
  const char* b_bytes = reinterpret_cast<const char*>(g.B) + (int64_t)seg * g.b_seg_stride * 2;
  const char* src = uniform_ptr(is_b ? b_bytes : a_bytes);
  const uint32_t pitch = (uint32_t)((is_b ? g.ldb : g.lda) * 2);   // bytes per source row (< 2^24, checked on the host)
  // transposing role: byte offset of this thread's 8 columns inside a source row
  const uint32_t col_bytes = (uint32_t)(((GK && !is_b) ? seg * TM : n0) + t_cg * 8) * 2u;

  uint32_t a_off[8];   // straight role: byte offset of (row of round j, this thread's chunk) at k step 0
  if constexpr (!GK) {
#pragma unroll
    for (int j = 0; j < 8; ++j) a_off[j] = __umul24((uint32_t)s_rows_a[j * 16 + s_row], pitch) + (uint32_t)(k_begin + s_chunk * 8) * 2u;
  }

  // LDS write offsets (8 per thread) and read offsets (32-row block i of this wave, k-substep ks)
  uint32_t w_off[8];
#pragma unroll
  for (int x = 0; x < 8; ++x) w_off[x] = (transposing ? tile_off(t_cg * 8 + x, t_kg) : tile_off(x * 16 + s_row, s_chunk)) + (is_b ? (uint32_t)A_TILE_BYTES : 0u);
  uint32_t rd_a[2][4], rd_b[2][4];
  {
    const int m = lane & 31, hi = lane >> 5;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        rd_a[i][ks] = tile_off(wm * 64 + i * 32 + m, hi + 2 * ks);
        rd_b[i][ks] = tile_off(wn * 64 + i * 32 + m, hi + 2 * ks) + (uint32_t)A_TILE_BYTES;
      }
  }

  uint4 R[D][8];
  int k_use[8], k_pend[8];   // GATHER_K: list values for the step being issued / the one after
  int k_ahead = 0;           // GATHER_K: one list entry on its way from global memory to the LDS window

  auto list_at = [&](int pos) { return g.idx[list_begin + min(pos, list_len - 1)]; };
  auto load_kid = [&](int step, int (&dst)[8]) {
    const uint32_t a = kring + (uint32_t)((((step & 15) << 6) + t_kg * 8) * 4);
    const u32x4_t lo = *(PIT_LDS u32x4_t*)(uintptr_t)a;
    const u32x4_t hi = *(PIT_LDS u32x4_t*)(uintptr_t)(a + 16);
    dst[0] = lo.x; dst[1] = lo.y; dst[2] = lo.z; dst[3] = lo.w;
    dst[4] = hi.x; dst[5] = hi.y; dst[6] = hi.z; dst[7] = hi.w;
  };
  auto issue = [&](int step, uint4 (&r)[8]) {
    if constexpr (GK) {
#pragma unroll
      for (int j = 0; j < 8; ++j) r[j] = load16(src, __umul24((uint32_t)k_use[j], pitch) + col_bytes);
    } else {
      if (is_b) {
        const int base = k_begin + min(step * TK + t_kg * 8, k_len - 8);
#pragma unroll
        for (int j = 0; j < 8; ++j) r[j] = load16(src, __umul24((uint32_t)(base + j), pitch) + col_bytes);
      } else {
        // byte distance from this thread's chunk at step 0; a chunk past the slab end re-reads the last one
        const uint32_t kofs = (uint32_t)((min(step * TK + s_chunk * 8, k_len - 8) - s_chunk * 8) * 2);
#pragma unroll
        for (int j = 0; j < 8; ++j) r[j] = load16(src, a_off[j] + kofs);
      }
    }
  };
  // byte offsets of the 8 loads of `step` (same addresses as issue())
  auto issue_offsets = [&](int step, uint32_t (&off)[8]) {
    if constexpr (GK) {
#pragma unroll
      for (int j = 0; j < 8; ++j) off[j] = __umul24((uint32_t)k_use[j], pitch) + col_bytes;
    } else {
      if (is_b) {
        const int base = k_begin + min(step * TK + t_kg * 8, k_len - 8);
#pragma unroll
        for (int j = 0; j < 8; ++j) off[j] = __umul24((uint32_t)(base + j), pitch) + col_bytes;
      } else {
        const uint32_t kofs = (uint32_t)((min(step * TK + s_chunk * 8, k_len - 8) - s_chunk * 8) * 2);
#pragma unroll
        for (int j = 0; j < 8; ++j) off[j] = a_off[j] + kofs;
      }
    }
  };
  // zero what lies past the end of the k extent (last, partial step only)
  auto zero_tail = [&](int step, uint4 (&r)[8]) {
    if (transposing) {
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (step * TK + t_kg * 8 + j >= len) r[j] = make_uint4(0, 0, 0, 0);
    } else if (step * TK + s_chunk * 8 >= len) {
#pragma unroll
      for (int j = 0; j < 8; ++j) r[j] = make_uint4(0, 0, 0, 0);
    }
  };
  // the 8 x 16 B this thread will write to LDS for `step`: transposed (or straight) and, in the
  // last partial step, with everything past the end of the k extent zeroed
  auto prepare = [&](int step, uint4 (&r)[8], uint4 (&o)[8], bool may_be_last) {
    if (may_be_last && tail != 0 && step == nsteps - 1) zero_tail(step, r);
    if (transposing) {
      transpose8x8_b16(r, o);
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) o[j] = r[j];
    }
  };
  auto read_frags = [&](uint32_t t, int ks, u32x4_t (&af)[2], u32x4_t (&bf)[2]) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      af[i] = lds_read_frag(t + rd_a[i][ks]);
      bf[i] = lds_read_frag(t + rd_b[i][ks]);
    }
  };
  auto mfma4 = [&](const u32x4_t (&af)[2], const u32x4_t (&bf)[2]) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) acc[i][j] = mfma32<BF>(af[i], bf[j], acc[i][j]);
  };
  // One step.  MFMAs of `step` read LDS buffer `buf`; the tile of step + 1, already transposed in
  // the registers o[], goes to the other buffer; the tile of step + 2 is taken out of ring slot r
  // and transposed into o[]; the loads of step + 1 + D refill ring slot rl (the one emptied by the
  // previous step).  A wavefront issues in order and an MFMA keeps the matrix pipe busy for 32
  // clocks, so everything else is placed BETWEEN consecutive MFMAs, about 30 clocks' worth each:
  //   MFMA 0..7    one LDS read (operands of the next k-substep), one LDS write, one global load
  //   MFMA 8..11   one LDS read, a quarter of the transpose (4 v_perm_b32) ... MFMA 12..15 likewise
  // `steady` = compile-time true in the branch-free loop (all parts on, order pinned).
  auto body = [&](int step, int buf, uint4 (&o)[8], uint4 (&r)[8], uint4 (&rl)[8],
                  bool do_write, bool do_prep, bool do_issue, bool steady) {
    const uint32_t t = lds0 + buf * STAGE_BYTES, tw = lds0 + (buf ^ 1) * STAGE_BYTES;
    u32x4_t fa[2][2], fb[2][2];
    read_frags(t, 0, fa[0], fb[0]);
    if (!steady && do_prep && tail != 0 && step + 2 == nsteps - 1) zero_tail(step + 2, r);
    uint32_t goff[8];
    if (do_issue) issue_offsets(step + 1 + D, goff);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int ks = i >> 2, q = i & 3;
      acc[q >> 1][q & 1] = mfma32<BF>(fa[ks & 1][q >> 1], fb[ks & 1][q & 1], acc[q >> 1][q & 1]);
      if (i < 12) {   // operands of k-substep ks + 1: A block 0, B block 0, A block 1, B block 1
        const int nb = (ks + 1) & 1;
        if (q == 0) fa[nb][0] = lds_read_frag(t + rd_a[0][ks + 1]);
        if (q == 1) fb[nb][0] = lds_read_frag(t + rd_b[0][ks + 1]);
        if (q == 2) fa[nb][1] = lds_read_frag(t + rd_a[1][ks + 1]);
        if (q == 3) fb[nb][1] = lds_read_frag(t + rd_b[1][ks + 1]);
      }
      if (i < 8) {
        if (do_write) lds_write_b128(tw + w_off[i], o[i]);
        if (do_issue) rl[i] = load16(src, goff[i]);
      } else if (do_prep) {
        o[i - 8] = transposing ? transpose8x8_row(r, i - 8) : r[i - 8];
      }
      if (steady) PIT_SCHED_FENCE();   // keep the slots in this order (the scheduler would cluster the MFMAs)
    }
    PIT_SCHED_FENCE();
    __syncthreads();
  };

  if (nsteps > 0) {
    if constexpr (GK) {
      // list window for steps 0..15
      int v[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) v[q] = list_at(q * 256 + tid);
#pragma unroll
      for (int q = 0; q < 4; ++q) s_kidx[q * 256 + tid] = v[q];
      __syncthreads();
    }
    // prologue: loads of tiles 0 .. D; tile 0 into LDS, tile 1 transposed into o[].  Tile t >= 2
    // travels through ring slot (t - 2) % D; slot D-1 is filled by step 0.
    uint4 o[8], r0[8], r1[8];
    if constexpr (GK) load_kid(0, k_use);
    issue(0, r0);
    if constexpr (GK) load_kid(min(1, nsteps - 1), k_use);
    issue(min(1, nsteps - 1), r1);
#pragma unroll
    for (int s = 0; s + 1 < D; ++s) {
      if constexpr (GK) load_kid(min(2 + s, nsteps - 1), k_use);
      issue(min(2 + s, nsteps - 1), R[s]);
    }
    if constexpr (GK) {
      load_kid(min(1 + D, nsteps - 1), k_use);
      load_kid(min(2 + D, nsteps - 1), k_pend);
    }
    prepare(0, r0, o, true);
#pragma unroll
    for (int x = 0; x < 8; ++x) lds_write_b128(lds0 + w_off[x], o[x]);
    if (nsteps > 1) prepare(1, r1, o, true);
    __syncthreads();

    int it = 0;
    // steady state, 4 steps per trip: every step here has step + 2 + D < nsteps; no conditionals
    // around memory operations
    for (; it + 5 + D < nsteps; it += 4) {
#pragma unroll
      for (int uu = 0; uu < 4; ++uu) {
        const int step = it + uu;
        body(step, uu & 1, o, R[uu % D], R[(uu + D - 1) % D], true, true, true, true);
        if constexpr (GK) {
          // list entries for the loads of the next step, and the sliding window's refill
#pragma unroll
          for (int j = 0; j < 8; ++j) k_use[j] = k_pend[j];
          load_kid(min(step + 3 + D, nsteps - 1), k_pend);
          if (uu == 0) k_ahead = list_at((step + 12) * TK + tid);
          if (uu == 3) s_kidx[((step + 9) * TK + tid) & (KRING - 1)] = k_ahead;   // entries of steps it+12 .. it+15
        }
      }
    }
    // drain
    for (; it < nsteps; it += 4) {
#pragma unroll
      for (int uu = 0; uu < 4; ++uu) {
        const int step = it + uu;
        if (step >= nsteps) break;
        body(step, uu & 1, o, R[uu % D], R[(uu + D - 1) % D], step + 1 < nsteps, step + 2 < nsteps, step + 1 + D < nsteps, false);
        if constexpr (GK) {
#pragma unroll
          for (int j = 0; j < 8; ++j) k_use[j] = k_pend[j];
          load_kid(min(step + 3 + D, nsteps - 1), k_pend);
        }
      }
    }
  }

  // ---------------------------------------------------------------- SWrite
  const int m_base = GK ? seg * TM : 0;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int r = wm * 64 + i * 32 + 8 * (e >> 2) + (lane >> 5) * 4 + (e & 3);
      int64_t crow;
      if constexpr (GK) crow = m_base + r;
      else              crow = s_rows_c[r];
      if (crow < 0) continue;
      float scale = 1.f;
      if constexpr (!GK && EPI == EPI_STORE) { if (g.gate) scale = g.gate[crow]; }
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int col = n0 + wn * 64 + j * 32 + (lane & 31);
        float v = acc[i][j][e];
        if constexpr (EPI == EPI_GELU) v = gelu_erf(v);
        if constexpr (EPI == EPI_STORE) v *= scale;
        if constexpr (EPI == EPI_ATOMIC) {
          atomicAdd(reinterpret_cast<float*>(g.C) + crow * g.ldc + col, v);
        } else if constexpr (CT == 0) {
          reinterpret_cast<float*>(g.C)[crow * g.ldc + col] = v;
        } else {
          reinterpret_cast<uint16_t*>(g.C)[crow * g.ldc + col] = f32_to_in<BF>(v);
        }
      }
    }
  }
}

// Zero rows of C that no index entry names (single-segment GATHER_M): the list is ascending, so a
// row is uncovered iff a binary search misses it.  One wave per row, 16-byte stores.
template <int ESIZE>
__global__ void __launch_bounds__(256)
k_zero_uncovered(void* C, int64_t ldc, int M, int N, const int32_t* seg_ptr, const int32_t* idx) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= M) return;
  int lo = 0, hi = seg_ptr[1] - seg_ptr[0];
  const int32_t* list = idx + seg_ptr[0];
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (list[mid] < row) lo = mid + 1; else hi = mid;
  }
  if (lo < seg_ptr[1] - seg_ptr[0] && list[lo] == row) return;
  char* p = reinterpret_cast<char*>(C) + (int64_t)row * ldc * ESIZE;
  const int64_t nbytes = (int64_t)N * ESIZE;
  for (int64_t b = (int64_t)(threadIdx.x & 63) * 16; b < nbytes; b += 64 * 16)
    *reinterpret_cast<uint4*>(p + b) = make_uint4(0, 0, 0, 0);
}

__global__ void __launch_bounds__(256) k_zero_rows(void* C, int64_t ld_bytes, int M, int64_t row_bytes) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= M) return;
  char* p = reinterpret_cast<char*>(C) + (int64_t)row * ld_bytes;
  for (int64_t b = (int64_t)(threadIdx.x & 63) * 16; b < row_bytes; b += 64 * 16)
    *reinterpret_cast<uint4*>(p + b) = make_uint4(0, 0, 0, 0);
}



}  // namespace

static int gemm_ring_depth() {
  static const int v = [] { const char* e = getenv("PIT_GEMM_RING"); return e ? atoi(e) : 2; }();
  return v == 4 ? 4 : 2;
}

template <bool BF, bool GK, int EPI, int CT>
static int launch_one(const GemmArgs& g, dim3 grid, hipStream_t st) {
  if (gemm_ring_depth() == 4) hipLaunchKernelGGL((k_sread_gemm<BF, GK, EPI, CT, 4>), grid, dim3(256), 0, st, g);
  else                        hipLaunchKernelGGL((k_sread_gemm<BF, GK, EPI, CT, 2>), grid, dim3(256), 0, st, g);
  PIT_LAUNCH_CHECK();
  return PIT_OK;
}

template <bool BF>
static int launch_bf(bool gather_k, int epi, int ct, const GemmArgs& g, dim3 grid, hipStream_t st) {
  if (gather_k) {
    if (epi != EPI_STORE) return PIT_EINVAL;
    return ct ? launch_one<BF, true, EPI_STORE, 1>(g, grid, st) : launch_one<BF, true, EPI_STORE, 0>(g, grid, st);
  }
  switch (epi) {
    case EPI_STORE:  return ct ? launch_one<BF, false, EPI_STORE, 1>(g, grid, st) : launch_one<BF, false, EPI_STORE, 0>(g, grid, st);
    case EPI_ATOMIC: return ct ? PIT_EINVAL : launch_one<BF, false, EPI_ATOMIC, 0>(g, grid, st);
    case EPI_GELU:   return ct ? launch_one<BF, false, EPI_GELU, 1>(g, grid, st) : PIT_EINVAL;
    default: return PIT_EINVAL;
  }
}

int launch_sread_gemm(bool bf, bool gather_k, int epi, int c_is_in_type, const GemmArgs& g, int max_tiles, hipStream_t st) {
  if (max_tiles <= 0 || g.N <= 0) return PIT_OK;
  // the kernel addresses each operand with 32-bit byte offsets from a per-segment base and
  // multiplies row numbers by the row pitch in 24 bits
  const int64_t a_rows = gather_k ? g.K : g.M;
  if (g.lda * 2 >= (1ll << 24) || g.ldb * 2 >= (1ll << 24) || a_rows >= (1ll << 24) || g.K >= (1ll << 24)) return PIT_ESHAPE;
  if (a_rows * g.lda * 2 >= (1ll << 32) || (int64_t)g.K * g.ldb * 2 >= (1ll << 32)) return PIT_ESHAPE;
  dim3 grid((unsigned)(g.N / TN), (unsigned)max_tiles);
  return bf ? launch_bf<true>(gather_k, epi, c_is_in_type, g, grid, st)
            : launch_bf<false>(gather_k, epi, c_is_in_type, g, grid, st);
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
  if (!ix || !ix->seg_ptr) return PIT_EINVAL;
  if (in_dt != PIT_BF16 && in_dt != PIT_F16) return PIT_EINVAL;
  if (c_dt != PIT_F32 && c_dt != in_dt) return PIT_EINVAL;
  if (mode != PIT_GEMM_GATHER_M && mode != PIT_GEMM_GATHER_K) return PIT_EINVAL;
  if (M < 0 || N < 0 || K < 0 || mt <= 0) return PIT_ESHAPE;
  if (N % TN) return PIT_ESHAPE;
  const int c_esize = c_dt == PIT_F32 ? 4 : 2;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  if (M == 0 || N == 0) return PIT_OK;
  if (!d_C || !aligned(d_C, 16) || ldc < N || (ldc * c_esize) % 16) return PIT_EINVAL;
  if (K > 0) {
    if (!d_A || !d_B || !ix->idx) return PIT_EINVAL;
    if (!aligned(d_A, 16) || !aligned(d_B, 16) || lda % 8 || ldb % 8 || ldb < N) return PIT_EINVAL;
  }

  GemmArgs g = {};
  g.A = d_A; g.lda = lda; g.B = d_B; g.ldb = ldb; g.b_seg_stride = 0;
  g.C = d_C; g.ldc = ldc; g.seg_ptr = ix->seg_ptr; g.idx = ix->idx; g.gate = nullptr;
  g.nseg = ix->nseg; g.M = M; g.N = N; g.K = K;

  if (mode == PIT_GEMM_GATHER_K) {
    if (mt != TM || M % TM) return PIT_ESHAPE;
    if (ix->nseg != M / TM) return PIT_ECAPACITY;
    if (K > 0 && lda < M) return PIT_EINVAL;
    g.slab = 0;
    return launch_sread_gemm(in_dt == PIT_BF16, true, EPI_STORE, c_dt != PIT_F32, g, ix->nseg, st);
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
  const int tiles_per_seg = (int)ceil_div(M, TM);
  if (ix->nseg == 1) {
    if (zero_uncovered) {
      if (c_esize == 4) hipLaunchKernelGGL(k_zero_uncovered<4>, dim3((unsigned)ceil_div(M, 4)), dim3(256), 0, st, d_C, ldc, M, N, ix->seg_ptr, ix->idx);
      else              hipLaunchKernelGGL(k_zero_uncovered<2>, dim3((unsigned)ceil_div(M, 4)), dim3(256), 0, st, d_C, ldc, M, N, ix->seg_ptr, ix->idx);
      PIT_LAUNCH_CHECK();
    }
    return launch_sread_gemm(in_dt == PIT_BF16, false, EPI_STORE, c_dt != PIT_F32, g, tiles_per_seg, st);
  }
  if (c_dt != PIT_F32) return PIT_EINVAL;
  { const int rc = launch_zero_rows(d_C, ldc * 4, M, (int64_t)N * 4, st); if (rc != PIT_OK) return rc; }
  const int64_t max_tiles = (int64_t)ix->nseg * tiles_per_seg;
  if (max_tiles > 65535) return PIT_ESHAPE;
  return launch_sread_gemm(in_dt == PIT_BF16, false, EPI_ATOMIC, 0, g, (int)max_tiles, st);
}
