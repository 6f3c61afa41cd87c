// pit_sread_gemm: the SRead -> dense MFMA tile -> SWrite kernels (paper Section 3.1, sparse kernel
// template) for gfx950, and their host-side validation and launch.
//
// A workgroup (256 threads = 4 wavefronts) computes a 128 x 128 dense tile of C with bf16 or f16
// inputs and fp32 accumulation.  There is one kernel per PIT-axis of MatMul (paper Table 1):
//
//   k_gather_k_direct  GATHER_K: A is K-major (At[k][m]); the tile's k-list comes from the index and
//             names the rows of At and of B to multiply.  Operands go global -> registers directly
//             and are transposed inside each lane; the four waves split the k-list and reduce
//             their partial tiles through LDS at the end (details above the kernel).
//   k_gather_m  GATHER_M: A is K-minor (A[m][k]); the tile's 128 row numbers come from the index
//             once, the k loop walks a contiguous k range; B rows are contiguous.  Operands are
//             staged through LDS, 2 x 2 waves of 64 x 64 with v_mfma_f32_32x32x16, 64 k per step.
//
// k_gather_m in detail.  Both operand tiles are K-MINOR in LDS ([128 x][64 k], 128 B per row) and
// are read with ds_read_b128.  The K-major source (rows of B) is transposed in registers on the way
// in: a thread loads an 8 k x 8 column block (8 x 16 B, one source row each), interleaves the 16-bit
// elements with v_perm_b32 and writes 8 tile rows of 16 B.  Global loads run 2 steps ahead in a
// register ring.  The steady-state loop is branch-free: all loads are unconditional (k past the end
// of the slab is clamped and zeroed on the way into LDS, in the last step only).  Inside a step the
// LDS reads of k-substep s+1, the transposes and the LDS writes of the next tile are interleaved
// with the MFMAs of k-substep s, so the LDS pipe and the matrix pipe work at the same time although
// there is a single wavefront per SIMD.
//
// SWrite.  The GATHER_M epilogue stores accumulator rows to the row numbers held in LDS (compact or
// from the index), optionally with a GELU + round to the input type (first MoE matmul) or a per-row
// gate (second MoE matmul).  GATHER_K writes the rows of its m-tile in place.  Several k-slabs per
// row (micro-tiles along k) have a kernel of their own, k_slab_strip, which keeps C in LDS.
#include "pit_gemm.hpp"
#include <type_traits>

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
// GELU(x) = x (1 + erf(x / sqrt 2)) / 2 with erf from the rational approximation 7.1.26 of Abramowitz & Stegun
// (|error| <= 1.5e-7, far below the rounding of the result to bf16 / fp16): a fifth of the
// instructions of erff; the GELU epilogue of the first MoE matmul is a quarter of its workgroups' run time otherwise.
__device__ __forceinline__ float gelu_erf_fast(float x) {
  const float z = fabsf(x) * 0.70710678118654752f;
  const float t = __frcp_rn(1.0f + 0.3275911f * z);
  const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
  const float e = 1.0f - poly * __expf(-z * z);          // erf(|x| / sqrt 2)
  return 0.5f * x * (1.0f + copysignf(e, x));
}

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

// Dword jj (k = 2 jj, 2 jj + 1) of column x of the 8 x 8 transpose below (one v_perm_b32).
__device__ __forceinline__ uint32_t transpose8x8_dword(const uint4 (&r)[8], int x, int jj) {
  const int i = x >> 1;
  const uint32_t sel = (x & 1) ? 0x07060302u : 0x05040100u;
  const uint32_t a = i == 0 ? r[2 * jj].x : i == 1 ? r[2 * jj].y : i == 2 ? r[2 * jj].z : r[2 * jj].w;
  const uint32_t b = i == 0 ? r[2 * jj + 1].x : i == 1 ? r[2 * jj + 1].y : i == 2 ? r[2 * jj + 1].z : r[2 * jj + 1].w;
  return __builtin_amdgcn_perm(b, a, sel);
}
// JA consecutive 16-bit columns of one k-row as loaded (JA = 8: 16 bytes, 4: 8 bytes, 2: 4 bytes)
template <int JA> struct ACols { uint32_t d[JA / 2]; };
// Dword jj (k = 2 jj, 2 jj + 1) of column x out of 8 k-rows of JA columns each (one v_perm_b32).
template <int JA>
__device__ __forceinline__ uint32_t transpose_cols_dword(const ACols<JA> (&r)[8], int x, int jj) {
  const uint32_t sel = (x & 1) ? 0x07060302u : 0x05040100u;
  return __builtin_amdgcn_perm(r[2 * jj + 1].d[x >> 1], r[2 * jj].d[x >> 1], sel);
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
// the same for 2 * JA bytes
template <int JA>
__device__ __forceinline__ ACols<JA> load_cols(const char* base, uint32_t byte_off) {
  ACols<JA> r;
  const uintptr_t a = reinterpret_cast<uintptr_t>(base) + byte_off;
  if constexpr (JA == 8) {
    const u32x4_t v = *(const u32x4_t __attribute__((address_space(1)))*)a;
    r.d[0] = v[0]; r.d[1] = v[1]; r.d[2] = v[2]; r.d[3] = v[3];
  } else if constexpr (JA == 4) {
    const u32x2_t v = *(const u32x2_t __attribute__((address_space(1)))*)a;
    r.d[0] = v[0]; r.d[1] = v[1];
  } else {
    static_assert(JA == 2, "columns per lane");
    r.d[0] = *(const uint32_t __attribute__((address_space(1)))*)a;
  }
  return r;
}

// nothing may be scheduled across this point
#define PIT_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

// GATHER_M (A K-minor, rows gathered; B K-major, contiguous k).  CT: 0 = fp32 C, 1 = C in the input type.
template <bool BF, int EPI, int CT>
__global__ void __launch_bounds__(256)
k_gather_m(const GemmArgs g) {
  constexpr int D = 2;   // depth of the register ring of global loads, in steps
  __shared__ __attribute__((aligned(1024))) char smem[2 * STAGE_BYTES];
  __shared__ int s_rows_a[TM];   // GATHER_M: source row of A per tile row
  __shared__ int s_rows_c[TM];   // destination row of C per tile row (-1 = skip)
  const uint32_t lds0 = (uint32_t)(uintptr_t)(PIT_LDS char*)smem;

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int wm = wv >> 1, wn = wv & 1;

  // ---------------------------------------------------------------- which tile is this workgroup?
  // Consecutive workgroup ids go to different XCDs (8, each with its own L2).  Renumber so that XCD
  // x works on row tiles x, x + 8, x + 16, .. and runs all column tiles of a row tile back to back:
  // they read the same gathered A rows through the same L2.  (Row tiles stay interleaved over the
  // XCDs because the grid is sized for the worst case and the surplus row tiles sit at its end.)
  // With one k-slab per segment (micro-tiles along k) every row tile has its own few B rows and
  // the plain order measures faster.
  int tile_row, tile_col;
  {
    const int tn = gridDim.x, tm = gridDim.y;
    const int lin = blockIdx.x + tn * blockIdx.y;
    const int full = g.slab_per_seg ? 0 : (tm >> 3) << 3;   // row tiles dealt out in rounds of 8
    if (lin < full * tn) {
      const int x = lin & 7, i = lin >> 3;
      tile_row = (i / tn) * 8 + x;
      tile_col = i % tn;
    } else {
      tile_row = lin / tn;
      tile_col = lin - tile_row * tn;
    }
  }
  const int n0 = tile_col * TN;

  int seg, list_begin, list_len;   // the row-list slice of this tile
  int k_begin = 0, k_len = 0;      // contiguous k range
  {
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

  const int len = k_len;                           // extent of the k loop (slab width)
  const int nsteps = (len + TK - 1) / TK;
  const int tail = len % TK;                       // != 0: the last step is partial

  // ---- loader roles: threads 0..127 fill the A tile, threads 128..255 the B tile (wave-uniform)
  const bool is_b = __builtin_amdgcn_readfirstlane(tid >> 7) != 0;
  const int u = tid & 127;
  const int t_cg = u & 15, t_kg = u >> 4;                               // transposing role: 8 k x 8 columns
  const int s_chunk = u & 7, s_row = (((u >> 3) & 1) << 3) | (u >> 4);  // straight role (A): rows r, r+8 per 16 lanes
  const bool transposing = is_b;

  const char* a_bytes = reinterpret_cast<const char*>(g.A);
  const char* b_bytes = reinterpret_cast<const char*>(g.B) + (int64_t)seg * g.b_seg_stride * 2;
  const char* src = uniform_ptr(is_b ? b_bytes : a_bytes);
  const uint32_t pitch = (uint32_t)((is_b ? g.ldb : g.lda) * 2);   // bytes per source row (< 2^24, checked on the host)
  // transposing role: byte offset of this thread's 8 columns inside a source row
  const uint32_t col_bytes = (uint32_t)(n0 + t_cg * 8) * 2u;

  uint32_t a_off[8];   // straight role: byte offset of (row of round j, this thread's chunk) at k step 0
#pragma unroll
  for (int j = 0; j < 8; ++j) a_off[j] = __umul24((uint32_t)s_rows_a[j * 16 + s_row], pitch) + (uint32_t)(k_begin + s_chunk * 8) * 2u;

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

  auto issue = [&](int step, uint4 (&r)[8]) {
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
  };
  // byte offsets of the 8 loads of `step` (same addresses as issue())
  auto issue_offsets = [&](int step, uint32_t (&off)[8]) {
    if (is_b) {
      const int base = k_begin + min(step * TK + t_kg * 8, k_len - 8);
#pragma unroll
      for (int j = 0; j < 8; ++j) off[j] = __umul24((uint32_t)(base + j), pitch) + col_bytes;
    } else {
      const uint32_t kofs = (uint32_t)((min(step * TK + s_chunk * 8, k_len - 8) - s_chunk * 8) * 2);
#pragma unroll
      for (int j = 0; j < 8; ++j) off[j] = a_off[j] + kofs;
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
      // operands swapped: the accumulator holds the 32 x 32 block transposed (lane = row of C, registers =
      // columns, four consecutive ones at a time), which is what the stores below want
      acc[q >> 1][q & 1] = mfma32<BF>(fb[ks & 1][q & 1], fa[ks & 1][q >> 1], acc[q >> 1][q & 1]);
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
    // prologue: loads of tiles 0 .. D; tile 0 into LDS, tile 1 transposed into o[].  Tile t >= 2
    // travels through ring slot (t - 2) % D; slot D-1 is filled by step 0.
    uint4 o[8], r0[8], r1[8];
    issue(0, r0);
    issue(min(1, nsteps - 1), r1);
#pragma unroll
    for (int s = 0; s + 1 < D; ++s) issue(min(2 + s, nsteps - 1), R[s]);
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
      for (int uu = 0; uu < 4; ++uu)
        body(it + uu, uu & 1, o, R[uu % D], R[(uu + D - 1) % D], true, true, true, true);
    }
    // drain
    for (; it < nsteps; it += 4) {
#pragma unroll
      for (int uu = 0; uu < 4; ++uu) {
        const int step = it + uu;
        if (step >= nsteps) break;
        body(step, uu & 1, o, R[uu % D], R[(uu + D - 1) % D], step + 1 < nsteps, step + 2 < nsteps, step + 1 + D < nsteps, false);
      }
    }
  }

  // ---------------------------------------------------------------- SWrite
  // lane l holds row (l % 32) of each of its two row blocks and, per register quad, 4 consecutive
  // columns: one row number and (optionally) one gate value per lane and block, 16-byte stores
  // (8-byte ones for 16-bit output), 16 store instructions per wave instead of 64 scalar ones
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int r = wm * 64 + i * 32 + (lane & 31);
    const int64_t crow = s_rows_c[r];
    if (crow < 0) continue;
    float scale = 1.f;
    if constexpr (EPI == EPI_STORE) { if (g.gate) scale = g.gate[crow]; }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
#pragma unroll
      for (int gq = 0; gq < 4; ++gq) {
        const int col = n0 + wn * 64 + j * 32 + 8 * gq + 4 * (lane >> 5);
        float v[4];
#pragma unroll
        for (int x = 0; x < 4; ++x) {
          v[x] = acc[i][j][4 * gq + x];
          if constexpr (EPI == EPI_GELU) v[x] = gelu_erf_fast(v[x]);
          if constexpr (EPI == EPI_STORE) v[x] *= scale;
        }
        if constexpr (CT == 0) {
          *reinterpret_cast<float4*>(reinterpret_cast<float*>(g.C) + crow * g.ldc + col) = make_float4(v[0], v[1], v[2], v[3]);
        } else {
          const uint32_t lo = (uint32_t)f32_to_in<BF>(v[0]) | ((uint32_t)f32_to_in<BF>(v[1]) << 16);
          const uint32_t hi = (uint32_t)f32_to_in<BF>(v[2]) | ((uint32_t)f32_to_in<BF>(v[3]) << 16);
          *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(g.C) + crow * g.ldc + col) = make_uint2(lo, hi);
        }
      }
    }
  }
}

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
          w[x] = (uint32_t)f32_to_in<BF>(acc[ja][2 * x][e]) | ((uint32_t)f32_to_in<BF>(acc[ja][2 * x + 1][e]) << 16);
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
  auto tile_of = [&](int lin) -> DirectTile {
    const int x = lin & 7, qq = total >> 3, rr = total & 7;
    const int lp = x * qq + min(x, rr) + (lin >> 3);
    constexpr int GM = 4;
    const int band = lp / (GM * tn), within = lp - band * (GM * tn);
    const int rows = min(GM, tm_tiles - band * GM);
    DirectTile t;
    t.seg = band * GM + within % rows;
    t.n0 = (within / rows) * TN;
    const int list_begin = g.seg_ptr[t.seg];
    t.list_len = g.seg_ptr[t.seg + 1] - list_begin;
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

// compute units of the current device rounded down to a multiple of 8 (one share per XCD)
static int compute_units() {
  static int cached[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  if (cached[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 8) n = 256;
    cached[dev] = n & ~7;
  }
  return cached[dev];
}

template <bool BF, bool GK, int EPI, int CT>
static int launch_one(const GemmArgs& g, dim3 grid, hipStream_t st) {
  if constexpr (GK) {
    static_assert(EPI == EPI_STORE, "GATHER_K has the plain store epilogue only");
    // one workgroup fits on a compute unit: with more tiles than compute units the workgroups loop
    const int total = (int)(grid.x * grid.y), cus = compute_units();
    if (g.slab == 64 || g.slab == 32) {
      // lower tiles: two-wave workgroups; as many as the registers let a compute unit hold (64 rows: two,
      // 32 rows: four, i.e. two waves per SIMD)
      const int resident = (g.slab == 64 ? 2 : 4) * cus;
      const unsigned wgs = (unsigned)(total <= resident ? total : resident);
      if (g.slab == 64) hipLaunchKernelGGL((k_gather_k_direct<BF, CT, 2, 4>), dim3(wgs), dim3(128), 0, st, g, (int)grid.y);
      else              hipLaunchKernelGGL((k_gather_k_direct<BF, CT, 2, 2>), dim3(wgs), dim3(128), 0, st, g, (int)grid.y);
    } else if (total >= 2 * cus) {      // two workgroups of two waves per compute unit
      hipLaunchKernelGGL((k_gather_k_direct<BF, CT, 2, 8>), dim3((unsigned)(2 * cus)), dim3(128), 0, st, g, (int)grid.y);
    } else {
      const unsigned wgs = (unsigned)(total <= cus ? total : cus);
      hipLaunchKernelGGL((k_gather_k_direct<BF, CT, 4, 8>), dim3(wgs), dim3(256), 0, st, g, (int)grid.y);
    }
    PIT_LAUNCH_CHECK();
    return PIT_OK;
  } else {
    hipLaunchKernelGGL((k_gather_m<BF, EPI, CT>), grid, dim3(256), 0, st, g);
    PIT_LAUNCH_CHECK();
    return PIT_OK;
  }
}

template <bool BF>
static int launch_bf(bool gather_k, int epi, int ct, const GemmArgs& g, dim3 grid, hipStream_t st) {
  if (gather_k) {
    if (epi != EPI_STORE) return PIT_EINVAL;
    return ct ? launch_one<BF, true, EPI_STORE, 1>(g, grid, st) : launch_one<BF, true, EPI_STORE, 0>(g, grid, st);
  }
  switch (epi) {
    case EPI_STORE:  return ct ? launch_one<BF, false, EPI_STORE, 1>(g, grid, st) : launch_one<BF, false, EPI_STORE, 0>(g, grid, st);
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
    if ((mt != 128 && mt != 64 && mt != 32) || M % mt) return PIT_ESHAPE;
    if (ix->nseg != M / mt) return PIT_ECAPACITY;
    if (K > 0 && lda < M) return PIT_EINVAL;
    g.slab = mt;       // GATHER_K: the tile height (= micro-tile height of the index)
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
