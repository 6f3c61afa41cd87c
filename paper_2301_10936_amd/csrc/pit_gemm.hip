// pit_sread_gemm: host-side validation and launch of the SRead/MFMA/SWrite kernel.
#include "pit_gemm.hpp"
#include <cstdlib>

namespace pit {
namespace {

template <bool BF>
__device__ __forceinline__ f32x16_t mfma32(const uint4& a, const uint4& b, const f32x16_t& c) {
  if constexpr (BF)
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
}

__device__ __forceinline__ uint2 lds_read_tr(uint32_t lds_base, uint32_t byte_off) {
  PIT_LDS v4i16_t* p = (PIT_LDS v4i16_t*)(uintptr_t)(lds_base + byte_off);
  return __builtin_bit_cast(uint2, __builtin_amdgcn_ds_read_tr16_b64_v4i16(p));
}
__device__ __forceinline__ uint4 lds_read_b128(uint32_t lds_base, uint32_t byte_off) {
  PIT_LDS u32x4_t* p = (PIT_LDS u32x4_t*)(uintptr_t)(lds_base + byte_off);
  return __builtin_bit_cast(uint4, *p);
}
__device__ __forceinline__ void lds_write_b128(uint32_t lds_base, uint32_t byte_off, const uint4& v) {
  PIT_LDS u32x4_t* p = (PIT_LDS u32x4_t*)(uintptr_t)(lds_base + byte_off);
  *p = __builtin_bit_cast(u32x4_t, v);
}

// byte offset of 16-byte chunk c (8 columns) of k-row k inside a K-major tile
__device__ __forceinline__ uint32_t kmajor_off(int k, int c) {
  return (uint32_t)(k * 256 + ((((c >> 2) ^ (k & 3)) << 6) | ((c & 3) << 4)));
}
// byte offset of 16-byte chunk c (8 k) of row m inside a K-minor tile
__device__ __forceinline__ uint32_t kminor_off(int m, int c) {
  return (uint32_t)(m * 128 + ((c ^ ((m >> 1) & 7)) << 4));
}

// MFMA operand (8 consecutive k of one column, for this lane) out of a K-major tile:
// column block cb (32 columns), k-substep ks (16 k).
__device__ __forceinline__ uint4 frag_kmajor(uint32_t tile, int cb, int ks, int lane) {
  const int k = ks * 16 + (lane >> 5) * 8 + ((lane & 15) >> 2);
  const int col = cb * 32 + ((lane >> 4) & 1) * 16 + (lane & 3) * 4;   // 4 columns = 8 bytes
  const int seg = col >> 5;
  const uint32_t in_seg = (uint32_t)(col & 31) * 2;
  const uint2 lo = lds_read_tr(tile, (uint32_t)(k * 256) + (uint32_t)(((seg ^ (k & 3)) << 6)) + in_seg);
  const int k2 = k + 4;
  const uint2 hi = lds_read_tr(tile, (uint32_t)(k2 * 256) + (uint32_t)(((seg ^ (k2 & 3)) << 6)) + in_seg);
  return make_uint4(lo.x, lo.y, hi.x, hi.y);
}
__device__ __forceinline__ uint4 frag_kminor(uint32_t tile, int mb, int ks, int lane) {
  const int m = mb * 32 + (lane & 31);
  return lds_read_b128(tile, kminor_off(m, ks * 2 + (lane >> 5)));
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

// GK = true: GATHER_K (A K-major), false: GATHER_M (A K-minor).  CT: 0 = fp32 C, 1 = C in the input type.
template <bool BF, bool GK, int EPI, int CT>
__global__ void __launch_bounds__(256)
k_sread_gemm(const GemmArgs g) {
  __shared__ __attribute__((aligned(1024))) char smem[2 * STAGE_BYTES];
  __shared__ int s_rows_a[TM];   // GATHER_M: source row of A per tile row (-1 = padding)
  __shared__ int s_rows_c[TM];   // destination row of C per tile row (-1 = skip)
  const uint32_t lds0 = (uint32_t)(uintptr_t)(PIT_LDS char*)smem;

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int wm = wv >> 1, wn = wv & 1;
  const int n0 = blockIdx.x * TN;

  // ---------------------------------------------------------------- which tile is this workgroup?
  int seg, list_begin, list_len;   // GATHER_K: the k-list; GATHER_M: the row list slice of this tile
  int k_begin = 0, k_len = 0;      // GATHER_M: contiguous k range
  if constexpr (GK) {
    seg = blockIdx.y;
    list_begin = g.seg_ptr[seg];
    list_len = g.seg_ptr[seg + 1] - list_begin;
  } else {
    // linear tile number -> (segment, tile inside segment); every wave does the same search
    const int tile = blockIdx.y;
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
      int ra = -1, rc = -1;
      if (tid < list_len) {
        const int v = g.idx[list_begin + tid];
        ra = g.a_gather ? v : list_begin + tid;
        rc = g.c_scatter ? v : list_begin + tid;
      }
      s_rows_a[tid] = ra;
      s_rows_c[tid] = rc;
    }
    __syncthreads();
  }

  const uint16_t* __restrict__ A = reinterpret_cast<const uint16_t*>(g.A);
  const uint16_t* __restrict__ B = reinterpret_cast<const uint16_t*>(g.B) + (int64_t)seg * g.b_seg_stride;

  f32x16_t acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int nsteps = GK ? (list_len + TK - 1) / TK : (k_len + TK - 1) / TK;

  // per-thread load slots
  //   K-major tile: 4 rounds; round r loads k-row r*16 + (tid>>4), 16-byte chunk tid & 15
  //   K-minor tile: 4 rounds; round r loads tile row r*32 + (tid>>3), 16-byte chunk tid & 7
  const int km_row = tid >> 4, km_chunk = tid & 15;
  const int kn_row = tid >> 3, kn_chunk = tid & 7;

  int64_t a_row_off[4];   // GATHER_M: element offset of this thread's 4 A rows (or -1)
  if constexpr (!GK) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int ra = s_rows_a[r * 32 + kn_row];
      a_row_off[r] = ra < 0 ? -1 : (int64_t)ra * g.lda;
    }
  }

  uint4 ra_[4], rb_[4];
  int kid[4];             // GATHER_K: k of this thread's 4 rows in the step being loaded

  auto load_kidx = [&](int step) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int kk = step * TK + r * 16 + km_row;
      kid[r] = kk < list_len ? g.idx[list_begin + kk] : -1;
    }
  };
  auto load_global = [&](int step) {
    if constexpr (GK) {
      const int m0 = seg * TM;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        ra_[r] = make_uint4(0, 0, 0, 0);
        rb_[r] = make_uint4(0, 0, 0, 0);
        if (kid[r] >= 0) {
          ra_[r] = *reinterpret_cast<const uint4*>(A + (int64_t)kid[r] * g.lda + m0 + km_chunk * 8);
          rb_[r] = *reinterpret_cast<const uint4*>(B + (int64_t)kid[r] * g.ldb + n0 + km_chunk * 8);
        }
      }
    } else {
      const int kofs = step * TK;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        ra_[r] = make_uint4(0, 0, 0, 0);
        rb_[r] = make_uint4(0, 0, 0, 0);
        const int ka = kofs + kn_chunk * 8;
        if (a_row_off[r] >= 0 && ka < k_len)
          ra_[r] = *reinterpret_cast<const uint4*>(A + a_row_off[r] + k_begin + ka);
        const int kb = kofs + r * 16 + km_row;
        if (kb < k_len)
          rb_[r] = *reinterpret_cast<const uint4*>(B + (int64_t)(k_begin + kb) * g.ldb + n0 + km_chunk * 8);
      }
    }
  };
  auto store_lds = [&](int buf) {
    const uint32_t a_t = lds0 + buf * STAGE_BYTES, b_t = a_t + A_TILE_BYTES;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      if constexpr (GK) lds_write_b128(a_t, kmajor_off(r * 16 + km_row, km_chunk), ra_[r]);
      else              lds_write_b128(a_t, kminor_off(r * 32 + kn_row, kn_chunk), ra_[r]);
      lds_write_b128(b_t, kmajor_off(r * 16 + km_row, km_chunk), rb_[r]);
    }
  };
  auto compute = [&](int buf, int nks) {
    const uint32_t a_t = lds0 + buf * STAGE_BYTES, b_t = a_t + A_TILE_BYTES;
    for (int ks = 0; ks < nks; ++ks) {
      uint4 af[2], bf[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        if constexpr (GK) af[i] = frag_kmajor(a_t, wm * 2 + i, ks, lane);
        else              af[i] = frag_kminor(a_t, wm * 2 + i, ks, lane);
        bf[i] = frag_kmajor(b_t, wn * 2 + i, ks, lane);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = mfma32<BF>(af[i], bf[j], acc[i][j]);
    }
  };

  if (nsteps > 0) {
    if constexpr (GK) load_kidx(0);
    load_global(0);
    store_lds(0);
    if constexpr (GK) { if (nsteps > 1) load_kidx(1); }
    __syncthreads();
    for (int it = 0; it < nsteps; ++it) {
      const bool more = it + 1 < nsteps;
      if (more) load_global(it + 1);
      if constexpr (GK) { if (it + 2 < nsteps) load_kidx(it + 2); }
      const int rem = (GK ? list_len : k_len) - it * TK;
      compute(it & 1, rem >= TK ? 4 : (rem + 15) / 16);
      if (more) store_lds((it + 1) & 1);
      __syncthreads();
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


// ------------------------------------------------------------------------------------------------
// Pipelined kernel.  Every operand tile is K-MINOR in LDS ([128 x][64 k], 128 B per row) and is read
// with ds_read_b128 (about twice the rate of the 8-byte transposing read).  K-major sources (rows of
// At and of B) are transposed in registers on their way in: a thread loads an 8 k x 8 column block
// (8 x 16 B, one row each), interleaves the 16-bit elements with v_perm_b32 and writes 8 rows of
// 16 B.  Global loads run D steps ahead in a register ring, so HBM/L2 latency is covered with a
// single wavefront per SIMD.  The steady-state loop is branch-free: all loads are unconditional
// (positions past the end of a list are clamped to its last entry and the rows are zeroed on the
// way into LDS, in the last step only), index values are fetched one step before the loads that
// use them and ahead of that step's data loads, so waiting for them never drains the data loads.
//
// Global loads are laid out so that 16 consecutive lanes read 256 contiguous bytes of one source
// row (the address unit merges 4 neighbouring lanes into one 64-byte request; lanes that jump
// between rows cost one request each, four times the address-unit time).
//
// LDS address of 16-byte chunk c (8 k) of tile row m, with a = m >> 4, h = (m >> 3) & 1, l = m & 7:
//   256-byte bank row = a * 8 + c,   16-byte slot = h * 8 + ((l + a + c) & 7)
// The LDS serves 16 lanes per clock and conflicts are decided by the slot.  All three access
// shapes put 16 lanes on 16 different slots:
//   operand read        16 consecutive rows (a fixed; h, l vary), one chunk
//   transposing write   rows 8*cg + x for 16 consecutive cg (l = x fixed; a, h vary), one chunk
//   straight write      rows m and m + 8 (h differs), all 8 chunks each
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t tile_off(int m, int c) {
  const int a = m >> 4, h = (m >> 3) & 1, l = m & 7;
  return (uint32_t)((((a << 3) | c) << 8) | (((h << 3) | ((l + a + c) & 7)) << 4));
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

__device__ __forceinline__ u32x4_t lds_read_frag(uint32_t addr) {
  return *(PIT_LDS u32x4_t*)(uintptr_t)addr;
}
template <bool BF>
__device__ __forceinline__ f32x16_t mfma32v(const u32x4_t& a, const u32x4_t& b, const f32x16_t& c) {
  if constexpr (BF)
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
}

// KS = 1: 256 threads, one k-group.  KS = 2: 512 threads; two groups of 4 wavefronts work on the SAME
// 128 x 128 tile, group g taking the g-th 64-wide half of every 128-wide k step with its own LDS
// buffers and accumulators; the two partial tiles are added through LDS before SWrite.  That puts
// two wavefronts on every SIMD (one can issue MFMAs while the other waits on the memory pipes)
// without shrinking the tile or going through global memory.
template <bool BF, bool GK, int EPI, int CT, int D, int KS, int ABL = 0>
__global__ void __launch_bounds__(256 * KS)
k_sread_gemm3(const GemmArgs g) {
  static_assert(D == 2 || D == 4, "ring depth must divide the unroll factor 4");
  static_assert(KS == 1 || KS == 2, "one or two k-groups");
  constexpr int TKS = TK * KS;                     // k extent of one step of the whole workgroup
  __shared__ __attribute__((aligned(1024))) char smem[KS * 2 * STAGE_BYTES];
  __shared__ int s_rows_a[TM];
  __shared__ int s_rows_c[TM];

  const int tid_all = threadIdx.x;
  const int grp = KS == 1 ? 0 : __builtin_amdgcn_readfirstlane(tid_all >> 8);
  const uint32_t lds0 = (uint32_t)(uintptr_t)(PIT_LDS char*)smem + (uint32_t)grp * 2u * STAGE_BYTES;
  const int tid = tid_all & 255, lane = tid & 63, wv = tid >> 6;
  const int wm = wv >> 1, wn = wv & 1;
  const int n0 = blockIdx.x * TN;

  int seg, list_begin, list_len;
  int k_begin = 0, k_len = 0;
  if constexpr (GK) {
    seg = blockIdx.y;
    list_begin = g.seg_ptr[seg];
    list_len = g.seg_ptr[seg + 1] - list_begin;
  } else {
    const int tile = blockIdx.y;
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
    if (tid_all < TM) {
      // rows past the end of the list read the list's last row (a valid address); their results
      // are never stored
      const int v = g.idx[list_begin + min(tid_all, list_len - 1)];
      s_rows_a[tid_all] = g.a_gather ? v : list_begin + min(tid_all, list_len - 1);
      s_rows_c[tid_all] = tid_all < list_len ? (g.c_scatter ? v : list_begin + tid_all) : -1;
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
  const int nsteps = (len + TKS - 1) / TKS;
  const int tail = len % TKS;                      // != 0: the last step is partial
  const int kpos0 = grp * TK;                      // this group's offset inside a step

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

  // LDS write offsets
  uint32_t w_off[8];
#pragma unroll
  for (int x = 0; x < 8; ++x) w_off[x] = transposing ? tile_off(t_cg * 8 + x, t_kg) : tile_off(x * 16 + s_row, s_chunk);
  const uint32_t w_tile = is_b ? (uint32_t)A_TILE_BYTES : 0u;
  // LDS read offsets.  For the 32-row block i of this wave and k-substep ks the operand address is
  //   rdX[(ks + i) & 3] + i * 4096 + ks * 512
  // (the slot rotates with a + c, and both the block and the substep add 2 to that sum).
  uint32_t rd_a[4], rd_b[4];
  {
    const int m = lane & 31, hi = lane >> 5;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      rd_a[q] = tile_off(wm * 64 + m, hi + 2 * q) - (uint32_t)q * 512u;
      rd_b[q] = tile_off(wn * 64 + m, hi + 2 * q) - (uint32_t)q * 512u + (uint32_t)A_TILE_BYTES;
    }
  }

  uint4 R[D][8];
  int k_use[8], k_pend[8];   // GATHER_K: list values for the step being issued / the one after
  int k_ahead = 0;           // GATHER_K: one list entry on its way from global memory to the LDS ring

  // GATHER_K keeps a sliding window of the k-list in LDS (16 steps x 64 entries).  Every 4th step
  // each thread fetches one entry 12 steps ahead and stores it 3 steps later, so no load in the
  // loop ever depends on a load issued less than 3 steps before it.
  constexpr int KRING = 16 * TKS;
  __shared__ __attribute__((aligned(32))) int s_kidx[GK ? KRING : 4];
  const uint32_t kring = (uint32_t)(uintptr_t)(PIT_LDS char*)s_kidx;
  auto list_at = [&](int pos) { return g.idx[list_begin + min(pos, list_len - 1)]; };
  auto load_kid = [&](int step, int (&dst)[8]) {
    const uint32_t a = kring + (uint32_t)(((step & 15) * TKS + kpos0 + t_kg * 8) * 4);
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
        const int base = k_begin + min(step * TKS + kpos0 + t_kg * 8, k_len - 8);
#pragma unroll
        for (int j = 0; j < 8; ++j) r[j] = load16(src, __umul24((uint32_t)(base + j), pitch) + col_bytes);
      } else {
        // byte distance from this thread's chunk at step 0; a chunk past the slab end re-reads the last one
        const uint32_t kofs = (uint32_t)((min(step * TKS + kpos0 + s_chunk * 8, k_len - 8) - s_chunk * 8) * 2);
#pragma unroll
        for (int j = 0; j < 8; ++j) r[j] = load16(src, a_off[j] + kofs);
      }
    }
  };
  // zero what lies past the end of the k extent (last, partial step only)
  auto zero_tail = [&](int step, uint4 (&r)[8]) {
    if (transposing) {
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (step * TKS + kpos0 + t_kg * 8 + j >= len) r[j] = make_uint4(0, 0, 0, 0);
    } else {
      if (step * TKS + kpos0 + s_chunk * 8 >= len) {
#pragma unroll
        for (int j = 0; j < 8; ++j) r[j] = make_uint4(0, 0, 0, 0);
      }
    }
  };
  auto stage = [&](int buf, int step, uint4 (&r)[8], bool may_be_last) {
    if (may_be_last && tail != 0 && step == nsteps - 1) zero_tail(step, r);
    const uint32_t t = lds0 + buf * STAGE_BYTES + w_tile;
    if (transposing) {
      uint4 o[8];
      transpose8x8_b16(r, o);
#pragma unroll
      for (int x = 0; x < 8; ++x) lds_write_b128(t, w_off[x], o[x]);
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) lds_write_b128(t, w_off[j], r[j]);
    }
  };
  auto compute = [&](int buf) {
    const uint32_t t = lds0 + buf * STAGE_BYTES;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      u32x4_t af[2], bf[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        af[i] = lds_read_frag(t + rd_a[(ks + i) & 3] + i * 4096 + ks * 512);
        bf[i] = lds_read_frag(t + rd_b[(ks + i) & 3] + i * 4096 + ks * 512);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = mfma32v<BF>(af[i], bf[j], acc[i][j]);
    }
  };

  if (nsteps > 0) {
    if constexpr (GK) {
      // list window for steps 0..15
      int v[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) v[q] = list_at(q * 256 * KS + tid_all);
#pragma unroll
      for (int q = 0; q < 4; ++q) s_kidx[q * 256 * KS + tid_all] = v[q];
      __syncthreads();
    }
    // prologue: steps 0 .. D-1 into the ring, step 0 into LDS, step D into the freed slot
#pragma unroll
    for (int s = 0; s < D; ++s) {
      if (s < nsteps) {
        if constexpr (GK) load_kid(s, k_use);
        issue(s, R[s]);
      }
    }
    if constexpr (GK) {
      load_kid(min(D, nsteps - 1), k_use);
      load_kid(min(D + 1, nsteps - 1), k_pend);
    }
    stage(0, 0, R[0], true);
    if (D < nsteps) issue(D, R[0]);
    __syncthreads();
    if (KS == 2 && grp == 1) __syncthreads();   // group 1 runs one barrier behind group 0 from here on

    int it = 0;
    // steady state, 4 steps per trip: every step here has step + 1 + D < nsteps; no conditionals
    // around memory operations
    for (; it + 4 + D < nsteps; it += 4) {
#pragma unroll
      for (int uu = 0; uu < 4; ++uu) {
        const int step = it + uu;
        if constexpr (GK) {
#pragma unroll
          for (int j = 0; j < 8; ++j) k_use[j] = k_pend[j];
          load_kid(min(step + 2 + D, nsteps - 1), k_pend);
          if (uu == 0) k_ahead = list_at((step + 12) * TKS + tid_all);
          // the list fetch stays ahead of this step's data loads in program order: the memory
          // counter is in-order, so waiting for it later never drains the younger data loads
          __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (GK) {
          if (uu == 3) s_kidx[((step + 9) * TKS + tid_all) & (KRING - 1)] = k_ahead;   // entries of steps it+12 .. it+15
        }
        // KS == 2: the two groups run half a step out of phase (group 1 entered the loop one
        // barrier late): while one feeds the matrix cores from LDS, the other moves the next
        // tiles (global loads, transposes, LDS stores)
        if constexpr (!(ABL & 1)) compute(uu & 1);
        if (KS == 2) __syncthreads();
        if constexpr (!(ABL & 2)) stage((uu + 1) & 1, step + 1, R[(uu + 1) % D], false);
        if constexpr (!(ABL & 4)) issue(step + 1 + D, R[(uu + 1) % D]);
        __syncthreads();
      }
    }
    // drain
    for (; it < nsteps; it += 4) {
#pragma unroll
      for (int uu = 0; uu < 4; ++uu) {
        const int step = it + uu;
        if (step >= nsteps) break;
        if constexpr (GK) {
          if (step + 1 + D < nsteps) {
#pragma unroll
            for (int j = 0; j < 8; ++j) k_use[j] = k_pend[j];
            load_kid(min(step + 2 + D, nsteps - 1), k_pend);
          }
        }
        compute(uu & 1);
        if (KS == 2) __syncthreads();
        if (step + 1 < nsteps) stage((uu + 1) & 1, step + 1, R[(uu + 1) % D], true);
        if (step + 1 + D < nsteps) issue(step + 1 + D, R[(uu + 1) % D]);
        __syncthreads();
      }
    }
    if (KS == 2 && grp == 0) __syncthreads();   // pairs with group 1's extra barrier at loop entry
  }

  if constexpr (KS == 2) {
    // add the second group's partial tile to the first's through LDS (the operand buffers are free:
    // the k loop ended with a barrier)
    float* red = reinterpret_cast<float*>(smem);     // [64 accumulators][256 threads]
    if (grp == 1) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int e = 0; e < 16; ++e) red[((i * 2 + j) * 16 + e) * 256 + tid] = acc[i][j][e];
    }
    __syncthreads();
    if (grp == 1) return;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] += red[((i * 2 + j) * 16 + e) * 256 + tid];
  }

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

static int gemm_variant() {
  static const int v = [] { const char* e = getenv("PIT_GEMM_VARIANT"); return e ? atoi(e) : 22; }();
  return v;
}

template <bool BF, bool GK, int EPI, int CT>
static int launch_one(const GemmArgs& g, dim3 grid, hipStream_t st) {
  if constexpr (BF && GK && EPI == EPI_STORE && CT == 0) {
    static const int abl = [] { const char* e = getenv("PIT_GEMM_ABL"); return e ? atoi(e) : 0; }();
    switch (abl) {
      case 1: hipLaunchKernelGGL((k_sread_gemm3<BF, GK, EPI, CT, 2, 2, 1>), grid, dim3(512), 0, st, g); return PIT_OK;
      case 2: hipLaunchKernelGGL((k_sread_gemm3<BF, GK, EPI, CT, 2, 2, 2>), grid, dim3(512), 0, st, g); return PIT_OK;
      case 3: hipLaunchKernelGGL((k_sread_gemm3<BF, GK, EPI, CT, 2, 2, 3>), grid, dim3(512), 0, st, g); return PIT_OK;
      case 4: hipLaunchKernelGGL((k_sread_gemm3<BF, GK, EPI, CT, 2, 2, 4>), grid, dim3(512), 0, st, g); return PIT_OK;
      case 5: hipLaunchKernelGGL((k_sread_gemm3<BF, GK, EPI, CT, 2, 2, 5>), grid, dim3(512), 0, st, g); return PIT_OK;
      case 6: hipLaunchKernelGGL((k_sread_gemm3<BF, GK, EPI, CT, 2, 2, 6>), grid, dim3(512), 0, st, g); return PIT_OK;
      case 7: hipLaunchKernelGGL((k_sread_gemm3<BF, GK, EPI, CT, 2, 2, 7>), grid, dim3(512), 0, st, g); return PIT_OK;
      default: break;
    }
  }
  switch (gemm_variant()) {
    case 0: hipLaunchKernelGGL((k_sread_gemm<BF, GK, EPI, CT>), grid, dim3(256), 0, st, g); break;
    case 2: hipLaunchKernelGGL((k_sread_gemm3<BF, GK, EPI, CT, 2, 1>), grid, dim3(256), 0, st, g); break;
    case 4: hipLaunchKernelGGL((k_sread_gemm3<BF, GK, EPI, CT, 4, 1>), grid, dim3(256), 0, st, g); break;
    default: hipLaunchKernelGGL((k_sread_gemm3<BF, GK, EPI, CT, 2, 2>), grid, dim3(512), 0, st, g); break;
  }
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
