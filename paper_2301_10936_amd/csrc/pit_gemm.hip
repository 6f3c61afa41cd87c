// pit_sread_gemm: host-side validation and launch of the SRead/MFMA/SWrite kernel.
#include "pit_gemm.hpp"

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

template <bool BF, bool GK, int EPI, int CT>
static int launch_one(const GemmArgs& g, dim3 grid, hipStream_t st) {
  hipLaunchKernelGGL((k_sread_gemm<BF, GK, EPI, CT>), grid, dim3(256), 0, st, g);
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
