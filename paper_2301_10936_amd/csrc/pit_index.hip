// Online sparsity detection (paper Section 3.3) for gfx950.
//
// The paper's detector appends coordinates with atomicAdd and accepts whatever order the scheduler
// produces.  Here the list is canonical (ascending per segment) and the detector uses no atomics:
//   pass 1  streams the tensor once (coalesced 16-byte loads where the layout allows it) and turns
//           "micro-tile contains a non-zero" into one bit per micro-tile with wavefront ballots.
//           The bitmap is laid out [segment][PIT coordinate / 64] as 64-bit words.
//   pass 2  one workgroup per segment: popcounts give the segment's start (exclusive prefix over
//           all earlier words), a block scan gives each word's offset, and every set bit is
//           written to its slot (lane b of a wave owns bit b, so stores are coalesced).
// The tensor itself is never re-formatted.
#include "pit_common.hpp"
#include <algorithm>

namespace pit {
namespace {

typedef unsigned long long u64;

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }

// ----------------------------------------------------------------------------------------------
// zero tests on raw bits: -0 is zero, NaN/Inf/subnormals are non-zero
// ----------------------------------------------------------------------------------------------
template <int ESIZE> struct Elem;
template <> struct Elem<1> { typedef uint8_t  T; static __device__ __forceinline__ bool nz(T v) { return v != 0; } };
template <> struct Elem<2> { typedef uint16_t T; static __device__ __forceinline__ bool nz(T v) { return (v & 0x7FFFu) != 0; } };
template <> struct Elem<4> { typedef uint32_t T; static __device__ __forceinline__ bool nz(T v) { return (v & 0x7FFFFFFFu) != 0; } };

template <int ESIZE>
__device__ __forceinline__ bool any_nz16(const uint4& v) {
  if (ESIZE == 1) return (v.x | v.y | v.z | v.w) != 0;
  if (ESIZE == 2) return ((v.x | v.y | v.z | v.w) & 0x7FFF7FFFu) != 0;
  return ((v.x | v.y | v.z | v.w) & 0x7FFFFFFFu) != 0;
}

// ----------------------------------------------------------------------------------------------
// pass 1, generic: one lane per micro-tile, any shape, any dtype, either PIT dimension.
// wave (s, w) covers PIT coordinates 64w .. 64w+63 of segment s.
// ----------------------------------------------------------------------------------------------
template <int ESIZE>
__global__ void __launch_bounds__(256)
k_bitmap_generic(const void* __restrict__ src, int64_t ld, int mt_rows, int mt_cols, int pit_dim,
                 int nseg, int npit, int W, u64* __restrict__ words, uint32_t* __restrict__ occ) {
  typedef typename Elem<ESIZE>::T T;
  const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (wave >= (int64_t)nseg * W) return;
  const int s = (int)(wave / W), w = (int)(wave % W);
  const int c = w * 64 + lane_id();
  uint32_t bits = 0;
  bool flag = false;
  if (c < npit) {
    const int64_t r0 = (int64_t)(pit_dim == 0 ? c : s) * mt_rows;
    const int64_t c0 = (int64_t)(pit_dim == 0 ? s : c) * mt_cols;
    const T* p = reinterpret_cast<const T*>(src) + r0 * ld + c0;
    const bool small = mt_rows * mt_cols <= 32;
    for (int r = 0; r < mt_rows; ++r) {
      for (int q = 0; q < mt_cols; ++q) {
        if (Elem<ESIZE>::nz(p[(int64_t)r * ld + q])) {
          flag = true;
          if (small) bits |= 1u << (r * mt_cols + q);
        }
      }
    }
    if (occ) occ[(int64_t)s * npit + c] = bits;
  }
  const u64 b = __ballot(flag);
  if (lane_id() == 0) words[(int64_t)s * W + w] = b;
}

// ----------------------------------------------------------------------------------------------
// pass 1, fast path A: PIT-axis = rows, micro-tile = 1 x mt_cols with mt_bytes in {16..1024}, a
// power of two.  A workgroup covers 64 rows x 1 KiB of columns; a wave issues 16 row loads of
// 1 KiB (64 lanes x 16 B, fully coalesced) at once and ballots each of them.
// ----------------------------------------------------------------------------------------------
template <int ESIZE>
__global__ void __launch_bounds__(256)
k_bitmap_rows(const void* __restrict__ src, int64_t ld_bytes, int rows, int row_bytes, int lpm /*lanes per micro-tile*/,
              int nseg, int W, u64* __restrict__ words) {
  __shared__ uint32_t part[4][64];
  const int wv = threadIdx.x >> 6, ln = lane_id();
  const int r0 = blockIdx.y * 64 + wv * 16;
  const int byte0 = blockIdx.x * 1024 + ln * 16;
  const char* base = reinterpret_cast<const char*>(src) + byte0;
  const bool col_ok = byte0 < row_bytes;
  uint4 v[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    v[i] = make_uint4(0, 0, 0, 0);
    if (col_ok && r0 + i < rows) v[i] = *reinterpret_cast<const uint4*>(base + (int64_t)(r0 + i) * ld_bytes);
  }
  const int nmt = 64 / lpm;
  const u64 lmask = lpm == 64 ? ~0ull : ((1ull << lpm) - 1ull);
  const int sh = (ln < nmt ? ln : 0) * lpm;
  uint32_t acc = 0;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const u64 b = __ballot(any_nz16<ESIZE>(v[i]));
    acc |= (((b >> sh) & lmask) != 0 ? 1u : 0u) << i;
  }
  part[wv][ln] = acc;
  __syncthreads();
  if (wv == 0 && ln < nmt) {
    const int s = blockIdx.x * nmt + ln;
    if (s < nseg) {
      const u64 word = (u64)part[0][ln] | ((u64)part[1][ln] << 16) | ((u64)part[2][ln] << 32) | ((u64)part[3][ln] << 48);
      words[(int64_t)s * W + blockIdx.y] = word;
    }
  }
}

// ----------------------------------------------------------------------------------------------
// pass 1, fast path B: PIT-axis = columns, byte mask, micro-tile = mt_rows x 1.
// A wave covers one segment (mt_rows rows) x 1024 columns; a lane owns 16 columns and keeps one
// occupancy word per column (bit r = row r of the micro-tile is non-zero).
// ----------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
k_bitmap_cols_u8(const uint8_t* __restrict__ src, int64_t ld, int mt_rows, int cols, int nseg, int npit, int W,
                 u64* __restrict__ words, uint32_t* __restrict__ occ) {
  const int chunks = (W * 64 + 1023) / 1024;
  const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (wave >= (int64_t)nseg * chunks) return;
  const int s = (int)(wave / chunks), ch = (int)(wave % chunks);
  const int c0 = ch * 1024 + lane_id() * 16;
  if (c0 >= W * 64) return;
  uint32_t o[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) o[j] = 0;
  if (c0 < cols) {
    const uint8_t* p = src + (int64_t)s * mt_rows * ld + c0;
    for (int r0 = 0; r0 < mt_rows; r0 += 8) {
      uint4 v[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        v[i] = make_uint4(0, 0, 0, 0);
        if (r0 + i < mt_rows) v[i] = *reinterpret_cast<const uint4*>(p + (int64_t)(r0 + i) * ld);
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const uint32_t d[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
        const uint32_t rb = (r0 + i) < 32 ? (1u << ((r0 + i) & 31)) : 0x80000000u;  // rows >= 32 only feed the flag
#pragma unroll
        for (int j = 0; j < 16; ++j)
          if ((d[j >> 2] >> ((j & 3) * 8)) & 0xFFu) o[j] |= rb;
      }
    }
  }
  uint32_t flags = 0;
#pragma unroll
  for (int j = 0; j < 16; ++j) flags |= (o[j] != 0 ? 1u : 0u) << j;
  reinterpret_cast<uint16_t*>(words)[((int64_t)s * W) * 4 + (c0 >> 4)] = (uint16_t)flags;
  if (occ && c0 < cols) {
    uint4* q = reinterpret_cast<uint4*>(occ + (int64_t)s * npit + c0);
    q[0] = make_uint4(o[0], o[1], o[2], o[3]);
    q[1] = make_uint4(o[4], o[5], o[6], o[7]);
    q[2] = make_uint4(o[8], o[9], o[10], o[11]);
    q[3] = make_uint4(o[12], o[13], o[14], o[15]);
  }
}

// ----------------------------------------------------------------------------------------------
// pass 1 for routing decisions: segment e, bit t  <=>  expert_id[t] == e
// ----------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
k_bitmap_route(const int32_t* __restrict__ expert_id, int T, int E, int W, u64* __restrict__ words) {
  const int w = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (w >= W) return;
  const int t = w * 64 + lane_id();
  const int e = t < T ? expert_id[t] : -1;
  for (int e0 = 0; e0 < E; e0 += 64) {
    u64 mine = 0;
    const int n = min(64, E - e0);
    for (int j = 0; j < n; ++j) {
      const u64 b = __ballot(e == e0 + j);
      if (lane_id() == j) mine = b;
    }
    if (lane_id() < n) words[(int64_t)(e0 + lane_id()) * W + w] = mine;
  }
}

// ----------------------------------------------------------------------------------------------
// per-segment popcount (only used when there are many segments)
// ----------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
k_seg_count(const u64* __restrict__ words, int nseg, int W, int32_t* __restrict__ cnt) {
  const int s = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (s >= nseg) return;
  int c = 0;
  for (int w = lane_id(); w < W; w += 64) c += __popcll(words[(int64_t)s * W + w]);
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) c += __shfl_xor(c, d);
  if (lane_id() == 0) cnt[s] = c;
}

// ----------------------------------------------------------------------------------------------
// pass 2: scan + ordered emit, one workgroup (256 threads) per segment
// ----------------------------------------------------------------------------------------------
__device__ __forceinline__ int block_sum_256(int v, int* sm) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d);
  __syncthreads();
  if (lane_id() == 0) sm[threadIdx.x >> 6] = v;
  __syncthreads();
  return sm[0] + sm[1] + sm[2] + sm[3];
}

__global__ void __launch_bounds__(256)
k_emit(const u64* __restrict__ words, const int32_t* __restrict__ seg_cnt, const uint32_t* __restrict__ occ,
       int nseg, int npit, int W, int cap, int total_items,
       int32_t* __restrict__ seg_ptr, int32_t* __restrict__ idx, uint32_t* __restrict__ bits,
       int32_t* __restrict__ status) {
  __shared__ int red[4];
  __shared__ int wsum[4];
  __shared__ u64 wd[256];
  __shared__ int off[256];
  const int s = blockIdx.x;
  const int tid = threadIdx.x, wv = tid >> 6, ln = lane_id();

  // start of this segment = number of set bits in all earlier segments
  int part = 0;
  if (seg_cnt) {
    for (int i = tid; i < s; i += 256) part += seg_cnt[i];
  } else {
    const int64_t n = (int64_t)s * W;
    for (int64_t i = tid; i < n; i += 256) part += __popcll(words[i]);
  }
  const int base = block_sum_256(part, red);

  int running = base;
  for (int w0 = 0; w0 < W; w0 += 256) {
    const int w = w0 + tid;
    const u64 word = w < W ? words[(int64_t)s * W + w] : 0ull;
    const int pc = __popcll(word);
    // inclusive scan over the 256 threads
    int inc = pc;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int t = __shfl_up(inc, d);
      if (ln >= d) inc += t;
    }
    __syncthreads();            // previous iteration's readers of wd/off/wsum are done
    if (ln == 63) wsum[wv] = inc;
    __syncthreads();
    int wave_base = 0;
    for (int i = 0; i < wv; ++i) wave_base += wsum[i];
    const int chunk_total = wsum[0] + wsum[1] + wsum[2] + wsum[3];
    wd[tid] = word;
    off[tid] = running + wave_base + inc - pc;
    __syncthreads();
    const int nw = min(256, W - w0);
    for (int i = wv; i < nw; i += 4) {
      const u64 x = wd[i];
      if ((x >> ln) & 1ull) {
        const int pos = off[i] + __popcll(x & ((1ull << ln) - 1ull));
        const int c = (w0 + i) * 64 + ln;
        if (pos < cap) {
          idx[pos] = c;
          if (bits) bits[pos] = occ[(int64_t)s * npit + c];
        }
      }
    }
    running += chunk_total;
  }
  if (tid == 0) {
    seg_ptr[s] = base;
    if (s == nseg - 1) {
      seg_ptr[nseg] = running;
      if (status) *status = total_items - running;
    }
  }
}

// Same result with more workgroups, for segments of up to 1024 words (65 536 micro-tiles): one
// workgroup per chunk of 16 words.  The chunk's own words are requested before the words that are
// only counted, so the kernel has a single round trip to memory ahead of its stores.
constexpr int EMIT_CH = 16;

__global__ void __launch_bounds__(256)
k_emit_chunked(const u64* __restrict__ words, const int32_t* __restrict__ seg_cnt, const uint32_t* __restrict__ occ,
               int nseg, int npit, int W, int cap, int total_items,
               int32_t* __restrict__ seg_ptr, int32_t* __restrict__ idx, uint32_t* __restrict__ bits,
               int32_t* __restrict__ status) {
  __shared__ int red[4];
  __shared__ int wsum[4];
  const int c = blockIdx.x, s = blockIdx.y;
  const int tid = threadIdx.x, wv = tid >> 6, ln = lane_id();
  const int w_first = c * EMIT_CH;
  const int64_t row0 = (int64_t)s * W;

  // wave wv emits words w_first + 4 wv .. + 3 (every lane holds all four)
  u64 mine[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int w = w_first + wv * 4 + i;
    mine[i] = w < W ? words[row0 + w] : 0ull;
  }
  // set bits ahead of this chunk: earlier segments, then the earlier words of this segment
  int part = 0;
  if (seg_cnt) {
    for (int i = tid; i < s; i += 256) part += seg_cnt[i];
    for (int i = tid; i < w_first; i += 256) part += __popcll(words[row0 + i]);
  } else {
    const int64_t n = row0 + w_first;
    for (int64_t i = tid; i < n; i += 256) part += __popcll(words[i]);
  }
  const int base = block_sum_256(part, red);

  int pc[4], wave_total = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) { pc[i] = __popcll(mine[i]); wave_total += pc[i]; }
  if (ln == 0) wsum[wv] = wave_total;
  __syncthreads();
  int off = base;
  for (int i = 0; i < wv; ++i) off += wsum[i];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const u64 x = mine[i];
    if ((x >> ln) & 1ull) {
      const int pos = off + __popcll(x & ((1ull << ln) - 1ull));
      const int coord = (w_first + wv * 4 + i) * 64 + ln;
      if (pos < cap) {
        idx[pos] = coord;
        if (bits) bits[pos] = occ[(int64_t)s * npit + coord];
      }
    }
    off += pc[i];
  }
  if (tid == 0) {
    if (c == 0) seg_ptr[s] = base;
    if (s == nseg - 1 && c == (int)gridDim.x - 1) {
      const int total = base + wsum[0] + wsum[1] + wsum[2] + wsum[3];
      seg_ptr[nseg] = total;
      if (status) *status = total_items - total;
    }
  }
}

// total number of set bits of the bitmap (CoverAlgo): one atomic per workgroup into a zeroed counter
__global__ void __launch_bounds__(256)
k_count_bits(const u64* __restrict__ words, int64_t nwords, int32_t* __restrict__ count) {
  __shared__ int red[4];
  int part = 0;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < nwords; i += (int64_t)gridDim.x * 256)
    part += __popcll(words[i]);
  const int total = block_sum_256(part, red);
  if (threadIdx.x == 0 && total != 0) atomicAdd(count, total);
}

__global__ void k_fill_i32(int32_t* p, int n, int32_t v) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

struct Layout {
  int nseg, npit, W;
  size_t words_bytes, occ_bytes, cnt_bytes;
};

Layout make_layout(int rows, int cols, int mt_rows, int mt_cols, int pit_dim, int want_bits) {
  Layout L;
  const int gr = rows / mt_rows, gc = cols / mt_cols;
  L.nseg = pit_dim == 0 ? gc : gr;
  L.npit = pit_dim == 0 ? gr : gc;
  L.W = (L.npit + 63) / 64;
  L.words_bytes = (size_t)L.nseg * L.W * 8;
  L.occ_bytes = want_bits ? (((size_t)L.nseg * L.npit * 4 + 15) & ~(size_t)15) : 0;
  L.cnt_bytes = ((size_t)L.nseg * 4 + 15) & ~(size_t)15;
  return L;
}

// k_emit_chunked serves segments of up to 1024 words (segment number in the grid's y), k_emit (one
// workgroup per segment) the rest.
inline bool use_chunked_emit(const Layout& L) { return L.W <= 1024 && L.nseg <= 65535; }
// many earlier words per workgroup => precompute per-segment counts in a separate launch
inline bool use_seg_count(const Layout& L) { return (int64_t)L.nseg * L.W > (use_chunked_emit(L) ? 16384 : 65536); }

int launch_emit(const Layout& L, const u64* words, int32_t* cnt, const uint32_t* occ, const pit_index* out,
                int total_items, int32_t* status, hipStream_t st) {
  if (L.nseg == 0 || L.npit == 0) {
    const int n = L.nseg + 1;
    hipLaunchKernelGGL(k_fill_i32, dim3((n + 255) / 256), dim3(256), 0, st, out->seg_ptr, n, 0);
    PIT_LAUNCH_CHECK();
    if (status) {
      hipLaunchKernelGGL(k_fill_i32, dim3(1), dim3(64), 0, st, status, 1, total_items);
      PIT_LAUNCH_CHECK();
    }
    return PIT_OK;
  }
  const int32_t* cnt_arg = nullptr;
  if (use_seg_count(L)) {
    hipLaunchKernelGGL(k_seg_count, dim3((L.nseg + 3) / 4), dim3(256), 0, st, words, L.nseg, L.W, cnt);
    PIT_LAUNCH_CHECK();
    cnt_arg = cnt;
  }
  if (use_chunked_emit(L)) {
    hipLaunchKernelGGL(k_emit_chunked, dim3((unsigned)ceil_div(L.W, EMIT_CH), (unsigned)L.nseg), dim3(256), 0, st,
                       words, cnt_arg, occ, L.nseg, L.npit, L.W, out->cap, total_items, out->seg_ptr, out->idx,
                       out->bits, status);
  } else {
    hipLaunchKernelGGL(k_emit, dim3(L.nseg), dim3(256), 0, st, words, cnt_arg, occ, L.nseg, L.npit, L.W, out->cap,
                       total_items, out->seg_ptr, out->idx, out->bits, status);
  }
  PIT_LAUNCH_CHECK();
  return PIT_OK;
}

}  // namespace
}  // namespace pit

using namespace pit;

// pass 1: the bitmap of non-empty micro-tiles (and, if occ != nullptr, their element occupancy)
static int launch_bitmap(const Layout& L, const void* d_src, int esize, int rows, int cols, int64_t ld,
                         int mt_rows, int mt_cols, int pit_dim, bool want_bits, u64* words, uint32_t* occ,
                         hipStream_t st) {
  const int64_t mt_bytes = (int64_t)mt_cols * esize;
  const int64_t row_bytes = (int64_t)cols * esize;
  const bool vec_ok = aligned(d_src, 16) && (ld * esize) % 16 == 0 && row_bytes % 16 == 0 && row_bytes < (1ll << 31);
  if (pit_dim == 0 && mt_rows == 1 && !want_bits && vec_ok && mt_bytes >= 16 && mt_bytes <= 1024 &&
      (mt_bytes & (mt_bytes - 1)) == 0) {
    const int lpm = (int)(mt_bytes / 16);
    dim3 grid((unsigned)ceil_div(row_bytes, 1024), (unsigned)ceil_div(rows, 64));
    if (esize == 1)      hipLaunchKernelGGL(k_bitmap_rows<1>, grid, dim3(256), 0, st, d_src, ld * esize, rows, (int)row_bytes, lpm, L.nseg, L.W, words);
    else if (esize == 2) hipLaunchKernelGGL(k_bitmap_rows<2>, grid, dim3(256), 0, st, d_src, ld * esize, rows, (int)row_bytes, lpm, L.nseg, L.W, words);
    else                 hipLaunchKernelGGL(k_bitmap_rows<4>, grid, dim3(256), 0, st, d_src, ld * esize, rows, (int)row_bytes, lpm, L.nseg, L.W, words);
  } else if (pit_dim == 1 && mt_cols == 1 && esize == 1 && vec_ok && cols % 16 == 0) {
    const int chunks = (L.W * 64 + 1023) / 1024;
    const int64_t waves = (int64_t)L.nseg * chunks;
    hipLaunchKernelGGL(k_bitmap_cols_u8, dim3((unsigned)ceil_div(waves, 4)), dim3(256), 0, st,
                       reinterpret_cast<const uint8_t*>(d_src), ld, mt_rows, cols, L.nseg, L.npit, L.W, words, occ);
  } else {
    const int64_t waves = (int64_t)L.nseg * L.W;
    dim3 grid((unsigned)ceil_div(waves, 4));
    if (esize == 1)      hipLaunchKernelGGL(k_bitmap_generic<1>, grid, dim3(256), 0, st, d_src, ld, mt_rows, mt_cols, pit_dim, L.nseg, L.npit, L.W, words, occ);
    else if (esize == 2) hipLaunchKernelGGL(k_bitmap_generic<2>, grid, dim3(256), 0, st, d_src, ld, mt_rows, mt_cols, pit_dim, L.nseg, L.npit, L.W, words, occ);
    else                 hipLaunchKernelGGL(k_bitmap_generic<4>, grid, dim3(256), 0, st, d_src, ld, mt_rows, mt_cols, pit_dim, L.nseg, L.npit, L.W, words, occ);
  }
  PIT_LAUNCH_CHECK();
  return PIT_OK;
}

extern "C" size_t pit_build_index_workspace(int rows, int cols, int mt_rows, int mt_cols, int pit_dim, int want_bits) {
  if (rows < 0 || cols < 0 || mt_rows <= 0 || mt_cols <= 0 || (pit_dim != 0 && pit_dim != 1)) return 0;
  if (rows % mt_rows || cols % mt_cols) return 0;
  const Layout L = make_layout(rows, cols, mt_rows, mt_cols, pit_dim, want_bits);
  return L.words_bytes + L.occ_bytes + L.cnt_bytes + 64;
}

extern "C" int pit_build_index(const void* d_src, int dt, int rows, int cols, int64_t ld,
                               int mt_rows, int mt_cols, int pit_dim,
                               const pit_index* out, void* d_ws, size_t ws_bytes, pit_stream stream) {
  const int esize = dtype_size(dt);
  if (!out || !out->seg_ptr || esize == 0 || (pit_dim != 0 && pit_dim != 1)) return PIT_EINVAL;
  if (rows < 0 || cols < 0 || mt_rows <= 0 || mt_cols <= 0) return PIT_ESHAPE;
  if (rows % mt_rows || cols % mt_cols) return PIT_ESHAPE;
  if (ld < cols) return PIT_EINVAL;
  const bool want_bits = out->bits != nullptr;
  if (want_bits && (int64_t)mt_rows * mt_cols > 32) return PIT_EINVAL;
  const Layout L = make_layout(rows, cols, mt_rows, mt_cols, pit_dim, want_bits);
  if (out->nseg != L.nseg) return PIT_ECAPACITY;
  if ((int64_t)out->cap < (int64_t)L.nseg * L.npit) return PIT_ECAPACITY;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  if (L.nseg == 0 || L.npit == 0) return launch_emit(L, nullptr, nullptr, nullptr, out, 0, nullptr, st);
  if (!d_src || !out->idx || !d_ws || !aligned(d_ws, 8) || !aligned(d_src, esize)) return PIT_EINVAL;
  if (ws_bytes < pit_build_index_workspace(rows, cols, mt_rows, mt_cols, pit_dim, want_bits)) return PIT_ECAPACITY;

  char* ws = reinterpret_cast<char*>(d_ws);
  u64* words = reinterpret_cast<u64*>(ws);
  uint32_t* occ = want_bits ? reinterpret_cast<uint32_t*>(ws + L.words_bytes) : nullptr;
  int32_t* cnt = reinterpret_cast<int32_t*>(ws + L.words_bytes + L.occ_bytes);

  const int rc = launch_bitmap(L, d_src, esize, rows, cols, ld, mt_rows, mt_cols, pit_dim, want_bits, words, occ, st);
  if (rc != PIT_OK) return rc;
  return launch_emit(L, words, cnt, occ, out, 0, nullptr, st);
}

// The count does not depend on the PIT-axis; byte masks with column-shaped micro-tiles take the
// layout whose bitmap pass reads rows of the mask with 16-byte loads.
static int cover_count_axis(int esize, int mt_rows, int mt_cols) { return (esize == 1 && mt_cols == 1 && mt_rows > 1) ? 1 : 0; }

extern "C" size_t pit_cover_count_workspace(int rows, int cols, int mt_rows, int mt_cols) {
  return std::max(pit_build_index_workspace(rows, cols, mt_rows, mt_cols, 0, 0),
                  pit_build_index_workspace(rows, cols, mt_rows, mt_cols, 1, 0));
}

extern "C" int pit_cover_count(const void* d_src, int dt, int rows, int cols, int64_t ld, int mt_rows, int mt_cols,
                               int32_t* d_count, void* d_ws, size_t ws_bytes, pit_stream stream) {
  const int esize = dtype_size(dt);
  if (!d_count || esize == 0) return PIT_EINVAL;
  if (rows < 0 || cols < 0 || mt_rows <= 0 || mt_cols <= 0) return PIT_ESHAPE;
  if (rows % mt_rows || cols % mt_cols) return PIT_ESHAPE;
  if (ld < cols) return PIT_EINVAL;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  hipLaunchKernelGGL(k_fill_i32, dim3(1), dim3(64), 0, st, d_count, 1, 0);
  PIT_LAUNCH_CHECK();
  const int pit_dim = cover_count_axis(esize, mt_rows, mt_cols);
  const Layout L = make_layout(rows, cols, mt_rows, mt_cols, pit_dim, 0);
  if (L.nseg == 0 || L.npit == 0) return PIT_OK;
  if (!d_src || !d_ws || !aligned(d_ws, 8) || !aligned(d_src, esize)) return PIT_EINVAL;
  if (ws_bytes < pit_cover_count_workspace(rows, cols, mt_rows, mt_cols)) return PIT_ECAPACITY;
  u64* words = reinterpret_cast<u64*>(d_ws);
  const int rc = launch_bitmap(L, d_src, esize, rows, cols, ld, mt_rows, mt_cols, pit_dim, false, words, nullptr, st);
  if (rc != PIT_OK) return rc;
  const int64_t nwords = (int64_t)L.nseg * L.W;
  const unsigned blocks = (unsigned)std::min<int64_t>(ceil_div(nwords, 256), 1024);
  hipLaunchKernelGGL(k_count_bits, dim3(blocks), dim3(256), 0, st, words, nwords, d_count);
  PIT_LAUNCH_CHECK();
  return PIT_OK;
}

extern "C" int pit_select_kernel(const pit_kernel_candidate* cand, int ncand, const int64_t* num_tiles,
                                 const int64_t* grid_tiles, int nsamples, double* cost_out, int* best_out) {
  if (!cand || !best_out || ncand <= 0 || nsamples < 0) return PIT_EINVAL;
  if (nsamples > 0 && (!num_tiles || !grid_tiles)) return PIT_EINVAL;
  int best = -1;
  double best_cost = 0.0;
  for (int j = 0; j < ncand; ++j) {
    if (!(cand[j].tile_cost >= 0.0) || cand[j].mt_rows <= 0 || cand[j].mt_cols <= 0) return PIT_EINVAL;
    double cost = 0.0;
    for (int i = 0; i < nsamples; ++i) {
      const int64_t n = cand[j].dense ? grid_tiles[(int64_t)i * ncand + j] : num_tiles[(int64_t)i * ncand + j];
      if (n < 0) return PIT_EINVAL;
      cost += (double)n * cand[j].tile_cost;
    }
    if (cost_out) cost_out[j] = cost;
    if (best < 0 || cost < best_cost) { best = j; best_cost = cost; }
  }
  *best_out = best;
  return PIT_OK;
}

extern "C" size_t pit_build_route_index_workspace(int T, int E) {
  if (T < 0 || E <= 0) return 0;
  const Layout L = make_layout(T, E, 1, 1, 0, 0);
  return L.words_bytes + L.cnt_bytes + 64;
}

extern "C" int pit_build_route_index(const int32_t* d_expert_id, int T, int E, const pit_index* out,
                                     int32_t* d_status, void* d_ws, size_t ws_bytes, pit_stream stream) {
  if (!out || !out->seg_ptr) return PIT_EINVAL;
  if (T < 0 || E <= 0) return PIT_ESHAPE;
  if (out->nseg != E || out->cap < T) return PIT_ECAPACITY;
  if (out->bits) return PIT_EINVAL;
  const Layout L = make_layout(T, E, 1, 1, 0, 0);
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  if (T == 0) return launch_emit(L, nullptr, nullptr, nullptr, out, 0, d_status, st);
  if (!d_expert_id || !out->idx || !d_ws || !aligned(d_ws, 8)) return PIT_EINVAL;
  if (ws_bytes < pit_build_route_index_workspace(T, E)) return PIT_ECAPACITY;
  char* ws = reinterpret_cast<char*>(d_ws);
  u64* words = reinterpret_cast<u64*>(ws);
  int32_t* cnt = reinterpret_cast<int32_t*>(ws + L.words_bytes);
  hipLaunchKernelGGL(k_bitmap_route, dim3((L.W + 3) / 4), dim3(256), 0, st, d_expert_id, T, E, L.W, words);
  PIT_LAUNCH_CHECK();
  return launch_emit(L, words, cnt, nullptr, out, T, d_status, st);
}
