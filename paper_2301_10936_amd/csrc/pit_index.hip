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
// pass 1, fast path B: PIT-axis = columns, byte mask, micro-tile = mt_rows x 1, with the element
// occupancy of every micro-tile.  A workgroup covers one segment (mt_rows rows) x 1024 columns; a
// lane owns 16 columns and keeps one occupancy word per column (bit r = row r of the micro-tile is
// non-zero).  The four waves split the rows (wave w takes rows w, w + 4, ...), so that a 32-row
// micro-tile is one batch of 8 row loads per wave; their partial words are OR-ed through LDS.
// ----------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
k_bitmap_cols_u8(const uint8_t* __restrict__ src, int64_t ld, int mt_rows, int cols, int nseg, int npit, int W,
                 u64* __restrict__ words, uint32_t* __restrict__ occ) {
  __shared__ uint4 part[3][4][64];
  const int chunks = (W * 64 + 1023) / 1024;
  const int s = blockIdx.x / chunks, ch = blockIdx.x % chunks;
  const int wv = threadIdx.x >> 6, ln = lane_id();
  const int c0 = ch * 1024 + ln * 16;
  uint32_t o[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) o[j] = 0;
  if (c0 < cols) {
    const uint8_t* p = src + (int64_t)s * mt_rows * ld + c0;
    for (int r0 = wv; r0 < mt_rows; r0 += 32) {
      uint4 v[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        v[i] = make_uint4(0, 0, 0, 0);
        if (r0 + 4 * i < mt_rows) v[i] = *reinterpret_cast<const uint4*>(p + (int64_t)(r0 + 4 * i) * ld);
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int r = r0 + 4 * i;
        const uint32_t d[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
        const uint32_t rb = r < 32 ? (1u << (r & 31)) : 0x80000000u;  // rows >= 32 only feed the flag
#pragma unroll
        for (int j = 0; j < 16; ++j)
          if ((d[j >> 2] >> ((j & 3) * 8)) & 0xFFu) o[j] |= rb;
      }
    }
  }
  if (wv > 0) {
#pragma unroll
    for (int q = 0; q < 4; ++q) part[wv - 1][q][ln] = make_uint4(o[4 * q], o[4 * q + 1], o[4 * q + 2], o[4 * q + 3]);
  }
  __syncthreads();
  if (wv != 0 || c0 >= W * 64) return;
#pragma unroll
  for (int w = 0; w < 3; ++w)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const uint4 t = part[w][q][ln];
      o[4 * q] |= t.x; o[4 * q + 1] |= t.y; o[4 * q + 2] |= t.z; o[4 * q + 3] |= t.w;
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
// pass 1, fast path C: any micro-tile of mt_rows x mt_bytes with mt_bytes a power of two up to
// 1 KiB, either PIT-axis, no occupancy bits.  A workgroup streams 64 rows x 1 KiB exactly like
// path A (16 coalesced row loads of 16 B per lane in flight per wave); what differs is how the
// per-lane results become bitmap bits.
//   F       flags per lane: 16 / mt_bytes for micro-tiles narrower than one load, else 1 (then
//           lpm = mt_bytes / 16 lanes share a micro-tile and a ballot joins them)
//   rows    the rows of one micro-tile are OR-ed in registers and flushed at its last row; the
//           flush ORs the tile flags into an LDS bit matrix of the workgroup's micro-tiles, laid
//           out the way the bitmap wants them: PIT_DIM 1 -> [tile row][tile column bits],
//           PIT_DIM 0 -> [tile column][tile row bits]
//   output  direct != 0: the workgroup owns whole 32/64-bit units of the bitmap and stores them;
//           direct == 0: micro-tiles or bitmap units are shared between workgroups, which then
//           OR their parts into a bitmap the host has cleared (OR commutes: the result does not
//           depend on the order of arrival).
// ----------------------------------------------------------------------------------------------
template <int ESIZE, int F>
__device__ __forceinline__ uint32_t tile_flags(const uint4& v) {
  constexpr uint32_t M = ESIZE == 1 ? 0xFFFFFFFFu : (ESIZE == 2 ? 0x7FFF7FFFu : 0x7FFFFFFFu);
  const uint32_t d[4] = {v.x & M, v.y & M, v.z & M, v.w & M};
  uint32_t r = 0;
  if (F == 1) {
    r = (d[0] | d[1] | d[2] | d[3]) != 0 ? 1u : 0u;
  } else if (F == 2) {
    r = ((d[0] | d[1]) != 0 ? 1u : 0u) | ((d[2] | d[3]) != 0 ? 2u : 0u);
  } else if (F == 4) {
#pragma unroll
    for (int k = 0; k < 4; ++k) r |= (d[k] != 0 ? 1u : 0u) << k;
  } else if (F == 8) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      r |= ((d[k] & 0xFFFFu) != 0 ? 1u : 0u) << (2 * k);
      r |= ((d[k] >> 16) != 0 ? 1u : 0u) << (2 * k + 1);
    }
  } else {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      // bit 7 of every non-zero byte, then the four of them gathered into bits 24..27
      const uint32_t t = (((d[k] & 0x7F7F7F7Fu) + 0x7F7F7F7Fu) | d[k]) & 0x80808080u;
      r |= ((((t >> 7) * 0x01020408u) >> 24) & 0xFu) << (4 * k);
    }
  }
  return r;
}

template <int ESIZE, int F, int PIT_DIM>
__global__ void __launch_bounds__(256)
k_bitmap_tiles(const void* __restrict__ src, int64_t ld_bytes, int rows, int row_bytes, int mt_rows, int lpm,
               int nseg, int W, int direct, uint32_t* __restrict__ words32) {
  __shared__ uint32_t T[2048];   // PIT_DIM 1: [64 tile rows][32 x 32 column bits]; PIT_DIM 0: [1024 tile columns][2 x 32 row bits]
  const int tid = threadIdx.x, wv = tid >> 6, ln = lane_id();
  const int strip = blockIdx.x;
  const int rblk = blockIdx.y * 64;
  const int rbase = rblk + wv * 16;
  const int64_t byte0 = (int64_t)strip * 1024 + ln * 16;
  const char* base = reinterpret_cast<const char*>(src) + byte0;
  const bool col_ok = byte0 < row_bytes;
  uint4 v[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    v[i] = make_uint4(0, 0, 0, 0);
    if (col_ok && rbase + i < rows) v[i] = *reinterpret_cast<const uint4*>(base + (int64_t)(rbase + i) * ld_bytes);
  }
  for (int i = tid; i < 2048; i += 256) T[i] = 0;
  __syncthreads();

  const int nb = F == 1 ? 64 / lpm : 64 * F;            // micro-tile columns per strip
  const u64 lmask = lpm >= 64 ? ~0ull : ((1ull << lpm) - 1ull);
  const int sh = (ln < nb ? ln : 0) * lpm;
  const int tr_first = rblk / mt_rows;
  int trl = rbase / mt_rows - tr_first;
  int rem = rbase % mt_rows;
  uint4 cur = make_uint4(0, 0, 0, 0);
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    if (rbase + i < rows) {
      cur.x |= v[i].x; cur.y |= v[i].y; cur.z |= v[i].z; cur.w |= v[i].w;
      ++rem;
      if (rem == mt_rows || i == 15) {
        const uint32_t fl = tile_flags<ESIZE, F>(cur);
        if (F == 1) {
          const u64 b = __ballot(fl != 0);
          if (b != 0) {
            const bool bit = ln < nb && ((b >> sh) & lmask) != 0;
            if (PIT_DIM == 1) {
              const u64 m = __ballot(bit);
              if (ln == 0) {
                atomicOr(&T[trl * 32], (uint32_t)m);
                if (m >> 32) atomicOr(&T[trl * 32 + 1], (uint32_t)(m >> 32));
              }
            } else if (bit) {
              atomicOr(&T[ln * 2 + (trl >> 5)], 1u << (trl & 31));
            }
          }
        } else if (fl != 0) {
          if (PIT_DIM == 1) {
            atomicOr(&T[trl * 32 + ((ln * F) >> 5)], fl << ((ln * F) & 31));
          } else {
#pragma unroll
            for (int q = 0; q < F; ++q)
              if ((fl >> q) & 1u) atomicOr(&T[(ln * F + q) * 2 + (trl >> 5)], 1u << (trl & 31));
          }
        }
        cur = make_uint4(0, 0, 0, 0);
      }
      if (rem == mt_rows) { rem = 0; ++trl; }
    }
  }
  __syncthreads();

  if (PIT_DIM == 1) {
    const int row_end = min(rows, rblk + 64);
    const int ntr = (row_end - 1) / mt_rows - tr_first + 1;
    if (nb >= 32) {
      const int nu = nb / 32;
      // with direct stores the last strip also clears the padding of the segment's last word
      const int nux = nu + ((direct && strip == (int)gridDim.x - 1) ? 2 : 0);
      for (int i = tid; i < ntr * nux; i += 256) {
        const int t = i / nux, j = i % nux;
        const int64_t u = (int64_t)strip * nu + j;
        if (u < 2 * (int64_t)W) {
          const uint32_t val = j < nu ? T[t * 32 + j] : 0u;
          uint32_t* p = words32 + (int64_t)(tr_first + t) * W * 2 + u;
          if (direct) *p = val;
          else if (val) atomicOr(p, val);
        }
      }
    } else {
      const int64_t bitpos = (int64_t)strip * nb;
      for (int t = tid; t < ntr; t += 256) {
        const uint32_t val = T[t * 32];
        if (val) atomicOr(words32 + (int64_t)(tr_first + t) * W * 2 + (bitpos >> 5), val << (bitpos & 31));
      }
    }
  } else {
    for (int tc = tid; tc < nb; tc += 256) {
      const int64_t seg = (int64_t)strip * nb + tc;
      if (seg >= nseg) continue;
      const uint32_t lo = T[tc * 2], hi = T[tc * 2 + 1];
      if (direct) {      // mt_rows == 1: the 64 rows of this workgroup are one whole word
        uint32_t* p = words32 + (seg * W + blockIdx.y) * 2;
        *reinterpret_cast<uint2*>(p) = make_uint2(lo, hi);
      } else {
        const u64 x = (u64)lo | ((u64)hi << 32);
        if (x == 0) continue;
        const int w = tr_first >> 6, off = tr_first & 63;
        const u64 a = x << off, b = off ? (x >> (64 - off)) : 0ull;
        uint32_t* p = words32 + (seg * W + w) * 2;
        if ((uint32_t)a) atomicOr(p, (uint32_t)a);
        if (a >> 32) atomicOr(p + 1, (uint32_t)(a >> 32));
        if ((uint32_t)b) atomicOr(p + 2, (uint32_t)b);
        if (b >> 32) atomicOr(p + 3, (uint32_t)(b >> 32));
      }
    }
  }
}

// ----------------------------------------------------------------------------------------------
// Producer with the bitmap for free: Xt[k][m] = ReLU(H[m][k]) and, per block of 128 tokens, one
// bit per channel "some activation is non-zero" (the bitmap of Xt at 1 x 128 micro-tiles, PIT-axis
// = channels), in one pass over H.
// A workgroup handles 128 tokens x 128 channels, wave w the channels 32 w .. 32 w + 31.  Lane l
// loads 8 token rows x 16 B (tokens 8 (l % 16) + j, channels 8 (l / 16) ..+7 of the wave's 32), i.e.
// an 8 x 8 block that it transposes in registers; its 8 stores then put 8 consecutive tokens of
// one channel each, and 16 lanes cover the 256 contiguous bytes of a channel's 128 tokens.
// Across the four waves a token row is read as 256 contiguous bytes.
// ----------------------------------------------------------------------------------------------
template <bool BF>
__device__ __forceinline__ uint32_t relu_pair(uint32_t v) {
  // per 16-bit half: negative and not NaN -> +0 (this includes -0 and -Inf); everything else unchanged
  constexpr uint32_t INF = BF ? 0x7F80u : 0x7C00u;
  const uint32_t lo = v & 0xFFFFu, hi = v >> 16;
  const uint32_t rl = ((lo & 0x8000u) && (lo & 0x7FFFu) <= INF) ? 0u : lo;
  const uint32_t rh = ((hi & 0x8000u) && (hi & 0x7FFFu) <= INF) ? 0u : hi;
  return rl | (rh << 16);
}

template <bool BF>
__global__ void __launch_bounds__(256)
k_relu_transpose_bitmap(const void* __restrict__ H, int64_t ldh_bytes, int tokens, int channels,
                        void* __restrict__ Xt, int64_t ldxt_bytes, int W, uint32_t* __restrict__ words32) {
  const int wv = threadIdx.x >> 6, ln = lane_id();
  const int tg = ln & 15, cg = ln >> 4;
  const int t0 = blockIdx.y * 128 + 8 * tg;                       // first of this lane's 8 tokens
  const int c0 = blockIdx.x * 128 + wv * 32 + 8 * cg;             // first of this lane's 8 channels
  const bool ok = c0 < channels;                                  // channels % 8 == 0: all 8 or none
  uint4 r[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    r[j] = make_uint4(0, 0, 0, 0);
    if (ok) r[j] = *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(H) + (int64_t)(t0 + j) * ldh_bytes + (int64_t)c0 * 2);
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    r[j].x = relu_pair<BF>(r[j].x); r[j].y = relu_pair<BF>(r[j].y);
    r[j].z = relu_pair<BF>(r[j].z); r[j].w = relu_pair<BF>(r[j].w);
  }
  // 8 x 8 transpose of 16-bit elements: o[c] = tokens t0 .. t0 + 7 of channel c0 + c
  uint4 o[8];
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
    o[2 * i] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
    o[2 * i + 1] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
  }
  uint32_t flags = 0;
#pragma unroll
  for (int c = 0; c < 8; ++c) {
    if (ok) *reinterpret_cast<uint4*>(reinterpret_cast<char*>(Xt) + (int64_t)(c0 + c) * ldxt_bytes + (int64_t)t0 * 2) = o[c];
    flags |= (((o[c].x | o[c].y | o[c].z | o[c].w) & 0x7FFF7FFFu) != 0 ? 1u : 0u) << c;
  }
  // OR over the 16 lanes that share the channels, then the four channel groups side by side
  flags |= __shfl_xor(flags, 1); flags |= __shfl_xor(flags, 2);
  flags |= __shfl_xor(flags, 4); flags |= __shfl_xor(flags, 8);
  const uint32_t word = (uint32_t)__shfl(flags, 0) | ((uint32_t)__shfl(flags, 16) << 8) |
                        ((uint32_t)__shfl(flags, 32) << 16) | ((uint32_t)__shfl(flags, 48) << 24);
  const int u = blockIdx.x * 4 + wv;                              // 32-bit unit inside the segment's bitmap row
  if (ln == 0 && u < 2 * W) words32[((int64_t)blockIdx.y * W) * 2 + u] = word;
}

// ----------------------------------------------------------------------------------------------
// pass 1 for routing decisions: segment e, bit t  <=>  expert_id[t] == e
// ----------------------------------------------------------------------------------------------
// A token whose id is outside [0, E) is listed nowhere; if zero_rows is given, its row of that matrix (the
// output of the layer that the index is built for) is cleared here, by the whole wave, so that the caller
// need not clear the matrix for the sake of tokens that normally do not exist.
__global__ void __launch_bounds__(256)
k_bitmap_route(const int32_t* __restrict__ expert_id, int T, int E, int W, u64* __restrict__ words,
               char* __restrict__ zero_rows, int64_t zero_ld_bytes, int zero_row_bytes) {
  const int w = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (w >= W) return;
  const int t = w * 64 + lane_id();
  const int e = t < T ? expert_id[t] : -1;
  if (zero_rows != nullptr) {
    u64 bad = __ballot(t < T && (e < 0 || e >= E));
    while (bad) {
      const int l = __builtin_ctzll(bad);
      bad &= bad - 1;
      char* row = zero_rows + (int64_t)(w * 64 + l) * zero_ld_bytes;
      for (int b = lane_id() * 16; b < zero_row_bytes; b += 64 * 16) *reinterpret_cast<uint4*>(row + b) = make_uint4(0, 0, 0, 0);
    }
  }
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
// Routing decisions of up to 8192 tokens over up to 64 experts: the whole index in ONE launch by one workgroup
// (a stable counting sort without atomics; the same lists as bitmap pass + ordered emit give).
//   1. a wave takes 64 consecutive tokens; six ballots over the bits of the expert id give every lane the set
//      of lanes with its expert, hence its rank among them and, in the first of them, their number:
//      tab[chunk][expert]
//   2. exclusive prefix of tab over the chunks (16 runs of chunks per expert, then the runs), totals per expert,
//      exclusive prefix over the experts = seg_ptr
//   3. token t goes to seg_ptr[e] + (tokens of e in earlier chunks) + (rank in its chunk)
// Tokens with an id outside [0, E) are listed nowhere, counted in *status, and their rows of zero_rows (if given)
// are cleared, as in k_bitmap_route.
// ----------------------------------------------------------------------------------------------
constexpr int ROUTE_ONE_MAX_T = 8192, ROUTE_ONE_CHUNKS = ROUTE_ONE_MAX_T / 64;
__global__ void __launch_bounds__(1024)
k_route_index_one(const int32_t* __restrict__ expert_id, int T, int E, int32_t* __restrict__ seg_ptr,
                  int32_t* __restrict__ idx, int32_t* __restrict__ status,
                  char* __restrict__ zero_rows, int64_t zero_ld_bytes, int zero_row_bytes) {
  __shared__ int tab[ROUTE_ONE_CHUNKS][64];
  __shared__ int run_sum[16][64];
  __shared__ int base[64];
  __shared__ int bad_s[16];
  const int tid = threadIdx.x, wv = tid >> 6, ln = tid & 63;
  const int C = (T + 63) >> 6;
  const int per = (C + 15) >> 4;                  // chunks per run; run g = chunks g * per .. g * per + per - 1
  int my_e[ROUTE_ONE_CHUNKS / 16], my_rank[ROUTE_ONE_CHUNKS / 16];
  int nbad = 0;
  // all of this wave's expert ids are requested before the first is used (unconditional loads at clamped
  // positions: one round trip to memory instead of one per chunk)
  int raw[ROUTE_ONE_CHUNKS / 16];
#pragma unroll
  for (int j = 0; j < ROUTE_ONE_CHUNKS / 16; ++j) raw[j] = expert_id[min((wv + 16 * j) * 64 + ln, T - 1)];
#pragma unroll
  for (int j = 0; j < ROUTE_ONE_CHUNKS / 16; ++j) {
    const int c = wv + 16 * j;
    my_e[j] = -1; my_rank[j] = 0;
    if (c >= C) continue;                         // (uniform per wave)
    const int t = c * 64 + ln;
    const int e = t < T ? raw[j] : -1;
    const bool valid = e >= 0 && e < E;
    u64 bad = __ballot(t < T && !valid);
    nbad += __builtin_popcountll(bad);
    if (zero_rows != nullptr) {
      while (bad) {
        const int l = __builtin_ctzll(bad);
        bad &= bad - 1;
        char* row = zero_rows + (int64_t)(c * 64 + l) * zero_ld_bytes;
        for (int b = ln * 16; b < zero_row_bytes; b += 64 * 16) *reinterpret_cast<uint4*>(row + b) = make_uint4(0, 0, 0, 0);
      }
    }
    u64 same = __ballot(valid);
#pragma unroll
    for (int bit = 0; bit < 6; ++bit) {
      const bool on = (e >> bit) & 1;
      const u64 b = __ballot(on);
      same &= on ? b : ~b;
    }
    const int rank = __builtin_popcountll(same & ((1ull << ln) - 1ull));
    tab[c][ln] = 0;                               // (this wave owns row c of the table)
    __builtin_amdgcn_wave_barrier();
    if (valid) {
      my_e[j] = e; my_rank[j] = rank;
      if (rank == 0) tab[c][e] = __builtin_popcountll(same);
    }
  }
  if (ln == 0) bad_s[wv] = nbad;
  __syncthreads();
  {
    const int e = ln, g = wv;                     // 16 waves = 16 runs of chunks, lane = expert
    int sum = 0;
    for (int c = g * per; c < min(C, (g + 1) * per); ++c) {
      const int x = tab[c][e];
      tab[c][e] = sum;
      sum += x;
    }
    run_sum[g][e] = sum;
  }
  __syncthreads();
  if (wv == 0) {
    int total = 0;
#pragma unroll
    for (int g = 0; g < 16; ++g) {
      const int x = run_sum[g][ln];
      run_sum[g][ln] = total;
      total += x;
    }
    int inc = total;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int x = __shfl_up(inc, d);
      if (ln >= d) inc += x;
    }
    base[ln] = inc - total;
    if (ln < E) seg_ptr[ln] = inc - total;
    if (ln == E - 1) seg_ptr[E] = inc;           // (experts beyond E have no tokens: total = 0 there)
    if (ln == 0 && status != nullptr) {
      int nb = 0;
#pragma unroll
      for (int w = 0; w < 16; ++w) nb += bad_s[w];
      *status = nb;
    }
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < ROUTE_ONE_CHUNKS / 16; ++j) {
    const int c = wv + 16 * j;
    const int e = my_e[j];
    if (c < C && e >= 0) idx[base[e] + run_sum[c / per][e] + tab[c][e] + my_rank[j]] = c * 64 + ln;
  }
}

// ----------------------------------------------------------------------------------------------
// two-level counts (only used when there are many segments): cnt[s] = set bits of segment s,
// blk[b] = set bits of segments 16 b .. 16 b + 15.  The start of segment s is then the sum of
// blk[0 .. s / 16) and cnt[16 (s / 16) .. s): two short loads per workgroup instead of a scan pass.
// ----------------------------------------------------------------------------------------------
constexpr int SEG_BLK = 16;

__global__ void __launch_bounds__(256)
k_seg_count(const u64* __restrict__ words, int nseg, int W, int32_t* __restrict__ cnt, int32_t* __restrict__ blk) {
  __shared__ int wsum[4];
  const int wv = threadIdx.x >> 6, ln = lane_id();
  int wave_total = 0;
  const int s0 = blockIdx.x * SEG_BLK + wv * 4;
  if (W <= 64) {       // one word per lane: the 4 segments of the wave are requested at once
    u64 x[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) x[j] = (s0 + j < nseg && ln < W) ? words[(int64_t)(s0 + j) * W + ln] : 0ull;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int c = __popcll(x[j]);
#pragma unroll
      for (int d = 32; d >= 1; d >>= 1) c += __shfl_xor(c, d);
      if (ln == 0 && s0 + j < nseg) cnt[s0 + j] = c;
      wave_total += c;
    }
  } else {
    for (int j = 0; j < 4; ++j) {
      const int s = s0 + j;
      if (s >= nseg) break;
      int c = 0;
      for (int w = ln; w < W; w += 64) c += __popcll(words[(int64_t)s * W + w]);
#pragma unroll
      for (int d = 32; d >= 1; d >>= 1) c += __shfl_xor(c, d);
      if (ln == 0) cnt[s] = c;
      wave_total += c;
    }
  }
  if (ln == 0) wsum[wv] = wave_total;
  __syncthreads();
  if (threadIdx.x == 0) blk[blockIdx.x] = wsum[0] + wsum[1] + wsum[2] + wsum[3];
}

// this thread's share of the number of set bits ahead of segment s (sum over the workgroup = the start)
__device__ __forceinline__ int seg_start_part(const int32_t* __restrict__ cnt, const int32_t* __restrict__ blk, int s,
                                              int tid, int nthreads) {
  int part = 0;
  for (int i = tid; i < s / SEG_BLK; i += nthreads) part += blk[i];
  for (int i = tid; i < s % SEG_BLK; i += nthreads) part += cnt[s - s % SEG_BLK + i];
  return part;
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

// this thread's share of the set bits of words[0 .. n): eight loads in flight per thread
__device__ __forceinline__ int popcount_part(const u64* __restrict__ words, int64_t n, int tid) {
  int part = 0;
  int64_t i = tid;
  for (; i + 7 * 256 < n; i += 8 * 256) {
    u64 x[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) x[j] = words[i + j * 256];
#pragma unroll
    for (int j = 0; j < 8; ++j) part += __popcll(x[j]);
  }
  for (; i < n; i += 256) part += __popcll(words[i]);
  return part;
}

__global__ void __launch_bounds__(256)
k_emit(const u64* __restrict__ words, const int32_t* __restrict__ cnt, const int32_t* __restrict__ blk, const uint32_t* __restrict__ occ,
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
  if (cnt) {
    part = seg_start_part(cnt, blk, s, tid, 256);
  } else {
    part = popcount_part(words, (int64_t)s * W, tid);
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
k_emit_chunked(const u64* __restrict__ words, const int32_t* __restrict__ cnt, const int32_t* __restrict__ blk, const uint32_t* __restrict__ occ,
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
  if (cnt) {
    part = seg_start_part(cnt, blk, s, tid, 256);
    part += popcount_part(words + row0, w_first, tid);
  } else {
    part = popcount_part(words, row0 + w_first, tid);
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

// Same result for many short segments (at most 64 words each): one wave per segment, no LDS and no
// barrier.  Lane w holds word w; empty words are skipped.
__global__ void __launch_bounds__(256)
k_emit_short(const u64* __restrict__ words, const int32_t* __restrict__ cnt, const int32_t* __restrict__ blk,
             const uint32_t* __restrict__ occ, int nseg, int npit, int W, int cap, int total_items,
             int32_t* __restrict__ seg_ptr, int32_t* __restrict__ idx, uint32_t* __restrict__ bits,
             int32_t* __restrict__ status) {
  const int ln = lane_id();
  const int s = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (s >= nseg) return;
  const u64 word = ln < W ? words[(int64_t)s * W + ln] : 0ull;
  int base = seg_start_part(cnt, blk, s, ln, 64);
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) base += __shfl_xor(base, d);
  const int pc = __popcll(word);
  int inc = pc;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int t = __shfl_up(inc, d);
    if (ln >= d) inc += t;
  }
  const int off = base + inc - pc;
  const int total = __shfl(inc, 63);
  int maxpc = pc;
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) maxpc = max(maxpc, __shfl_xor(maxpc, d));
  if (maxpc <= 8) {    // sparse segment: every lane walks the few set bits of its own word
    u64 x = word;
    int pos = off;
    while (x) {
      const int c = ln * 64 + __ffsll((long long)x) - 1;
      x &= x - 1ull;
      if (pos < cap) {
        idx[pos] = c;
        if (bits) bits[pos] = occ[(int64_t)s * npit + c];
      }
      ++pos;
    }
  }
  u64 live = maxpc <= 8 ? 0ull : __ballot(word != 0ull);
  while (live) {
    const int i = __ffsll((long long)live) - 1;
    live &= live - 1ull;
    const u64 x = ((u64)(uint32_t)__shfl((int)(uint32_t)(word >> 32), i) << 32) | (u64)(uint32_t)__shfl((int)(uint32_t)word, i);
    const int o = __shfl(off, i);
    if ((x >> ln) & 1ull) {
      const int pos = o + __popcll(x & ((1ull << ln) - 1ull));
      const int c = i * 64 + ln;
      if (pos < cap) {
        idx[pos] = c;
        if (bits) bits[pos] = occ[(int64_t)s * npit + c];
      }
    }
  }
  if (ln == 0) {
    seg_ptr[s] = base;
    if (s == nseg - 1) {
      seg_ptr[nseg] = base + total;
      if (status) *status = total_items - (base + total);
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
  L.cnt_bytes = (((size_t)L.nseg + (size_t)(L.nseg + SEG_BLK - 1) / SEG_BLK) * 4 + 15) & ~(size_t)15;   // cnt[nseg], blk[ceil(nseg / SEG_BLK)]
  return L;
}

// k_emit_short (one wave per segment) serves many segments of at most 64 words, k_emit_chunked
// segments of up to 1024 words (segment number in the grid's y), k_emit (one workgroup per segment)
// the rest.
inline bool use_short_emit(const Layout& L) { return L.W <= 64 && L.nseg >= 1024; }
inline bool use_chunked_emit(const Layout& L) { return L.W <= 1024 && L.nseg <= 65535; }
// many earlier words per workgroup => two-level per-segment counts in a launch of their own
inline bool use_seg_count(const Layout& L) {
  return use_short_emit(L) || (int64_t)L.nseg * L.W > (use_chunked_emit(L) ? 16384 : 65536);
}

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
  const int32_t* blk_arg = nullptr;
  if (use_seg_count(L)) {
    int32_t* blk = cnt + L.nseg;
    hipLaunchKernelGGL(k_seg_count, dim3((L.nseg + SEG_BLK - 1) / SEG_BLK), dim3(256), 0, st, words, L.nseg, L.W, cnt, blk);
    PIT_LAUNCH_CHECK();
    cnt_arg = cnt;
    blk_arg = blk;
  }
  if (use_short_emit(L)) {
    hipLaunchKernelGGL(k_emit_short, dim3((L.nseg + 3) / 4), dim3(256), 0, st, words, cnt_arg, blk_arg, occ, L.nseg,
                       L.npit, L.W, out->cap, total_items, out->seg_ptr, out->idx, out->bits, status);
  } else if (use_chunked_emit(L)) {
    hipLaunchKernelGGL(k_emit_chunked, dim3((unsigned)ceil_div(L.W, EMIT_CH), (unsigned)L.nseg), dim3(256), 0, st,
                       words, cnt_arg, blk_arg, occ, L.nseg, L.npit, L.W, out->cap, total_items, out->seg_ptr, out->idx,
                       out->bits, status);
  } else {
    hipLaunchKernelGGL(k_emit, dim3(L.nseg), dim3(256), 0, st, words, cnt_arg, blk_arg, occ, L.nseg, L.npit, L.W,
                       out->cap, total_items, out->seg_ptr, out->idx, out->bits, status);
  }
  PIT_LAUNCH_CHECK();
  return PIT_OK;
}

}  // namespace
}  // namespace pit

using namespace pit;

// fast path C serves power-of-two micro-tile widths up to 1 KiB on 16-byte aligned rows
static bool tiles_path_ok(const Layout& L, int esize, int rows, int64_t row_bytes, int64_t mt_bytes, bool vec_ok) {
  return vec_ok && mt_bytes <= 1024 && (mt_bytes & (mt_bytes - 1)) == 0 && rows <= 65535 * 64 &&
         (int64_t)L.nseg * L.W * 2 < (1ll << 31) && esize <= mt_bytes;
}

template <int ESIZE, int F>
static void launch_tiles_ef(int pit_dim, dim3 grid, hipStream_t st, const void* src, int64_t ld_bytes, int rows,
                            int row_bytes, int mt_rows, int lpm, int nseg, int W, int direct, uint32_t* words32) {
  if (pit_dim == 0)
    hipLaunchKernelGGL((k_bitmap_tiles<ESIZE, F, 0>), grid, dim3(256), 0, st, src, ld_bytes, rows, row_bytes, mt_rows, lpm, nseg, W, direct, words32);
  else
    hipLaunchKernelGGL((k_bitmap_tiles<ESIZE, F, 1>), grid, dim3(256), 0, st, src, ld_bytes, rows, row_bytes, mt_rows, lpm, nseg, W, direct, words32);
}

template <int ESIZE>
static void launch_tiles_e(int f, int pit_dim, dim3 grid, hipStream_t st, const void* src, int64_t ld_bytes, int rows,
                           int row_bytes, int mt_rows, int lpm, int nseg, int W, int direct, uint32_t* words32) {
#define PIT_TILES_CASE(FF) launch_tiles_ef<ESIZE, FF>(pit_dim, grid, st, src, ld_bytes, rows, row_bytes, mt_rows, lpm, nseg, W, direct, words32)
  if (f == 1) PIT_TILES_CASE(1);
  else if (f == 2) PIT_TILES_CASE(2);
  else if (f == 4) PIT_TILES_CASE(4);
  else if constexpr (ESIZE <= 2) {      // f <= 16 / ESIZE
    if (f == 8) PIT_TILES_CASE(8);
    else if constexpr (ESIZE == 1) PIT_TILES_CASE(16);
  }
#undef PIT_TILES_CASE
}

static int launch_bitmap_tiles(const Layout& L, const void* d_src, int esize, int rows, int row_bytes, int64_t ld_bytes,
                               int mt_rows, int mt_bytes, int pit_dim, u64* words, hipStream_t st) {
  const int f = mt_bytes >= 16 ? 1 : 16 / mt_bytes;
  const int lpm = mt_bytes >= 16 ? mt_bytes / 16 : 1;
  const int nb = f == 1 ? 64 / lpm : 64 * f;
  // a workgroup (64 rows x 1 KiB) owns whole units of the bitmap in these cases only
  const int direct = pit_dim == 0 ? (mt_rows == 1) : (64 % mt_rows == 0 && nb % 32 == 0);
  uint32_t* words32 = reinterpret_cast<uint32_t*>(words);
  if (!direct) {
    const int n = (int)((int64_t)L.nseg * L.W * 2);
    hipLaunchKernelGGL(k_fill_i32, dim3((n + 255) / 256), dim3(256), 0, st, reinterpret_cast<int32_t*>(words32), n, 0);
    PIT_LAUNCH_CHECK();
  }
  dim3 grid((unsigned)ceil_div(row_bytes, 1024), (unsigned)ceil_div(rows, 64));
  if (esize == 1)      launch_tiles_e<1>(f, pit_dim, grid, st, d_src, ld_bytes, rows, row_bytes, mt_rows, lpm, L.nseg, L.W, direct, words32);
  else if (esize == 2) launch_tiles_e<2>(f, pit_dim, grid, st, d_src, ld_bytes, rows, row_bytes, mt_rows, lpm, L.nseg, L.W, direct, words32);
  else                 launch_tiles_e<4>(f, pit_dim, grid, st, d_src, ld_bytes, rows, row_bytes, mt_rows, lpm, L.nseg, L.W, direct, words32);
  PIT_LAUNCH_CHECK();
  return PIT_OK;
}

// A byte mask over rows (one column, 1 x 1 micro-tiles, a single segment: which token rows of a padded
// batch are valid) of at most 65536 rows is small enough for ONE workgroup to do everything, in one
// launch instead of two: thread t takes `per` consecutive rows (one 16-byte load when the mask is
// contiguous), counts them, a scan over the workgroup gives its position in the list, and it writes
// its row numbers there in ascending order.  Same result as the two-pass path, bit for bit.
__global__ void __launch_bounds__(1024) k_index_rowmask(const uint8_t* __restrict__ src, int64_t ld, int rows,
                                                        int32_t* __restrict__ seg_ptr, int32_t* __restrict__ idx) {
  __shared__ int s_wave[16];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int per = (rows + 1023) / 1024;          // <= 64
  const int r0 = tid * per;
  u64 flags = 0;
  if (ld == 1 && per == 16 && (reinterpret_cast<uintptr_t>(src) & 15) == 0 && r0 + 16 <= rows) {
    const uint4 v = *reinterpret_cast<const uint4*>(src + r0);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 16; ++i)
      if ((w[i >> 2] >> (8 * (i & 3))) & 0xffu) flags |= 1ull << i;
  } else {
    for (int i = 0; i < per; ++i)
      if (r0 + i < rows && src[(int64_t)(r0 + i) * ld] != 0) flags |= 1ull << i;
  }
  const int c = __popcll(flags);
  int inc = c;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int t = __shfl_up(inc, d);
    if (lane >= d) inc += t;
  }
  if (lane == 63) s_wave[wv] = inc;
  __syncthreads();
  int base = 0, total = 0;
#pragma unroll
  for (int w = 0; w < 16; ++w) {
    const int x = s_wave[w];
    if (w < wv) base += x;
    total += x;
  }
  int pos = base + inc - c;
  while (flags) {
    const int b = __builtin_ctzll(flags);
    flags &= flags - 1;
    idx[pos++] = r0 + b;
  }
  if (tid == 0) { seg_ptr[0] = 0; seg_ptr[1] = total; }
}

// pass 1: the bitmap of non-empty micro-tiles (and, if occ != nullptr, their element occupancy)
static int launch_bitmap(const Layout& L, const void* d_src, int esize, int rows, int cols, int64_t ld,
                         int mt_rows, int mt_cols, int pit_dim, bool want_bits, u64* words, uint32_t* occ,
                         hipStream_t st) {
  const int64_t mt_bytes = (int64_t)mt_cols * esize;
  const int64_t row_bytes = (int64_t)cols * esize;
  const bool vec_ok = aligned(d_src, 16) && (ld * esize) % 16 == 0 && row_bytes % 16 == 0 && row_bytes < (1ll << 31);
  if (pit_dim == 0 && mt_rows == 1 && !want_bits && vec_ok && mt_bytes >= 16 && mt_bytes <= 1024 &&
      (mt_bytes & (mt_bytes - 1)) == 0 && rows <= 65535 * 64) {          // (64 rows per workgroup, grid.y limit)
    const int lpm = (int)(mt_bytes / 16);
    dim3 grid((unsigned)ceil_div(row_bytes, 1024), (unsigned)ceil_div(rows, 64));
    if (esize == 1)      hipLaunchKernelGGL(k_bitmap_rows<1>, grid, dim3(256), 0, st, d_src, ld * esize, rows, (int)row_bytes, lpm, L.nseg, L.W, words);
    else if (esize == 2) hipLaunchKernelGGL(k_bitmap_rows<2>, grid, dim3(256), 0, st, d_src, ld * esize, rows, (int)row_bytes, lpm, L.nseg, L.W, words);
    else                 hipLaunchKernelGGL(k_bitmap_rows<4>, grid, dim3(256), 0, st, d_src, ld * esize, rows, (int)row_bytes, lpm, L.nseg, L.W, words);
  } else if (want_bits == false && tiles_path_ok(L, esize, rows, row_bytes, mt_bytes, vec_ok)) {
    return launch_bitmap_tiles(L, d_src, esize, rows, (int)row_bytes, ld * esize, mt_rows, (int)mt_bytes, pit_dim, words, st);
  } else if (pit_dim == 1 && mt_cols == 1 && esize == 1 && vec_ok && cols % 16 == 0) {
    const int chunks = (L.W * 64 + 1023) / 1024;
    hipLaunchKernelGGL(k_bitmap_cols_u8, dim3((unsigned)((int64_t)L.nseg * chunks)), dim3(256), 0, st,
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

  if (esize == 1 && cols == 1 && mt_rows == 1 && mt_cols == 1 && pit_dim == 0 && !want_bits && rows <= 65536) {
    hipLaunchKernelGGL(k_index_rowmask, dim3(1), dim3(1024), 0, st, reinterpret_cast<const uint8_t*>(d_src), ld, rows,
                       out->seg_ptr, out->idx);
    PIT_LAUNCH_CHECK();
    return PIT_OK;
  }

  char* ws = reinterpret_cast<char*>(d_ws);
  u64* words = reinterpret_cast<u64*>(ws);
  uint32_t* occ = want_bits ? reinterpret_cast<uint32_t*>(ws + L.words_bytes) : nullptr;
  int32_t* cnt = reinterpret_cast<int32_t*>(ws + L.words_bytes + L.occ_bytes);

  const int rc = launch_bitmap(L, d_src, esize, rows, cols, ld, mt_rows, mt_cols, pit_dim, want_bits, words, occ, st);
  if (rc != PIT_OK) return rc;
  return launch_emit(L, words, cnt, occ, out, 0, nullptr, st);
}

extern "C" size_t pit_relu_channel_major_index_workspace(int tokens, int channels) {
  if (tokens < 0 || channels < 0 || tokens % 128 || channels % 8) return 0;
  return pit_build_index_workspace(channels, tokens, 1, 128, 0, 0);
}

extern "C" int pit_relu_channel_major_index(const void* d_H, int64_t ldh, int tokens, int channels, int dt,
                                            void* d_Xt, int64_t ldxt, const pit_index* out,
                                            void* d_ws, size_t ws_bytes, pit_stream stream) {
  // out == nullptr: ReLU and layout change only (the bitmap still goes to the workspace, nothing is emitted)
  if ((out && (!out->seg_ptr || out->bits)) || (dt != PIT_BF16 && dt != PIT_F16)) return PIT_EINVAL;
  if (tokens < 0 || channels < 0 || tokens % 128 || channels % 8) return PIT_ESHAPE;
  // the index of Xt[channels][tokens] at 1 x 128 micro-tiles with the channel as PIT coordinate
  const Layout L = make_layout(channels, tokens, 1, 128, 0, 0);
  if (out && out->nseg != L.nseg) return PIT_ECAPACITY;
  if (out && (int64_t)out->cap < (int64_t)L.nseg * L.npit) return PIT_ECAPACITY;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  if (L.nseg == 0 || L.npit == 0) return out ? launch_emit(L, nullptr, nullptr, nullptr, out, 0, nullptr, st) : PIT_OK;
  if (ldh < channels || ldxt < tokens || ldh % 8 || ldxt % 8) return PIT_EINVAL;
  if (!d_H || !d_Xt || (out && !out->idx) || !d_ws || !aligned(d_ws, 8) || !aligned(d_H, 16) || !aligned(d_Xt, 16)) return PIT_EINVAL;
  if (ws_bytes < pit_relu_channel_major_index_workspace(tokens, channels)) return PIT_ECAPACITY;
  if (tokens / 128 > 65535) return PIT_ESHAPE;

  char* ws = reinterpret_cast<char*>(d_ws);
  u64* words = reinterpret_cast<u64*>(ws);
  int32_t* cnt = reinterpret_cast<int32_t*>(ws + L.words_bytes + L.occ_bytes);
  dim3 grid((unsigned)ceil_div(channels, 128), (unsigned)(tokens / 128));
  if (dt == PIT_BF16)
    hipLaunchKernelGGL(k_relu_transpose_bitmap<true>, grid, dim3(256), 0, st, d_H, ldh * 2, tokens, channels, d_Xt,
                       ldxt * 2, L.W, reinterpret_cast<uint32_t*>(words));
  else
    hipLaunchKernelGGL(k_relu_transpose_bitmap<false>, grid, dim3(256), 0, st, d_H, ldh * 2, tokens, channels, d_Xt,
                       ldxt * 2, L.W, reinterpret_cast<uint32_t*>(words));
  PIT_LAUNCH_CHECK();
  return out ? launch_emit(L, words, cnt, nullptr, out, 0, nullptr, st) : PIT_OK;
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
    if (!(cand[j].tile_cost >= 0.0) || !(cand[j].fixed_cost >= 0.0) || cand[j].mt_rows <= 0 || cand[j].mt_cols <= 0) return PIT_EINVAL;
    double cost = 0.0;
    for (int i = 0; i < nsamples; ++i) {
      const int64_t n = cand[j].dense ? grid_tiles[(int64_t)i * ncand + j] : num_tiles[(int64_t)i * ncand + j];
      if (n < 0) return PIT_EINVAL;
      cost += cand[j].fixed_cost + (double)n * cand[j].tile_cost;
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
  return pit::launch_route_index(d_expert_id, T, E, out, d_status, d_ws, ws_bytes, nullptr, 0, 0, stream);
}

int pit::launch_route_index(const int32_t* d_expert_id, int T, int E, const pit_index* out, int32_t* d_status,
                            void* d_ws, size_t ws_bytes, void* zero_rows, int64_t zero_ld_bytes, int zero_row_bytes,
                            pit_stream stream) {
  if (!out || !out->seg_ptr) return PIT_EINVAL;
  if (zero_rows && (zero_row_bytes % 16 || zero_ld_bytes % 16 || !aligned(zero_rows, 16))) return PIT_EINVAL;
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
  if (T <= ROUTE_ONE_MAX_T && E <= 64) {
    hipLaunchKernelGGL(k_route_index_one, dim3(1), dim3(1024), 0, st, d_expert_id, T, E, out->seg_ptr, out->idx, d_status,
                       reinterpret_cast<char*>(zero_rows), zero_ld_bytes, zero_row_bytes);
    PIT_LAUNCH_CHECK();
    return PIT_OK;
  }
  hipLaunchKernelGGL(k_bitmap_route, dim3((L.W + 3) / 4), dim3(256), 0, st, d_expert_id, T, E, L.W, words,
                     reinterpret_cast<char*>(zero_rows), zero_ld_bytes, zero_row_bytes);
  PIT_LAUNCH_CHECK();
  return launch_emit(L, words, cnt, nullptr, out, T, d_status, st);
}

// ----------------------------------------------------------------------------------------------
// Debug aid: validate an index before handing it to a product kernel (the kernels themselves trust it).
// ----------------------------------------------------------------------------------------------
namespace pit {
namespace {
// one workgroup per segment; counts entries outside [0, npit), entries not strictly above their predecessor in
// the segment, and segment bounds that are not 0 <= seg_ptr[s] <= seg_ptr[s + 1] <= cap (seg_ptr[0] must be 0)
__global__ void __launch_bounds__(256)
k_check_index(const int32_t* __restrict__ seg_ptr, const int32_t* __restrict__ idx, int nseg, int cap, int npit,
              int32_t* __restrict__ bad) {
  __shared__ int red[4];
  const int s = blockIdx.x;
  const int b = seg_ptr[s], e = seg_ptr[s + 1];
  int n = 0;
  const bool bounds_ok = b >= 0 && e >= b && e <= cap && (s != 0 || b == 0);
  if (!bounds_ok) {
    n = threadIdx.x == 0 ? 1 : 0;
  } else {
    for (int j = b + (int)threadIdx.x; j < e; j += 256) {
      const int v = idx[j];
      if (v < 0 || v >= npit || (j > b && idx[j - 1] >= v)) ++n;
    }
  }
  const int total = block_sum_256(n, red);
  if (threadIdx.x == 0 && total != 0) atomicAdd(bad, total);
}
}  // namespace
}  // namespace pit

extern "C" int pit_check_index(const pit_index* ix, int npit, int32_t* d_bad, pit_stream stream) {
  if (!ix || !ix->seg_ptr || !d_bad || ix->nseg < 0 || ix->cap < 0 || npit < 0) return PIT_EINVAL;
  if (ix->nseg > 0 && ix->cap > 0 && !ix->idx) return PIT_EINVAL;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  hipLaunchKernelGGL(k_fill_i32, dim3(1), dim3(64), 0, st, d_bad, 1, 0);
  PIT_LAUNCH_CHECK();
  if (ix->nseg == 0) return PIT_OK;
  hipLaunchKernelGGL(k_check_index, dim3((unsigned)ix->nseg), dim3(256), 0, st, ix->seg_ptr, ix->idx, ix->nseg, ix->cap, npit, d_bad);
  PIT_LAUNCH_CHECK();
  return PIT_OK;
}

// ----------------------------------------------------------------------------------------------
// pit_build_index for callers that cannot allocate: the workspace (bitmap words, occupancy words,
// per-segment counts) lives in a file-scope device array instead of a caller's buffer.  Each GPU
// holds its own copy of the array at its own address; host code never uses the array's name as a
// pointer, only the address hipGetSymbolAddress reports for the current device.
// ----------------------------------------------------------------------------------------------
namespace pit {
namespace {
constexpr size_t kStaticScratchBytes = (size_t)1 << 20;
}  // namespace
}  // namespace pit
static __device__ __align__(256) unsigned char scratch[pit::kStaticScratchBytes];

#include <mutex>
namespace pit {
namespace {
// device address of `scratch` on the current device, looked up once per device
int static_scratch(void** out) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* ptr[kMaxDevices] = {};
  int dev = -1;
  PIT_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return PIT_EINVAL;
  std::lock_guard<std::mutex> lock(mu);
  if (ptr[dev] == nullptr) {
    void* p = nullptr;
    PIT_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (p == nullptr) return PIT_EINVAL;
    ptr[dev] = p;
  }
  *out = ptr[dev];
  return PIT_OK;
}
}  // namespace
}  // namespace pit

extern "C" size_t pit_build_index_static_capacity(void) { return pit::kStaticScratchBytes; }

extern "C" int pit_build_index_static(const void* d_src, int dt, int rows, int cols, int64_t ld,
                                      int mt_rows, int mt_cols, int pit_dim,
                                      const pit_index* out, pit_stream stream) {
  // argument errors are reported exactly as by pit_build_index, before the scratch array is touched
  const int esize = dtype_size(dt);
  if (!out || !out->seg_ptr || esize == 0 || (pit_dim != 0 && pit_dim != 1)) return PIT_EINVAL;
  if (rows < 0 || cols < 0 || mt_rows <= 0 || mt_cols <= 0) return PIT_ESHAPE;
  if (rows % mt_rows || cols % mt_cols) return PIT_ESHAPE;
  const size_t need = pit_build_index_workspace(rows, cols, mt_rows, mt_cols, pit_dim, out->bits != nullptr);
  if (need > kStaticScratchBytes) return PIT_ECAPACITY;
  void* ws = nullptr;
  const int rc = static_scratch(&ws);
  if (rc != PIT_OK) return rc;
  // (every path of pit_build_index either writes each workspace word it later reads or clears it
  // with a fill kernel first, so what the previous call left in the array does not matter)
  return pit_build_index(d_src, dt, rows, cols, ld, mt_rows, mt_cols, pit_dim, out, ws, kStaticScratchBytes, stream);
}
