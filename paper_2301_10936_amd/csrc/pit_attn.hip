// pit_sparse_attn: dynamic sparse attention with the key axis as PIT-axis (paper Section 5.1,
// Longformer; Table 1, BatchMatMul).  Micro-tile = 32 queries x 1 key.
//
//   1. The index of the [S x S] byte mask (32 x 1 micro-tiles, PIT-axis = keys) gives, for every
//      block of 32 queries, the ascending list of keys at least one of them attends to, and per
//      listed key a 32-bit word saying which of the 32 queries do.  It is built in one launch
//      (k_mask_index_q32: the lists sit at fixed places, one workgroup per query block), or by
//      pit_build_index when the mask cannot be read 16 bytes at a time.
//   2. One workgroup per (query block, head); its 4 wavefronts take the key list in chunks of 32
//      keys, round-robin, each with its own running softmax state, merged at the end.  A wave's
//      loop has no workgroup barrier and keeps the loads of its next chunk (and the list entries
//      of the one after) in flight while it computes.
//      Per chunk (everything is laid out so that lane % 32 == query):
//        SRead   the K and V rows of the listed keys are gathered into LDS as [key][d], each
//                128-byte row fetched by 8 lanes at once; K operands are read back row-wise (a K
//                row is d-contiguous, which is what the A operand wants).
//        S^T   = K' . Q^T           4 x v_mfma_f32_32x32x16 (input type), fp32
//        mask, running max / sum per query, P^T = exp2(S^T*c - m)        fp32, in registers
//        O^T  += V'^T . P^T         v_mfma_f32_32x32x16 in the input type; V'^T operands come from
//                LDS with the transposing read; the accumulator layout of S^T is already the
//                B-operand layout of this product up to a permutation of the keys inside the chunk,
//                which is free because keys are a PIT-axis here (the same permutation is applied to V').
//      SWrite is a plain store: queries of a block are contiguous.
// Precision of P in the second product: P rounded to bf16 would by itself cost about 1.7e-3 relative
// Frobenius error.  With fp16 inputs P is rounded to fp16 (11-bit significand, 4 MFMAs per chunk).
// With bf16 inputs V stays bf16 -- every finite bf16 value is used as it is, no range restriction --
// and P enters as the sum of two bf16 terms, P = hi + lo with hi = P rounded to bf16 and lo = the
// exact fp32 remainder rounded to bf16 (relative error of the pair below 2^-17), in 8 MFMAs per chunk
// that share their V operands.
#include "pit_common.hpp"

namespace pit {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef short v4i16_t __attribute__((__vector_size__(8)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
#define PIT_LDS __attribute__((address_space(3)))

constexpr int QB = 32;          // queries per block (micro-tile height)
constexpr int KC = 32;          // keys per chunk
constexpr int HD = 64;          // head dimension
constexpr int V_TILE_BYTES = KC * HD * 2;   // 4 KiB

template <bool BF>
__device__ __forceinline__ f32x16_t mfma_in(const uint4& a, const uint4& b, const f32x16_t& c) {
  if constexpr (BF)
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
}
__device__ __forceinline__ uint32_t pack_f16x2(float a, float b) {
  const uint16_t lo = __builtin_bit_cast(uint16_t, (_Float16)a), hi = __builtin_bit_cast(uint16_t, (_Float16)b);
  return (uint32_t)lo | ((uint32_t)hi << 16);
}
// hi2 = {a, b} rounded to bf16 (nearest even, one v_cvt_pk_bf16_f32); lo2 = the remainders a - hi(a), b - hi(b)
// (exact in fp32, of either sign) rounded to bf16 the same way.  hi + lo reproduces the fp32 value to 2^-17 relative.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void split_bf16x2(float a, float b, uint32_t& hi2, uint32_t& lo2) {
  const f32x2_t v = {a, b};
  hi2 = __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
  const f32x2_t r = {a - __builtin_bit_cast(float, hi2 << 16), b - __builtin_bit_cast(float, hi2 & 0xFFFF0000u)};
  lo2 = __builtin_bit_cast(uint32_t, __builtin_convertvector(r, bf16x2_t));
}
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __builtin_bit_cast(uint32_t, f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0;
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// Direct global -> LDS load of 16 bytes per lane: lane i's bytes land at lds_wave_base + 16 i (base and
// lds_wave_base are wave-uniform).  Nothing passes through registers and no LDS write is issued by the wave.
__device__ __forceinline__ void dma16(const char* base, uint32_t byte_off, uint32_t lds_wave_base) {
  const uint32_t m0v = __builtin_amdgcn_readfirstlane(lds_wave_base);
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :: "s"(m0v), "v"(byte_off), "s"(reinterpret_cast<uint64_t>(base)) : "memory", "m0");
}
// The same for 4 bytes per lane (lane i's dword lands at lds_wave_base + 4 i); lanes that are switched off
// neither load nor write.
__device__ __forceinline__ void dma4(const void* base, uint32_t byte_off, uint32_t lds_wave_base) {
  const uint32_t m0v = __builtin_amdgcn_readfirstlane(lds_wave_base);
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
               :: "s"(m0v), "v"(byte_off), "s"(reinterpret_cast<uint64_t>(base)) : "memory", "m0");
}
// The compiler's own wait counts know nothing of these loads, so the chunk loop issues and awaits every one of
// its loads by hand -- and all of them land in LDS, never in a register that the compiler might copy while
// the load is still under way.  wait_loads: every vector-memory operation of this wave has completed.
__device__ __forceinline__ void wait_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
// wait for this wave's LDS operations (reads of a tile must have returned before a direct load refills it)
__device__ __forceinline__ void wait_lds() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// byte offset of 16-byte chunk c16 (8 d) of key row r inside a V tile [32 keys][64 d]; the two
// 64-byte halves of a row are swapped on rows with (r >> 1) odd so that the 4 consecutive rows a
// transposing read touches land in 4 different quarters of the 256-byte bank row.
__device__ __forceinline__ uint32_t v_off(int r, int c16) {
  return (uint32_t)(r * 128 + ((((c16 >> 2) ^ ((r >> 1) & 1)) << 6) | ((c16 & 3) << 4)));
}

// OT: 0 = fp32, 1 = bf16, 2 = fp16 output
template <bool BF, int OT>
__global__ void __launch_bounds__(256, 3)
k_sparse_attn(const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
              const int32_t* __restrict__ seg_ptr, const int32_t* __restrict__ idx, const uint32_t* __restrict__ bits,
              int list_stride, void* __restrict__ O, int S, float scale_log2e) {
  // per wave (private): two V tiles and one K tile of 4 KiB; after the loop the first 8 KiB carry the
  // wave's partial output to wave 0 (32 floats per lane, laid out [value][lane])
  __shared__ __attribute__((aligned(1024))) char s_kv[4][3 * V_TILE_BYTES];
  // per wave, for two chunks: the 32 listed keys, then their 32 occupancy words
  __shared__ __attribute__((aligned(256))) uint32_t s_list[4][2][2 * KC];
  __shared__ float s_ml[3][2][64];

  // Consecutive workgroup ids go to different XCDs (8, each with its own L2): renumber so that an XCD
  // works on a contiguous run of (head, query block) pairs, i.e. on the K and V of one or two heads
  // (1 MiB per head at S = 4096), which then stay in its L2.
  int qb, head;
  {
    const int nqb = gridDim.x, total = nqb * gridDim.y;
    const int lin = blockIdx.x + nqb * blockIdx.y;
    const int x = lin & 7, qq = total >> 3, rr = total & 7;
    const int lp = x * qq + min(x, rr) + (lin >> 3);
    head = lp / nqb;
    qb = lp - head * nqb;
  }
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int h = lane >> 5, ql = lane & 31;
  // list_stride > 0: the list of query block qb starts at qb * list_stride and seg_ptr[qb] is its length
  // (k_mask_index_q32 below); else seg_ptr is the exclusive prefix pit_build_index writes
  const int list_begin = list_stride > 0 ? qb * list_stride : seg_ptr[qb];
  const int list_len = list_stride > 0 ? seg_ptr[qb] : seg_ptr[qb + 1] - list_begin;
  const int nchunks = (list_len + KC - 1) / KC;
  const int64_t head_off = (int64_t)head * S * HD;

  // Q^T operand: lane holds query ql, d = 16*ks + 8*h + (0..7)
  uint4 qf[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks)
    qf[ks] = *reinterpret_cast<const uint4*>(Q + head_off + (int64_t)(qb * QB + ql) * HD + ks * 16 + h * 8);

  float m_run = -INFINITY, l_run = 0.f;
  f32x16_t o[2];
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) o[t][e] = 0.f;

  const uint32_t v_lds0 = (uint32_t)(uintptr_t)(PIT_LDS char*)s_kv[wv];
  const uint32_t k_lds = v_lds0 + 2 * V_TILE_BYTES;
  const char* k_head = reinterpret_cast<const char*>(K + head_off);
  const char* v_head = reinterpret_cast<const char*>(V + head_off);

  // This wave's chunks are wv, wv + 4, ...  The tiles and the mask words in LDS are private to the wave, so
  // the loop needs no workgroup barrier, and it is software-pipelined: while chunk i is computed, the list
  // entries of chunk i + 2 and the K and V rows of chunk i + 1 are under way.
  const int my_chunks = nchunks > wv ? (nchunks - wv + 3) >> 2 : 0;
  // SRead.  The K and V rows of a chunk (32 x 128 B each) travel global -> LDS directly, 8 lanes x 16 B per
  // row, so that every 128-byte line is requested once; the place of a 16-byte piece inside its row of the
  // tile (the bank swizzle) is expressed by which piece of the source row a lane asks for.
  // Every load is unconditional: positions past the end of the list (in the last chunk, and in the chunk
  // requested beyond the wave's last one) repeat the list's last key with an occupancy word of zero -- a
  // listed key's rows are valid addresses, and with probabilities of exactly zero its finite V contributes
  // nothing.  (The loop only runs when the list is not empty.)
  const uint32_t my_row = (uint32_t)(lane >> 3), my_slot = (uint32_t)(lane & 7);
  auto key_request = [&](int i, int slot) {                          // issue only
    const int kk = (wv + 4 * i) * KC + ql;
    const uint32_t pos = (uint32_t)(list_begin + min(kk, list_len - 1)) * 4u;
    const uint32_t at = (uint32_t)(uintptr_t)(PIT_LDS char*)&s_list[wv][slot][0];
    if (lane < KC) {
      dma4(idx, pos, at);
      dma4(bits, pos, at + KC * 4);
    }
  };
  // (after the entries have landed) positions past the end of the list get an occupancy word of zero
  auto key_finish = [&](int i, int slot) {
    if (!(i < my_chunks && (wv + 4 * i) * KC + ql < list_len)) s_list[wv][slot][KC + ql] = 0u;
    __builtin_amdgcn_wave_barrier();
  };
  // byte offset of this lane's row of the key tile, instruction `it` (tile rows 8 it + lane / 8)
  auto row_offsets = [&](int slot, uint32_t (&ro)[4]) {
#pragma unroll
    for (int it = 0; it < 4; ++it) ro[it] = s_list[wv][slot][it * 8 + (int)my_row] * (uint32_t)(HD * 2);
  };
  auto request_v = [&](const uint32_t (&ro)[4], uint32_t v_lds) {
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const uint32_t r = (uint32_t)it * 8u + my_row;                    // v_off(r, c16) == r * 128 + 16 * my_slot
      const uint32_t c16 = ((((my_slot >> 2) ^ ((r >> 1) & 1u)) << 2) | (my_slot & 3u));
      dma16(v_head, ro[it] + c16 * 16u, v_lds + (uint32_t)it * 1024u);
    }
  };
  // K tile [32 keys][8 pieces of 16 B], piece index XOR-ed with (key >> 1) & 7: the operand reads (lane: key
  // ql, piece 2 ks + h) are free of bank conflicts
  auto request_k = [&](const uint32_t (&ro)[4]) {
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const uint32_t r = (uint32_t)it * 8u + my_row;
      dma16(k_head, ro[it] + ((my_slot ^ ((r >> 1) & 7u)) << 4), k_lds + (uint32_t)it * 1024u);
    }
  };

  uint32_t ro[4];
  if (my_chunks > 0) {
    key_request(0, 0);
    key_request(1, 1);
    wait_loads();
    key_finish(0, 0);
    key_finish(1, 1);
    row_offsets(0, ro);
    request_v(ro, v_lds0);
    request_k(ro);
  }
  // one chunk; vb = i % 2.  On entry the rows of chunk i (V in tile vb, K) and the list entries of chunk i + 1
  // (in slot vb ^ 1) were requested during the previous chunk.
  auto step = [&](int i, int vb) {
    const uint32_t v_lds = v_lds0 + (uint32_t)vb * V_TILE_BYTES;
    wait_loads();                            // everything requested so far has landed
    key_finish(i + 1, vb ^ 1);
    row_offsets(vb ^ 1, ro);
    wait_lds();                              // (the other V tile was read by the previous chunk)
    request_v(ro, v_lds0 + (uint32_t)(vb ^ 1) * V_TILE_BYTES);

    f32x16_t st;
#pragma unroll
    for (int e = 0; e < 16; ++e) st[e] = 0.f;
    u32x4_t ka[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
      ka[ks] = *(PIT_LDS u32x4_t*)(uintptr_t)(k_lds + (uint32_t)(ql * 128 + (((2 * ks + h) ^ ((ql >> 1) & 7)) << 4)));
    u32x4_t bwv[4];
#pragma unroll
    for (int g = 0; g < 4; ++g)
      bwv[g] = *(PIT_LDS u32x4_t*)(uintptr_t)((uint32_t)(uintptr_t)(PIT_LDS char*)&s_list[wv][vb][KC + g * 8 + h * 4]);
    wait_lds();                              // the K tile and this chunk's occupancy words are in registers:
    request_k(ro);                           // the tile takes the next chunk's rows, the slot the list entries
    key_request(i + 2, vb);                  // of the chunk after it
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) st = mfma_in<BF>(__builtin_bit_cast(uint4, ka[ks]), qf[ks], st);
    {
      // st[j] = S^T[key 8*(j/4) + 4*h + j%4][query ql]
      float mx = -INFINITY;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const bool on = (bwv[g][e] >> ql) & 1u;
          const float sc = on ? st[g * 4 + e] * scale_log2e : -INFINITY;
          st[g * 4 + e] = sc;
          mx = fmaxf(mx, sc);
        }
      }
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m_run, mx);
      const float m_safe = m_new == -INFINITY ? 0.f : m_new;
      // (the arguments are <= 0 or -inf: the bare hardware exp2 needs no range handling here)
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_safe);
      float psum = 0.f;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const float pe = __builtin_amdgcn_exp2f(st[e] - m_safe);
        st[e] = pe;
        psum += pe;
      }
      psum += __shfl_xor(psum, 32);
      l_run = l_run * alpha + psum;
      // the running output is rescaled only when some query's maximum moved (alpha == 1 otherwise)
      if (__builtin_amdgcn_ballot_w64(m_new != m_run) != 0ull) {
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int e = 0; e < 16; ++e) o[t][e] *= alpha;
      }
      m_run = m_new;
      // O^T += V'^T . P^T ; k-step t covers chunk keys 16t .. 16t+15 in the order the accumulator holds them
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        uint4 pb, pl = make_uint4(0, 0, 0, 0);
        if constexpr (BF) {
          uint32_t hi2[4], lo2[4];
#pragma unroll
          for (int x = 0; x < 4; ++x) split_bf16x2(st[8 * t + 2 * x], st[8 * t + 2 * x + 1], hi2[x], lo2[x]);
          pb = make_uint4(hi2[0], hi2[1], hi2[2], hi2[3]);
          pl = make_uint4(lo2[0], lo2[1], lo2[2], lo2[3]);
        } else {
          pb.x = pack_f16x2(st[8 * t + 0], st[8 * t + 1]);
          pb.y = pack_f16x2(st[8 * t + 2], st[8 * t + 3]);
          pb.z = pack_f16x2(st[8 * t + 4], st[8 * t + 5]);
          pb.w = pack_f16x2(st[8 * t + 6], st[8 * t + 7]);
        }
#pragma unroll
        for (int dt = 0; dt < 2; ++dt) {
          const int r0 = 16 * t + 4 * h + ((lane & 15) >> 2);
          const int col = dt * 32 + ((lane >> 4) & 1) * 16 + (lane & 3) * 4;
          const int r1 = r0 + 8;
          const uint32_t a0 = v_lds + (uint32_t)(r0 * 128 + ((((col >> 5) ^ ((r0 >> 1) & 1)) << 6) | ((col & 31) * 2)));
          const uint32_t a1 = v_lds + (uint32_t)(r1 * 128 + ((((col >> 5) ^ ((r1 >> 1) & 1)) << 6) | ((col & 31) * 2)));
          const uint2 lo = __builtin_bit_cast(uint2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((PIT_LDS v4i16_t*)(uintptr_t)a0));
          const uint2 hi = __builtin_bit_cast(uint2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((PIT_LDS v4i16_t*)(uintptr_t)a1));
          const uint4 vt = make_uint4(lo.x, lo.y, hi.x, hi.y);
          o[dt] = mfma_in<BF>(vt, pb, o[dt]);
          if constexpr (BF) o[dt] = mfma_in<BF>(vt, pl, o[dt]);
        }
      }
    }
  };
  for (int i = 0; i < my_chunks; i += 2) {      // the two V tiles alternate
    step(i, 0);
    if (i + 1 < my_chunks) step(i + 1, 1);
  }
  // the rows requested beyond the last chunk are still arriving in this wave's tiles, which now carry its
  // partial result to wave 0
  wait_loads();
  wait_lds();

  // merge the 4 wavefronts' partial (m, l, O) per lane; wave 0 finishes
  if (wv > 0) {
    float* dst = reinterpret_cast<float*>(s_kv[wv]);      // this wave's own tiles: nobody else reads them
    s_ml[wv - 1][0][lane] = m_run;
    s_ml[wv - 1][1][lane] = l_run;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int e = 0; e < 16; ++e) dst[(t * 16 + e) * 64 + lane] = o[t][e];
  }
  __syncthreads();
  if (wv != 0) return;
  float m_all = m_run;
#pragma unroll
  for (int w = 0; w < 3; ++w) m_all = fmaxf(m_all, s_ml[w][0][lane]);
  const float m_safe = m_all == -INFINITY ? 0.f : m_all;
  float a = exp2f(m_run - m_safe);
  float l_all = l_run * a;
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) o[t][e] *= a;
#pragma unroll
  for (int w = 0; w < 3; ++w) {
    const float* src = reinterpret_cast<const float*>(s_kv[w + 1]);
    a = exp2f(s_ml[w][0][lane] - m_safe);
    l_all += s_ml[w][1][lane] * a;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int e = 0; e < 16; ++e) o[t][e] += src[(t * 16 + e) * 64 + lane] * a;
  }
  const float inv = l_all > 0.f ? 1.f / l_all : 0.f;
  // o[dt][4*g + e] = O[query ql][d = 32*dt + 8*g + 4*h + e]
  const int64_t row = head_off + (int64_t)(qb * QB + ql) * HD;
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int d = dt * 32 + g * 8 + h * 4;
      const float v0 = o[dt][4 * g] * inv, v1 = o[dt][4 * g + 1] * inv, v2 = o[dt][4 * g + 2] * inv, v3 = o[dt][4 * g + 3] * inv;
      if constexpr (OT == 0) {
        *reinterpret_cast<float4*>(reinterpret_cast<float*>(O) + row + d) = make_float4(v0, v1, v2, v3);
      } else if constexpr (OT == 1) {
        uint2 pk;
        pk.x = (uint32_t)f32_to_bf16_rne(v0) | ((uint32_t)f32_to_bf16_rne(v1) << 16);
        pk.y = (uint32_t)f32_to_bf16_rne(v2) | ((uint32_t)f32_to_bf16_rne(v3) << 16);
        *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(O) + row + d) = pk;
      } else {
        uint2 pk;
        pk.x = pack_f16x2(v0, v1);
        pk.y = pack_f16x2(v2, v3);
        *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(O) + row + d) = pk;
      }
    }
}

// ----------------------------------------------------------------------------------------------
// The index of the [S x S] byte mask at 32 x 1 (PIT-axis = keys) with occupancy words, in ONE launch
// (paper Section 3.3: detection of the non-zero micro-tiles and their ordered list).  The attention
// kernel is the only reader of this index, so the list of every query block may sit at a fixed place,
// qb * S, with its length beside it; no prefix over the blocks is needed and one workgroup can do
// detection, scan and ordered emit for its block without waiting for any other.
// A thread owns 16 consecutive keys and 8 of the block's 32 queries (16 B per row, a wave reads 1 KiB of
// a mask row at a time); the non-zero test runs on four bytes at once and leaves a byte of occupancy
// bits per key; the four bytes of a key (one per group of 8 queries) make the key's word.
// Entries are written in ascending key order: threads, waves and passes of 4096 keys are in key order
// and positions come from an exclusive scan of the per-thread counts.
// ----------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(1024)
k_mask_index_q32(const uint8_t* __restrict__ mask, int S, int32_t* __restrict__ cnt,
                 int32_t* __restrict__ idx, uint32_t* __restrict__ bits) {
  // 4 groups of 256 threads: group g tests queries 8 g .. 8 g + 7 for the 16 keys of thread tid % 256 (8 loads per
  // thread: the 16 waves of the workgroup have the whole 128 KiB of a pass under way at once); the groups' bytes
  // of occupancy bits meet in LDS, and the first group makes the words, scans and writes the list.
  __shared__ uint4 s_part[3][256];
  __shared__ int s_wave[4];
  const int qb = blockIdx.x, tid = threadIdx.x, lane = tid & 63;
  const int grp = tid >> 8, ct = tid & 255, wv = ct >> 6;
  const uint8_t* base = mask + (int64_t)qb * QB * S + (int64_t)(8 * grp) * S;
  int32_t* out_i = idx + (int64_t)qb * S;
  uint32_t* out_b = bits + (int64_t)qb * S;
  int run = 0;                                    // entries written by earlier passes (uniform)
  for (int c_base = 0; c_base < S; c_base += 4096) {
    const int c0 = c_base + ct * 16;
    uint32_t acc[4] = {0u, 0u, 0u, 0u};           // [4 keys]: byte j = the group's 8 queries' bits of key 4 w + j
    if (c0 < S) {
      uint4 v[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = *reinterpret_cast<const uint4*>(base + (int64_t)i * S + c0);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const uint32_t d[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          // bit 7 of every non-zero byte, moved to bit i of that byte
          const uint32_t nz = (((d[w] & 0x7F7F7F7Fu) + 0x7F7F7F7Fu) | d[w]) & 0x80808080u;
          acc[w] |= nz >> (7 - i);
        }
      }
    }
    if (grp > 0) s_part[grp - 1][ct] = make_uint4(acc[0], acc[1], acc[2], acc[3]);
    __syncthreads();
    uint32_t o[16];
    int mine = 0, inc = 0;
    if (grp == 0) {
      const uint4 p1 = s_part[0][ct], p2 = s_part[1][ct], p3 = s_part[2][ct];
      const uint32_t a1[4] = {p1.x, p1.y, p1.z, p1.w}, a2[4] = {p2.x, p2.y, p2.z, p2.w}, a3[4] = {p3.x, p3.y, p3.z, p3.w};
      uint32_t flags = 0;
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const int w = j >> 2;
        const uint32_t b = (uint32_t)(j & 3);
        // byte b of the four groups' words -> bytes 0..3 of the key's occupancy word (selector 0x0c = zero byte)
        const uint32_t lo = __builtin_amdgcn_perm(a1[w], acc[w], 0x0c0c0000u | ((4u + b) << 8) | b);
        const uint32_t hi = __builtin_amdgcn_perm(a3[w], a2[w], 0x00000c0cu | ((4u + b) << 24) | (b << 16));
        o[j] = lo | hi;
        flags |= (o[j] != 0 ? 1u : 0u) << j;
      }
      mine = __builtin_popcount(flags);
      inc = mine;
#pragma unroll
      for (int dd = 1; dd < 64; dd <<= 1) {
        const int t = __shfl_up(inc, dd);
        if (lane >= dd) inc += t;
      }
      if (lane == 63) s_wave[wv] = inc;
    }
    __syncthreads();
    int total = 0;
    int pos = run + inc - mine;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const int x = s_wave[w];
      if (w < wv) pos += x;
      total += x;
    }
    if (grp == 0) {
#pragma unroll
      for (int j = 0; j < 16; ++j)
        if (o[j] != 0) {
          out_i[pos] = c0 + j;
          out_b[pos] = o[j];
          ++pos;
        }
    }
    run += total;
    __syncthreads();                              // s_wave and s_part are rewritten by the next pass
  }
  if (tid == 0) cnt[qb] = run;
}

struct AttnWs {
  size_t seg_ptr_off, idx_off, bits_off, build_off, total;
  int nseg, cap;
};
AttnWs attn_layout(int S) {
  AttnWs w;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o += (bytes + 255) & ~(size_t)255; return at; };
  w.nseg = S / QB;
  w.cap = w.nseg * S;
  w.seg_ptr_off = take((size_t)(w.nseg + 1) * 4);
  w.idx_off = take((size_t)(w.cap > 0 ? w.cap : 1) * 4);
  w.bits_off = take((size_t)(w.cap > 0 ? w.cap : 1) * 4);
  w.build_off = take(pit_build_index_workspace(S, S, QB, 1, 1, 1));
  w.total = o;
  return w;
}

}  // namespace
}  // namespace pit

using namespace pit;

extern "C" size_t pit_sparse_attn_workspace(int H, int S, int D) {
  if (H < 0 || S < 0 || D != HD || S % QB) return 0;
  return attn_layout(S).total;
}

extern "C" int pit_sparse_attn(const void* d_Q, const void* d_K, const void* d_V, const uint8_t* d_mask,
                               void* d_O, int o_dt, int H, int S, int D, float scale, int in_dt,
                               void* d_ws, size_t ws_bytes, pit_stream stream) {
  if (in_dt != PIT_BF16 && in_dt != PIT_F16) return PIT_EINVAL;
  if (o_dt != PIT_F32 && o_dt != PIT_BF16 && o_dt != PIT_F16) return PIT_EINVAL;
  if (H < 0 || S < 0) return PIT_ESHAPE;
  if (D != HD || S % QB) return PIT_ESHAPE;
  if (H == 0 || S == 0) return PIT_OK;
  if (H > 65535) return PIT_ESHAPE;
  if (!d_Q || !d_K || !d_V || !d_mask || !d_O || !d_ws) return PIT_EINVAL;
  if (!aligned(d_Q, 16) || !aligned(d_K, 16) || !aligned(d_V, 16) || !aligned(d_O, 16) || !aligned(d_ws, 256)) return PIT_EINVAL;
  const AttnWs L = attn_layout(S);
  if (ws_bytes < L.total) return PIT_ECAPACITY;
  char* ws = reinterpret_cast<char*>(d_ws);
  pit_index ix;
  ix.seg_ptr = reinterpret_cast<int32_t*>(ws + L.seg_ptr_off);
  ix.idx = reinterpret_cast<int32_t*>(ws + L.idx_off);
  ix.bits = reinterpret_cast<uint32_t*>(ws + L.bits_off);
  ix.nseg = L.nseg;
  ix.cap = L.cap;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  // one launch when the mask rows can be read 16 bytes at a time (S is a multiple of 32, so the base decides),
  // else the general index build (bitmap pass + ordered emit) with the same lists behind an exclusive prefix
  int list_stride = 0;
  if (aligned(d_mask, 16) && (int64_t)L.nseg * S < (1ll << 31)) {
    list_stride = S;
    hipLaunchKernelGGL(k_mask_index_q32, dim3((unsigned)L.nseg), dim3(1024), 0, st, d_mask, S, ix.seg_ptr, ix.idx, ix.bits);
    PIT_LAUNCH_CHECK();
  } else {
    const int rc = pit_build_index(d_mask, PIT_U8, S, S, S, QB, 1, 1, &ix, ws + L.build_off, L.total - L.build_off, stream);
    if (rc != PIT_OK) return rc;
  }

  const float c = scale * 1.4426950408889634f;
  const uint16_t* q = reinterpret_cast<const uint16_t*>(d_Q);
  const uint16_t* k = reinterpret_cast<const uint16_t*>(d_K);
  const uint16_t* v = reinterpret_cast<const uint16_t*>(d_V);
  dim3 grid((unsigned)L.nseg, (unsigned)H);
#define PIT_ATTN_LAUNCH(BF, OT) \
  hipLaunchKernelGGL((k_sparse_attn<BF, OT>), grid, dim3(256), 0, st, q, k, v, ix.seg_ptr, ix.idx, ix.bits, list_stride, d_O, S, c)
  const int ot = o_dt == PIT_F32 ? 0 : (o_dt == PIT_BF16 ? 1 : 2);
  if (in_dt == PIT_BF16) {
    if (ot == 0) PIT_ATTN_LAUNCH(true, 0); else if (ot == 1) PIT_ATTN_LAUNCH(true, 1); else PIT_ATTN_LAUNCH(true, 2);
  } else {
    if (ot == 0) PIT_ATTN_LAUNCH(false, 0); else if (ot == 1) PIT_ATTN_LAUNCH(false, 1); else PIT_ATTN_LAUNCH(false, 2);
  }
#undef PIT_ATTN_LAUNCH
  PIT_LAUNCH_CHECK();
  return PIT_OK;
}
