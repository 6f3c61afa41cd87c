// Device-side helpers shared by the SRead / MFMA / SWrite kernels (gfx950): LDS accessors, MFMA wrappers,
// output rounding, the GELU of the MoE epilogue, in-lane 8 x 8 transposes of 16-bit elements, and
// global loads at a wave-uniform base plus a 32-bit per-lane offset.
#pragma once
#include "pit_gemm.hpp"

namespace pit {
namespace {

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
// Two fp32 values rounded (nearest-even) to the 16-bit input type and packed, a in the low half: one
// v_cvt_pk_bf16_f32 on gfx950 for bf16 (the same rounding as f32_to_bf16_rne for every finite value and for
// infinities; a NaN stays a NaN).
typedef __bf16 pit_bf16x2_t __attribute__((ext_vector_type(2)));
typedef _Float16 pit_f16x2_t __attribute__((ext_vector_type(2)));
typedef float pit_f32x2_t __attribute__((ext_vector_type(2)));
template <bool BF> __device__ __forceinline__ uint32_t pack2_in(float a, float b) {
  const pit_f32x2_t v = {a, b};
  if constexpr (BF) return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, pit_bf16x2_t));
  else return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, pit_f16x2_t));
}
// GELU(x) = x (1 + erf(x / sqrt 2)) / 2 with erf(z) = 1 - 2^(-q(z)) for z >= 0, q the polynomial of degree 5 without
// constant term fitted (weighted least squares, reweighted towards the minimax fit) to -log2(erfc z) on [0, 4.2];
// beyond 4.2 q keeps growing (q >= 28.6 there: erfc itself is below 3e-9) until 2^-q underflows to zero.
// |error of erf| <= 7e-7 in fp32, far below the rounding of the result to bf16 / fp16.  One transcendental
// (v_exp_f32) and a dozen other instructions: half of the rational approximation 7.1.26 of Abramowitz & Stegun
// (a reciprocal and an exponential), a tenth of erff -- the GELU epilogue of the first MoE matmul is a quarter of
// its workgroups' run time with the library function.
__device__ __forceinline__ float gelu_erf_fast(float x) {
  const float z = fabsf(x) * 0.70710678118654752f;
  const float q = z * (1.6278890371f + z * (0.9185093641f + z * (0.1486656219f + z * (-0.02959003858f + z * 0.00294415676f))));
  const float e = 1.0f - __builtin_amdgcn_exp2f(-q);     // erf(|x| / sqrt 2)
  return 0.5f * x * (1.0f + copysignf(e, x));
}

// JA consecutive 16-bit columns of one k-row as loaded (JA = 8: 16 bytes, 4: 8 bytes, 2: 4 bytes)
template <int JA> struct ACols { uint32_t d[JA / 2]; };
// Dword jj (k = 2 jj, 2 jj + 1) of column x out of 8 k-rows of JA columns each (one v_perm_b32).
template <int JA>
__device__ __forceinline__ uint32_t transpose_cols_dword(const ACols<JA> (&r)[8], int x, int jj) {
  const uint32_t sel = (x & 1) ? 0x07060302u : 0x05040100u;
  return __builtin_amdgcn_perm(r[2 * jj + 1].d[x >> 1], r[2 * jj].d[x >> 1], sel);
}
// r[j] = 8 consecutive columns of k-row j (16-bit elements); result = 8 consecutive k of column x (4 v_perm_b32).
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


}  // namespace
}  // namespace pit
