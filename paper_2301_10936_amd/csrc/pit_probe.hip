// Measurement probes for gfx950, built into a library of their own (libpit_probe.so) that only
// bench_micro.py --probe loads: the issue rate of the two MFMA shapes the kernels use, from registers
// only (what a kernel built on a shape can reach at best), and an empty kernel (the floor of a launch).
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

// NACC independent accumulators, one MFMA each per trip; operands are loop-invariant registers
template <int NACC>
__global__ void __launch_bounds__(256) k_rate_16x16x32(int iters, float* out) {
  const u32x4_t av = {0x3f803f80u + threadIdx.x, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};
  const u32x4_t bv = {0x3f803f80u, 0x3f803f80u + threadIdx.x, 0x3f803f80u, 0x3f803f80u};
  const bf16x8_t a = __builtin_bit_cast(bf16x8_t, av), b = __builtin_bit_cast(bf16x8_t, bv);
  f32x4_t acc[NACC];
#pragma unroll
  for (int i = 0; i < NACC; ++i) acc[i] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  for (int t = 0; t < iters; ++t) {
#pragma unroll
    for (int i = 0; i < NACC; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NACC; ++i) s += acc[i][0] + acc[i][3];
  if (s == 12345.678f) out[0] = s;      // keeps the loop alive; practically never true
}
template <int NACC>
__global__ void __launch_bounds__(256) k_rate_32x32x16(int iters, float* out) {
  const u32x4_t av = {0x3f803f80u + threadIdx.x, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};
  const u32x4_t bv = {0x3f803f80u, 0x3f803f80u + threadIdx.x, 0x3f803f80u, 0x3f803f80u};
  const bf16x8_t a = __builtin_bit_cast(bf16x8_t, av), b = __builtin_bit_cast(bf16x8_t, bv);
  f32x16_t acc[NACC];
#pragma unroll
  for (int i = 0; i < NACC; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
  for (int t = 0; t < iters; ++t) {
#pragma unroll
    for (int i = 0; i < NACC; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NACC; ++i) s += acc[i][0] + acc[i][15];
  if (s == 12345.678f) out[0] = s;
}
__global__ void k_empty() {}
}  // namespace

// shape 0: v_mfma_f32_16x16x32_bf16 (16384 FLOP), 1: v_mfma_f32_32x32x16_bf16 (32768 FLOP); 8 independent
// accumulators; `blocks` workgroups of 4 waves, `iters` trips.  Returns the FLOPs the launch performs (0 on error).
extern "C" double pit_probe_mfma(int shape, int blocks, int iters, float* d_out, void* stream) {
  if (blocks <= 0 || iters <= 0 || !d_out) return 0.0;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  if (shape == 0) hipLaunchKernelGGL(k_rate_16x16x32<8>, dim3(blocks), dim3(256), 0, st, iters, d_out);
  else if (shape == 1) hipLaunchKernelGGL(k_rate_32x32x16<8>, dim3(blocks), dim3(256), 0, st, iters, d_out);
  else return 0.0;
  if (hipGetLastError() != hipSuccess) return 0.0;
  return (double)blocks * 4.0 * iters * 8.0 * (shape == 0 ? 16384.0 : 32768.0);
}

extern "C" int pit_probe_empty(void* stream) {
  hipLaunchKernelGGL(k_empty, dim3(1), dim3(64), 0, reinterpret_cast<hipStream_t>(stream));
  return hipGetLastError() == hipSuccess ? 0 : -1;
}
