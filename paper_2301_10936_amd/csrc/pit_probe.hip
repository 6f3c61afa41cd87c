// Measurement probes for gfx950, built into a library of their own (libpit_probe.so) that only
// bench_micro.py --probe loads: the issue rate of the two MFMA shapes the kernels use, from registers
// only (what a kernel built on a shape can reach at best), an empty kernel (the floor of a launch), and a
// read-only streaming kernel (what the memory system delivers to a kernel that reads weights once).
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

// Read-only streaming: workgroup w = g * per_group + i reads `rows` pieces of `piece` bytes at
// base + g * group_stride + i * wg_stride + r * pitch (16 bytes per lane, four loads in flight per lane), as a
// GEMM tile reads its slice of the weights.
__global__ void __launch_bounds__(256) k_stream(const char* base, int per_group, long group_stride, long wg_stride,
                                                int rows, int piece, long pitch, float* out) {
  const int lanes_per_row = piece / 16, rows_per_pass = 256 / lanes_per_row;
  const int r0 = threadIdx.x / lanes_per_row, c = (threadIdx.x % lanes_per_row) * 16;
  const char* p = base + (long)(blockIdx.x / per_group) * group_stride + (long)(blockIdx.x % per_group) * wg_stride +
                  (long)r0 * pitch + c;
  const long step = (long)rows_per_pass * pitch;
  float acc = 0.f;
  for (int r = 0; r + 4 * rows_per_pass <= rows; r += 4 * rows_per_pass) {
    float4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = *reinterpret_cast<const float4*>(p + u * step);
#pragma unroll
    for (int u = 0; u < 4; ++u) acc += v[u].x + v[u].y + v[u].z + v[u].w;
    p += 4 * step;
  }
  if (acc == 12345.678f) out[0] = acc;
}
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

// `blocks` workgroups in groups of `per_group`; workgroup i of group g reads `rows` pieces of `piece` bytes (a power
// of two, 16 .. 4096), piece r at d_src + g * group_stride + i * wg_stride + r * pitch.  rows must be a multiple of
// 4 * (4096 / piece); every address is checked against src_bytes on the host.  Returns the bytes the launch reads
// (0 on error, nothing launched).
extern "C" double pit_probe_stream(const void* d_src, size_t src_bytes, int blocks, int per_group, long group_stride,
                                   long wg_stride, int rows, int piece, long pitch, float* d_out, void* stream) {
  if (!d_src || !d_out || blocks <= 0 || per_group <= 0 || rows <= 0 || piece < 16 || piece > 4096 || (piece & (piece - 1))) return 0.0;
  if (rows % (4 * (4096 / piece)) || pitch < piece || wg_stride < 0 || group_stride < 0) return 0.0;
  const long last = (long)((blocks - 1) / per_group) * group_stride + (long)(per_group - 1) * wg_stride + (long)(rows - 1) * pitch + piece;
  if (last < 0 || (size_t)last > src_bytes || (reinterpret_cast<uintptr_t>(d_src) & 15) || (pitch & 15) || (wg_stride & 15) || (group_stride & 15)) return 0.0;
  hipLaunchKernelGGL(k_stream, dim3(blocks), dim3(256), 0, reinterpret_cast<hipStream_t>(stream),
                     reinterpret_cast<const char*>(d_src), per_group, group_stride, wg_stride, rows, piece, pitch, d_out);
  if (hipGetLastError() != hipSuccess) return 0.0;
  return (double)blocks * rows * piece;
}
