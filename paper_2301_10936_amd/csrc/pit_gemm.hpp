// Types, tile constants and host-side launchers shared by the SRead -> dense MFMA tile -> SWrite
// kernels for gfx950 (paper Section 3.1, sparse kernel template).  The kernels themselves:
//   pit_gemm.hip    GATHER_K (k is the PIT-axis, operands register-direct) and the k-slab strips
//   pit_gemm_m.hip  GATHER_M with whole-row micro-tiles (operands staged through LDS by direct loads)
// Their device-side helpers are in pit_gemm_dev.hpp.
#pragma once
#include "pit_common.hpp"

namespace pit {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef short v4i16_t __attribute__((__vector_size__(8)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
#define PIT_LDS __attribute__((address_space(3)))

constexpr int TM = 128, TN = 128;   // GATHER_K: rows (at most) and columns of a tile

enum { EPI_STORE = 0, EPI_GELU = 2 };

struct GemmArgs {
  const void* A; int64_t lda;
  const void* B; int64_t ldb; int64_t b_seg_stride;   // elements between the B matrices of two segments (MoE), else 0
  void* C; int64_t ldc;
  const int32_t* seg_ptr; const int32_t* idx;
  const float* gate;                                   // per C row (EPI_STORE with scatter), or nullptr
  int nseg, M, N, K;
  int slab;          // GATHER_M: k extent of one segment's slab (K when nseg == 1 or per-segment weights)
                     // GATHER_K: rows of a tile = micro-tile height of the index (128, 64 or 32)
  int a_gather;      // GATHER_M: 1 = A rows come from idx, 0 = A rows are seg_ptr[s] + r (compact)
  int c_scatter;     // GATHER_M: 1 = C rows go to idx, 0 = C rows are seg_ptr[s] + r (compact)
  int slab_per_seg;  // GATHER_M: 1 = segment s covers k in [s*slab, (s+1)*slab), 0 = every segment covers [0, K)
  int k_stagger;     // GATHER_M, set by the launcher: 1 = tiles of different segments / column tiles start their walk
                     // over k at different steps (per-segment B)
  int xcd_cols;      // GATHER_M, set by the launcher: the 8 XCDs form 8 / xcd_cols row groups x xcd_cols column groups
  int zero_rest;     // GATHER_M, one segment: 1 = the rows of C that the list does not name are set to zero by the
                     // workgroups of the grid that have no tile
};

// Host-side launchers shared by pit_sread_gemm and pit_moe_dispatch_gemm.
// GATHER_M with operands staged through LDS by direct loads (pit_gemm_m.hip).  total_rows = upper bound of the
// number of listed rows over all segments (the grid is sized for the worst case; the counts stay on the device).
int launch_gather_m(bool bf, int epi, int c_is_in_type, const GemmArgs& g, int64_t total_rows, hipStream_t st);
int launch_zero_rows(void* C, int64_t ld_bytes, int M, int64_t row_bytes, hipStream_t st);

}  // namespace pit
