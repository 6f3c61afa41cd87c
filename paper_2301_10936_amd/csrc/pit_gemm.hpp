// SRead -> dense MFMA tile -> SWrite kernel for gfx950 (paper Section 3.1, sparse kernel template).
//
// One workgroup (256 threads = 4 wavefronts, 2 x 2) computes a 128 x 128 dense tile of C with
// v_mfma_f32_32x32x16 (bf16 or f16 inputs, fp32 accumulation), stepping 64 along k.
//
// SRead.  Two gathers are supported, one per PIT-axis of MatMul (paper Table 1):
//   GATHER_K  A is K-major (At[k][m]); the tile's k-list comes from the index; step i of the k-loop
//             loads rows k_list[64i .. 64i+63] of At (128 m = 256 B each) and the SAME rows of B.
//   GATHER_M  A is K-minor (A[m][k]); the tile's 128 row numbers come from the index once, the
//             k-loop walks a contiguous k range; B rows are contiguous.
// Operand tiles live in LDS in the layout the MFMA operand reads want:
//   K-major tile [64 k][128 x] (256 B per k, one full LDS bank row): read with ds_read_tr16_b64
//             (the transposing LDS read), which hands each lane 4 consecutive k of one column.
//             A 32-lane half of that read touches 4 consecutive k-rows x 64 B; the 64-byte segment
//             index is XOR-ed with (k & 3) so the four rows fall into different bank quarters.
//   K-minor tile [128 m][64 k] (128 B per row): read with ds_read_b128 (8 consecutive k of one
//             row); the 16-byte chunk index is XOR-ed with ((m >> 1) & 7) so that 16 consecutive
//             rows hit 16 different 16-byte slots of the 256-byte bank row.
// SWrite.  The epilogue stores accumulator rows to the row numbers held in LDS (identity or the
// index), optionally with a GELU + round to the input type (first MoE matmul) or a per-row gate
// (second MoE matmul).
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

constexpr int TM = 128, TN = 128, TK = 64;
constexpr int A_TILE_BYTES = TM * TK * 2;   // 16 KiB either layout
constexpr int B_TILE_BYTES = TK * TN * 2;   // 16 KiB
constexpr int STAGE_BYTES = A_TILE_BYTES + B_TILE_BYTES;

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
};

// Host-side launchers shared by pit_sread_gemm and pit_moe_dispatch_gemm.
int launch_sread_gemm(bool bf, bool gather_k, int epi, int c_is_in_type, const GemmArgs& g, int max_tiles, hipStream_t st);
int launch_zero_rows(void* C, int64_t ld_bytes, int M, int64_t row_bytes, hipStream_t st);

}  // namespace pit
