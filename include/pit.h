/*
 * pit.h -- C ABI of the MI355X (gfx950) dynamic-sparse GEMM hot path.
 *
 * The library implements the run-time half of permutation-invariant transformation (PIT):
 *   1. online sparsity detection  -- find the non-zero micro-tiles of a tensor that stays in its
 *      ordinary dense storage and list their coordinates along the PIT-axis      (paper Section 3.3)
 *   2. SRead   -- gather the listed micro-tiles from global memory into dense operand tiles on chip
 *      (LDS, or straight into registers)
 *   3. dense tile compute on the matrix cores (bf16/fp16 inputs, fp32 accumulation)
 *   4. SWrite  -- write the dense result tile back to the original coordinates
 *                                                    (paper Section 3.1, sparse kernel template)
 * Gathering along m (rows of A and C) or along k (columns of A together with rows of B) leaves
 * C = A.B unchanged because both are PIT-axes of MatMul (paper Section 3.2, Theorem 1, Table 1).
 *
 * General rules of this ABI
 *   - Every pointer named `d_*` or documented "device" is a DEVICE pointer owned by the caller; the
 *     library never frees or keeps it after the call has been enqueued.  pit_index itself is a host
 *     struct holding device pointers.
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the default stream).
 *     No call synchronises with the host, allocates device memory, or reads results back: counts
 *     and indices stay on the device.
 *   - Every function returns PIT_OK (0) or a negative pit_status.  After PIT_EHIP,
 *     pit_last_hip_error() returns the HIP error code of the failing runtime call.
 *   - Matrices are row-major with an explicit leading dimension counted in ELEMENTS.
 *   - 16-bit inputs are PIT_BF16 or PIT_F16; accumulation is always fp32.
 */
#ifndef PIT_H_
#define PIT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef void* pit_stream;

typedef enum pit_status {
  PIT_OK = 0,
  PIT_EINVAL = -1,    /* NULL pointer, unknown enum value, misaligned pointer or leading dimension */
  PIT_ESHAPE = -2,    /* a dimension is not a multiple of the micro-tile / tile the kernel needs   */
  PIT_ECAPACITY = -3, /* index capacity or workspace too small for the worst case                  */
  PIT_EHIP = -4       /* a HIP runtime call failed; see pit_last_hip_error()                       */
} pit_status;

typedef enum pit_dtype { PIT_U8 = 0, PIT_F16 = 1, PIT_BF16 = 2, PIT_F32 = 3 } pit_dtype;

/*
 * The sparse index (paper Section 3.1 "SparseIdx", Section 3.3).
 * A *segment* is one line of the micro-tile grid that runs along the PIT-axis.  For segment s,
 * idx[seg_ptr[s] .. seg_ptr[s+1]) holds the micro-tile coordinates along the PIT-axis of the
 * micro-tiles that contain a non-zero, in ASCENDING order (the paper allows any order; this
 * library fixes one so that results are reproducible bit for bit).
 * bits (optional, may be NULL): for micro-tiles of at most 32 elements, bits[j] has bit
 * (r*mt_cols + c) set iff element (r,c) of the micro-tile listed at idx[j] is non-zero.
 */
typedef struct pit_index {
  int32_t*  seg_ptr; /* device, [nseg + 1]                               */
  int32_t*  idx;     /* device, [cap]                                    */
  uint32_t* bits;    /* device, [cap] or NULL                            */
  int32_t   nseg;    /* host: number of segments the caller sized seg_ptr for */
  int32_t   cap;     /* host: capacity of idx (and bits) in entries      */
} pit_index;

/* HIP error code of the last failing runtime call on this thread (0 if none). */
int pit_last_hip_error(void);

/* Library version: major*10000 + minor*100 + patch. */
int pit_version(void);

/* ---------------------------------------------------------------------------------------------
 * 1. Online sparsity detection (paper Section 3.3)
 * ------------------------------------------------------------------------------------------- */

/* Bytes of device workspace pit_build_index needs for this problem (0 on invalid arguments). */
size_t pit_build_index_workspace(int rows, int cols, int mt_rows, int mt_cols, int pit_dim, int want_bits);

/*
 * Build the canonical index of the [rows x cols] tensor `d_src` (leading dimension `ld` elements),
 * cut into mt_rows x mt_cols micro-tiles.  The tensor is only read; it is never re-formatted.
 *   dt       element type.  The zero test is numeric x != 0: -0.0 is zero; NaN, Inf and
 *            subnormals are non-zero.  PIT_U8 treats any non-zero byte as non-zero.
 *   pit_dim  storage dimension that is the PIT-axis: 0 = rows (one segment per micro-tile column),
 *            1 = columns (one segment per micro-tile row).
 *   out      out->nseg must equal the number of segments, out->cap must be at least the number of
 *            micro-tiles (the worst case), else PIT_ECAPACITY.  out->bits may be non-NULL only if
 *            mt_rows*mt_cols <= 32.
 *   d_ws     workspace of at least pit_build_index_workspace(...) bytes, 8-byte aligned.
 * Errors: PIT_EINVAL (NULL/misaligned pointers, bad enum), PIT_ESHAPE (rows % mt_rows or
 * cols % mt_cols non-zero, or a dimension <= 0), PIT_ECAPACITY, PIT_EHIP.
 * rows*cols == 0 is not an error: seg_ptr is all zeros.
 */
int pit_build_index(const void* d_src, int dt, int rows, int cols, int64_t ld,
                    int mt_rows, int mt_cols, int pit_dim,
                    const pit_index* out, void* d_ws, size_t ws_bytes, pit_stream stream);

/*
 * pit_build_index for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and errors as
 * pit_build_index, without d_ws / ws_bytes: the workspace is a fixed device array inside the
 * library (pit_build_index_static_capacity() bytes, 1 MiB, held by every GPU the library has run
 * on until the process ends).  The call allocates nothing and frees nothing.
 *   PIT_ECAPACITY  if pit_build_index_workspace(...) for this problem exceeds the capacity
 *                  (e.g. a 4096 x 4096 byte mask at 1 x 1); nothing is enqueued then.
 * All calls on one GPU share that GPU's array: calls that may overlap in time on one GPU (other
 * streams, other threads) race on it and must be serialised by the caller; calls enqueued on one
 * stream are ordered and safe.  The array keeps the previous call's contents; the build either
 * overwrites or clears every word it reads, so no clearing is needed between calls.
 */
size_t pit_build_index_static_capacity(void);
int pit_build_index_static(const void* d_src, int dt, int rows, int cols, int64_t ld,
                           int mt_rows, int mt_cols, int pit_dim,
                           const pit_index* out, pit_stream stream);

/*
 * Debug aid.  The product kernels trust the index they are given: an entry outside the operand
 * makes them read or write out of bounds (checking every entry inside the k loop would cost a
 * compare and a branch per gathered row on the hot path; an index built by this library is in
 * range by construction).  A caller that builds or edits an index itself can validate it first:
 * *d_bad (device, int32) receives the number of violations -- entries outside [0, npit), entries
 * not strictly above their predecessor within a segment, and segment bounds that are not
 * 0 = seg_ptr[0] <= seg_ptr[s] <= seg_ptr[s + 1] <= cap.  npit = number of micro-tile coordinates
 * along the PIT-axis.  Enqueued on `stream`; the caller reads *d_bad back when it wants to know.
 */
int pit_check_index(const pit_index* ix, int npit, int32_t* d_bad, pit_stream stream);

/* Bytes of device workspace pit_build_route_index needs. */
size_t pit_build_route_index_workspace(int T, int E);

/*
 * Index of a top-1 routing decision (paper Section 5.1, Switch Transformer): segment e lists, in
 * ascending order, the tokens t with d_expert_id[t] == e.  Equivalent to pit_build_index on the
 * [T x E] one-hot routing matrix with 1x1 micro-tiles and pit_dim = 0, without materialising it.
 * out->nseg must be E and out->cap >= T.  Tokens whose id is outside [0, E) are listed nowhere;
 * if d_status is non-NULL, *d_status is set to the number of such tokens (else 0).
 */
int pit_build_route_index(const int32_t* d_expert_id, int T, int E, const pit_index* out,
                          int32_t* d_status, void* d_ws, size_t ws_bytes, pit_stream stream);

/* Bytes of device workspace pit_relu_channel_major_index needs (0 on invalid arguments). */
size_t pit_relu_channel_major_index_workspace(int tokens, int channels);

/*
 * The producer of activation sparsity, fused with the layout change and the detection: reads the
 * pre-activation d_H [tokens x channels] (row-major, leading dimension ldh elements) once, writes
 * d_Xt [channels x tokens] = ReLU(H)^T (leading dimension ldxt >= tokens) -- the layout paper
 * Section 3.2 asks for when k is the PIT-axis of the product that follows -- and the index that
 * pit_build_index(d_Xt, dt, channels, tokens, ldxt, 1, 128, 0, ...) would give on it (paper Section 3.3):
 * one segment per block of 128 tokens listing, in ascending order, the channels with a non-zero
 * activation in that block.  The tensor is not read a second time for the detection.
 *   dt       PIT_BF16 or PIT_F16.  ReLU(x) = max(x, 0): both zeros and every negative value give +0,
 *            NaN is passed through unchanged (and counts as non-zero), +Inf stays.
 *   tokens   multiple of 128;  channels  multiple of 8;  ldh, ldxt multiples of 8; d_H, d_Xt 16-byte aligned.
 *   out      out->nseg == tokens / 128, out->cap >= (tokens / 128) * channels, out->bits NULL.
 *            NULL: no index is written (ReLU and layout change only; the workspace is still needed) --
 *            what the detection adds to the pass can be timed as the difference.
 *   d_ws     workspace of at least pit_relu_channel_major_index_workspace(...) bytes, 8-byte aligned.
 * d_H and d_Xt must not overlap.  Errors as for pit_build_index.  tokens*channels == 0 is not an error.
 */
int pit_relu_channel_major_index(const void* d_H, int64_t ldh, int tokens, int channels, int dt,
                                 void* d_Xt, int64_t ldxt, const pit_index* out,
                                 void* d_ws, size_t ws_bytes, pit_stream stream);

/* ---------------------------------------------------------------------------------------------
 * 1b. Micro-tile and kernel selection (paper Section 3.2, Algorithm 1)
 * ------------------------------------------------------------------------------------------- */

/* Bytes of device workspace pit_cover_count needs for this problem (0 on invalid arguments). */
size_t pit_cover_count_workspace(int rows, int cols, int mt_rows, int mt_cols);

/*
 * CoverAlgo of Algorithm 1: the number of mt_rows x mt_cols micro-tiles needed to cover every
 * non-zero of the [rows x cols] tensor `d_src` (same zero test and arguments as pit_build_index;
 * the count does not depend on which axis is the PIT-axis).  *d_count (device, int32) receives
 * the count when the enqueued work completes; the caller reads it back when it wants to decide.
 * Errors as pit_build_index.  rows*cols == 0 gives 0.
 */
int pit_cover_count(const void* d_src, int dt, int rows, int cols, int64_t ld, int mt_rows, int mt_cols,
                    int32_t* d_count, void* d_ws, size_t ws_bytes, pit_stream stream);

/*
 * One (dense computation tile, PIT-axis) pair of Algorithm 1's double loop: the micro-tile shape
 * the pair induces on the sparse operand, the profiled running time of its sparse kernel per
 * covered micro-tile (any unit, the same for all candidates), and whether it is the dense
 * kernel, which processes every micro-tile of the grid whatever the data (the fallback for low
 * sparsity).
 */
typedef struct pit_kernel_candidate {
  int32_t mt_rows, mt_cols;
  int32_t dense;       /* 0 = sparse kernel, 1 = dense kernel */
  double  tile_cost;
  double  fixed_cost;  /* cost of one run that does not depend on the number of micro-tiles (launches, index
                          build, set-up and stores of the output), same unit as tile_cost; 0 gives the
                          paper's formula exactly (Algorithm 1: CoverAlgo x tile_cost) */
} pit_kernel_candidate;

/*
 * Kernel selection (Algorithm 1).  HOST-only: no device work, no stream.
 *   cand       [ncand] candidates (host)
 *   num_tiles  [nsamples x ncand] (host, row-major): CoverAlgo of sample i for candidate j, e.g.
 *              read back from pit_cover_count; ignored for dense candidates
 *   grid_tiles [nsamples x ncand] (host): number of micro-tiles of candidate j in sample i's whole
 *              grid (rows/mt_rows * cols/mt_cols); used for dense candidates
 *   cost_out   [ncand] (host) or NULL: receives sum over samples of (fixed_cost + tiles * tile_cost)
 *   best_out   receives the index of the cheapest candidate, the first one among equals
 * Errors: PIT_EINVAL (NULL pointers, ncand <= 0, nsamples < 0, negative counts or costs).
 * The fixed term is this library's addition to the paper's cost model: on this GPU a step of a few
 * tens of microseconds has a constant part (two or three launches, the output's stores) that a purely
 * proportional model charges to no one; the offline profile measures it with the tile cost.
 */
int pit_select_kernel(const pit_kernel_candidate* cand, int ncand, const int64_t* num_tiles,
                      const int64_t* grid_tiles, int nsamples, double* cost_out, int* best_out);

/* ---------------------------------------------------------------------------------------------
 * 2-4. SRead -> dense MFMA tile -> SWrite  (paper Section 3.1; Section 2.3 for the two cases)
 * ------------------------------------------------------------------------------------------- */

typedef enum pit_gemm_mode {
  /*
   * PIT-axis = m.  A is [M x K] row-major (k contiguous).  The index has nseg = K / mt segments,
   * segment s covering the k-slab [s*mt, (s+1)*mt); its list names the rows m whose 1 x mt
   * micro-tile in that slab is non-zero.  For every segment: C[rows, :] += A[rows, slab] . B[slab, :].
   * nseg == 1 (mt == K, whole-row micro-tiles: padded batches) stores each listed row once;
   * rows not listed are zero-filled if zero_uncovered != 0, else left untouched.
   * nseg  > 1 (micro-tiles along k): every element of C is written, rows that no slab lists as
   * zeros, so C needs no clearing and zero_uncovered is ignored.  c_dt must be PIT_F32.  The slabs'
   * partial products are added in an order that depends on the shape only (no atomics): the result
   * is the same bits from run to run.  The lists must be ascending, as pit_build_index builds them.
   * Limits of this case (else PIT_ESHAPE): lda, ldb < 2^23 elements, M, K < 2^24, M*lda and K*ldb
   * < 2^31 elements, M <= 32 * 65535.
   */
  PIT_GEMM_GATHER_M = 0,
  /*
   * PIT-axis = k.  A is supplied K-MAJOR: d_A is At [K x M] row-major (m contiguous), the layout
   * the paper asks for when the operand would otherwise be contiguous along the PIT-axis
   * (Section 3.2).  Micro-tile = mt consecutive m (one k): the index has nseg = M / mt
   * segments, segment s listing the k whose micro-tile At[k, s*mt .. (s+1)*mt) is non-zero.
   * C[s*mt .. (s+1)*mt, :] = sum over listed k of At[k, rows]^T . B[k, :].  Plain stores; every
   * element of C is written.  mt is 128, 64 or 32: the dense tile is mt rows x 128 columns (paper
   * Section 3.2: the micro-tile takes the dense tile's extent on the other axes).  A lower tile
   * follows a finer sparsity pattern -- fewer all-zero micro-tiles are multiplied (Table 3, "sparsity
   * ratio after cover") -- and reads B once per mt rows of C instead of once per 128; which one is
   * cheaper for given data is what pit_select_kernel decides.
   */
  PIT_GEMM_GATHER_K = 1,
  /*
   * The dense kernel Algorithm 1 falls back to at low sparsity (paper Section 3.2): the GATHER_K tile
   * (A supplied K-major, mt = tile height 128, 64 or 32) with identity addressing -- every k is
   * multiplied, no index is built or read; ix is ignored and may be NULL.
   */
  PIT_GEMM_DENSE_K = 2
} pit_gemm_mode;

/*
 * C[M x N] = A . B over the listed micro-tiles only.  B is [K x N] row-major, dense.
 *   in_dt  PIT_BF16 or PIT_F16 (A and B);  c_dt  PIT_F32, or PIT_BF16 / PIT_F16 (rounded once from the
 *          fp32 accumulator, nearest-even; not available when nseg > 1 in GATHER_M mode).
 *   ix     index built by pit_build_index on A (or on a row mask) with the micro-tile named above.
 * Shape rules (else PIT_ESHAPE): N % 128 == 0; GATHER_M: mt % 32 == 0 and K % mt == 0;
 * GATHER_K and DENSE_K: mt in {32, 64, 128}, M % mt == 0.  Pointers 16-byte aligned, leading dimensions % 8 == 0.
 * Index entries outside the valid coordinate range are a caller error (not checked by this call:
 * see pit_check_index).  Grid limits (else PIT_ESHAPE): the worst-case number of row tiles of
 * GATHER_M, M / 128 + nseg, must not exceed 65520.
 */
int pit_sread_gemm(int mode, const void* d_A, int64_t lda, const void* d_B, int64_t ldb,
                   void* d_C, int64_t ldc, int M, int N, int K, int in_dt, int c_dt,
                   const pit_index* ix, int mt, int zero_uncovered, pit_stream stream);

/* Bytes of device workspace pit_select_and_run_gemm needs (0 on invalid arguments). */
size_t pit_select_and_run_gemm_workspace(int M, int K);

/*
 * Algorithm 1 (paper Section 3.2) followed by the kernel it selects, for C[M x N] = A . B with A
 * supplied K-major (d_At is [K x M] row-major, m contiguous).
 * Selection (host, as pit_select_kernel): cand / num_tiles / grid_tiles / nsamples describe the
 * (dense tile, PIT-axis) pairs to choose from and CoverAlgo's counts on the caller's sparsity
 * samples (e.g. from pit_cover_count on earlier activations).  A sparse candidate must have
 * mt_rows == 1 and mt_cols in {32, 64, 128} (micro-tiles of mt_cols consecutive m of one k: the tile
 * heights the GATHER_K kernel offers); a dense candidate stands for PIT_GEMM_DENSE_K at tile height
 * mt_cols.  nsamples == 0 selects candidate 0.
 * Run (device, on `stream`): a sparse winner builds the index of d_At at its micro-tile in the
 * workspace (pit_build_index) and launches pit_sread_gemm(PIT_GEMM_GATHER_K) at that tile height; a
 * dense winner launches PIT_GEMM_DENSE_K.  *chosen (host, may be NULL) receives the winner's index.
 *   d_ws  at least pit_select_and_run_gemm_workspace(M, K) bytes, 256-byte aligned.
 * Errors: as pit_select_kernel, pit_build_index and pit_sread_gemm; PIT_ESHAPE if a candidate's
 * micro-tile is not one the kernels offer or M is not a multiple of it.
 */
int pit_select_and_run_gemm(const pit_kernel_candidate* cand, int ncand, const int64_t* num_tiles,
                            const int64_t* grid_tiles, int nsamples,
                            const void* d_At, int64_t lda, const void* d_B, int64_t ldb,
                            void* d_C, int64_t ldc, int M, int N, int K, int in_dt, int c_dt,
                            void* d_ws, size_t ws_bytes, int* chosen, pit_stream stream);

/* ---------------------------------------------------------------------------------------------
 * Mixture of experts (paper Section 2.1 "Mixture-of-Experts", Section 5.1 "Switch Transformer"):
 * SRead loads each expert's tokens, the expert FFN runs on dense tiles, SWrite puts every result
 * row back at its token's position.  No padding to a capacity, no token dropping.
 * ------------------------------------------------------------------------------------------- */

/* Bytes of device workspace pit_moe_dispatch_gemm needs (index + hidden activations + scratch). */
size_t pit_moe_workspace(int T, int d_model, int d_ff, int E);

/*
 * Y[t, :] = gate[t] * ( act( X[t, :] . W1[e] ) . W2[e] ),   e = d_expert_id[t]   (top-1).
 *   d_X   [T x d_model] in_dt, row-major, contiguous.     d_Y  [T x d_model] y_dt (PIT_F32/BF16/F16).
 *   d_W1  [E][d_model][d_ff] in_dt, contiguous.            d_W2 [E][d_ff][d_model] in_dt, contiguous.
 *   d_gate [T] fp32 or NULL (= 1).    act: 0 = erf-form GELU x (1 + erf(x / sqrt 2)) / 2 (erf evaluated
 *   to 7e-7 absolute error, below the rounding of the hidden row to the input type), 1 = identity.
 *   The hidden activations are kept in in_dt (rounded nearest-even) between the two matmuls.
 *   d_status (may be NULL): set to the number of tokens whose expert id is outside [0, E); those
 *   tokens' rows of Y are zero.
 * Shape rules: d_model % 128 == 0, d_ff % 128 == 0, T >= 0, E >= 1.
 */
int pit_moe_dispatch_gemm(const void* d_X, const int32_t* d_expert_id, const float* d_gate,
                          const void* d_W1, const void* d_W2, void* d_Y, int y_dt,
                          int T, int d_model, int d_ff, int E, int in_dt, int act,
                          int32_t* d_status, void* d_ws, size_t ws_bytes, pit_stream stream);

/* ---------------------------------------------------------------------------------------------
 * Dynamic sparse attention (paper Section 5.1 "Longformer"): PIT on the two batched matmuls of
 * attention with the key axis as PIT-axis; micro-tile = 32 queries x 1 key.
 * ------------------------------------------------------------------------------------------- */

/* Bytes of device workspace pit_sparse_attn needs. */
size_t pit_sparse_attn_workspace(int H, int S, int D);

/*
 * O[h] = softmax over allowed keys( scale * Q[h] . K[h]^T ) . V[h]   for h in [0, H).
 *   d_Q, d_K, d_V  [H][S][D] in_dt contiguous;  d_O [H][S][D] o_dt (PIT_F32/BF16/F16).
 *   d_mask  [S x S] uint8, shared by all heads: mask[i][j] != 0 lets query i attend to key j.
 *           The index is detected online at 32 x 1 granularity (32 queries x 1 key); inside a kept
 *           micro-tile the element mask is honoured exactly.  A query with no allowed key gives a
 *           zero row.
 * Precision: scores, softmax and accumulation in fp32.  V enters the second product in its own type
 * (every finite bf16 / fp16 value as it is: no range restriction; K and V must be finite in the rows of
 * listed keys -- a key that some query of a block attends to meets the other 31 queries with a
 * probability of exactly zero, and 0 x Inf is not 0); the softmax numerators enter it as a two-term
 * bf16 sum (relative error < 2^-15) for bf16 inputs and rounded to fp16 for fp16 inputs.
 * Shape rules: D == 64, S % 32 == 0.
 */
int pit_sparse_attn(const void* d_Q, const void* d_K, const void* d_V, const uint8_t* d_mask,
                    void* d_O, int o_dt, int H, int S, int D, float scale, int in_dt,
                    void* d_ws, size_t ws_bytes, pit_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* PIT_H_ */
