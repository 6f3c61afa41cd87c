// pit_moe_dispatch_gemm: top-1 mixture-of-experts FFN (paper Section 5.1, Switch Transformer).
//   route index (counting sort by expert, ascending tokens)            -- pit_build_route_index
//   matmul 1: SRead gathers each expert's token rows, GELU epilogue, hidden rows stored compactly
//             in expert-sorted order
//   matmul 2: reads the compact hidden rows, SWrite scatters every result row to its token's slot
// Nothing is padded to a capacity: an expert with c tokens costs ceil(c / 128) row tiles.
#include "pit_gemm.hpp"

namespace pit {
namespace {
struct MoeWs {
  size_t seg_ptr_off, idx_off, h_off, route_off, total;
};
MoeWs moe_layout(int T, int d_ff, int E) {
  MoeWs w;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o += (bytes + 255) & ~(size_t)255; return at; };
  w.seg_ptr_off = take((size_t)(E + 1) * 4);
  w.idx_off = take((size_t)(T > 0 ? T : 1) * 4);
  w.h_off = take((size_t)(T > 0 ? T : 1) * d_ff * 2);
  w.route_off = take(pit_build_route_index_workspace(T, E));
  w.total = o;
  return w;
}
}  // namespace
}  // namespace pit

using namespace pit;

extern "C" size_t pit_moe_workspace(int T, int d_model, int d_ff, int E) {
  if (T < 0 || d_model <= 0 || d_ff <= 0 || E <= 0) return 0;
  return moe_layout(T, d_ff, E).total;
}

extern "C" int pit_moe_dispatch_gemm(const void* d_X, const int32_t* d_expert_id, const float* d_gate,
                                     const void* d_W1, const void* d_W2, void* d_Y, int y_dt,
                                     int T, int d_model, int d_ff, int E, int in_dt, int act,
                                     int32_t* d_status, void* d_ws, size_t ws_bytes, pit_stream stream) {
  if (in_dt != PIT_BF16 && in_dt != PIT_F16) return PIT_EINVAL;
  if (y_dt != PIT_F32 && y_dt != in_dt) return PIT_EINVAL;
  if (act != 0 && act != 1) return PIT_EINVAL;
  if (T < 0 || E <= 0 || d_model <= 0 || d_ff <= 0) return PIT_ESHAPE;
  if (d_model % TN || d_ff % TN) return PIT_ESHAPE;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  const MoeWs L = moe_layout(T, d_ff, E);
  if (!d_ws || !aligned(d_ws, 256)) return PIT_EINVAL;
  if (ws_bytes < L.total) return PIT_ECAPACITY;
  char* ws = reinterpret_cast<char*>(d_ws);
  pit_index ix;
  ix.seg_ptr = reinterpret_cast<int32_t*>(ws + L.seg_ptr_off);
  ix.idx = reinterpret_cast<int32_t*>(ws + L.idx_off);
  ix.bits = nullptr;
  ix.nseg = E;
  ix.cap = T;
  if (T == 0) return pit_build_route_index(d_expert_id, 0, E, &ix, d_status, ws + L.route_off, L.total - L.route_off, stream);
  if (!d_X || !d_expert_id || !d_W1 || !d_W2 || !d_Y) return PIT_EINVAL;
  if (!aligned(d_X, 16) || !aligned(d_W1, 16) || !aligned(d_W2, 16) || !aligned(d_Y, 16)) return PIT_EINVAL;

  // tokens with an invalid expert id are listed nowhere; their rows of Y are cleared by the index build itself
  // (every other row is written by the second matmul's SWrite)
  const int y_esize = y_dt == PIT_F32 ? 4 : 2;
  int rc = launch_route_index(d_expert_id, T, E, &ix, d_status, ws + L.route_off, L.total - L.route_off,
                              d_Y, (int64_t)d_model * y_esize, d_model * y_esize, stream);
  if (rc != PIT_OK) return rc;

  void* H = ws + L.h_off;
  const bool bf = in_dt == PIT_BF16;

  GemmArgs g1 = {};
  g1.A = d_X; g1.lda = d_model; g1.B = d_W1; g1.ldb = d_ff; g1.b_seg_stride = (int64_t)d_model * d_ff;
  g1.C = H; g1.ldc = d_ff; g1.seg_ptr = ix.seg_ptr; g1.idx = ix.idx; g1.gate = nullptr;
  g1.nseg = E; g1.M = T; g1.N = d_ff; g1.K = d_model;
  g1.slab = d_model; g1.a_gather = 1; g1.c_scatter = 0; g1.slab_per_seg = 0;
  rc = launch_gather_m(bf, act == 0 ? EPI_GELU : EPI_STORE, 1, g1, T, st);
  if (rc != PIT_OK) return rc;

  GemmArgs g2 = {};
  g2.A = H; g2.lda = d_ff; g2.B = d_W2; g2.ldb = d_model; g2.b_seg_stride = (int64_t)d_ff * d_model;
  g2.C = d_Y; g2.ldc = d_model; g2.seg_ptr = ix.seg_ptr; g2.idx = ix.idx; g2.gate = d_gate;
  g2.nseg = E; g2.M = T; g2.N = d_model; g2.K = d_ff;
  g2.slab = d_ff; g2.a_gather = 0; g2.c_scatter = 1; g2.slab_per_seg = 0;
  return launch_gather_m(bf, EPI_STORE, y_dt != PIT_F32, g2, T, st);
}
