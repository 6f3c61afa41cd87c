// Internal helpers shared by the HIP translation units of the PIT hot-path library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/pit.h"

namespace pit {

// Thread-local HIP error code of the last failing runtime call (see pit_last_hip_error()).
int& last_hip_error();

inline int hip_fail(hipError_t e) {
  last_hip_error() = (int)e;
  return PIT_EHIP;
}

#define PIT_HIP_TRY(expr)                                   \
  do {                                                      \
    hipError_t e__ = (expr);                                \
    if (e__ != hipSuccess) return ::pit::hip_fail(e__);     \
  } while (0)

// Launch check: catches invalid configurations right after a kernel launch.
#define PIT_LAUNCH_CHECK() PIT_HIP_TRY(hipGetLastError())

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
inline int dtype_size(int dt) {
  switch (dt) {
    case PIT_U8: return 1;
    case PIT_F16: case PIT_BF16: return 2;
    case PIT_F32: return 4;
    default: return 0;
  }
}
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

constexpr int kWave = 64;

// pit_build_route_index that also clears, in `zero_rows` (row pitch zero_ld_bytes, zero_row_bytes per row, both
// multiples of 16), the rows of the tokens whose expert id is out of range (zero_rows == nullptr: nothing cleared).
int launch_route_index(const int32_t* d_expert_id, int T, int E, const pit_index* out, int32_t* d_status,
                       void* d_ws, size_t ws_bytes, void* zero_rows, int64_t zero_ld_bytes, int zero_row_bytes,
                       pit_stream stream);

}  // namespace pit
