// Host-side helpers: argument checks that run before any HIP call, launch-error mapping.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <cmath>
#include "../../include/perf.h"

namespace perf {

inline bool dtype_ok(int d) { return d == PERF_F32 || d == PERF_BF16; }
inline bool layout_ok(int l) { return l == PERF_ROW_MAJOR || l == PERF_COL_MAJOR; }
inline int64_t dtype_size(int d) { return d == PERF_BF16 ? 2 : 4; }
inline bool aligned(const void *p, int64_t a) { return (reinterpret_cast<uintptr_t>(p) % (uintptr_t)a) == 0; }

inline perf_status launch_status()
{
    return hipGetLastError() == hipSuccess ? PERF_OK : PERF_ERR_LAUNCH;
}

constexpr int64_t kMaxGridX = 2147483647;  // HIP grid.x limit
constexpr int64_t kMaxGridYZ = 65535;

}  // namespace perf
