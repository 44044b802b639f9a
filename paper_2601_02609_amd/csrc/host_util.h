// Host-side helpers shared by the translation units of libcce.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cce {

// hipError_t of the last failed HIP call made by this thread (reported by cce_last_hip_error).
extern thread_local int g_last_hip_error;

static inline bool hip_ok(hipError_t e) {
    if (e != hipSuccess) { g_last_hip_error = (int)e; return false; }
    return true;
}

static inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

}  // namespace cce
