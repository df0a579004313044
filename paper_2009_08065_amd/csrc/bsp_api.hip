// Host-only helpers of the C ABI: status strings, error bookkeeping, the compression rate.
#include "bsp_common.h"

namespace bsp {
static thread_local int g_last_hip_error = 0;
void set_last_hip_error(int e) { g_last_hip_error = e; }
}  // namespace bsp

extern "C" int bsp_last_hip_error(void) { return bsp::g_last_hip_error; }

extern "C" const char *bsp_status_string(int status) {
    switch (status) {
        case BSP_OK: return "ok";
        case BSP_ERR_NULL: return "a required pointer is NULL";
        case BSP_ERR_SHAPE: return "bad shape (dimension <= 0, M % R != 0, R outside [1,64], misaligned or too large)";
        case BSP_ERR_DTYPE: return "unsupported dtype or enum value";
        case BSP_ERR_CAPACITY: return "output or workspace buffer too small";
        case BSP_ERR_FORMAT: return "malformed compact storage";
        case BSP_ERR_HIP: return "a HIP call failed (see bsp_last_hip_error)";
        default: return "unknown status";
    }
}

// Dense parameters over kept parameters (Sec. 4.4: 1.428x <=> 30 % sparsity).
extern "C" double bsp_compression_rate(int64_t M, int64_t N, int32_t R, int64_t kept_cols_total) {
    if (kept_cols_total <= 0) return __builtin_inf();
    return ((double)M * (double)N) / ((double)R * (double)kept_cols_total);
}

extern "C" const char *bsp_version(void) { return "bsp 0.1 (gfx950)"; }
