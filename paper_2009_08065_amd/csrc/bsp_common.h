// Internal helpers shared by the gfx950 kernels of the block-structured-pruning library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "bsp.h"

namespace bsp {

constexpr int kWave = 64;

// ---- status / error bookkeeping -------------------------------------------------------
void set_last_hip_error(int e);

inline int check_launch() {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_last_hip_error((int)e);
        return BSP_ERR_HIP;
    }
    return BSP_OK;
}

inline bool valid_dtype(int d) { return d == BSP_F32 || d == BSP_BF16 || d == BSP_F16; }
inline size_t dtype_size(int d) { return d == BSP_F32 ? 4 : 2; }
inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// ---- element types ----------------------------------------------------------------------
// bf16 is carried as its 16 raw bits; fp16 as _Float16.
struct bf16_t {
    uint16_t bits;
};

__device__ __forceinline__ float bf16_to_float(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// Round-to-nearest-even fp32 -> bf16; NaN stays NaN (quiet).
__device__ __forceinline__ uint16_t float_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

template <int DT>
struct elem;
template <>
struct elem<BSP_F32> {
    using type = float;
    static __device__ __forceinline__ float load(const void *p, int64_t i) { return ((const float *)p)[i]; }
    static __device__ __forceinline__ void store(void *p, int64_t i, float v) { ((float *)p)[i] = v; }
    static __device__ __forceinline__ uint32_t bits(float v) { return __float_as_uint(v); }
};
template <>
struct elem<BSP_BF16> {
    using type = uint16_t;
    static __device__ __forceinline__ float load(const void *p, int64_t i) {
        return bf16_to_float(((const uint16_t *)p)[i]);
    }
    static __device__ __forceinline__ void store(void *p, int64_t i, float v) {
        ((uint16_t *)p)[i] = float_to_bf16(v);
    }
    // the stored 16 bits of v (round-to-nearest-even), for packing two values into one word
    static __device__ __forceinline__ uint32_t bits(float v) { return float_to_bf16(v); }
};
template <>
struct elem<BSP_F16> {
    using type = _Float16;
    static __device__ __forceinline__ float load(const void *p, int64_t i) {
        return (float)((const _Float16 *)p)[i];
    }
    static __device__ __forceinline__ void store(void *p, int64_t i, float v) {
        ((_Float16 *)p)[i] = (_Float16)v;  // v_cvt_f16_f32, round-to-nearest-even
    }
    static __device__ __forceinline__ uint32_t bits(float v) {
        return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)v);
    }
};

// Dispatch a callable templated on the dtype tag.
#define BSP_DISPATCH_DTYPE(dt, NAME, ...)                  \
    switch (dt) {                                          \
        case BSP_F32: { constexpr int NAME = BSP_F32; __VA_ARGS__; } break;   \
        case BSP_BF16: { constexpr int NAME = BSP_BF16; __VA_ARGS__; } break; \
        default: { constexpr int NAME = BSP_F16; __VA_ARGS__; } break;        \
    }

}  // namespace bsp
