// Device helpers shared by the matrix-core kernels of the layer: operand types, the 16x16x32 matrix
// instruction, the transposing LDS read and the packed conversion to 16-bit floats.
#pragma once
#include <type_traits>

#include "bsp_common.h"

namespace bsp {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

template <int DT>
__device__ __forceinline__ f32x4 mfma16(uint4 a, uint4 b, f32x4 c) {
    if constexpr (DT == BSP_BF16)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c,
                                                       0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0,
                                                      0, 0);
}

__device__ __forceinline__ uint2 tr_read(const uint8_t *lds_base, uint32_t off) {
    s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(lds_base + off));
    return __builtin_bit_cast(uint2, v);
}
// The same read at an LDS address given as an integer (the dynamic LDS block starts at 0 in kernels without
// static LDS variables; through its symbol every address costs an addition of that base).
__device__ __forceinline__ uint2 tr_read_at(uint32_t lds_addr) {
    s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(uintptr_t)lds_addr);
    return __builtin_bit_cast(uint2, v);
}

// Two fp32 -> two 16-bit floats (round-to-nearest-even, hardware conversion), packed.
template <int DT>
__device__ __forceinline__ uint32_t cvt_pk(float a, float b) {
    if constexpr (DT == BSP_BF16)
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{a, b}, bf16x2));
    else
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{a, b}, f16x2));
}

extern __shared__ __attribute__((aligned(16))) uint8_t smem_x[];

// f(integral_constant<int, I>) for I = B .. E - 1: a loop whose index is a constant inside the body, so that
// register arrays indexed by it stay in registers.
template <int B, int E, typename F>
__device__ __forceinline__ void static_for(F &&f) {
    if constexpr (B < E) {
        f(std::integral_constant<int, B>{});
        static_for<B + 1, E>(f);
    }
}

}  // namespace
}  // namespace bsp
