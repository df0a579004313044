// Device helpers shared by the tiled matrix-core kernels of the layer: the X tile's place in LDS, its copy-in,
// the streaming store of Y and the checked raise of a kernel's dynamic-LDS limit.
#pragma once
#include "bsp_common.h"
#include "bsp_linear_internal.h"
#include "bsp_mfma_device.h"

namespace bsp {
namespace {

// 16 bytes of Y leave as a streaming store: Y is written once, and as ordinary stores its 50 to 70 MB per layer
// push the operand stream and the tiles of X, which other workgroups are about to read, out of the L2
// (measured on the BERT-large set at 5x: 8 to 12 % shorter launches).
__device__ __forceinline__ void store_y16(void *p, uint4 v) {
    __builtin_nontemporal_store(u32x4{v.x, v.y, v.z, v.w}, reinterpret_cast<u32x4 *>(p));
}

constexpr uint32_t kXTileBytes = 131072;  // a tile of 64 tokens x 1024 columns

// Distance in LDS between the 16-token sub-tiles of a workgroup's X tile: a constant, so that
// sub-tile offsets fold into the immediate field of the LDS instructions.
template <int NSUB>
constexpr uint32_t sub_stride() { return NSUB == 4 ? kSubStride4 : 65536u; }
// Placement of column c (token quad p) inside sub-tile 0 of a tile of NSUB sub-tiles.
template <int NSUB>
__device__ __forceinline__ uint32_t tile_col_offset(uint32_t c, uint32_t p) {
    if constexpr (NSUB == 4) return lds_col_offset4(c, p);
    else return lds_col_offset(c, p);
}
// Bytes of LDS a tile of NSUB sub-tiles and npad columns occupies.
template <int NSUB>
constexpr size_t tile_bytes(int64_t npad) {
    if (NSUB == 4) return npad <= 512 ? 3 * (size_t)kSubStride4 + (size_t)npad * 32
                                      : 65536 + 3 * (size_t)kSubStride4 + (size_t)(npad - 512) * 32;
    return (size_t)(NSUB - 1) * 65536 + (size_t)npad * 32;
}

// Copy the workgroup's X tile into LDS, transposed.  Unit of work = 4 columns x 4 tokens per
// lane (four 8-byte loads, a 4x4 transpose of 16-bit values in registers, four 8-byte LDS
// stores); all the loads of a batch are issued before the first store so their latencies overlap.
// The tile holds columns [col0, col0 + width) of X (width a multiple of 4), at LDS columns 0 .. width-1.
template <int NSUB>
__device__ __forceinline__ void stage_x_chunk(const uint16_t *__restrict__ X, int64_t T, int64_t N, int32_t col0,
                                              int32_t width, int64_t t0) {
    constexpr int kBatch = 4;
    const int cquads = width >> 2;
    const int units = cquads * (4 * NSUB);
    for (int u0 = threadIdx.x; u0 < units; u0 += blockDim.x * kBatch) {
        uint2 a[kBatch][4];
#pragma unroll
        for (int k = 0; k < kBatch; ++k) {
            const int u = u0 + k * blockDim.x;
            const int cq = u % cquads, tq = u / cquads;
            const int c = cq << 2;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int64_t t = t0 + 4 * tq + i;
                a[k][i] = (u < units && t < T && col0 + c < N)
                              ? *reinterpret_cast<const uint2 *>(X + t * N + col0 + c)
                              : make_uint2(0u, 0u);
            }
        }
#pragma unroll
        for (int k = 0; k < kBatch; ++k) {
            const int u = u0 + k * blockDim.x;
            if (u >= units) break;
            const int cq = u % cquads, tq = u / cquads;
            const int c = cq << 2;
            const uint32_t sub = (uint32_t)(tq >> 2), pq = (uint32_t)(tq & 3);
            uint8_t *dst = smem_x + sub * sub_stride<NSUB>() + tile_col_offset<NSUB>((uint32_t)c, pq);
            uint2 w;  // columns c+1 .. c+3 lie 8, 16, 24 LDS rows further on
            w.x = (a[k][0].x & 0xffffu) | (a[k][1].x << 16);
            w.y = (a[k][2].x & 0xffffu) | (a[k][3].x << 16);
            *reinterpret_cast<uint2 *>(dst) = w;
            w.x = (a[k][0].x >> 16) | (a[k][1].x & 0xffff0000u);
            w.y = (a[k][2].x >> 16) | (a[k][3].x & 0xffff0000u);
            *reinterpret_cast<uint2 *>(dst + 8 * 32) = w;
            w.x = (a[k][0].y & 0xffffu) | (a[k][1].y << 16);
            w.y = (a[k][2].y & 0xffffu) | (a[k][3].y << 16);
            *reinterpret_cast<uint2 *>(dst + 16 * 32) = w;
            w.x = (a[k][0].y >> 16) | (a[k][1].y & 0xffff0000u);
            w.y = (a[k][2].y >> 16) | (a[k][3].y & 0xffff0000u);
            *reinterpret_cast<uint2 *>(dst + 24 * 32) = w;
        }
    }
}

template <int NSUB>
__device__ __forceinline__ void stage_x_tile(const uint16_t *__restrict__ X, int64_t T, int64_t N, int32_t npad,
                                             int64_t t0) {
    stage_x_chunk<NSUB>(X, T, N, 0, npad, t0);
}

template <typename K>
int raise_lds_limit(K kern, size_t lds, size_t &configured) {
    if (lds <= configured) return BSP_OK;
    hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) {
        set_last_hip_error((int)e);
        return BSP_ERR_HIP;
    }
    configured = lds;
    return BSP_OK;
}

}  // namespace
}  // namespace bsp
