// The transposed product of the block-structure-pruned layer:
//   Z[t, n] = bias[n] + sum over the kept columns (b, c) with col_idx[b, c] == n of
//             sum_r U[t, bR + r] * vals[b, r, c]
// With Y = X Wp^T + bias the layer of Sec. 3.1 (Wp: the matrix after Alg. 1), this is the
// gradient with respect to the layer's input (dX = dY Wp), and it is the layer itself when the
// pruned groups are row segments of column blocks (the other division of Alg. 1) and the
// matrix is stored transposed.
//
// Per row-block the product is a small dense one (tokens x R times R x kept columns) whose
// result is scattered to the kept columns' positions.  A workgroup owns a tile of tokens x a
// range of output columns as fp32 sums in LDS; its wavefronts walk the row-blocks, take the
// kept columns that fall into the range 16 at a time through the matrix cores (contraction
// depth R), and add the 16 x 16 results into the tile with LDS atomics, so no sum leaves the
// compute unit before it is complete.  The tile is rounded once on the way out.
#include "bsp_common.h"

namespace bsp {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));

constexpr int kTok = 64;            // tokens per workgroup
constexpr int kCols = 256;          // output columns per workgroup
constexpr int kPitch = kCols + 1;   // tile row pitch in words: the 16 tokens of one scatter hit 16 different banks
constexpr int kWaves = 8;
constexpr int kThreads = kWaves * kWave;
constexpr int kTable = 1024;        // row-blocks per pass over the range table

template <int DT>
struct mfma16;
template <>
struct mfma16<BSP_BF16> {
    static __device__ __forceinline__ f32x4 run(uint2 a, uint2 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, a), __builtin_bit_cast(s16x4, b), c,
                                                         0, 0, 0);
    }
};
template <>
struct mfma16<BSP_F16> {
    static __device__ __forceinline__ f32x4 run(uint2 a, uint2 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(f16x4, a), __builtin_bit_cast(f16x4, b), c, 0,
                                                     0, 0);
    }
};

__device__ __forceinline__ void lds_add(float *p, float v) {
    (void)__hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// first position p in [0, n) with a[p] >= key (a ascending), n if none
__device__ __forceinline__ int lower_bound(const int32_t *__restrict__ a, int n, int key) {
    int lo = 0, hi = n;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (a[mid] < key) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// ---------------------------------------------------------------------------------------
// Matrix-core kernel.  16-bit values, R % 4 == 0, R <= 64, k_align % 4 == 0, U 8-byte aligned.
// grid.x = token tiles, grid.y = column ranges.  NK = contraction chunks of 16 (ceil(R / 16)).
//
// v_mfma_f32_16x16x16 with A = the value panel transposed (row = kept column, k = r) and
// B = U (k = r, column = token): lane l supplies A[l % 16][4 (l / 16) ..+3] and
// B[4 (l / 16) ..+3][l % 16], the latter four consecutive elements of a row of U; it receives
// D[4 (l / 16) + i][l % 16], i.e. four kept columns of one token.
// ---------------------------------------------------------------------------------------
template <int DT, int NK>
__global__ __launch_bounds__(kThreads) void linear_t_mfma_kernel(const uint16_t *__restrict__ U, int64_t T, int64_t M,
                                                                 int64_t N, int64_t B, int32_t R,
                                                                 const int32_t *__restrict__ blk_cnt,
                                                                 const int32_t *__restrict__ blk_ptr,
                                                                 const int32_t *__restrict__ col_idx,
                                                                 const uint16_t *__restrict__ vals,
                                                                 const void *__restrict__ bias, void *__restrict__ Z) {
    extern __shared__ __align__(16) unsigned char smem[];
    float *tile = reinterpret_cast<float *>(smem);                                    // [kTok][kPitch]
    uint32_t *range = reinterpret_cast<uint32_t *>(smem + sizeof(float) * kTok * kPitch);  // [kTable]: lo | hi << 16

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, kg = lane >> 4;
    const int64_t t0 = (int64_t)blockIdx.x * kTok;
    const int cr0 = (int)blockIdx.y * kCols;

    for (int i = tid; i < kTok * kPitch; i += kThreads) tile[i] = 0.0f;

    // this lane's rows of U (B operand), one per 16-token sub-tile; tokens past T read row 0 and are zeroed
    const uint16_t *urow[4];
    bool tok_ok[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const int64_t t = t0 + 16 * s + l16;
        tok_ok[s] = t < T;
        urow[s] = U + (tok_ok[s] ? t : 0) * M + 4 * kg;
    }

    for (int64_t bc = 0; bc < B; bc += kTable) {
        const int nb = (int)((B - bc) < kTable ? (B - bc) : kTable);
        __syncthreads();  // the tile is zeroed / the previous pass has read the table
        for (int i = tid; i < nb; i += kThreads) {
            const int64_t b = bc + i;
            const int32_t *cols = col_idx + blk_ptr[b];
            const int k = blk_cnt[b];
            const int lo = k ? lower_bound(cols, k, cr0) : 0;
            const int hi = k ? lower_bound(cols, k, cr0 + kCols) : 0;
            range[i] = (uint32_t)lo | ((uint32_t)hi << 16);
        }
        __syncthreads();

        for (int i = wave; i < nb; i += kWaves) {
            const uint32_t lh = __builtin_amdgcn_readfirstlane(range[i]);
            const int lo = (int)(lh & 0xffffu), hi = (int)(lh >> 16);
            if (lo >= hi) continue;
            const int64_t b = bc + i;
            const int64_t base = blk_ptr[b];
            const int kp = blk_ptr[b + 1] - blk_ptr[b];
            const int32_t *cols = col_idx + base;
            const uint16_t *panel = vals + (int64_t)R * base;

            uint2 ub[NK][4];
#pragma unroll
            for (int kc = 0; kc < NK; ++kc) {
                const bool k_ok = 16 * kc + 4 * kg < R;
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    ub[kc][s] = make_uint2(0u, 0u);
                    if (k_ok && tok_ok[s]) ub[kc][s] = *reinterpret_cast<const uint2 *>(urow[s] + b * R + 16 * kc);
                }
            }

            for (int g0 = lo & ~3; g0 < hi; g0 += 16) {
                // A operand: kept column g0 + l16, rows 16 kc + 4 kg ..+3 of the panel
                const int pa = g0 + l16;
                const bool a_ok = pa >= lo && pa < hi;
                const uint16_t *ap = panel + (a_ok ? pa : lo);
                uint2 av[NK];
#pragma unroll
                for (int kc = 0; kc < NK; ++kc) {
                    const int r = 16 * kc + 4 * kg;
                    av[kc] = make_uint2(0u, 0u);
                    if (a_ok && r < R) {
                        const uint16_t *q = ap + (int64_t)r * kp;
                        av[kc].x = (uint32_t)q[0] | ((uint32_t)q[kp] << 16);
                        av[kc].y = (uint32_t)q[2 * (int64_t)kp] | ((uint32_t)q[3 * (int64_t)kp] << 16);
                    }
                }
                // the four kept columns whose sums this lane receives
                const int pd = g0 + 4 * kg;
                int4 cd = make_int4(0, 0, 0, 0);
                if (pd < hi) cd = *reinterpret_cast<const int4 *>(cols + pd);  // pd + 3 < kp: kp % 4 == 0
                const int cdv[4] = {cd.x, cd.y, cd.z, cd.w};

                f32x4 acc[4];
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    acc[s] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int kc = 0; kc < NK; ++kc) acc[s] = mfma16<DT>::run(av[kc], ub[kc][s], acc[s]);
                }
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int p = pd + v;
                    if (p >= lo && p < hi) {
                        float *dst = tile + l16 * kPitch + (cdv[v] - cr0);
#pragma unroll
                        for (int s = 0; s < 4; ++s) lds_add(dst + 16 * s * kPitch, acc[s][v]);
                    }
                }
            }
        }
    }
    __syncthreads();

    // write the tile out: bias added in fp32, one rounding
    const int ncol = (int)((N - cr0) < kCols ? (N - cr0) : kCols);
    if (ncol == kCols && (N & 7) == 0 && (reinterpret_cast<uintptr_t>(Z) & 15) == 0) {
        // 8 columns per lane: a wavefront writes two rows of 512 bytes
        for (int i = tid; i < kTok * (kCols / 8); i += kThreads) {
            const int tok = i / (kCols / 8), c8 = (i % (kCols / 8)) * 8;
            const int64_t t = t0 + tok;
            if (t >= T) continue;
            uint32_t w[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float v0 = tile[tok * kPitch + c8 + 2 * q], v1 = tile[tok * kPitch + c8 + 2 * q + 1];
                if (bias) {
                    v0 += elem<DT>::load(bias, cr0 + c8 + 2 * q);
                    v1 += elem<DT>::load(bias, cr0 + c8 + 2 * q + 1);
                }
                w[q] = elem<DT>::bits(v0) | (elem<DT>::bits(v1) << 16);
            }
            *reinterpret_cast<uint4 *>((uint16_t *)Z + t * N + cr0 + c8) = make_uint4(w[0], w[1], w[2], w[3]);
        }
    } else {
        for (int i = tid; i < kTok * kCols; i += kThreads) {
            const int tok = i / kCols, c = i % kCols;
            const int64_t t = t0 + tok;
            if (t >= T || c >= ncol) continue;
            float v = tile[tok * kPitch + c];
            if (bias) v += elem<DT>::load(bias, cr0 + c);
            elem<DT>::store(Z, t * N + cr0 + c, v);
        }
    }
}

// ---------------------------------------------------------------------------------------
// General kernel: any dtype, any R in [1, 64], any k_align.  Same tile, fp32 fused
// multiply-adds; a thread owns one kept column of the row-block at a time and walks the tokens.
// ---------------------------------------------------------------------------------------
constexpr int kGenTok = 32, kGenThreads = 256;

template <int DT>
__global__ __launch_bounds__(kGenThreads) void linear_t_general_kernel(const void *__restrict__ U, int64_t T, int64_t M,
                                                                      int64_t N, int64_t B, int32_t R,
                                                                      const int32_t *__restrict__ blk_cnt,
                                                                      const int32_t *__restrict__ blk_ptr,
                                                                      const int32_t *__restrict__ col_idx,
                                                                      const void *__restrict__ vals,
                                                                      const void *__restrict__ bias,
                                                                      void *__restrict__ Z) {
    __shared__ float tile[kGenTok][kPitch];
    __shared__ float us[kGenTok][64];
    const int tid = threadIdx.x;
    const int64_t t0 = (int64_t)blockIdx.x * kGenTok;
    const int cr0 = (int)blockIdx.y * kCols;
    for (int i = tid; i < kGenTok * kPitch; i += kGenThreads) (&tile[0][0])[i] = 0.0f;
    for (int64_t b = 0; b < B; ++b) {
        const int k = blk_cnt[b];
        if (k == 0) continue;  // uniform over the workgroup
        const int64_t base = blk_ptr[b];
        const int kp = blk_ptr[b + 1] - blk_ptr[b];
        __syncthreads();
        for (int i = tid; i < kGenTok * R; i += kGenThreads) {
            const int tok = i / R, r = i % R;
            const int64_t t = t0 + tok;
            us[tok][r] = t < T ? elem<DT>::load(U, t * M + b * R + r) : 0.0f;
        }
        __syncthreads();
        for (int p = tid; p < k; p += kGenThreads) {
            const int col = col_idx[base + p] - cr0;
            if (col < 0 || col >= kCols) continue;
            float acc[kGenTok];
#pragma unroll
            for (int tok = 0; tok < kGenTok; ++tok) acc[tok] = 0.0f;
            for (int r = 0; r < R; ++r) {
                const float w = elem<DT>::load(vals, (int64_t)R * base + (int64_t)r * kp + p);
#pragma unroll
                for (int tok = 0; tok < kGenTok; ++tok) acc[tok] = __builtin_fmaf(us[tok][r], w, acc[tok]);
            }
            // the kept columns of one row-block are distinct: no two threads share a cell
#pragma unroll
            for (int tok = 0; tok < kGenTok; ++tok) tile[tok][col] += acc[tok];
        }
    }
    __syncthreads();
    const int ncol = (int)((N - cr0) < kCols ? (N - cr0) : kCols);
    for (int i = tid; i < kGenTok * kCols; i += kGenThreads) {
        const int tok = i / kCols, c = i % kCols;
        const int64_t t = t0 + tok;
        if (t >= T || c >= ncol) continue;
        float v = tile[tok][c];
        if (bias) v += elem<DT>::load(bias, cr0 + c);
        elem<DT>::store(Z, t * N + cr0 + c, v);
    }
}

template <int DT>
void launch_mfma(int nk, dim3 grid, size_t lds, hipStream_t s, const uint16_t *U, int64_t T, int64_t M, int64_t N,
                 int64_t B, int32_t R, const int32_t *blk_cnt, const int32_t *blk_ptr, const int32_t *col_idx,
                 const uint16_t *vals, const void *bias, void *Z) {
#define BSP_LT_CASE(NK)                                                                                             \
    case NK: {                                                                                                      \
        auto k = linear_t_mfma_kernel<DT, NK>;                                                                      \
        static bool raised = false; /* per instantiation: dynamic LDS above 64 KB must be asked for once */         \
        if (!raised) {                                                                                              \
            (void)hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, \
                                      (int)lds);                                                                    \
            raised = true;                                                                                          \
        }                                                                                                           \
        k<<<grid, kThreads, lds, s>>>(U, T, M, N, B, R, blk_cnt, blk_ptr, col_idx, vals, bias, Z);                  \
    } break;
    switch (nk) {
        BSP_LT_CASE(1)
        BSP_LT_CASE(2)
        BSP_LT_CASE(3)
        default:
        BSP_LT_CASE(4)
    }
#undef BSP_LT_CASE
}

}  // namespace
}  // namespace bsp

using namespace bsp;

extern "C" int bsp_linear_transposed(const void *U, int udt, int64_t T, int64_t M, int64_t N, int32_t R,
                                     int32_t k_align, const int32_t *blk_cnt, const int32_t *blk_ptr,
                                     const int32_t *col_idx, const void *vals, const void *bias, void *Z,
                                     void *stream) {
    if (!U || !blk_cnt || !blk_ptr || !Z) return BSP_ERR_NULL;
    if (!valid_dtype(udt)) return BSP_ERR_DTYPE;
    if (T < 0 || M <= 0 || N <= 0 || R < 1 || R > 64 || M % R != 0) return BSP_ERR_SHAPE;
    if (!(k_align == 1 || k_align == 8 || k_align == 16 || k_align == 32 || k_align == 64)) return BSP_ERR_SHAPE;
    if (T == 0) return BSP_OK;
    const int64_t B = M / R;
    const int64_t ranges = (N + kCols - 1) / kCols;
    if (ranges > 65535 || N > 65535) return BSP_ERR_SHAPE;  // kept-column positions travel as 16 bits
    hipStream_t s = (hipStream_t)stream;
    const bool mfma_ok = udt != BSP_F32 && R % 4 == 0 && k_align % 4 == 0 && col_idx && vals && aligned(U, 8) &&
                         aligned(col_idx, 16);
    if (mfma_ok) {
        const int64_t tiles = (T + kTok - 1) / kTok;
        if (tiles >= ((int64_t)1 << 31)) return BSP_ERR_SHAPE;
        const dim3 grid((unsigned)tiles, (unsigned)ranges);
        const size_t lds = sizeof(float) * kTok * kPitch + sizeof(uint32_t) * kTable;
        const int nk = (R + 15) / 16;
        if (udt == BSP_BF16)
            launch_mfma<BSP_BF16>(nk, grid, lds, s, (const uint16_t *)U, T, M, N, B, R, blk_cnt, blk_ptr, col_idx,
                                  (const uint16_t *)vals, bias, Z);
        else
            launch_mfma<BSP_F16>(nk, grid, lds, s, (const uint16_t *)U, T, M, N, B, R, blk_cnt, blk_ptr, col_idx,
                                 (const uint16_t *)vals, bias, Z);
    } else {
        const int64_t tiles = (T + kGenTok - 1) / kGenTok;
        if (tiles >= ((int64_t)1 << 31)) return BSP_ERR_SHAPE;
        const dim3 grid((unsigned)tiles, (unsigned)ranges);
        BSP_DISPATCH_DTYPE(udt, DT, {
            linear_t_general_kernel<DT><<<grid, kGenThreads, 0, s>>>(U, T, M, N, B, R, blk_cnt, blk_ptr, col_idx, vals,
                                                                     bias, Z);
        });
    }
    return check_launch();
}
