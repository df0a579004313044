// The block-structure-pruned linear layer (Sec. 3.1, Sec. 4.4):
//   Y[t, bR + r] = bias[bR + r] + sum_c X[t, col_idx[b, c]] * vals[b, r, c]
// i.e. per row-block a gather of the kept columns of X followed by a small dense product.
#include "bsp_common.h"
#include "bsp_linear_internal.h"

namespace bsp {
namespace {

constexpr int kThreads = 256;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------------------
// General kernel: any dtype, any R in [1, 64], any k_align.  fp32 fused multiply-adds,
// kept columns ascending.  Workgroup = 64 tokens x one row-block; the gathered X tile and the
// value panel are staged through LDS in chunks of 64 kept columns.
// ---------------------------------------------------------------------------------------
constexpr int kGenTok = 64, kGenChunk = 64;

template <int DT>
__global__ __launch_bounds__(kThreads) void linear_general_kernel(const void *__restrict__ X, int64_t T, int64_t M,
                                                                  int64_t N, int32_t R,
                                                                  const int32_t *__restrict__ blk_ptr,
                                                                  const int32_t *__restrict__ col_idx,
                                                                  const void *__restrict__ vals,
                                                                  const void *__restrict__ bias,
                                                                  void *__restrict__ Y) {
    __shared__ float Xs[kGenTok][kGenChunk + 1];
    __shared__ float Ws[64][kGenChunk + 1];
    const int64_t b = blockIdx.y;
    const int64_t t0 = (int64_t)blockIdx.x * kGenTok;
    const int64_t base = blk_ptr[b];
    const int kp = blk_ptr[b + 1] - blk_ptr[b];
    const int tl = threadIdx.x & 63, rg = threadIdx.x >> 6;
    float acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.0f;
    for (int c0 = 0; c0 < kp; c0 += kGenChunk) {
        const int cc = threadIdx.x & 63;
        const bool cin = c0 + cc < kp;
        const int64_t col = cin ? col_idx[base + c0 + cc] : 0;
        for (int i = 0; i < kGenTok / 4; ++i) {
            const int tok = i * 4 + rg;
            const int64_t t = t0 + tok;
            Xs[tok][cc] = (cin && t < T) ? elem<DT>::load(X, t * N + col) : 0.0f;
        }
        for (int r = rg; r < R; r += 4)
            Ws[r][cc] = cin ? elem<DT>::load(vals, (int64_t)R * base + (int64_t)r * kp + c0 + cc) : 0.0f;
        __syncthreads();
        const int lim = (kp - c0) < kGenChunk ? (kp - c0) : kGenChunk;
        for (int q = 0; q < lim; ++q) {
            const float x = Xs[tl][q];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int r = rg + 4 * i;
                if (r < R) acc[i] = __builtin_fmaf(x, Ws[r][q], acc[i]);
            }
        }
        __syncthreads();
    }
    const int64_t t = t0 + tl;
    if (t < T) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int r = rg + 4 * i;
            if (r < R) {
                const int64_t m = b * R + r;
                const float bv = bias ? elem<DT>::load(bias, m) : 0.0f;
                elem<DT>::store(Y, t * M + m, acc[i] + bv);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// Matrix-core kernel, direct-gather form (no LDS): one wavefront = 16 tokens x one row-block,
// v_mfma_f32_16x16x32 with A = value panel rows (16 x 32), B = gathered X (32 x 16 tokens).
// Needs kp_b % 32 == 0.  Kept as the simple matrix-core path for shapes the tiled kernel
// does not take.
// ---------------------------------------------------------------------------------------
template <int DT>
struct mfma_op;
template <>
struct mfma_op<BSP_BF16> {
    using vec = bf16x8;
    static __device__ __forceinline__ f32x4 run(uint4 a, uint4 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c,
                                                       0, 0, 0);
    }
};
template <>
struct mfma_op<BSP_F16> {
    using vec = f16x8;
    static __device__ __forceinline__ f32x4 run(uint4 a, uint4 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0,
                                                      0, 0);
    }
};

template <int DT>
__global__ __launch_bounds__(kThreads) void linear_mfma_direct_kernel(const uint16_t *__restrict__ X, int64_t T,
                                                                      int64_t M, int64_t N, int32_t R,
                                                                      const int32_t *__restrict__ blk_ptr,
                                                                      const int32_t *__restrict__ col_idx,
                                                                      const uint16_t *__restrict__ vals,
                                                                      const void *__restrict__ bias,
                                                                      void *__restrict__ Y) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l16 = lane & 15, g = lane >> 4;
    const int64_t b = blockIdx.y;
    const int64_t t = (int64_t)blockIdx.x * 64 + wave * 16 + l16;  // this lane's token (B operand / output column)
    const int64_t base = blk_ptr[b];
    const int kp = blk_ptr[b + 1] - blk_ptr[b];
    const bool tok_ok = t < T;
    const uint16_t *xrow = X + (tok_ok ? t : 0) * N;
    for (int sub = 0; sub * 16 < R; ++sub) {
        const int r = sub * 16 + l16;  // this lane's panel row (A operand)
        const bool row_ok = r < R;
        const uint16_t *wrow = vals + (int64_t)R * base + (int64_t)(row_ok ? r : 0) * kp;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        for (int kk = 0; kk < kp; kk += 32) {
            uint4 a = make_uint4(0, 0, 0, 0);
            if (row_ok) a = *reinterpret_cast<const uint4 *>(wrow + kk + 8 * g);
            const int4 c0 = *reinterpret_cast<const int4 *>(col_idx + base + kk + 8 * g);
            const int4 c1 = *reinterpret_cast<const int4 *>(col_idx + base + kk + 8 * g + 4);
            uint4 x = make_uint4(0, 0, 0, 0);
            if (tok_ok) {
                x.x = (uint32_t)xrow[c0.x] | ((uint32_t)xrow[c0.y] << 16);
                x.y = (uint32_t)xrow[c0.z] | ((uint32_t)xrow[c0.w] << 16);
                x.z = (uint32_t)xrow[c1.x] | ((uint32_t)xrow[c1.y] << 16);
                x.w = (uint32_t)xrow[c1.z] | ((uint32_t)xrow[c1.w] << 16);
            }
            acc = mfma_op<DT>::run(a, x, acc);
        }
        // acc[v] = Y[t, bR + sub*16 + 4g + v]
        if (tok_ok) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int rr = sub * 16 + 4 * g + v;
                if (rr < R) {
                    const int64_t m = b * R + rr;
                    const float bv = bias ? elem<DT>::load(bias, m) : 0.0f;
                    elem<DT>::store(Y, t * M + m, acc[v] + bv);
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// fp32 matrix-core kernel, direct-gather form: a workgroup of four wavefronts = 16 tokens x one row-block.
// v_mfma_f32_16x16x4_f32 with A = value panel (16 rows x 4 kept columns: lane (row, k) holds one value),
// B = gathered X (4 kept columns x 16 tokens: lane (token, k) holds one value).  The kept columns of the
// row-block are dealt to the four wavefronts in quarters (a layer of this kind is a latency case: a few
// hundred kept columns, little work, so the chain of dependent loads is what is cut), their partial sums
// meet in LDS.  Any R, any k_align.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void linear_f32_mfma_kernel(const float *__restrict__ X, int64_t T, int64_t M,
                                                                   int64_t N, int32_t R,
                                                                   const int32_t *__restrict__ blk_ptr,
                                                                   const int32_t *__restrict__ col_idx,
                                                                   const float *__restrict__ vals,
                                                                   const float *__restrict__ bias,
                                                                   float *__restrict__ Y) {
    __shared__ float red[3][4][64];  // partial sums of wavefronts 1 .. 3: [wavefront][register][lane]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l16 = lane & 15, g = lane >> 4;
    const int64_t b = blockIdx.y;
    const int64_t t = (int64_t)blockIdx.x * 16 + l16;  // this lane's token (B operand / output column)
    const int64_t base = blk_ptr[b];
    const int kp = blk_ptr[b + 1] - blk_ptr[b];
    const bool tok_ok = t < T;
    const float *xrow = X + (tok_ok ? t : 0) * N;
    const int nsteps = (kp + 3) >> 2, per = (nsteps + 3) >> 2;
    const int s_lo = wave * per, s_hi = min(nsteps, s_lo + per);
    for (int sub = 0; sub * 16 < R; ++sub) {
        const int r = sub * 16 + l16;  // this lane's panel row (A operand)
        const bool row_ok = r < R;
        const float *wrow = vals + (int64_t)R * base + (int64_t)(row_ok ? r : 0) * kp;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        constexpr int kU = 8;  // steps whose loads are in flight together
        for (int s0 = s_lo; s0 < s_hi; s0 += kU) {
            float a[kU], x[kU];
            int c[kU];
#pragma unroll
            for (int u = 0; u < kU; ++u) {
                const int k = 4 * (s0 + u) + g;
                const bool ok = s0 + u < s_hi && k < kp;
                c[u] = ok ? col_idx[base + k] : 0;
                a[u] = (ok && row_ok) ? wrow[k] : 0.0f;
            }
#pragma unroll
            for (int u = 0; u < kU; ++u) {
                const int k = 4 * (s0 + u) + g;
                const bool ok = s0 + u < s_hi && k < kp;
                x[u] = (ok && tok_ok) ? xrow[c[u]] : 0.0f;
            }
#pragma unroll
            for (int u = 0; u < kU; ++u) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[u], x[u], acc, 0, 0, 0);
        }
        if (wave > 0) {
#pragma unroll
            for (int v = 0; v < 4; ++v) red[wave - 1][v][lane] = acc[v];
        }
        __syncthreads();
        if (wave == 0 && tok_ok) {
            // acc[v] = Y[t, bR + sub*16 + 4g + v] before the bias
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int rr = sub * 16 + 4 * g + v;
                if (rr < R) {
                    const int64_t m = b * R + rr;
                    const float sum = ((acc[v] + red[0][v][lane]) + red[1][v][lane]) + red[2][v][lane];
                    Y[t * M + m] = sum + (bias ? bias[m] : 0.0f);
                }
            }
        }
        __syncthreads();  // the partial sums are reused by the next 16 rows
    }
}

}  // namespace
}  // namespace bsp

using namespace bsp;

extern "C" int bsp_linear(const void *X, int xdt, int64_t T, int64_t M, int64_t N, int32_t R, int32_t k_align,
                          const int32_t *blk_cnt, const int32_t *blk_ptr, const int32_t *col_idx, const void *vals,
                          const void *bias, void *Y, void *stream) {
    if (!X || !blk_cnt || !blk_ptr || !Y) return BSP_ERR_NULL;
    if (!valid_dtype(xdt)) return BSP_ERR_DTYPE;
    if (T < 0 || M <= 0 || N <= 0 || R < 1 || R > 64 || M % R != 0) return BSP_ERR_SHAPE;
    if (!(k_align == 1 || k_align == 8 || k_align == 16 || k_align == 32 || k_align == 64)) return BSP_ERR_SHAPE;
    if (T == 0) return BSP_OK;
    const int64_t B = M / R;
    const int64_t tok_tiles = (T + 63) / 64;
    if (B > 65535 || tok_tiles >= ((int64_t)1 << 31)) return BSP_ERR_SHAPE;
    if (!aligned(X, 16) || (vals && !aligned(vals, 16))) return BSP_ERR_SHAPE;
    // col_idx / vals may be NULL only for an all-empty storage; the kernels never touch them then.
    hipStream_t s = (hipStream_t)stream;
    dim3 grid((unsigned)tok_tiles, (unsigned)B, 1);
    const bool mfma_ok = xdt != BSP_F32 && k_align % 32 == 0 && col_idx && vals && aligned(col_idx, 16);
    if (mfma_ok && aligned(Y, 16) && tiled_supported(xdt, N, k_align)) {
        TiledArgs a{};
        a.xdt = xdt;
        a.X = (const uint16_t *)X;
        a.T = T; a.M = M; a.N = N; a.B = B; a.R = R;
        a.blk_ptr = blk_ptr;
        a.col_idx = col_idx;
        a.vals = (const uint16_t *)vals;
        a.bias = bias;
        a.Y = Y;
        return launch_linear_tiled(a, false, s);
    }
    if (mfma_ok) {
        if (xdt == BSP_BF16)
            linear_mfma_direct_kernel<BSP_BF16><<<grid, kThreads, 0, s>>>((const uint16_t *)X, T, M, N, R, blk_ptr,
                                                                          col_idx, (const uint16_t *)vals, bias, Y);
        else
            linear_mfma_direct_kernel<BSP_F16><<<grid, kThreads, 0, s>>>((const uint16_t *)X, T, M, N, R, blk_ptr,
                                                                         col_idx, (const uint16_t *)vals, bias, Y);
    } else if (xdt == BSP_F32) {
        const int64_t tiles16 = (T + 15) / 16;
        if (tiles16 >= ((int64_t)1 << 31)) return BSP_ERR_SHAPE;
        linear_f32_mfma_kernel<<<dim3((unsigned)tiles16, (unsigned)B, 1), kThreads, 0, s>>>(
            (const float *)X, T, M, N, R, blk_ptr, col_idx, (const float *)vals, (const float *)bias, (float *)Y);
    } else {
        BSP_DISPATCH_DTYPE(xdt, DT, {
            linear_general_kernel<DT><<<grid, kThreads, 0, s>>>(X, T, M, N, R, blk_ptr, col_idx, vals, bias, Y);
        });
    }
    return check_launch();
}
