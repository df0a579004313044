// Group sums of squares, norms, reweighting factors and the regulariser's gradient
// (Sec. 3.2, Eq. 3; norm step of Alg. 1; the refresh and the penalised step of Alg. 2).
//
// A group is a column segment of a row-block, so one lane owns whole groups: it walks the
// R rows of its columns with one fused multiply-add per row, rows ascending.  No cross-lane
// reduction touches a group's sum, which keeps the result independent of the launch shape.
// Consecutive lanes read consecutive 16-byte vectors of a row, so every load instruction of
// a wavefront covers 1 KiB of contiguous HBM.  The path is HBM-bound: W is read once.
#include "bsp_common.h"

namespace bsp {
namespace {

constexpr int kThreads = 256;

template <int DT, int VEC>
struct vec_io;

// 16-byte vector of 4 fp32.
template <>
struct vec_io<BSP_F32, 4> {
    static __device__ __forceinline__ void load(const void *p, int64_t i, float (&v)[4]) {
        float4 q = *reinterpret_cast<const float4 *>((const float *)p + i);
        v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
    }
    static __device__ __forceinline__ void store(void *p, int64_t i, const float (&v)[4]) {
        *reinterpret_cast<float4 *>((float *)p + i) = make_float4(v[0], v[1], v[2], v[3]);
    }
};
// 16-byte vector of 8 bf16.
template <>
struct vec_io<BSP_BF16, 8> {
    static __device__ __forceinline__ void load(const void *p, int64_t i, float (&v)[8]) {
        uint4 q = *reinterpret_cast<const uint4 *>((const uint16_t *)p + i);
        uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            v[2 * k] = __uint_as_float(w[k] << 16);
            v[2 * k + 1] = __uint_as_float(w[k] & 0xffff0000u);
        }
    }
    static __device__ __forceinline__ void store(void *p, int64_t i, const float (&v)[8]) {
        uint32_t w[4];
#pragma unroll
        for (int k = 0; k < 4; ++k)
            w[k] = (uint32_t)float_to_bf16(v[2 * k]) | ((uint32_t)float_to_bf16(v[2 * k + 1]) << 16);
        *reinterpret_cast<uint4 *>((uint16_t *)p + i) = make_uint4(w[0], w[1], w[2], w[3]);
    }
};
// 16-byte vector of 8 fp16.
template <>
struct vec_io<BSP_F16, 8> {
    typedef _Float16 h8 __attribute__((ext_vector_type(8)));
    static __device__ __forceinline__ void load(const void *p, int64_t i, float (&v)[8]) {
        h8 q = *reinterpret_cast<const h8 *>((const _Float16 *)p + i);
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = (float)q[k];
    }
    static __device__ __forceinline__ void store(void *p, int64_t i, const float (&v)[8]) {
        h8 q;
#pragma unroll
        for (int k = 0; k < 8; ++k) q[k] = (_Float16)v[k];
        *reinterpret_cast<h8 *>((_Float16 *)p + i) = q;
    }
};
// 4-byte vector of 2 bf16 / 2 fp16: a wavefront load covers 256 contiguous bytes, the width the
// vector memory pipeline sustains best, and a row-block offers 4x more lanes than with 16-byte vectors.
template <>
struct vec_io<BSP_BF16, 2> {
    static __device__ __forceinline__ void load(const void *p, int64_t i, float (&v)[2]) {
        const uint32_t w = *reinterpret_cast<const uint32_t *>((const uint16_t *)p + i);
        v[0] = __uint_as_float(w << 16);
        v[1] = __uint_as_float(w & 0xffff0000u);
    }
    static __device__ __forceinline__ void store(void *p, int64_t i, const float (&v)[2]) {
        *reinterpret_cast<uint32_t *>((uint16_t *)p + i) = (uint32_t)float_to_bf16(v[0]) | ((uint32_t)float_to_bf16(v[1]) << 16);
    }
};
template <>
struct vec_io<BSP_F16, 2> {
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    static __device__ __forceinline__ void load(const void *p, int64_t i, float (&v)[2]) {
        const h2 q = *reinterpret_cast<const h2 *>((const _Float16 *)p + i);
        v[0] = (float)q[0];
        v[1] = (float)q[1];
    }
    static __device__ __forceinline__ void store(void *p, int64_t i, const float (&v)[2]) {
        h2 q;
        q[0] = (_Float16)v[0];
        q[1] = (_Float16)v[1];
        *reinterpret_cast<h2 *>((_Float16 *)p + i) = q;
    }
};
// Scalar fallback for unaligned or ragged rows.
template <int DT>
struct vec_io<DT, 1> {
    static __device__ __forceinline__ void load(const void *p, int64_t i, float (&v)[1]) {
        v[0] = elem<DT>::load(p, i);
    }
    static __device__ __forceinline__ void store(void *p, int64_t i, const float (&v)[1]) {
        elem<DT>::store(p, i, v[0]);
    }
};

template <int VEC>
__device__ __forceinline__ void store_f32(float *p, int64_t i, const float (&v)[VEC]) {
    if constexpr (VEC == 1) {
        p[i] = v[0];
    } else if constexpr (VEC == 2) {
        *reinterpret_cast<float2 *>(p + i) = make_float2(v[0], v[1]);
    } else {
#pragma unroll
        for (int k = 0; k < VEC; k += 4)
            *reinterpret_cast<float4 *>(p + i + k) = make_float4(v[k], v[k + 1], v[k + 2], v[k + 3]);
    }
}
template <int VEC>
__device__ __forceinline__ void load_f32(const float *p, int64_t i, float (&v)[VEC]) {
    if constexpr (VEC == 1) {
        v[0] = p[i];
    } else if constexpr (VEC == 2) {
        const float2 q = *reinterpret_cast<const float2 *>(p + i);
        v[0] = q.x;
        v[1] = q.y;
    } else {
#pragma unroll
        for (int k = 0; k < VEC; k += 4) {
            float4 q = *reinterpret_cast<const float4 *>(p + i + k);
            v[k] = q.x; v[k + 1] = q.y; v[k + 2] = q.z; v[k + 3] = q.w;
        }
    }
}

__device__ __forceinline__ float alpha_of(float s, float root, float eps, int mode) {
    float den = (mode == BSP_ALPHA_NORM) ? (root + eps) : (s + eps);
    return 1.0f / den;  // IEEE division (the library is built without fast-math)
}

// grid.x covers the N / VEC column vectors, grid.y the row-blocks.
template <int DT, int VEC>
__global__ __launch_bounds__(kThreads) void group_norms_kernel(const void *__restrict__ W, int64_t N, int32_t R,
                                                               float eps, int mode, float *__restrict__ sumsq,
                                                               float *__restrict__ norm,
                                                               float *__restrict__ alpha) {
    const int64_t jv = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t j = jv * VEC;
    if (j >= N) return;
    const int64_t b = blockIdx.y;
    float acc[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[v] = 0.0f;
    int64_t off = b * R * N + j;
#pragma unroll 8
    for (int32_t r = 0; r < R; ++r, off += N) {
        float w[VEC];
        vec_io<DT, VEC>::load(W, off, w);
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[v] = __builtin_fmaf(w[v], w[v], acc[v]);
    }
    const int64_t o = b * N + j;
    if (sumsq) store_f32<VEC>(sumsq, o, acc);
    if (norm || alpha) {
        float root[VEC], a[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            root[v] = __builtin_sqrtf(acc[v]);
            a[v] = alpha_of(acc[v], root[v], eps, mode);
        }
        if (norm) store_f32<VEC>(norm, o, root);
        if (alpha) store_f32<VEC>(alpha, o, a);
    }
}

// Group sums of the other division (Eq. 2; Alg. 1 as printed): a group is a row segment of C columns.  In the
// flat row-major array the groups are consecutive runs of C elements, so a workgroup takes 256 groups = 256 C
// contiguous elements, copies them with coalesced loads into LDS (one group per padded row: the stride C + 1 keeps
// the lanes on different banks) and every lane then walks its own group with one fused multiply-add per element,
// columns ascending: the same chain as the column groups', and bit for bit what group_norms gives on the
// transposed matrix.  (A cross-lane shuffle tree would be shorter, but it adds in another order.)
template <int DT>
__global__ __launch_bounds__(kThreads) void rowseg_norms_kernel(const void *__restrict__ W, int64_t groups, int32_t C,
                                                                float eps, int mode, float *__restrict__ sumsq,
                                                                float *__restrict__ norm, float *__restrict__ alpha) {
    extern __shared__ float seg[];  // [kThreads][C + 1]
    const int64_t g0 = (int64_t)blockIdx.x * kThreads;
    const int ng = (int)((groups - g0) < kThreads ? (groups - g0) : kThreads);
    const int n = ng * C;
    for (int e = threadIdx.x; e < n; e += kThreads) {
        const int i = e / C, c = e - i * C;
        seg[i * (C + 1) + c] = elem<DT>::load(W, g0 * C + e);
    }
    __syncthreads();
    if ((int)threadIdx.x >= ng) return;
    float acc = 0.0f;
    const float *mine = seg + threadIdx.x * (C + 1);
    for (int c = 0; c < C; ++c) acc = __builtin_fmaf(mine[c], mine[c], acc);
    const int64_t o = g0 + threadIdx.x;
    if (sumsq) sumsq[o] = acc;
    if (norm || alpha) {
        const float root = __builtin_sqrtf(acc);
        if (norm) norm[o] = root;
        if (alpha) alpha[o] = alpha_of(acc, root, eps, mode);
    }
}

// Refresh and gradient in one pass over W (Alg. 2 at a milestone: the factors are recomputed and the next
// step's regulariser gradient uses them).  The same arithmetic as group_norms_kernel followed by the gradient
// kernels, operation for operation, so the results are bit-identical to the two separate calls; the R = RT
// rows of the lane's groups stay in registers between the norm pass and the scaling pass (RT == 0: any R,
// the second pass re-reads the rows).
template <int DT, int VEC, int RT>
__global__ __launch_bounds__(kThreads) void norms_grad_kernel(const void *__restrict__ W, int64_t N, int32_t R, float eps,
                                                              int mode, float lambda, int accumulate,
                                                              float *__restrict__ sumsq, float *__restrict__ norm,
                                                              float *__restrict__ alpha, void *__restrict__ G) {
    const int64_t jv = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t j = jv * VEC;
    if (j >= N) return;
    const int64_t b = blockIdx.y;
    const int64_t base = b * R * N + j;
    constexpr int RC = RT > 0 ? RT : 1;
    float cache[RC][VEC];
    float acc[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[v] = 0.0f;
    auto row_step = [&](int32_t r) {
        float w[VEC];
        vec_io<DT, VEC>::load(W, base + (int64_t)r * N, w);
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            if constexpr (RT > 0) cache[r][v] = w[v];
            acc[v] = __builtin_fmaf(w[v], w[v], acc[v]);
        }
    };
    if constexpr (RT > 0) {
#pragma unroll
        for (int32_t r = 0; r < RT; ++r) row_step(r);
    } else {
#pragma unroll 4
        for (int32_t r = 0; r < R; ++r) row_step(r);
    }
    float root[VEC], a[VEC], coef[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
        root[v] = __builtin_sqrtf(acc[v]);
        a[v] = alpha_of(acc[v], root[v], eps, mode);
        coef[v] = lambda * a[v];
        if (mode == BSP_ALPHA_NORM) coef[v] = (acc[v] > 0.0f) ? coef[v] / __builtin_sqrtf(acc[v]) : 0.0f;
    }
    const int64_t o = b * N + j;
    if (sumsq) store_f32<VEC>(sumsq, o, acc);
    if (norm) store_f32<VEC>(norm, o, root);
    if (alpha) store_f32<VEC>(alpha, o, a);
    auto out_step = [&](int32_t r) {
        const int64_t off = base + (int64_t)r * N;
        float w[VEC], g[VEC];
        if constexpr (RT > 0) {
#pragma unroll
            for (int v = 0; v < VEC; ++v) w[v] = cache[r][v];
        } else {
            vec_io<DT, VEC>::load(W, off, w);
        }
        if (accumulate) {
            vec_io<DT, VEC>::load(G, off, g);
#pragma unroll
            for (int v = 0; v < VEC; ++v) g[v] = __builtin_fmaf(coef[v], w[v], g[v]);
        } else {
#pragma unroll
            for (int v = 0; v < VEC; ++v) g[v] = coef[v] * w[v];
        }
        vec_io<DT, VEC>::store(G, off, g);
    };
    if constexpr (RT > 0) {
#pragma unroll
        for (int32_t r = 0; r < RT; ++r) out_step(r);
    } else {
#pragma unroll 4
        for (int32_t r = 0; r < R; ++r) out_step(r);
    }
}

// Gradient of the regulariser.  RT > 0: the R = RT rows of the lane's groups stay in
// registers between the norm pass and the scaling pass, so W is read from HBM once.
// RT == 0: any R; the second pass re-reads the rows (cache hits in the common case).
template <int DT, int VEC, int RT, bool NEED_S, bool PEN>
__global__ __launch_bounds__(kThreads) void penalty_grad_kernel(const void *__restrict__ W, int64_t N, int32_t R,
                                                                const float *__restrict__ alpha, float lambda,
                                                                int mode, int accumulate, void *__restrict__ G,
                                                                double *__restrict__ partial) {
    const int64_t jv = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t j = jv * VEC;
    const int64_t b = blockIdx.y;
    double pen = 0.0;
    if (j < N) {
        const int64_t base = b * R * N + j;
        float coef[VEC], a[VEC];
        load_f32<VEC>(alpha, b * N + j, a);
#pragma unroll
        for (int v = 0; v < VEC; ++v) coef[v] = lambda * a[v];

        constexpr int RC = RT > 0 ? RT : 1;
        float cache[RC][VEC];
        if constexpr (NEED_S || PEN || RT > 0) {
            float s[VEC];
            double sd[VEC];
#pragma unroll
            for (int v = 0; v < VEC; ++v) { s[v] = 0.0f; sd[v] = 0.0; }
            auto row_step = [&](int32_t r) {
                float w[VEC];
                vec_io<DT, VEC>::load(W, base + (int64_t)r * N, w);
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    if constexpr (RT > 0) cache[r][v] = w[v];
                    if constexpr (NEED_S) s[v] = __builtin_fmaf(w[v], w[v], s[v]);
                    if constexpr (PEN) sd[v] += (double)w[v] * (double)w[v];
                }
            };
            if constexpr (RT > 0) {
#pragma unroll
                for (int32_t r = 0; r < RT; ++r) row_step(r);
            } else {
#pragma unroll 4
                for (int32_t r = 0; r < R; ++r) row_step(r);
            }
            if constexpr (NEED_S || PEN) {
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    if (mode == BSP_ALPHA_NORM) {
                        if constexpr (PEN) pen += (double)lambda * (double)a[v] * sqrt(sd[v]);
                        coef[v] = (s[v] > 0.0f) ? coef[v] / __builtin_sqrtf(s[v]) : 0.0f;
                    } else {
                        if constexpr (PEN) pen += 0.5 * (double)lambda * (double)a[v] * sd[v];
                    }
                }
            }
        }
        auto out_step = [&](int32_t r) {
            const int64_t off = base + (int64_t)r * N;
            float w[VEC], g[VEC];
            if constexpr (RT > 0) {
#pragma unroll
                for (int v = 0; v < VEC; ++v) w[v] = cache[r][v];
            } else {
                vec_io<DT, VEC>::load(W, off, w);
            }
            if (accumulate) {
                vec_io<DT, VEC>::load(G, off, g);
#pragma unroll
                for (int v = 0; v < VEC; ++v) g[v] = __builtin_fmaf(coef[v], w[v], g[v]);
            } else {
#pragma unroll
                for (int v = 0; v < VEC; ++v) g[v] = coef[v] * w[v];
            }
            vec_io<DT, VEC>::store(G, off, g);
        };
        if constexpr (RT > 0) {
#pragma unroll
            for (int32_t r = 0; r < RT; ++r) out_step(r);
        } else {
#pragma unroll 4
            for (int32_t r = 0; r < R; ++r) out_step(r);
        }
    }
    if constexpr (PEN) {
        // fixed-order reduction: lanes by xor-shuffle, wavefronts in index order
        __shared__ double wsum[kThreads / kWave];
#pragma unroll
        for (int o = kWave / 2; o > 0; o >>= 1) pen += __shfl_xor(pen, o, kWave);
        if ((threadIdx.x & (kWave - 1)) == 0) wsum[threadIdx.x / kWave] = pen;
        __syncthreads();
        if (threadIdx.x == 0) {
            double t = 0.0;
            for (int w = 0; w < kThreads / kWave; ++w) t += wsum[w];
            partial[(int64_t)blockIdx.y * gridDim.x + blockIdx.x] = t;
        }
    }
}

// Squared-norm form without the penalty value: coef depends on alpha only, so the gradient is a
// plain element-wise product; one lane per 16-byte vector of W, rows of W along grid.y (and grid.z
// beyond 65535 rows).
template <int DT, int VEC>
__global__ __launch_bounds__(kThreads) void penalty_grad_sq_kernel(const void *__restrict__ W, int64_t M, int64_t N, int32_t R,
                                                                   const float *__restrict__ alpha, float lambda,
                                                                   int accumulate, void *__restrict__ G) {
    const int64_t j = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * VEC;
    if (j >= N) return;
    const int64_t m = (int64_t)blockIdx.z * 65535 + blockIdx.y;
    if (m >= M) return;
    float a[VEC], w[VEC], g[VEC];
    load_f32<VEC>(alpha, (m / R) * N + j, a);
    vec_io<DT, VEC>::load(W, m * N + j, w);
    if (accumulate) {
        vec_io<DT, VEC>::load(G, m * N + j, g);
#pragma unroll
        for (int v = 0; v < VEC; ++v) g[v] = __builtin_fmaf(lambda * a[v], w[v], g[v]);
    } else {
#pragma unroll
        for (int v = 0; v < VEC; ++v) g[v] = (lambda * a[v]) * w[v];
    }
    vec_io<DT, VEC>::store(G, m * N + j, g);
}

// One workgroup sums the per-workgroup partials in index order.
__global__ __launch_bounds__(kThreads) void penalty_finish_kernel(const double *__restrict__ partial, int64_t n,
                                                                  double *__restrict__ out) {
    __shared__ double wsum[kThreads / kWave];
    double t = 0.0;
    for (int64_t i = threadIdx.x; i < n; i += kThreads) t += partial[i];
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) t += __shfl_xor(t, o, kWave);
    if ((threadIdx.x & (kWave - 1)) == 0) wsum[threadIdx.x / kWave] = t;
    __syncthreads();
    if (threadIdx.x == 0) {
        double r = 0.0;
        for (int w = 0; w < kThreads / kWave; ++w) r += wsum[w];
        *out = r;
    }
}

template <int DT>
constexpr int native_vec() { return DT == BSP_F32 ? 1 : 2; }  // 4 bytes per lane

inline int check_matrix(const void *W, int wdt, int64_t M, int64_t N, int32_t R) {
    if (!W) return BSP_ERR_NULL;
    if (!valid_dtype(wdt)) return BSP_ERR_DTYPE;
    if (M <= 0 || N <= 0 || R < 1 || R > 64 || M % R != 0) return BSP_ERR_SHAPE;
    return BSP_OK;
}

inline dim3 grid_for(int64_t N, int vec, int64_t B) {
    int64_t nv = (N + vec - 1) / vec;
    return dim3((unsigned)((nv + kThreads - 1) / kThreads), (unsigned)B, 1);
}

}  // namespace
}  // namespace bsp

using namespace bsp;

extern "C" int bsp_group_norms(const void *W, int wdt, int64_t M, int64_t N, int32_t R, float eps, int mode,
                               float *sumsq, float *norm, float *alpha, void *stream) {
    int st = check_matrix(W, wdt, M, N, R);
    if (st != BSP_OK) return st;
    if (mode != BSP_ALPHA_SQNORM && mode != BSP_ALPHA_NORM) return BSP_ERR_DTYPE;
    const int64_t B = M / R;
    if (B > 65535) return BSP_ERR_SHAPE;
    if (!sumsq && !norm && !alpha) return BSP_OK;
    hipStream_t s = (hipStream_t)stream;
    BSP_DISPATCH_DTYPE(wdt, DT, {
        constexpr int V = native_vec<DT>();
        // (4-byte lanes: 16-byte lanes were measured slower here, on small and on large matrices alike)
        const bool vec_ok = (N % V == 0) && aligned(W, 16) && (!sumsq || aligned(sumsq, 16)) &&
                            (!norm || aligned(norm, 16)) && (!alpha || aligned(alpha, 16));
        if (vec_ok)
            group_norms_kernel<DT, V><<<grid_for(N, V, B), kThreads, 0, s>>>(W, N, R, eps, mode, sumsq, norm, alpha);
        else
            group_norms_kernel<DT, 1><<<grid_for(N, 1, B), kThreads, 0, s>>>(W, N, R, eps, mode, sumsq, norm, alpha);
    });
    return check_launch();
}

extern "C" int bsp_rowseg_norms(const void *W, int wdt, int64_t M, int64_t N, int32_t C, float eps, int mode,
                                float *sumsq, float *norm, float *alpha, void *stream) {
    if (!W) return BSP_ERR_NULL;
    if (!valid_dtype(wdt)) return BSP_ERR_DTYPE;
    if (M <= 0 || N <= 0 || C < 1 || C > 64 || N % C != 0 || M * (N / C) >= ((int64_t)1 << 31)) return BSP_ERR_SHAPE;
    if (mode != BSP_ALPHA_SQNORM && mode != BSP_ALPHA_NORM) return BSP_ERR_DTYPE;
    if (!sumsq && !norm && !alpha) return BSP_OK;
    const int64_t groups = M * (N / C);
    const unsigned grid = (unsigned)((groups + kThreads - 1) / kThreads);
    const size_t lds = (size_t)kThreads * (C + 1) * sizeof(float);
    hipStream_t s = (hipStream_t)stream;
    BSP_DISPATCH_DTYPE(wdt, DT, {
        // (C = 64 needs 65 KB of dynamic LDS, above the default limit)
        auto kern = rowseg_norms_kernel<DT>;
        static thread_local size_t configured = 0;
        if (lds > 65536 && lds > configured) {
            hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) {
                set_last_hip_error((int)e);
                return BSP_ERR_HIP;
            }
            configured = lds;
        }
        kern<<<grid, kThreads, lds, s>>>(W, groups, C, eps, mode, sumsq, norm, alpha);
    });
    return check_launch();
}

extern "C" size_t bsp_penalty_grad_workspace_bytes(int64_t M, int64_t N, int32_t R) {
    if (M <= 0 || N <= 0 || R < 1 || M % R != 0) return 0;
    return (size_t)(M / R) * (size_t)((N + kThreads - 1) / kThreads) * sizeof(double);
}

namespace {
template <int DT, int VEC, int RT>
int launch_penalty(const void *W, int64_t N, int32_t R, int64_t B, const float *alpha, float lambda, int mode,
                   int accumulate, void *G, double *penalty, double *partial, hipStream_t s) {
    dim3 grid = grid_for(N, VEC, B);
    const bool need_s = (mode == BSP_ALPHA_NORM);
    if (penalty) {
        if (need_s)
            penalty_grad_kernel<DT, VEC, RT, true, true><<<grid, kThreads, 0, s>>>(W, N, R, alpha, lambda, mode, accumulate, G, partial);
        else
            penalty_grad_kernel<DT, VEC, RT, false, true><<<grid, kThreads, 0, s>>>(W, N, R, alpha, lambda, mode, accumulate, G, partial);
        int st = check_launch();
        if (st != BSP_OK) return st;
        penalty_finish_kernel<<<1, kThreads, 0, s>>>(partial, (int64_t)grid.x * grid.y, penalty);
    } else {
        if (need_s)
            penalty_grad_kernel<DT, VEC, RT, true, false><<<grid, kThreads, 0, s>>>(W, N, R, alpha, lambda, mode, accumulate, G, nullptr);
        else
            penalty_grad_kernel<DT, VEC, 0, false, false><<<grid, kThreads, 0, s>>>(W, N, R, alpha, lambda, mode, accumulate, G, nullptr);
    }
    return check_launch();
}
}  // namespace

extern "C" int bsp_penalty_grad(const void *W, int wdt, int64_t M, int64_t N, int32_t R, const float *alpha,
                                float lambda, int mode, int accumulate, void *grad, double *penalty, void *ws,
                                size_t ws_bytes, void *stream) {
    int st = check_matrix(W, wdt, M, N, R);
    if (st != BSP_OK) return st;
    if (!alpha || !grad) return BSP_ERR_NULL;
    if (mode != BSP_ALPHA_SQNORM && mode != BSP_ALPHA_NORM) return BSP_ERR_DTYPE;
    const int64_t B = M / R;
    if (B > 65535) return BSP_ERR_SHAPE;
    if (penalty) {
        if (!ws) return BSP_ERR_NULL;
        if (ws_bytes < bsp_penalty_grad_workspace_bytes(M, N, R) || !aligned(ws, 8)) return BSP_ERR_CAPACITY;
    }
    hipStream_t s = (hipStream_t)stream;
    double *partial = (double *)ws;
    if (mode == BSP_ALPHA_SQNORM && !penalty) {
        const unsigned gy = (unsigned)(M < 65535 ? M : 65535), gz = (unsigned)((M + 65534) / 65535);
        BSP_DISPATCH_DTYPE(wdt, DT, {
            constexpr int V16 = DT == BSP_F32 ? 4 : 8;  // 16 bytes per lane: every lane is independent here
            const bool vec_ok = (N % V16 == 0) && aligned(W, 16) && aligned(grad, 16) && aligned(alpha, 16);
            if (vec_ok) {
                const int64_t nv = N / V16;
                const unsigned bs = nv >= 256 ? 256 : (unsigned)((nv + 63) / 64 * 64);
                penalty_grad_sq_kernel<DT, V16><<<dim3((unsigned)((nv + bs - 1) / bs), gy, gz), bs, 0, s>>>(
                    W, M, N, R, alpha, lambda, accumulate, grad);
            } else {
                penalty_grad_sq_kernel<DT, 1><<<dim3((unsigned)((N + 255) / 256), gy, gz), 256, 0, s>>>(
                    W, M, N, R, alpha, lambda, accumulate, grad);
            }
        });
        return check_launch();
    }
    BSP_DISPATCH_DTYPE(wdt, DT, {
        constexpr int V = native_vec<DT>();
        const bool vec_ok = (N % V == 0) && aligned(W, 16) && aligned(grad, 16) && aligned(alpha, 16);
        if (!vec_ok)
            st = launch_penalty<DT, 1, 0>(W, N, R, B, alpha, lambda, mode, accumulate, grad, penalty, partial, s);
        else if (R == 8)
            st = launch_penalty<DT, V, 8>(W, N, R, B, alpha, lambda, mode, accumulate, grad, penalty, partial, s);
        else if (R == 16)
            st = launch_penalty<DT, V, 16>(W, N, R, B, alpha, lambda, mode, accumulate, grad, penalty, partial, s);
        else
            st = launch_penalty<DT, V, 0>(W, N, R, B, alpha, lambda, mode, accumulate, grad, penalty, partial, s);
    });
    return st;
}

#define BSP_NG_LAUNCH(VV, RT) \
    norms_grad_kernel<DT, VV, RT><<<grid, kThreads, 0, s>>>(W, N, R, eps, mode, lambda, accumulate, sumsq, norm, alpha, grad)
extern "C" int bsp_group_norms_grad(const void *W, int wdt, int64_t M, int64_t N, int32_t R, float eps, int mode,
                                    float lambda, int accumulate, float *sumsq, float *norm, float *alpha, void *grad,
                                    void *stream) {
    int st = check_matrix(W, wdt, M, N, R);
    if (st != BSP_OK) return st;
    if (!grad) return BSP_ERR_NULL;
    if (mode != BSP_ALPHA_SQNORM && mode != BSP_ALPHA_NORM) return BSP_ERR_DTYPE;
    const int64_t B = M / R;
    if (B > 65535) return BSP_ERR_SHAPE;
    hipStream_t s = (hipStream_t)stream;
    BSP_DISPATCH_DTYPE(wdt, DT, {
        constexpr int V = native_vec<DT>();
        const bool vec_ok = (N % V == 0) && aligned(W, 16) && aligned(grad, 16) && (!sumsq || aligned(sumsq, 16)) &&
                            (!norm || aligned(norm, 16)) && (!alpha || aligned(alpha, 16));
        const dim3 grid = vec_ok ? grid_for(N, V, B) : grid_for(N, 1, B);
        if (!vec_ok) BSP_NG_LAUNCH(1, 0);
        else if (R == 8) BSP_NG_LAUNCH(V, 8);
        else if (R == 16) BSP_NG_LAUNCH(V, 16);
        else if (R == 32) BSP_NG_LAUNCH(V, 32);
        else BSP_NG_LAUNCH(V, 0);
    });
#undef BSP_NG_LAUNCH
    return check_launch();
}
