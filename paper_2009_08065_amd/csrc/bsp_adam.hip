// One weight update of Alg. 2: Adam on the mixed loss (reweighted training: the regulariser's
// gradient of Eq. 3, with the factors held fixed, is added to the incoming gradient on the fly)
// or on the prediction loss followed by W = W * Mask (retraining), in one pass over the state.
//
// Per parameter 16 bytes are read (w, g, m, v) and 12 written (w, m, v); the factor and the mask
// byte of a group are read once per R parameters.  The path is HBM-bound and every lane owns
// whole groups (a column segment of a row-block), so no reduction crosses lanes.
// Adam itself is Kingma & Ba's Algorithm 1, evaluated in fp32 with one rounding per operation.
#include "bsp_common.h"

#include <cmath>

namespace bsp {
namespace {

constexpr int kThreads = 256;

struct AdamScalars {
    float lr, beta1, beta2, omb1, omb2, c1, c2, eps;
};

// grid.x covers the columns, one per lane (4-byte lanes stream faster here than 16-byte ones: measured 5.4 against
// 5.1 TB/s on 0.8 G parameters), grid.y the row-blocks.  REG: the regulariser's gradient is added (alpha != nullptr);
// MASK: pruned groups are written as +0 (keep != nullptr).
template <int GDT, bool REG, bool MASK>
__global__ __launch_bounds__(kThreads) void adam_step_kernel(float *__restrict__ W, const void *__restrict__ G,
                                                             float *__restrict__ m, float *__restrict__ v, int64_t N,
                                                             int32_t R, const float *__restrict__ alpha, float lambda,
                                                             int mode, const uint8_t *__restrict__ keep, AdamScalars h) {
    const int64_t j = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (j >= N) return;
    const int64_t b = blockIdx.y;
    const int64_t base = b * R * N + j;
    float coef = 0.0f;
    bool kept = true;
    if constexpr (REG) {
        coef = lambda * alpha[b * N + j];
        if (mode == BSP_ALPHA_NORM) {  // the factor multiplies the norm itself: d||w||/dw = w / ||w||
            float s = 0.0f;
#pragma unroll 4
            for (int32_t r = 0; r < R; ++r) {
                const float w = W[base + (int64_t)r * N];
                s = __builtin_fmaf(w, w, s);
            }
            coef = (s > 0.0f) ? coef / __builtin_sqrtf(s) : 0.0f;
        }
    }
    if constexpr (MASK) kept = keep[b * N + j] != 0;
#pragma unroll 4
    for (int32_t r = 0; r < R; ++r) {
        const int64_t off = base + (int64_t)r * N;
        const float w = W[off];
        float g = elem<GDT>::load(G, off);
        if constexpr (REG) g = __builtin_fmaf(coef, w, g);
        const float t1 = h.beta1 * m[off];
        const float t2 = h.omb1 * g;
        const float mn = t1 + t2;
        const float t3 = h.beta2 * v[off];
        float t4 = h.omb2 * g;
        t4 = t4 * g;
        const float vn = t3 + t4;
        const float mh = mn / h.c1;
        const float vh = vn / h.c2;
        const float num = h.lr * mh;
        const float den = __builtin_sqrtf(vh) + h.eps;
        const float q = num / den;
        float wn = w - q;
        if constexpr (MASK) wn = kept ? wn : 0.0f;
        W[off] = wn;
        m[off] = mn;
        v[off] = vn;
    }
}

template <int GDT>
void launch_adam(dim3 grid, hipStream_t s, float *W, const void *G, float *m, float *v, int64_t N, int32_t R,
                 const float *alpha, float lambda, int mode, const uint8_t *keep, const AdamScalars &h) {
    if (alpha && keep)
        adam_step_kernel<GDT, true, true><<<grid, kThreads, 0, s>>>(W, G, m, v, N, R, alpha, lambda, mode, keep, h);
    else if (alpha)
        adam_step_kernel<GDT, true, false><<<grid, kThreads, 0, s>>>(W, G, m, v, N, R, alpha, lambda, mode, keep, h);
    else if (keep)
        adam_step_kernel<GDT, false, true><<<grid, kThreads, 0, s>>>(W, G, m, v, N, R, alpha, lambda, mode, keep, h);
    else
        adam_step_kernel<GDT, false, false><<<grid, kThreads, 0, s>>>(W, G, m, v, N, R, alpha, lambda, mode, keep, h);
}

}  // namespace
}  // namespace bsp

using namespace bsp;

extern "C" int bsp_adam_step(float *W, const void *G, int gdt, float *m, float *v, int64_t M, int64_t N, int32_t R,
                             const float *alpha, float lambda, int mode, const uint8_t *keep, float lr, float beta1,
                             float beta2, float eps, int64_t t, void *stream) {
    if (!W || !G || !m || !v) return BSP_ERR_NULL;
    if (!valid_dtype(gdt)) return BSP_ERR_DTYPE;
    if (M <= 0 || N <= 0 || R <= 0 || M % R != 0 || t < 1) return BSP_ERR_SHAPE;
    if (alpha && mode != BSP_ALPHA_SQNORM && mode != BSP_ALPHA_NORM) return BSP_ERR_DTYPE;
    const int64_t B = M / R;
    if (B > 65535) return BSP_ERR_SHAPE;
    AdamScalars h;
    h.lr = lr;
    h.beta1 = beta1;
    h.beta2 = beta2;
    h.omb1 = 1.0f - beta1;
    h.omb2 = 1.0f - beta2;
    h.c1 = (float)(1.0 - std::pow((double)beta1, (double)t));
    h.c2 = (float)(1.0 - std::pow((double)beta2, (double)t));
    h.eps = eps;
    hipStream_t s = (hipStream_t)stream;
    const dim3 grid((unsigned)((N + kThreads - 1) / kThreads), (unsigned)B);
    BSP_DISPATCH_DTYPE(gdt, GDT, { launch_adam<GDT>(grid, s, W, G, m, v, N, R, alpha, lambda, mode, keep, h); });
    return check_launch();
}
