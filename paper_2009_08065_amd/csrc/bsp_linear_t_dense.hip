// The transposed product as a dense product on the masked matrix:
//   Z[t, n] = bias[n] + sum_m U[t, m] * Wm[m, n],   Wm = W after Alg. 1 (pruned groups zero: bsp_mask_weights)
// -- the input gradient of the layer of Sec. 3.1 (dX = dY Wp), and the layer of the row-segment variant on a
// transposed matrix, computed without the compact storage.  It spends 1 / density times the multiplications of
// bsp_linear_transposed, but as one plain dense product, which is the vendor library's job: at the compression
// rates of the paper (1.4x to 5x) that is the faster way on this machine (measured on the BERT-large set at 5x:
// 52 against 171 us for the 3072 x 1024 matrix), and the gather form only wins from about 16x on.
//
// The product is handed to rocBLAS (rocblas_gemm_ex, fp32 accumulation), which is loaded when this entry point is
// first called, so that the rest of the library does not depend on it.  Row-major Z = U Wm is, in the column-major
// terms of BLAS, Z^T [N x T] = Wm^T [N x M] * U^T [M x T] with no operand transposed.
#include <dlfcn.h>

#include <mutex>

#include "bsp_common.h"

namespace bsp {
namespace {

// the few rocBLAS names this file needs, as the library's C interface declares them
typedef void *rb_handle;
typedef int (*rb_create_handle_t)(rb_handle *);
typedef int (*rb_set_stream_t)(rb_handle, hipStream_t);
typedef int (*rb_gemm_ex_t)(rb_handle, int, int, int, int, int, const void *, const void *, int, int, const void *, int,
                            int, const void *, const void *, int, int, void *, int, int, int, int, int32_t, uint32_t);
constexpr int kRbOpNone = 111;
constexpr int kRbF16 = 150, kRbF32 = 151, kRbBF16 = 168;
constexpr int kRbAlgoStandard = 0;

struct Blas {
    rb_create_handle_t create = nullptr;
    rb_set_stream_t set_stream = nullptr;
    rb_gemm_ex_t gemm_ex = nullptr;
    bool tried = false, ok = false;
};
std::mutex g_blas_lock;
Blas g_blas;
constexpr int kMaxDevices = 64;
rb_handle g_handle[kMaxDevices];  // one per device, made on the first call there

bool load_blas() {
    if (g_blas.tried) return g_blas.ok;
    g_blas.tried = true;
    void *lib = nullptr;
    for (const char *name : {"librocblas.so", "librocblas.so.5", "/opt/rocm/lib/librocblas.so"}) {
        lib = dlopen(name, RTLD_NOW | RTLD_LOCAL);
        if (lib) break;
    }
    if (!lib) return false;
    g_blas.create = (rb_create_handle_t)dlsym(lib, "rocblas_create_handle");
    g_blas.set_stream = (rb_set_stream_t)dlsym(lib, "rocblas_set_stream");
    g_blas.gemm_ex = (rb_gemm_ex_t)dlsym(lib, "rocblas_gemm_ex");
    g_blas.ok = g_blas.create && g_blas.set_stream && g_blas.gemm_ex;
    return g_blas.ok;
}

template <int DT>
__global__ __launch_bounds__(256) void fill_rows_kernel(const void *__restrict__ bias, int64_t T, int64_t N,
                                                        void *__restrict__ Z) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= T * N) return;
    elem<DT>::store(Z, i, elem<DT>::load(bias, i % N));
}

}  // namespace
}  // namespace bsp

using namespace bsp;

extern "C" int bsp_linear_transposed_dense(const void *U, int udt, int64_t T, int64_t M, int64_t N, const void *Wm,
                                           const void *bias, void *Z, void *stream) {
    if (!U || !Wm || !Z) return BSP_ERR_NULL;
    if (!valid_dtype(udt)) return BSP_ERR_DTYPE;
    if (T < 0 || M <= 0 || N <= 0 || T >= ((int64_t)1 << 31) || M >= ((int64_t)1 << 31) || N >= ((int64_t)1 << 31))
        return BSP_ERR_SHAPE;
    if (T == 0) return BSP_OK;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) {
        set_last_hip_error((int)e);
        return BSP_ERR_HIP;
    }
    if (dev < 0 || dev >= kMaxDevices) return BSP_ERR_SHAPE;
    rb_handle h = nullptr;
    {
        std::lock_guard<std::mutex> hold(g_blas_lock);
        if (!load_blas()) return BSP_ERR_HIP;  // (the dense-product library is not there)
        if (!g_handle[dev] && g_blas.create(&g_handle[dev]) != 0) {
            g_handle[dev] = nullptr;
            return BSP_ERR_HIP;
        }
        h = g_handle[dev];
    }
    hipStream_t s = (hipStream_t)stream;
    if (bias) {  // Z starts as the bias in every row and the product is added to it (in fp32, one rounding)
        if (T * N >= ((int64_t)1 << 39)) return BSP_ERR_SHAPE;
        const unsigned grid = (unsigned)((T * N + 255) / 256);
        BSP_DISPATCH_DTYPE(udt, DT, (fill_rows_kernel<DT><<<grid, 256, 0, s>>>(bias, T, N, Z)));
        const int st = check_launch();
        if (st != BSP_OK) return st;
    }
    const float alpha = 1.0f, beta = bias ? 1.0f : 0.0f;
    const int dt = udt == BSP_BF16 ? kRbBF16 : (udt == BSP_F16 ? kRbF16 : kRbF32);
    // one call at a time per device: the handle carries the stream
    std::lock_guard<std::mutex> hold(g_blas_lock);
    if (g_blas.set_stream(h, s) != 0) return BSP_ERR_HIP;
    const int rc = g_blas.gemm_ex(h, kRbOpNone, kRbOpNone, (int)N, (int)T, (int)M, &alpha, Wm, dt, (int)N, U, dt, (int)M,
                                  &beta, Z, dt, (int)N, Z, dt, (int)N, kRbF32, kRbAlgoStandard, 0, 0);
    return rc == 0 ? BSP_OK : BSP_ERR_HIP;
}
