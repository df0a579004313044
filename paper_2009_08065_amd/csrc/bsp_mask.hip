// Prune decision of Alg. 1 (a group whose norm is <= the threshold is removed) with the
// threshold either given or taken as a percentile of the group norms (Sec. 3.1).
//
// The percentile is an exact order statistic found by a most-significant-digit radix select
// on the bit patterns of the sums of squares: a histogram per digit, integer counters only,
// so the result does not depend on the order in which lanes or workgroups run.
//   row-block scope : one workgroup per row of the [B, N] array, 4 digits of 8 bits, all in LDS.
//   matrix scope    : 3 digits of 11 / 11 / 10 bits; every workgroup builds an LDS histogram of
//                     its share and flushes the non-empty bins to a global histogram; the next
//                     launch starts by locating the digit that holds the wanted rank.
// The final pass writes keep = (sumsq > threshold).
#include "bsp_common.h"

namespace bsp {
namespace {

constexpr int kThreads = 256;

// Order-preserving map from fp32 to uint32 (negative values below positive ones).
__device__ __forceinline__ uint32_t to_key(float f) {
    uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float from_key(uint32_t k) {
    uint32_t u = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
    return __uint_as_float(u);
}

// ------------------------------------------------------------------ threshold form
__global__ __launch_bounds__(kThreads) void mask_threshold_kernel(const float *__restrict__ s, int64_t n, float t,
                                                                  uint8_t *__restrict__ keep) {
    const double t2 = (double)t * (double)t;  // exact: a product of two fp32 fits in fp64
    const bool all = t < 0.0f;
    int64_t i = ((int64_t)blockIdx.x * kThreads + threadIdx.x) * 4;
    if (i + 3 < n && ((reinterpret_cast<uintptr_t>(s) | reinterpret_cast<uintptr_t>(keep)) & 15) == 0) {
        float4 v = *reinterpret_cast<const float4 *>(s + i);
        uchar4 k;
        k.x = all || (double)v.x > t2;
        k.y = all || (double)v.y > t2;
        k.z = all || (double)v.z > t2;
        k.w = all || (double)v.w > t2;
        *reinterpret_cast<uchar4 *>(keep + i) = k;
    } else {
        for (int e = 0; e < 4 && i + e < n; ++e) keep[i + e] = all || (double)s[i + e] > t2;
    }
}

// Wavefront 0 finds, in a histogram of `nbins` counters (nbins a multiple of 64), the bin that
// holds the element of rank `want` (1-based) and the rank inside that bin.  All lanes of the
// wavefront return the same pair.
template <typename H>
__device__ __forceinline__ void locate_rank(const H *hist, int nbins, uint32_t want, uint32_t &bin,
                                            uint32_t &rank_in_bin) {
    const int lane = threadIdx.x & (kWave - 1);
    const int per = nbins / kWave;
    uint32_t mine = 0;
    for (int i = 0; i < per; ++i) mine += hist[lane * per + i];
    uint32_t incl = mine;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        uint32_t up = __shfl_up(incl, o, kWave);
        if (lane >= o) incl += up;
    }
    const uint64_t reach = __ballot(incl >= want);
    const int owner = reach ? (__ffsll((long long)reach) - 1) : (kWave - 1);
    const uint32_t before = __shfl(incl - mine, owner, kWave);
    uint32_t cum = before, found_bin = (uint32_t)(owner * per + per - 1), found_rank = 1;
    bool done = false;
    for (int i = 0; i < per; ++i) {  // every lane walks the owner's bins: same result everywhere
        uint32_t c = hist[owner * per + i];
        if (!done && cum + c >= want) {
            found_bin = (uint32_t)(owner * per + i);
            found_rank = want - cum;
            done = true;
        }
        cum += c;
    }
    bin = found_bin;
    rank_in_bin = found_rank;
}

// ------------------------------------------------------------------ percentile, row-block scope
__global__ __launch_bounds__(kThreads) void mask_rank_block_kernel(const float *__restrict__ s, int64_t N,
                                                                   int64_t n_keep, uint8_t *__restrict__ keep,
                                                                   float *__restrict__ t_used) {
    __shared__ uint32_t hist[256];
    __shared__ uint32_t sh_prefix, sh_want;
    const float *row = s + (int64_t)blockIdx.x * N;
    uint8_t *krow = keep + (int64_t)blockIdx.x * N;
    const int64_t P = N - n_keep;
    float thr = -INFINITY;
    if (P > 0) {
        if (threadIdx.x == 0) {
            sh_prefix = 0;
            sh_want = (uint32_t)(P > N ? N : P);
        }
        for (int pass = 0; pass < 4; ++pass) {
            const int shift = 24 - 8 * pass;
            hist[threadIdx.x] = 0;
            __syncthreads();
            const uint32_t prefix = sh_prefix;
            for (int64_t i = threadIdx.x; i < N; i += kThreads) {
                const uint32_t key = to_key(row[i]);
                const bool in = pass == 0 || (key >> (shift + 8)) == (prefix >> (shift + 8));
                if (in) atomicAdd(&hist[(key >> shift) & 255u], 1u);
            }
            __syncthreads();
            if (threadIdx.x < kWave) {
                uint32_t bin, rank;
                locate_rank(hist, 256, sh_want, bin, rank);
                if (threadIdx.x == 0) {
                    sh_prefix = prefix | (bin << shift);
                    sh_want = rank;
                }
            }
            __syncthreads();
        }
        thr = from_key(sh_prefix);
    }
    for (int64_t i = threadIdx.x; i < N; i += kThreads) krow[i] = row[i] > thr;
    if (t_used && threadIdx.x == 0) t_used[blockIdx.x] = thr;
}

// ------------------------------------------------------------------ percentile, matrix scope
constexpr int kBits0 = 11, kBits2 = 10;  // digits: 11, 11, 10 bits
constexpr int kBins = 2048;  // per-pass stride in the global histogram

__device__ __forceinline__ int pass_shift(int pass) { return pass == 0 ? 21 : (pass == 1 ? 10 : 0); }
__device__ __forceinline__ int pass_bits(int pass) { return pass == 2 ? kBits2 : kBits0; }

// Wavefront 0 replays the digits chosen by passes 0 .. upto-1 from the global histograms.
__device__ __forceinline__ void resolve_prefix(const uint32_t *ghist, int upto, uint32_t P, uint32_t &prefix,
                                               uint32_t &want) {
    prefix = 0;
    want = P;
    for (int p = 0; p < upto; ++p) {
        uint32_t bin, rank;
        locate_rank(ghist + p * kBins, 1 << pass_bits(p), want, bin, rank);
        prefix |= bin << pass_shift(p);
        want = rank;
    }
}

__global__ __launch_bounds__(kThreads) void zero_u32_kernel(uint32_t *p, int n) {
    int i = blockIdx.x * kThreads + threadIdx.x;
    if (i < n) p[i] = 0;
}

__global__ __launch_bounds__(kThreads) void mask_rank_hist_kernel(const float *__restrict__ s, int64_t n, uint32_t P,
                                                                  int pass, uint32_t *__restrict__ ghist) {
    __shared__ uint32_t hist[kBins];
    __shared__ uint32_t sh_prefix;
    for (int i = threadIdx.x; i < kBins; i += kThreads) hist[i] = 0;
    if (threadIdx.x < kWave) {
        uint32_t prefix, want;
        resolve_prefix(ghist, pass, P, prefix, want);
        if (threadIdx.x == 0) sh_prefix = prefix;
    }
    __syncthreads();
    const uint32_t prefix = sh_prefix;
    const int shift = pass_shift(pass);
    const uint32_t dmask = (1u << pass_bits(pass)) - 1u;
    const int hi = shift + pass_bits(pass);  // bits above the digit must match the prefix
    const int64_t stride = (int64_t)gridDim.x * kThreads * 4;
    const bool vec = (reinterpret_cast<uintptr_t>(s) & 15) == 0;
    for (int64_t i = ((int64_t)blockIdx.x * kThreads + threadIdx.x) * 4; i < n; i += stride) {
        float v[4];
        int cnt = 4;
        if (vec && i + 3 < n) {
            float4 q = *reinterpret_cast<const float4 *>(s + i);
            v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
        } else {
            cnt = (int)((n - i) < 4 ? (n - i) : 4);
            for (int e = 0; e < cnt; ++e) v[e] = s[i + e];
        }
        for (int e = 0; e < cnt; ++e) {
            const uint32_t key = to_key(v[e]);
            const bool in = pass == 0 || (key >> hi) == (prefix >> hi);
            if (in) atomicAdd(&hist[(key >> shift) & dmask], 1u);
        }
    }
    __syncthreads();
    uint32_t *g = ghist + pass * kBins;
    for (int i = threadIdx.x; i < kBins; i += kThreads) {
        const uint32_t c = hist[i];
        if (c) atomicAdd(&g[i], c);
    }
}

__global__ __launch_bounds__(kThreads) void mask_rank_apply_kernel(const float *__restrict__ s, int64_t n, int64_t P,
                                                                   const uint32_t *__restrict__ ghist,
                                                                   uint8_t *__restrict__ keep,
                                                                   float *__restrict__ t_used) {
    __shared__ float sh_thr;
    if (threadIdx.x < kWave) {
        float thr = -INFINITY;
        if (P > 0) {
            uint32_t prefix, want;
            resolve_prefix(ghist, 3, (uint32_t)P, prefix, want);
            thr = from_key(prefix);
        }
        if (threadIdx.x == 0) {
            sh_thr = thr;
            if (t_used && blockIdx.x == 0) *t_used = thr;
        }
    }
    __syncthreads();
    const float thr = sh_thr;
    const int64_t stride = (int64_t)gridDim.x * kThreads * 4;
    const bool vec = ((reinterpret_cast<uintptr_t>(s) | reinterpret_cast<uintptr_t>(keep)) & 15) == 0;
    for (int64_t i = ((int64_t)blockIdx.x * kThreads + threadIdx.x) * 4; i < n; i += stride) {
        if (vec && i + 3 < n) {
            float4 q = *reinterpret_cast<const float4 *>(s + i);
            uchar4 k;
            k.x = q.x > thr; k.y = q.y > thr; k.z = q.z > thr; k.w = q.w > thr;
            *reinterpret_cast<uchar4 *>(keep + i) = k;
        } else {
            for (int e = 0; e < 4 && i + e < n; ++e) keep[i + e] = s[i + e] > thr;
        }
    }
}

inline unsigned grid_for_elems(int64_t n, int per_thread, unsigned cap) {
    int64_t g = (n + (int64_t)kThreads * per_thread - 1) / ((int64_t)kThreads * per_thread);
    if (g < 1) g = 1;
    if (cap && g > cap) g = cap;
    return (unsigned)g;
}

}  // namespace
}  // namespace bsp

using namespace bsp;

extern "C" size_t bsp_prune_mask_workspace_bytes(int64_t B, int64_t N, int scope) {
    (void)B; (void)N;
    return scope == BSP_SCOPE_MATRIX ? 3 * kBins * sizeof(uint32_t) : 0;
}

extern "C" int bsp_prune_mask(const float *sumsq, int64_t B, int64_t N, float t, int64_t n_keep, int scope,
                              uint8_t *keep, float *t_used, void *ws, size_t ws_bytes, void *stream) {
    if (!sumsq || !keep) return BSP_ERR_NULL;
    if (B <= 0 || N <= 0 || B * N >= ((int64_t)1 << 31)) return BSP_ERR_SHAPE;
    if (scope != BSP_SCOPE_BLOCK && scope != BSP_SCOPE_MATRIX) return BSP_ERR_DTYPE;
    hipStream_t s = (hipStream_t)stream;
    const int64_t n = B * N;
    if (n_keep < 0) {
        mask_threshold_kernel<<<grid_for_elems(n, 4, 0), kThreads, 0, s>>>(sumsq, n, t, keep);
        return check_launch();
    }
    if (scope == BSP_SCOPE_BLOCK) {
        mask_rank_block_kernel<<<(unsigned)B, kThreads, 0, s>>>(sumsq, N, n_keep, keep, t_used);
        return check_launch();
    }
    const int64_t P = n - n_keep;
    uint32_t *ghist = (uint32_t *)ws;
    if (P > 0) {
        if (!ws) return BSP_ERR_NULL;
        if (ws_bytes < bsp_prune_mask_workspace_bytes(B, N, scope) || !aligned(ws, 4)) return BSP_ERR_CAPACITY;
        zero_u32_kernel<<<(3 * kBins + kThreads - 1) / kThreads, kThreads, 0, s>>>(ghist, 3 * kBins);
        const unsigned g = grid_for_elems(n, 16, 2048);
        for (int pass = 0; pass < 3; ++pass)
            mask_rank_hist_kernel<<<g, kThreads, 0, s>>>(sumsq, n, (uint32_t)P, pass, ghist);
    }
    mask_rank_apply_kernel<<<grid_for_elems(n, 16, 4096), kThreads, 0, s>>>(sumsq, n, P, ghist, keep, t_used);
    return check_launch();
}
