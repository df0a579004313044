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
// PAD: counter b lives at hist[b + (b >> 5)] (one spare word per 32), which keeps the lane-strided
// walk below free of LDS bank conflicts for large histograms.
template <bool PAD, typename H>
__device__ __forceinline__ void locate_rank(const H *hist, int nbins, uint32_t want, uint32_t &bin,
                                            uint32_t &rank_in_bin) {
    const int lane = threadIdx.x & (kWave - 1);
    const int per = nbins / kWave;
    auto at = [&](int b) { return hist[PAD ? b + (b >> 5) : b]; };
    uint32_t mine = 0;
    for (int i = 0; i < per; ++i) mine += at(lane * per + i);
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
        uint32_t c = at(owner * per + i);
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
                locate_rank<false>(hist, 256, sh_want, bin, rank);
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
constexpr int kStage = kBins + kBins / 32;  // LDS copy of one histogram, padded

__device__ __forceinline__ int pass_shift(int pass) { return pass == 0 ? 21 : (pass == 1 ? 10 : 0); }
__device__ __forceinline__ int pass_bits(int pass) { return pass == 2 ? kBits2 : kBits0; }

// Workspace of the matrix-scope select: three global histograms, then the state words.
constexpr int kStatePrefix = 3 * kBins;      // key bits fixed so far
constexpr int kStateWant = 3 * kBins + 1;    // rank still wanted inside the current prefix
constexpr int kStateDone = 3 * kBins + 2;    // [3] workgroups that have flushed their histogram, per pass
constexpr int kWsWords = 3 * kBins + 8;

__global__ __launch_bounds__(kThreads) void mask_rank_init_kernel(uint32_t *ws, uint32_t P) {
    const int i = blockIdx.x * kThreads + threadIdx.x;
    if (i < kWsWords) ws[i] = i == kStateWant ? P : 0u;
}

// One digit of the select.  Every workgroup histograms its share in LDS and adds the non-empty
// bins to the pass's global histogram; the workgroup that finishes last (a ticket counter tells)
// locates the bin holding the wanted rank and publishes the longer prefix for the next launch.
__global__ __launch_bounds__(kThreads) void mask_rank_hist_kernel(const float *__restrict__ s, int64_t n, int pass,
                                                                  uint32_t *__restrict__ ws) {
    __shared__ uint32_t hist[kStage];
    __shared__ int s_last;
    const uint32_t prefix = ws[kStatePrefix];
    for (int i = threadIdx.x; i < kBins; i += kThreads) hist[i] = 0;
    __syncthreads();
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
        for (int e = 0; e < 4; ++e) {
            const uint32_t key = to_key(e < cnt ? v[e] : 0.0f);
            const bool in = e < cnt && (pass == 0 || (key >> hi) == (prefix >> hi));
            const uint32_t digit = (key >> shift) & dmask;
            if (pass == 0) {
                // The leading digit (sign, exponent, top mantissa bits) takes only a handful of values:
                // lanes with equal digits elect one lane that adds their count, instead of up to 64
                // serialized LDS atomics on one address.
                uint64_t todo = __ballot(in);
                while (todo) {
                    const int leader = __ffsll((long long)todo) - 1;
                    const uint32_t dl = (uint32_t)__builtin_amdgcn_readlane((int)digit, leader);  // leader is uniform
                    const uint64_t same = __ballot(in && digit == dl);
                    if ((int)(threadIdx.x & (kWave - 1)) == leader) atomicAdd(&hist[dl], (uint32_t)__popcll(same));
                    todo &= ~same;
                }
            } else if (in) {
                atomicAdd(&hist[digit], 1u);
            }
        }
    }
    __syncthreads();
    uint32_t *g = ws + pass * kBins;
    // Device-scope atomics are performed at the memory side, coherent across the chip's L2s.  The
    // additions return their old value and the ticket is taken only after every lane has its
    // returns, so the workgroup that draws the last ticket knows that all additions have landed;
    // no fence is used (a release fence would write back the whole L2 on this multi-L2 part).
    uint32_t seen = 0;
    for (int i = threadIdx.x; i < kBins; i += kThreads) {
        const uint32_t c = hist[i];
        if (c) seen |= atomicAdd(&g[i], c);
    }
    __shared__ uint32_t s_sink[kThreads / kWave];
    if ((threadIdx.x & (kWave - 1)) == 0) s_sink[threadIdx.x / kWave] = seen;  // needs the returns
    __syncthreads();
    if (threadIdx.x == 0) s_last = atomicAdd(&ws[kStateDone + pass], 1u) == gridDim.x - 1;
    __syncthreads();
    if (!s_last) return;
    const int nb = 1 << pass_bits(pass);
    for (int i = threadIdx.x; i < nb; i += kThreads)
        hist[i + (i >> 5)] = __hip_atomic_load(&g[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // read at the memory side
    __syncthreads();
    if (threadIdx.x < kWave) {
        uint32_t bin, rank;
        locate_rank<true>(hist, nb, __hip_atomic_load(&ws[kStateWant], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT), bin, rank);
        if (threadIdx.x == 0) {
            __hip_atomic_store(&ws[kStatePrefix], prefix | (bin << shift), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&ws[kStateWant], rank, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

__global__ __launch_bounds__(kThreads) void mask_rank_apply_kernel(const float *__restrict__ s, int64_t n, int64_t P,
                                                                   const uint32_t *__restrict__ ws,
                                                                   uint8_t *__restrict__ keep,
                                                                   float *__restrict__ t_used) {
    const float thr = P > 0 ? from_key(ws[kStatePrefix]) : -INFINITY;
    if (t_used && blockIdx.x == 0 && threadIdx.x == 0) *t_used = thr;
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
    return scope == BSP_SCOPE_MATRIX ? kWsWords * sizeof(uint32_t) : 0;
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
        mask_rank_init_kernel<<<(kWsWords + kThreads - 1) / kThreads, kThreads, 0, s>>>(ghist, (uint32_t)P);
        // few, large workgroups: every one of them ends with atomics on the same hot bins
        const unsigned g = grid_for_elems(n, 8, 1024);
        for (int pass = 0; pass < 3; ++pass) mask_rank_hist_kernel<<<g, kThreads, 0, s>>>(sumsq, n, pass, ghist);
    }
    mask_rank_apply_kernel<<<grid_for_elems(n, 8, 4096), kThreads, 0, s>>>(sumsq, n, P, ghist, keep, t_used);
    return check_launch();
}
