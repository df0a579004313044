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
#include <mutex>

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
// Three digits of 11 / 11 / 10 bits, one launch per digit plus the launch that writes the mask.
// Workgroups never talk to each other inside a launch: each one histograms its slice of the array in
// LDS and stores the histogram (2048 fine counters plus 64 coarse sums of 32 counters each) to its own
// slot of the workspace with plain stores.  The next launch starts, in every workgroup, by locating
// the digit that holds the wanted rank: it adds up the coarse sums of all slots, picks the coarse bin,
// adds up that bin's 32 fine counters, picks the fine bin.  That costs each workgroup two short
// dependent reads instead of a chip-wide atomic histogram and a last-workgroup election, needs no
// zeroed memory, and is deterministic (integer sums).
constexpr int kSelThreads = 1024;
constexpr int kBins = 2048;     // fine counters per digit (the 10-bit digit uses the lower half)
constexpr int kCoarse = 64;     // coarse sums per digit
constexpr int kSlot = kBins + kCoarse;
constexpr int kMaxSlots = 256;  // workgroups of a histogram launch
constexpr int kStateWords = 16; // state[k] = {key bits fixed after k digits, rank wanted inside them}, k = 1..3
constexpr int kDoneWord = 8;    // state word that counts the workgroups of mask_rank_apply_count_kernel that are done

__device__ __forceinline__ int pass_shift(int pass) { return pass == 0 ? 21 : (pass == 1 ? 10 : 0); }
__device__ __forceinline__ int pass_bits(int pass) { return pass == 2 ? 10 : 11; }
__device__ __forceinline__ const uint32_t *slots_of(const uint32_t *ws, int pass, int G) {
    return ws + kStateWords + (size_t)(pass & 1) * G * kSlot;  // digits alternate between two slot arrays
}

// Every workgroup of the launch after digit d's histogram: find digit d of the wanted element.
// Returns (in all threads) the key bits fixed so far and the rank wanted among the keys that share them.
__device__ __forceinline__ void resolve_digit(const uint32_t *__restrict__ ws, int d, int G, uint32_t P,
                                              uint32_t &prefix, uint32_t &want) {
    __shared__ uint32_t sh_coarse[kCoarse], sh_fine[32], sh_out[2];
    const uint32_t *slots = slots_of(ws, d, G);
    uint32_t prev_prefix = 0, prev_want = P;
    if (d > 0) {  // written by workgroup 0 of the previous launch
        prev_prefix = ws[2 * d];
        prev_want = ws[2 * d + 1];
    }
    if (threadIdx.x < kCoarse) sh_coarse[threadIdx.x] = 0;
    if (threadIdx.x < 32) sh_fine[threadIdx.x] = 0;
    __syncthreads();
    {
        const int c = threadIdx.x & (kCoarse - 1);
        uint32_t sum = 0;
        for (int g = threadIdx.x / kCoarse; g < G; g += kSelThreads / kCoarse) sum += slots[(size_t)g * kSlot + kBins + c];
        if (sum) atomicAdd(&sh_coarse[c], sum);
    }
    __syncthreads();
    if (threadIdx.x < kWave) {
        uint32_t bin, rank;
        locate_rank<false>(sh_coarse, kCoarse, prev_want, bin, rank);
        if (threadIdx.x == 0) {
            sh_out[0] = bin;
            sh_out[1] = rank;
        }
    }
    __syncthreads();
    const uint32_t cb = sh_out[0], want_c = sh_out[1];
    {
        const int f = threadIdx.x & 31;
        uint32_t sum = 0;
        for (int g = threadIdx.x / 32; g < G; g += kSelThreads / 32) sum += slots[(size_t)g * kSlot + cb * 32 + f];
        if (sum) atomicAdd(&sh_fine[f], sum);
    }
    __syncthreads();
    if (threadIdx.x < kWave) {
        const int lane = threadIdx.x;
        const uint32_t mine = lane < 32 ? sh_fine[lane] : 0u;
        uint32_t incl = mine;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) {
            const uint32_t up = __shfl_up(incl, o, kWave);
            if (lane >= o) incl += up;
        }
        const uint64_t reach = __ballot(lane < 32 && incl >= want_c);
        const int fb = reach ? (__ffsll((long long)reach) - 1) : 31;
        const uint32_t before = __shfl(incl - mine, fb, kWave);
        if (lane == 0) {
            sh_out[0] = prev_prefix | ((cb * 32 + (uint32_t)fb) << pass_shift(d));
            sh_out[1] = want_c - before;
        }
    }
    __syncthreads();
    prefix = sh_out[0];
    want = sh_out[1];
    __syncthreads();  // sh_out may be reused by a later call
}

// Histogram of digit PASS over the keys that share the digits found so far.
template <int PASS, int COPIES = 1>
__global__ __launch_bounds__(kSelThreads) void mask_rank_hist_kernel(const float *__restrict__ s, int64_t n,
                                                                     int64_t per_wg, uint32_t P,
                                                                     uint32_t *__restrict__ ws) {
    // The leading digit (sign, exponent, two mantissa bits) takes only a handful of values, so its LDS
    // counters are kept in COPIES copies picked by the lane: fewer lanes collide on one address.  (4 copies on
    // large inputs; 2 on small ones, whose launches are latency-bound anyway and then fit, with 17 KiB of LDS,
    // beside a workgroup that holds most of a compute unit's LDS.)
    __shared__ uint32_t hist[kBins * COPIES];
    const int G = gridDim.x;
    uint32_t prefix = 0, want = P;
    if constexpr (PASS > 0) {
        resolve_digit(ws, PASS - 1, G, P, prefix, want);
        if (blockIdx.x == 0 && threadIdx.x == 0) {
            ws[2 * PASS] = prefix;
            ws[2 * PASS + 1] = want;
        }
    } else {
        // the counter of the launch that writes the mask together with the storage's sizes starts at zero
        if (blockIdx.x == 0 && threadIdx.x == 0) ws[kDoneWord] = 0u;
    }
    for (int i = threadIdx.x; i < kBins * COPIES; i += kSelThreads) hist[i] = 0;
    __syncthreads();
    constexpr int shift = PASS == 0 ? 21 : (PASS == 1 ? 10 : 0);
    constexpr int bits = PASS == 2 ? 10 : 11;
    constexpr int hi = shift + bits;  // bits above the digit must match the prefix
    const int64_t lo = (int64_t)blockIdx.x * per_wg;  // per_wg is a multiple of 4
    const int64_t end = lo + per_wg < n ? lo + per_wg : n;
    const bool vec = (reinterpret_cast<uintptr_t>(s) & 15) == 0;
    const uint32_t copy = COPIES > 1 ? (threadIdx.x & (COPIES - 1)) : 0;
    auto count4 = [&](const float (&v)[4], int cnt) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t key = to_key(e < cnt ? v[e] : 0.0f);
            bool in = e < cnt;
            if constexpr (PASS > 0) in = in && (key >> hi) == (prefix >> hi);
            const uint32_t digit = (key >> shift) & ((1u << bits) - 1u);
            if (in) atomicAdd(&hist[digit * COPIES + copy], 1u);
        }
    };
    // Batches of kBatch 16-byte loads per thread are issued before any of them is used: one load per
    // round trip leaves the kernel waiting on memory latency at large sizes.
    constexpr int kBatch = 4;
    int64_t i = lo + (int64_t)threadIdx.x * 4;
    if (vec) {
        for (; i + (int64_t)(kBatch - 1) * kSelThreads * 4 + 3 < end; i += (int64_t)kBatch * kSelThreads * 4) {
            float4 q[kBatch];
#pragma unroll
            for (int k = 0; k < kBatch; ++k) q[k] = *reinterpret_cast<const float4 *>(s + i + (int64_t)k * kSelThreads * 4);
#pragma unroll
            for (int k = 0; k < kBatch; ++k) {
                const float v[4] = {q[k].x, q[k].y, q[k].z, q[k].w};
                count4(v, 4);
            }
        }
    }
    for (; i < end; i += kSelThreads * 4) {
        float v[4] = {0.f, 0.f, 0.f, 0.f};
        int cnt = 4;
        if (vec && i + 3 < end) {
            const float4 q = *reinterpret_cast<const float4 *>(s + i);
            v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
        } else {
            cnt = (int)((end - i) < 4 ? (end - i) : 4);
            for (int e = 0; e < cnt; ++e) v[e] = s[i + e];
        }
        count4(v, cnt);
    }
    __syncthreads();
    uint32_t *slot = ws + kStateWords + (size_t)(PASS & 1) * G * kSlot + (size_t)blockIdx.x * kSlot;
#pragma unroll
    for (int k = 0; k < kBins / kSelThreads; ++k) {
        const int bin = k * kSelThreads + threadIdx.x;
        uint32_t c = 0;
#pragma unroll
        for (int j = 0; j < COPIES; ++j) c += hist[bin * COPIES + j];
        slot[bin] = c;
        uint32_t sum = c;  // coarse sum: the 32 lanes of a half-wavefront hold one coarse bin
#pragma unroll
        for (int o = 1; o < 32; o <<= 1) sum += __shfl_xor(sum, o, kWave);
        if ((threadIdx.x & 31) == 0) slot[kBins + (bin >> 5)] = sum;
    }
}

__global__ __launch_bounds__(kSelThreads) void mask_rank_apply_kernel(const float *__restrict__ s, int64_t n,
                                                                      uint32_t P, int G,
                                                                      const uint32_t *__restrict__ ws,
                                                                      uint8_t *__restrict__ keep,
                                                                      float *__restrict__ t_used) {
    float thr = -INFINITY;
    if (P > 0) {
        uint32_t prefix, want;
        resolve_digit(ws, 2, G, P, prefix, want);
        thr = from_key(prefix);
    }
    if (t_used && blockIdx.x == 0 && threadIdx.x == 0) *t_used = thr;
    const bool vec = ((reinterpret_cast<uintptr_t>(s) | reinterpret_cast<uintptr_t>(keep)) & 15) == 0;
    // 16 consecutive groups per thread and round: four 16-byte loads in flight, one 16-byte store
    const int64_t stride = (int64_t)gridDim.x * kSelThreads * 16;
    for (int64_t i = ((int64_t)blockIdx.x * kSelThreads + threadIdx.x) * 16; i < n; i += stride) {
        if (vec && i + 15 < n) {
            float4 q[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) q[k] = *reinterpret_cast<const float4 *>(s + i + 4 * k);
            uint32_t w[4];
#pragma unroll
            for (int k = 0; k < 4; ++k)
                w[k] = (uint32_t)(q[k].x > thr) | ((uint32_t)(q[k].y > thr) << 8) | ((uint32_t)(q[k].z > thr) << 16) |
                       ((uint32_t)(q[k].w > thr) << 24);
            *reinterpret_cast<uint4 *>(keep + i) = make_uint4(w[0], w[1], w[2], w[3]);
        } else {
            for (int e = 0; e < 16 && i + e < n; ++e) keep[i + e] = s[i + e] > thr;
        }
    }
}

// The mask of the percentile together with the sizes of its compact storage: keep = (sumsq > threshold), blk_cnt[b] =
// kept groups of row b, blk_ptr = exclusive sums of the counts rounded up to k_align.  A wavefront takes whole rows
// (it has a row's flags in registers when it writes them, so the count is a population count away); the workgroup
// that finishes last -- elected by a counter that the first histogram launch of the same call has cleared -- adds
// up the counts.  Nothing waits on another workgroup.  Integer results: the same as the separate launches'.
__global__ __launch_bounds__(kSelThreads) void mask_rank_apply_count_kernel(const float *__restrict__ s, int64_t B,
                                                                            int64_t N, uint32_t P, int G,
                                                                            uint32_t *__restrict__ ws,
                                                                            uint8_t *__restrict__ keep,
                                                                            float *__restrict__ t_used,
                                                                            int32_t k_align,
                                                                            int32_t *__restrict__ blk_cnt,
                                                                            int32_t *__restrict__ blk_ptr) {
    __shared__ int sh_last, wsum[kSelThreads / kWave];
    uint32_t prefix, want;
    resolve_digit(ws, 2, G, P, prefix, want);
    const float thr = from_key(prefix);
    if (t_used && blockIdx.x == 0 && threadIdx.x == 0) *t_used = thr;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    constexpr int kRows = kSelThreads / kWave;  // rows a workgroup works on at a time
    const bool vec = ((reinterpret_cast<uintptr_t>(s) & 15) | (reinterpret_cast<uintptr_t>(keep) & 3) | (uintptr_t)(N & 3)) == 0;
    for (int64_t b = (int64_t)blockIdx.x * kRows + wave; b < B; b += (int64_t)gridDim.x * kRows) {
        const float *row = s + b * N;
        uint8_t *krow = keep + b * N;
        int cnt = 0;
        if (vec) {
            for (int64_t j = (int64_t)lane * 4; j < N; j += kWave * 4) {
                const float4 q = *reinterpret_cast<const float4 *>(row + j);
                const uint32_t w = (uint32_t)(q.x > thr) | ((uint32_t)(q.y > thr) << 8) | ((uint32_t)(q.z > thr) << 16) |
                                   ((uint32_t)(q.w > thr) << 24);
                *reinterpret_cast<uint32_t *>(krow + j) = w;
                cnt += __popc(w);
            }
        } else {
            for (int64_t j = lane; j < N; j += kWave) {
                const bool k = row[j] > thr;
                krow[j] = k;
                cnt += k;
            }
        }
#pragma unroll
        for (int o = kWave / 2; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o, kWave);
        if (lane == 0) blk_cnt[b] = cnt;
    }
    // The counts of this workgroup are visible on the device before it reports that it is done.  One thread fences for
    // the workgroup, after the barrier that orders its wavefronts' stores before it (a device-wide fence writes the
    // L2 of the workgroup's XCD back and costs microseconds while a layer kernel fills that L2: one per workgroup, not
    // one per thread), and one thread of the elected workgroup fences before the barrier behind which all read.
    __syncthreads();
    if (threadIdx.x == 0) {
        __threadfence();
        const uint32_t done = atomicAdd(&ws[kDoneWord], 1u);
        sh_last = done == gridDim.x - 1;
        if (sh_last) __threadfence();
    }
    __syncthreads();
    if (!sh_last) return;  // (uniform)
    // the last workgroup: every thread owns a run of consecutive row-blocks
    const int64_t per = (B + kSelThreads - 1) / kSelThreads;
    const int64_t lo = (int64_t)threadIdx.x * per, hi = lo + per < B ? lo + per : B;
    auto padded = [&](int64_t b) {
        const int c = __atomic_load_n(&blk_cnt[b], __ATOMIC_RELAXED);  // (written by other workgroups of this launch)
        return (c + k_align - 1) / k_align * k_align;
    };
    int mine = 0;
    for (int64_t b = lo; b < hi; ++b) mine += padded(b);
    int incl = mine;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        const int up = __shfl_up(incl, o, kWave);
        if (lane >= o) incl += up;
    }
    if (lane == kWave - 1) wsum[wave] = incl;
    __syncthreads();
    int run = incl - mine;
    for (int w = 0; w < wave; ++w) run += wsum[w];
    for (int64_t b = lo; b < hi; ++b) {
        blk_ptr[b] = run;
        run += padded(b);
    }
    if (threadIdx.x == kSelThreads - 1) blk_ptr[B] = run;  // the last thread's run ends at B (or is empty)
}

// ------------------------------------------------------------------ masked weights
// A stream over W in 16-byte lanes (4 fp32 or 8 sixteen-bit columns of one row): a vector whose columns are
// all kept is skipped, one whose columns are all pruned is overwritten with zeros without being read, a mixed
// one is read, masked and written back.  (Storing only the pruned elements, as sub-line masked stores, was
// measured three times slower: partial lines are read-modify-write at the memory anyway.)
template <int DT>
__global__ __launch_bounds__(kThreads) void mask_weights_vec_kernel(void *__restrict__ W, int64_t M, int64_t N,
                                                                    int32_t R, const uint8_t *__restrict__ keep) {
    using E = typename elem<DT>::type;
    constexpr int V = 16 / (int)sizeof(E);
    const int64_t j = ((int64_t)blockIdx.x * kThreads + threadIdx.x) * V;
    const int64_t m = (int64_t)blockIdx.z * 65535 + blockIdx.y;
    if (j >= N || m >= M) return;
    const uint8_t *k = keep + (m / R) * N + j;
    uint32_t f[V / 4];
#pragma unroll
    for (int i = 0; i < V / 4; ++i) f[i] = reinterpret_cast<const uint32_t *>(k)[i];
    uint32_t any_kept = 0, any_pruned = 0;
#pragma unroll
    for (int i = 0; i < V / 4; ++i) {
        // fold every flag byte onto its low bit
        uint32_t nz = (f[i] | (f[i] >> 1) | (f[i] >> 2) | (f[i] >> 3) | (f[i] >> 4) | (f[i] >> 5) | (f[i] >> 6) | (f[i] >> 7)) & 0x01010101u;
        f[i] = nz;
        any_kept |= nz;
        any_pruned |= nz ^ 0x01010101u;
    }
    if (!any_pruned) return;
    uint4 *p = reinterpret_cast<uint4 *>((E *)W + m * N + j);
    if (!any_kept) {
        *p = make_uint4(0u, 0u, 0u, 0u);
        return;
    }
    uint4 w = *p;
    uint32_t *wd = reinterpret_cast<uint32_t *>(&w);
    if constexpr (V == 4) {
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (!((f[0] >> (8 * c)) & 1u)) wd[c] = 0u;
    } else {
#pragma unroll
        for (int c = 0; c < 8; ++c)
            if (!((f[c >> 2] >> (8 * (c & 3))) & 1u)) wd[c >> 1] &= (c & 1) ? 0x0000ffffu : 0xffff0000u;
    }
    *p = w;
}

// Any shape and alignment: one lane per element.
template <int DT>
__global__ __launch_bounds__(kThreads) void mask_weights_kernel(void *__restrict__ W, int64_t M, int64_t N, int32_t R,
                                                                const uint8_t *__restrict__ keep) {
    using E = typename elem<DT>::type;
    const int64_t j = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t m = (int64_t)blockIdx.z * 65535 + blockIdx.y;
    if (j >= N || m >= M) return;
    if (keep[(m / R) * N + j] == 0) ((E *)W)[m * N + j] = E(0);
}

// ------------------------------------------------------------------ whole-block pruning and the other division
// Sum of squares of the R x C tiles from the column-group sums: fp32, columns ascending, starting from +0.
__global__ __launch_bounds__(kThreads) void tile_sumsq_kernel(const float *__restrict__ s, int64_t tiles, int32_t C,
                                                              float *__restrict__ ts) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= tiles) return;
    const float *p = s + i * C;  // the tiles of a row of the group array lie end to end (N % C == 0)
    float acc = 0.0f;
    for (int c = 0; c < C; ++c) acc = acc + p[c];
    ts[i] = acc;
}

// keep[b, j] = tkeep[b, j / C] != 0
__global__ __launch_bounds__(kThreads) void expand_tile_mask_kernel(const uint8_t *__restrict__ tkeep, int64_t n,
                                                                    int32_t C, uint8_t *__restrict__ keep) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < n) keep[i] = tkeep[i / C] != 0;  // (flat index / C = flat tile index, since N % C == 0)
}

// W[m, j] = +0 where keep_seg[m, j / C] == 0 (row segments of C columns)
template <int DT>
__global__ __launch_bounds__(kThreads) void mask_weights_rowseg_kernel(void *__restrict__ W, int64_t n, int32_t C,
                                                                       const uint8_t *__restrict__ keep_seg) {
    using E = typename elem<DT>::type;
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < n && keep_seg[i / C] == 0) ((E *)W)[i] = E(0);
}

// Workgroups of the histogram launches: about 16384 elements each (measured best on 0.25 M groups: fewer slots to
// sum at the start of the next launch weigh more than the shorter read), at most kMaxSlots.
inline int select_slots(int64_t n) {
    int64_t g = (n + 16383) / 16384;
    return (int)(g < 1 ? 1 : (g > kMaxSlots ? kMaxSlots : g));
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
    if (scope != BSP_SCOPE_MATRIX || B <= 0 || N <= 0) return 0;
    return ((size_t)kStateWords + 2 * (size_t)select_slots(B * N) * kSlot) * sizeof(uint32_t);
}

namespace {
int prune_mask_launch(const float *sumsq, int64_t B, int64_t N, float t, int64_t n_keep, int scope, uint8_t *keep,
                      float *t_used, void *ws, size_t ws_bytes, void *stream) {
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
    const int64_t P = n - n_keep > 0 ? n - n_keep : 0;
    uint32_t *w = (uint32_t *)ws;
    const int G = select_slots(n);
    if (P > 0) {
        if (!ws) return BSP_ERR_NULL;
        if (ws_bytes < bsp_prune_mask_workspace_bytes(B, N, scope) || !aligned(ws, 4)) return BSP_ERR_CAPACITY;
        int64_t per_wg = (n + G - 1) / G;
        per_wg = (per_wg + 3) / 4 * 4;
        if (n > ((int64_t)1 << 21))
            mask_rank_hist_kernel<0, 4><<<G, kSelThreads, 0, s>>>(sumsq, n, per_wg, (uint32_t)P, w);
        else
            mask_rank_hist_kernel<0, 2><<<G, kSelThreads, 0, s>>>(sumsq, n, per_wg, (uint32_t)P, w);
        mask_rank_hist_kernel<1><<<G, kSelThreads, 0, s>>>(sumsq, n, per_wg, (uint32_t)P, w);
        mask_rank_hist_kernel<2><<<G, kSelThreads, 0, s>>>(sumsq, n, per_wg, (uint32_t)P, w);
    }
    int64_t ga = (n + (int64_t)kSelThreads * 16 - 1) / ((int64_t)kSelThreads * 16);
    ga = ga < 1 ? 1 : (ga > 256 ? 256 : ga);  // a workgroup per compute unit at most: each starts by resolving the last digit
    mask_rank_apply_kernel<<<(unsigned)ga, kSelThreads, 0, s>>>(sumsq, n, (uint32_t)P, G, w, keep, t_used);
    return check_launch();
}

// Scratch of the entry point that allocates nothing: the percentile's state words and histogram slots at their
// largest (kMaxSlots workgroups per histogram launch, two slot arrays), about 4.1 MiB per GPU.  In host code the
// name below is only a handle; the array's device address is looked up once per device.
constexpr size_t kStaticScratchWords = (size_t)kStateWords + 2 * (size_t)kMaxSlots * kSlot;
constexpr int kMaxDevices = 64;
}  // namespace

static __device__ __align__(256) uint32_t scratch[kStaticScratchWords];

namespace {
std::mutex g_scratch_lock;
uint32_t *g_scratch_ptr[kMaxDevices];  // per device, filled on the first call there

int static_scratch(uint32_t **out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) {
        set_last_hip_error((int)e);
        return BSP_ERR_HIP;
    }
    if (dev < 0 || dev >= kMaxDevices) return BSP_ERR_SHAPE;
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));  // the address of this device's copy of the array
        if (e != hipSuccess || !p) {
            set_last_hip_error((int)e);
            return BSP_ERR_HIP;
        }
        g_scratch_ptr[dev] = (uint32_t *)p;
    }
    *out = g_scratch_ptr[dev];
    return BSP_OK;
}
}  // namespace

extern "C" int bsp_prune_mask(const float *sumsq, int64_t B, int64_t N, float t, int64_t n_keep, int scope,
                              uint8_t *keep, float *t_used, void *ws, size_t ws_bytes, void *stream) {
    return prune_mask_launch(sumsq, B, N, t, n_keep, scope, keep, t_used, ws, ws_bytes, stream);
}

extern "C" int bsp_prune_mask_static(const float *sumsq, int64_t B, int64_t N, float t, int64_t n_keep, int scope,
                                     uint8_t *keep, float *t_used, void *stream) {
    if (B <= 0 || N <= 0 || B * N >= ((int64_t)1 << 31)) return BSP_ERR_SHAPE;  // beyond what the scratch serves
    if (bsp_prune_mask_workspace_bytes(B, N, scope) > kStaticScratchWords * sizeof(uint32_t)) return BSP_ERR_CAPACITY;
    uint32_t *ws = nullptr;
    const int st = static_scratch(&ws);
    if (st != BSP_OK) return st;
    // every histogram launch overwrites the state words and all the slots the next launch reads, so nothing of
    // the previous call's contents has to be cleared
    return prune_mask_launch(sumsq, B, N, t, n_keep, scope, keep, t_used, ws, kStaticScratchWords * sizeof(uint32_t),
                             stream);
}

extern "C" int bsp_prune_mask_count(const float *sumsq, int64_t B, int64_t N, float t, int64_t n_keep, int scope,
                                    uint8_t *keep, float *t_used, int32_t k_align, int32_t *blk_cnt, int32_t *blk_ptr,
                                    void *ws, size_t ws_bytes, void *stream) {
    if (!sumsq || !keep || !blk_cnt || !blk_ptr) return BSP_ERR_NULL;
    if (B <= 0 || N <= 0 || B * N >= ((int64_t)1 << 31) || (B * (N + 63)) >= ((int64_t)1 << 31)) return BSP_ERR_SHAPE;
    if (k_align != 1 && k_align != 8 && k_align != 16 && k_align != 32 && k_align != 64) return BSP_ERR_SHAPE;
    const int64_t n = B * N;
    const int64_t P = n_keep >= 0 ? (n - n_keep > 0 ? n - n_keep : 0) : 0;
    if (n_keep < 0 || scope != BSP_SCOPE_MATRIX || P == 0) {
        // the forms whose mask comes from one launch (a given threshold, the row-block scope, nothing to prune):
        // the two stages one after the other
        const int st = prune_mask_launch(sumsq, B, N, t, n_keep, scope, keep, t_used, ws, ws_bytes, stream);
        if (st != BSP_OK) return st;
        return bsp_pack_count(keep, B, N, k_align, blk_cnt, blk_ptr, stream);
    }
    if (!ws) return BSP_ERR_NULL;
    if (ws_bytes < bsp_prune_mask_workspace_bytes(B, N, scope) || !aligned(ws, 4)) return BSP_ERR_CAPACITY;
    hipStream_t s = (hipStream_t)stream;
    uint32_t *w = (uint32_t *)ws;
    const int G = select_slots(n);
    int64_t per_wg = (n + G - 1) / G;
    per_wg = (per_wg + 3) / 4 * 4;
    if (n > ((int64_t)1 << 21))
        mask_rank_hist_kernel<0, 4><<<G, kSelThreads, 0, s>>>(sumsq, n, per_wg, (uint32_t)P, w);
    else
        mask_rank_hist_kernel<0, 2><<<G, kSelThreads, 0, s>>>(sumsq, n, per_wg, (uint32_t)P, w);
    mask_rank_hist_kernel<1><<<G, kSelThreads, 0, s>>>(sumsq, n, per_wg, (uint32_t)P, w);
    mask_rank_hist_kernel<2><<<G, kSelThreads, 0, s>>>(sumsq, n, per_wg, (uint32_t)P, w);
    constexpr int kRows = kSelThreads / kWave;
    int64_t ga = (B + kRows - 1) / kRows;
    ga = ga > 256 ? 256 : ga;  // a workgroup per compute unit at most: each starts by resolving the last digit
    mask_rank_apply_count_kernel<<<(unsigned)ga, kSelThreads, 0, s>>>(sumsq, B, N, (uint32_t)P, G, w, keep, t_used,
                                                                     k_align, blk_cnt, blk_ptr);
    return check_launch();
}

extern "C" int bsp_mask_weights(void *W, int wdt, int64_t M, int64_t N, int32_t R, const uint8_t *keep, void *stream) {
    if (!W || !keep) return BSP_ERR_NULL;
    if (!valid_dtype(wdt)) return BSP_ERR_DTYPE;
    if (M <= 0 || N <= 0 || R < 1 || R > 64 || M % R != 0) return BSP_ERR_SHAPE;
    hipStream_t s = (hipStream_t)stream;
    const unsigned gy = (unsigned)(M < 65535 ? M : 65535), gz = (unsigned)((M + 65534) / 65535);
    const int V = wdt == BSP_F32 ? 4 : 8;
    const bool vec = N % V == 0 && aligned(W, 16) && aligned(keep, 4);
    BSP_DISPATCH_DTYPE(wdt, DT, {
        if (vec)
            mask_weights_vec_kernel<DT><<<dim3((unsigned)((N / V + kThreads - 1) / kThreads), gy, gz), kThreads, 0, s>>>(
                W, M, N, R, keep);
        else
            mask_weights_kernel<DT><<<dim3((unsigned)((N + kThreads - 1) / kThreads), gy, gz), kThreads, 0, s>>>(W, M, N,
                                                                                                              R, keep);
    });
    return check_launch();
}

extern "C" int bsp_tile_sumsq(const float *sumsq, int64_t B, int64_t N, int32_t C, float *tile_sumsq, void *stream) {
    if (!sumsq || !tile_sumsq) return BSP_ERR_NULL;
    if (B <= 0 || N <= 0 || C < 1 || C > N || N % C != 0 || B * N >= ((int64_t)1 << 31)) return BSP_ERR_SHAPE;
    const int64_t tiles = B * (N / C);
    tile_sumsq_kernel<<<(unsigned)((tiles + kThreads - 1) / kThreads), kThreads, 0, (hipStream_t)stream>>>(sumsq, tiles, C,
                                                                                                     tile_sumsq);
    return check_launch();
}

extern "C" int bsp_expand_tile_mask(const uint8_t *tile_keep, int64_t B, int64_t N, int32_t C, uint8_t *keep,
                                    void *stream) {
    if (!tile_keep || !keep) return BSP_ERR_NULL;
    if (B <= 0 || N <= 0 || C < 1 || C > N || N % C != 0 || B * N >= ((int64_t)1 << 31)) return BSP_ERR_SHAPE;
    const int64_t n = B * N;
    expand_tile_mask_kernel<<<(unsigned)((n + kThreads - 1) / kThreads), kThreads, 0, (hipStream_t)stream>>>(tile_keep, n, C,
                                                                                                       keep);
    return check_launch();
}

extern "C" int bsp_mask_weights_rowseg(void *W, int wdt, int64_t M, int64_t N, int32_t C, const uint8_t *keep_seg,
                                       void *stream) {
    if (!W || !keep_seg) return BSP_ERR_NULL;
    if (!valid_dtype(wdt)) return BSP_ERR_DTYPE;
    if (M <= 0 || N <= 0 || C < 1 || C > N || N % C != 0 || M * N >= ((int64_t)1 << 40)) return BSP_ERR_SHAPE;
    const int64_t n = M * N;
    const int64_t grid = (n + kThreads - 1) / kThreads;
    if (grid >= ((int64_t)1 << 31)) return BSP_ERR_SHAPE;
    BSP_DISPATCH_DTYPE(wdt, DT, {
        mask_weights_rowseg_kernel<DT><<<(unsigned)grid, kThreads, 0, (hipStream_t)stream>>>(W, n, C, keep_seg);
    });
    return check_launch();
}
