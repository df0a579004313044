// Compact storage of a block-structure-pruned weight (Sec. 3.1: only the kept columns of a
// block need an index; Sec. 4.4: the kept values form a smaller dense panel).
//
//   bsp_pack_count : kept columns per row-block (ballot + popcount per wavefront) and the
//                    exclusive scan of the padded counts.
//   bsp_pack       : one workgroup per row-block compacts the ascending kept-column list
//                    (ballot + lane-prefix popcount, wavefronts in order) and copies the R x kp
//                    value panel, rows of W read with coalesced gathers, panel rows written
//                    contiguously.
// Integer work only; every result is independent of scheduling.
#include "bsp_common.h"

namespace bsp {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;

__device__ __forceinline__ int round_up(int k, int a) { return ((k + a - 1) / a) * a; }

// One workgroup per row of keep[B, N].
__global__ __launch_bounds__(kThreads) void pack_count_kernel(const uint8_t *__restrict__ keep, int64_t N,
                                                              int32_t *__restrict__ blk_cnt) {
    __shared__ int wsum[kWaves];
    const uint8_t *row = keep + (int64_t)blockIdx.x * N;
    int cnt = 0;
    if (((reinterpret_cast<uintptr_t>(row) | (uintptr_t)N) & 15) == 0) {  // 16 flags per load
        for (int64_t j = (int64_t)threadIdx.x * 16; j < N; j += kThreads * 16) {
            const uint4 q = *reinterpret_cast<const uint4 *>(row + j);
            const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
            for (int k = 0; k < 4; ++k)  // a flag is any non-zero byte: fold each byte onto its low bit
                cnt += __popc(((w[k] | (w[k] >> 1) | (w[k] >> 2) | (w[k] >> 3) | (w[k] >> 4) | (w[k] >> 5) | (w[k] >> 6) |
                                (w[k] >> 7)) & 0x01010101u));
        }
    } else {
        for (int64_t j = threadIdx.x; j < N; j += kThreads) cnt += row[j] != 0;
    }
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o, kWave);
    if ((threadIdx.x & (kWave - 1)) == 0) wsum[threadIdx.x / kWave] = cnt;
    __syncthreads();
    if (threadIdx.x == 0) {
        int t = 0;
        for (int w = 0; w < kWaves; ++w) t += wsum[w];
        blk_cnt[blockIdx.x] = t;
    }
}

// Single workgroup: blk_ptr = exclusive scan of the padded counts, blk_ptr[B] = total.
__global__ __launch_bounds__(kThreads) void pack_scan_kernel(const int32_t *__restrict__ blk_cnt, int64_t B,
                                                             int32_t k_align, int32_t *__restrict__ blk_ptr) {
    __shared__ int wsum[kWaves];
    __shared__ int carry;
    if (threadIdx.x == 0) carry = 0;
    __syncthreads();
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    for (int64_t base = 0; base < B; base += kThreads) {
        const int64_t b = base + threadIdx.x;
        const int kp = b < B ? round_up(blk_cnt[b], k_align) : 0;
        int incl = kp;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) {
            int up = __shfl_up(incl, o, kWave);
            if (lane >= o) incl += up;
        }
        if (lane == kWave - 1) wsum[wave] = incl;
        __syncthreads();
        int woff = 0;
        for (int w = 0; w < wave; ++w) woff += wsum[w];
        const int c = carry;
        if (b < B) blk_ptr[b] = c + woff + incl - kp;
        __syncthreads();
        if (threadIdx.x == kThreads - 1) carry = c + woff + incl;
        __syncthreads();
    }
    if (threadIdx.x == 0) blk_ptr[B] = carry;
}

// One or more workgroups per row-block (gridDim.y of them share a block when there are few blocks: each
// takes an equal run of 64-column chunks).  The keep row is cut into chunks of 64 columns, one wavefront
// ballot each: pass 1 counts the kept columns of every chunk, wavefront 0 scans the counts, pass 2
// writes each kept column index at (chunk offset + lane prefix) and copies its R values from W
// straight into the panel.  Reads of a W row touch consecutive columns, panel writes are
// contiguous in c.
constexpr int kMaxChunks = 1024;  // 64-column chunks handled with LDS-resident counts (N <= 65536)

constexpr int kPackThreads = 1024;  // 16 wavefronts: one 64-column chunk each for N = 1024, so the chunks'
                                    // load -> ballot -> gather chains run side by side
constexpr int kPackWaves = kPackThreads / kWave;

template <int WDT, int VDT>
__global__ __launch_bounds__(kPackThreads) void pack_kernel(const void *__restrict__ W, int64_t N, int32_t R,
                                                        const uint8_t *__restrict__ keep,
                                                        const int32_t *__restrict__ blk_cnt,
                                                        const int32_t *__restrict__ blk_ptr, int64_t capacity_cols,
                                                        int32_t *__restrict__ col_idx, void *__restrict__ vals) {
    __shared__ int chunk_off[kMaxChunks + 1];
    __shared__ int s_last;
    if (threadIdx.x == 0) s_last = -1;
    const int64_t b = blockIdx.x;
    const int64_t base = blk_ptr[b];
    const int kp = blk_ptr[b + 1] - blk_ptr[b];
    const int kb = blk_cnt[b];
    if (kp <= 0 || kb <= 0 || kb > kp || base < 0 || base + kp > capacity_cols) return;  // uniform per workgroup
    const uint8_t *krow = keep + b * N;
    int32_t *idx = col_idx + base;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int nchunks = (int)((N + kWave - 1) / kWave);
    const uint64_t lt = (1ull << lane) - 1ull;
    const int64_t vbase = (int64_t)R * base;
    const int64_t wbase = b * R * N;

    for (int c0 = 0; c0 < nchunks; c0 += kMaxChunks) {  // one round unless N > 65536
        const int nc = min(kMaxChunks, nchunks - c0);
        const int carry = c0 == 0 ? 0 : chunk_off[kMaxChunks];
        __syncthreads();
        for (int c = wave; c < nc; c += kPackWaves) {
            const int64_t j = (int64_t)(c0 + c) * kWave + lane;
            const uint64_t m = __ballot(j < N && krow[j] != 0);
            if (lane == 0) chunk_off[c] = __popcll(m);
        }
        __syncthreads();
        if (wave == 0) {  // exclusive scan of the chunk counts
            int run = carry;
            for (int cb = 0; cb < nc; cb += kWave) {
                const int c = cb + lane;
                const int v = c < nc ? chunk_off[c] : 0;
                int incl = v;
#pragma unroll
                for (int o = 1; o < kWave; o <<= 1) {
                    const int up = __shfl_up(incl, o, kWave);
                    if (lane >= o) incl += up;
                }
                if (c < nc) chunk_off[c] = run + incl - v;
                run += __shfl(incl, kWave - 1, kWave);
            }
            if (lane == 0) chunk_off[kMaxChunks] = run;
        }
        __syncthreads();
        // this workgroup's run of chunks
        const int per = (nchunks + (int)gridDim.y - 1) / (int)gridDim.y;
        const int mine_lo = max((int)blockIdx.y * per - c0, 0), mine_hi = min(((int)blockIdx.y + 1) * per - c0, nc);
        for (int c = mine_lo + wave; c < mine_hi; c += kPackWaves) {
            const int64_t j = (int64_t)(c0 + c) * kWave + lane;
            const bool k = j < N && krow[j] != 0;
            const uint64_t m = __ballot(k);
            const int pos = chunk_off[c] + __popcll(m & lt);
            if (k && pos < kb) {
                idx[pos] = (int32_t)j;
                if (pos == kb - 1) s_last = (int32_t)j;
#pragma unroll 8
                for (int r = 0; r < R; ++r)
                    elem<VDT>::store(vals, vbase + (int64_t)r * kp + pos, elem<WDT>::load(W, wbase + (int64_t)r * N + j));
            }
        }
    }
    __syncthreads();
    // pads: repeat the last kept column, zero values (written by the workgroup that placed that column)
    const int32_t last = s_last;
    if (last < 0) return;
    for (int c = kb + threadIdx.x; c < kp; c += kPackThreads) {
        idx[c] = last;
        for (int r = 0; r < R; ++r) elem<VDT>::store(vals, vbase + (int64_t)r * kp + c, 0.0f);
    }
}

// Format check; any violation sets *flag.
__global__ __launch_bounds__(kThreads) void validate_kernel(int64_t B, int64_t N, int32_t k_align,
                                                            const int32_t *__restrict__ blk_cnt,
                                                            const int32_t *__restrict__ blk_ptr,
                                                            const int32_t *__restrict__ col_idx, int64_t capacity_cols,
                                                            int32_t *flag) {
    const int64_t b = blockIdx.x;
    bool bad = false;
    const int64_t base = blk_ptr[b];
    const int64_t kp = (int64_t)blk_ptr[b + 1] - base;
    const int kb = blk_cnt[b];
    if (b == 0 && base != 0) bad = true;
    if (kb < 0 || kb > N || kp != (int64_t)round_up(kb, k_align) || base < 0 || base + kp > capacity_cols) bad = true;
    if (!bad) {
        for (int64_t c = threadIdx.x; c < kp; c += kThreads) {
            const int32_t j = col_idx[base + c];
            if (j < 0 || j >= N) bad = true;
            if (c < kb) {
                if (c > 0 && col_idx[base + c - 1] >= j) bad = true;
            } else if (j != col_idx[base + kb - 1]) {
                bad = true;
            }
        }
    }
    if (bad) atomicOr(flag, 1);
}

__global__ void set_i32_kernel(int32_t *p, int32_t v) { *p = v; }

}  // namespace
}  // namespace bsp

using namespace bsp;

static bool valid_align(int32_t a) { return a == 1 || a == 8 || a == 16 || a == 32 || a == 64; }

extern "C" int bsp_pack_count(const uint8_t *keep, int64_t B, int64_t N, int32_t k_align, int32_t *blk_cnt,
                              int32_t *blk_ptr, void *stream) {
    if (!keep || !blk_cnt || !blk_ptr) return BSP_ERR_NULL;
    if (B <= 0 || N <= 0 || N >= ((int64_t)1 << 31) - 64 || B >= ((int64_t)1 << 31) || !valid_align(k_align)) return BSP_ERR_SHAPE;
    if ((B * (N + 63)) >= ((int64_t)1 << 31)) return BSP_ERR_SHAPE;  // blk_ptr is int32
    hipStream_t s = (hipStream_t)stream;
    pack_count_kernel<<<(unsigned)B, kThreads, 0, s>>>(keep, N, blk_cnt);
    pack_scan_kernel<<<1, kThreads, 0, s>>>(blk_cnt, B, k_align, blk_ptr);
    return check_launch();
}

extern "C" int bsp_pack(const void *W, int wdt, int64_t M, int64_t N, int32_t R, const uint8_t *keep,
                        int32_t k_align, const int32_t *blk_cnt, const int32_t *blk_ptr, int64_t capacity_cols,
                        int32_t *col_idx, void *vals, int vdt, void *stream) {
    if (!W || !keep || !blk_cnt || !blk_ptr) return BSP_ERR_NULL;
    if (!valid_dtype(wdt) || !valid_dtype(vdt)) return BSP_ERR_DTYPE;
    if (M <= 0 || N <= 0 || R < 1 || R > 64 || M % R != 0 || !valid_align(k_align)) return BSP_ERR_SHAPE;
    if (capacity_cols < 0) return BSP_ERR_CAPACITY;
    if (capacity_cols == 0) return BSP_OK;
    if (!col_idx || !vals) return BSP_ERR_NULL;
    const int64_t B = M / R;
    hipStream_t s = (hipStream_t)stream;
    // few row-blocks: several workgroups per block, each with at least 1024 columns (a chunk per wavefront)
    int64_t split64 = (N + 1023) / 1024;
    if (split64 > 512 / B) split64 = 512 / B;
    const unsigned split = (unsigned)(split64 < 1 ? 1 : split64);
    BSP_DISPATCH_DTYPE(wdt, WDT, {
        BSP_DISPATCH_DTYPE(vdt, VDT, {
            pack_kernel<WDT, VDT><<<dim3((unsigned)B, split), kPackThreads, 0, s>>>(W, N, R, keep, blk_cnt, blk_ptr,
                                                                                capacity_cols, col_idx, vals);
        });
    });
    return check_launch();
}

extern "C" int bsp_packed_validate(int64_t M, int64_t N, int32_t R, int32_t k_align, const int32_t *blk_cnt,
                                   const int32_t *blk_ptr, const int32_t *col_idx, int64_t capacity_cols,
                                   int32_t *flag, void *stream) {
    if (!blk_cnt || !blk_ptr || !flag) return BSP_ERR_NULL;
    if (M <= 0 || N <= 0 || R < 1 || R > 64 || M % R != 0 || !valid_align(k_align)) return BSP_ERR_SHAPE;
    if (capacity_cols > 0 && !col_idx) return BSP_ERR_NULL;
    const int64_t B = M / R;
    hipStream_t s = (hipStream_t)stream;
    set_i32_kernel<<<1, 1, 0, s>>>(flag, 0);
    validate_kernel<<<(unsigned)B, kThreads, 0, s>>>(B, N, k_align, blk_cnt, blk_ptr, col_idx, capacity_cols, flag);
    int st = check_launch();
    if (st != BSP_OK) return st;
    int32_t h = 0;
    hipError_t e = hipMemcpyAsync(&h, flag, sizeof(h), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) {
        set_last_hip_error((int)e);
        return BSP_ERR_HIP;
    }
    return h ? BSP_ERR_FORMAT : BSP_OK;
}
