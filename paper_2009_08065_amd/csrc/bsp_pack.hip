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

// Kept flags of one row of keep, counted by one wavefront (the result in every lane).
__device__ __forceinline__ int count_row(const uint8_t *__restrict__ row, int64_t N, int lane) {
    int cnt = 0;
    if (((reinterpret_cast<uintptr_t>(row) | (uintptr_t)N) & 15) == 0) {  // 16 flags per load
        for (int64_t j = (int64_t)lane * 16; j < N; j += kWave * 16) {
            const uint4 q = *reinterpret_cast<const uint4 *>(row + j);
            const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
            for (int k = 0; k < 4; ++k)  // a flag is any non-zero byte: fold each byte onto its low bit
                cnt += __popc(((w[k] | (w[k] >> 1) | (w[k] >> 2) | (w[k] >> 3) | (w[k] >> 4) | (w[k] >> 5) | (w[k] >> 6) |
                                (w[k] >> 7)) & 0x01010101u));
        }
    } else {
        for (int64_t j = lane; j < N; j += kWave) cnt += row[j] != 0;
    }
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o, kWave);
    return cnt;
}

// One wavefront per row of keep[B, N] (kWaves rows per workgroup).
__global__ __launch_bounds__(kThreads) void pack_count_kernel(const uint8_t *__restrict__ keep, int64_t B, int64_t N,
                                                              int32_t *__restrict__ blk_cnt) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t b = (int64_t)blockIdx.x * kWaves + threadIdx.x / kWave;
    if (b >= B) return;  // whole wavefronts leave
    const int cnt = count_row(keep + b * N, N, lane);
    if (lane == 0) blk_cnt[b] = cnt;
}

// Single workgroup: blk_ptr = exclusive scan of the padded counts, blk_ptr[B] = total.  Every thread owns a
// run of consecutive row-blocks (sums it, the workgroup scans the run sums, the thread writes its run).
constexpr int kScanThreads = 1024;
__global__ __launch_bounds__(kScanThreads) void pack_scan_kernel(const int32_t *__restrict__ blk_cnt, int64_t B,
                                                                 int32_t k_align, int32_t *__restrict__ blk_ptr) {
    __shared__ int wsum[kScanThreads / kWave];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int64_t per = (B + kScanThreads - 1) / kScanThreads;
    const int64_t lo = (int64_t)threadIdx.x * per, hi = lo + per < B ? lo + per : B;
    int mine = 0;
    for (int64_t b = lo; b < hi; ++b) mine += round_up(blk_cnt[b], k_align);
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
        run += round_up(blk_cnt[b], k_align);
    }
    if (threadIdx.x == kScanThreads - 1) blk_ptr[B] = run;  // the last thread's run ends at B (or is empty)
}

// Small masks (at most kScanThreads rows and kSmallFlags flags): count and scan in one launch of one workgroup.
// Its wavefronts count the rows in turn, then thread b owns row-block b in the scan.  Saves a launch where the
// launches, not the bytes, are what takes the time: up to 32 K flags.  (One compute unit reads slowly: on the
// 0.25 M flags of a BERT-large matrix this kernel took 11 us against 3 + 3 for the two launches.)
constexpr int64_t kSmallFlags = (int64_t)1 << 15;
__global__ __launch_bounds__(kScanThreads) void pack_count_scan_kernel(const uint8_t *__restrict__ keep, int64_t B,
                                                                       int64_t N, int32_t k_align,
                                                                       int32_t *__restrict__ blk_cnt,
                                                                       int32_t *__restrict__ blk_ptr) {
    __shared__ int s_cnt[kScanThreads];
    __shared__ int wsum[kScanThreads / kWave];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    for (int64_t b = wave; b < B; b += kScanThreads / kWave) {
        const int cnt = count_row(keep + b * N, N, lane);
        if (lane == 0) s_cnt[b] = cnt;
    }
    __syncthreads();
    const bool live = threadIdx.x < B;
    const int cnt = live ? s_cnt[threadIdx.x] : 0;
    const int mine = round_up(cnt, k_align);
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
    if (live) {
        blk_cnt[threadIdx.x] = cnt;
        blk_ptr[threadIdx.x] = run;
        if (threadIdx.x == B - 1) blk_ptr[B] = run + mine;
    }
}

// Compaction in two stages.  Every workgroup first builds the ascending list of the row-block's kept columns
// in LDS (the keep row cut into chunks of 64 columns, one wavefront ballot each: count, scan, place).  Then it
// works by *output position*: consecutive lanes take consecutive positions of the panel, so panel rows are
// written contiguously (16-bit values two per lane, packed) and no lane idles on a pruned column.  gridDim.y
// workgroups share a row-block when there are few row-blocks: each repeats the cheap first stage and takes a
// run of positions.
constexpr int kPackThreads = 1024;  // 16 wavefronts
constexpr int kPackWaves = kPackThreads / kWave;
constexpr int kPackMaxCols = 16384;  // widest layer for this kernel: the kept-column list is 16-bit in LDS

__host__ __device__ inline size_t pack_lds_counts_bytes(int64_t N) { return (size_t)(((N + kWave - 1) / kWave + 1 + 3) / 4 * 4) * 4; }
inline size_t pack_lds_bytes(int64_t N) { return pack_lds_counts_bytes(N) + (size_t)((N + 7) / 8 * 8) * 2; }

template <int WDT, int VDT>
__global__ __launch_bounds__(kPackThreads) void pack_positions_kernel(const void *__restrict__ W, int64_t N, int32_t R,
                                                                      const uint8_t *__restrict__ keep,
                                                                      const int32_t *__restrict__ blk_cnt,
                                                                      const int32_t *__restrict__ blk_ptr,
                                                                      int64_t capacity_cols, int32_t *__restrict__ col_idx,
                                                                      void *__restrict__ vals) {
    // LDS sized by the launch for this layer's width (the counts of the 64-column chunks, then the kept-column
    // list): a narrow layer then leaves room for this kernel beside a workgroup that holds most of a compute
    // unit's LDS
    extern __shared__ __attribute__((aligned(16))) uint8_t pack_lds[];
    int *chunk_off = reinterpret_cast<int *>(pack_lds);
    uint16_t *s_cols = reinterpret_cast<uint16_t *>(pack_lds + pack_lds_counts_bytes(N));
    const int64_t b = blockIdx.x;
    const int64_t base = blk_ptr[b];
    const int kp = blk_ptr[b + 1] - blk_ptr[b];
    const int kb = blk_cnt[b];
    if (kp <= 0 || kb <= 0 || kb > kp || kb > N || base < 0 || base + kp > capacity_cols) return;  // uniform per workgroup
    const uint8_t *krow = keep + b * N;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int nchunks = (int)((N + kWave - 1) / kWave);
    const uint64_t lt = (1ull << lane) - 1ull;
    for (int c = wave; c < nchunks; c += kPackWaves) {
        const int64_t j = (int64_t)c * kWave + lane;
        const uint64_t m = __ballot(j < N && krow[j] != 0);
        if (lane == 0) chunk_off[c] = __popcll(m);
    }
    __syncthreads();
    if (wave == 0) {  // exclusive scan of the chunk counts
        int run = 0;
        for (int cb = 0; cb < nchunks; cb += kWave) {
            const int c = cb + lane;
            const int v = c < nchunks ? chunk_off[c] : 0;
            int incl = v;
#pragma unroll
            for (int o = 1; o < kWave; o <<= 1) {
                const int up = __shfl_up(incl, o, kWave);
                if (lane >= o) incl += up;
            }
            if (c < nchunks) chunk_off[c] = run + incl - v;
            run += __shfl(incl, kWave - 1, kWave);
        }
    }
    __syncthreads();
    for (int c = wave; c < nchunks; c += kPackWaves) {
        const int64_t j = (int64_t)c * kWave + lane;
        const bool k = j < N && krow[j] != 0;
        const uint64_t m = __ballot(k);
        const int pos = chunk_off[c] + __popcll(m & lt);
        if (k && pos < kb) s_cols[pos] = (uint16_t)j;
    }
    __syncthreads();
    // this workgroup's run of positions, whole 64-position pieces
    const int pieces = (kp + kWave - 1) / kWave;
    const int per = (pieces + (int)gridDim.y - 1) / (int)gridDim.y;
    const int p_lo = min((int)blockIdx.y * per, pieces) * kWave, p_hi = min(((int)blockIdx.y + 1) * per * kWave, kp);
    if (p_lo >= p_hi) return;
    const int last = s_cols[kb - 1];
    for (int pos = p_lo + threadIdx.x; pos < p_hi; pos += kPackThreads) col_idx[base + pos] = pos < kb ? (int)s_cols[pos] : last;
    // values: a unit is (row r, 64-position piece); wavefronts take units in turn.  Pads are +0.
    const int npc = (p_hi - p_lo + kWave - 1) / kWave;
    const int64_t vbase = (int64_t)R * base, wbase = b * R * N;
    constexpr bool kPairs = VDT != BSP_F32;  // 16-bit values: a lane packs two neighbours into one 4-byte store
    const bool pairs = kPairs && (kp & 1) == 0 && (vbase & 1) == 0 && (reinterpret_cast<uintptr_t>(vals) & 3) == 0;
    if (pairs) {
        const int npc2 = (p_hi - p_lo + 2 * kWave - 1) / (2 * kWave);
        for (int u = wave; u < R * npc2; u += kPackWaves) {
            const int r = u / npc2, pos = p_lo + (u % npc2) * (2 * kWave) + 2 * lane;
            if (pos >= p_hi) continue;
            const float v0 = pos < kb ? elem<WDT>::load(W, wbase + (int64_t)r * N + s_cols[pos]) : 0.0f;
            const float v1 = pos + 1 < kb ? elem<WDT>::load(W, wbase + (int64_t)r * N + s_cols[pos + 1]) : 0.0f;
            const uint32_t lo = elem<VDT>::bits(v0), hi = elem<VDT>::bits(v1);
            *reinterpret_cast<uint32_t *>((uint16_t *)vals + vbase + (int64_t)r * kp + pos) = lo | (hi << 16);
        }
    } else {
        for (int u = wave; u < R * npc; u += kPackWaves) {
            const int r = u / npc, pos = p_lo + (u % npc) * kWave + lane;
            if (pos >= p_hi) continue;
            const float v = pos < kb ? elem<WDT>::load(W, wbase + (int64_t)r * N + s_cols[pos]) : 0.0f;
            elem<VDT>::store(vals, vbase + (int64_t)r * kp + pos, v);
        }
    }
}

// The same for layers wider than kPackMaxCols: compaction and copy chunk by chunk, one lane per column.
// One or more workgroups per row-block (gridDim.y of them share a block when there are few blocks: each
// takes an equal run of 64-column chunks).  The keep row is cut into chunks of 64 columns, one wavefront
// ballot each: pass 1 counts the kept columns of every chunk, wavefront 0 scans the counts, pass 2
// writes each kept column index at (chunk offset + lane prefix) and copies its R values from W
// straight into the panel.  Reads of a W row touch consecutive columns, panel writes are
// contiguous in c.
constexpr int kMaxChunks = 1024;  // 64-column chunks handled with LDS-resident counts (N <= 65536)


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
    if (B <= kScanThreads && B * N <= kSmallFlags) {
        pack_count_scan_kernel<<<1, kScanThreads, 0, s>>>(keep, B, N, k_align, blk_cnt, blk_ptr);
    } else {
        pack_count_kernel<<<(unsigned)((B + kWaves - 1) / kWaves), kThreads, 0, s>>>(keep, B, N, blk_cnt);
        pack_scan_kernel<<<1, kScanThreads, 0, s>>>(blk_cnt, B, k_align, blk_ptr);
    }
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
            if (N <= kPackMaxCols)
                pack_positions_kernel<WDT, VDT><<<dim3((unsigned)B, split), kPackThreads, pack_lds_bytes(N), s>>>(
                    W, N, R, keep, blk_cnt, blk_ptr, capacity_cols, col_idx, vals);
            else
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
