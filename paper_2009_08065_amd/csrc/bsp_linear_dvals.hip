// Gradient of the block-structure-pruned layer with respect to its kept weights.
//   For Y = X Wp^T + bias (Sec. 3.1; Wp the matrix after Alg. 1) the chain rule gives dW[m, j] = sum_t dY[t, m] X[t, j],
//   and the weight update of Alg. 2 needs it on the kept groups only.  In the layout of the value panels:
//     D[R blk_ptr[b] + r kp_b + c] = sum_t dY[t, bR + r] X[t, col_idx[b, c]]   (c < k_b),   +0 on pad slots.
//
// Per row-block this is a dense product (R rows x tokens times tokens x kept columns) whose right operand is a gather
// of columns of X; the contraction runs over the tokens.  The sums of the whole matrix are few (2 to 3 MB as fp32)
// against a register file of 128 MB, so the tokens are split over the workgroups and a second, ordered pass adds the
// partial sums: two calls give the same bits.
//
// Work units.  The kept columns of a row-block that fall into one range of 1024 columns of X are cut into groups of
// 16 (one matrix-core result of 16 rows x 16 columns each, fp32) and up to 16 groups of one 16-row slab of a
// row-block form an item: what one wavefront accumulates (64 registers).  A strip is 16 consecutive items of one
// column range: what a workgroup of 16 wavefronts accumulates while it walks a run of token tiles.  Per tile of 32
// tokens the workgroup copies the range's columns of X into LDS transposed (64 bytes per column: a lane's operand,
// 8 consecutive tokens of its own kept column, is one 16-byte read) and every wavefront its slab's 16 columns of dY
// untransposed (the transposing LDS read delivers the other operand); the global loads of tile i + 1 are in flight
// while tile i is multiplied.
#include "bsp_common.h"
#include "bsp_mfma_device.h"

namespace bsp {
namespace {

constexpr int kDvTok = 32;               // tokens per tile: the contraction depth of one matrix instruction
constexpr int kDvRange = 1024;           // columns of X a tile holds
constexpr int kDvStrip = 16;             // items of a strip = of a workgroup
constexpr int kDvWaves = 8;              // each with 2 items: 128 accumulator registers of the 256 a wavefront may hold
constexpr int kDvPerWave = kDvStrip / kDvWaves;
constexpr int kDvThreads = kDvWaves * kWave;
constexpr int kDvXUnits = 2048 / kDvThreads;  // units of 4 columns x 4 tokens a thread copies per tile
constexpr int kDvGroups = 16;            // groups of 16 kept columns per item
constexpr int kDvReduceThreads = kDvGroups * kWave;  // the second pass: one wavefront per group of an item
constexpr int kDvQuads = kDvGroups / 4;
constexpr int kDvItemCols = kDvGroups * 16;
constexpr int kDvItemFloats = kDvGroups * 256;
constexpr uint32_t kDvXBytes = kDvRange * 64;     // 64 KiB
constexpr uint32_t kDvYBytes = kDvStrip * 1024;   // 16 KiB: per item 32 tokens x 16 rows
constexpr int kDvUnits = 256;            // workgroups of the product: one per compute unit
constexpr size_t kDvHeaderBytes = 256;

struct DvItem {
    int32_t b;      // row-block
    int32_t pos0;   // index into col_idx of the item's first kept column
    int32_t ncols;  // kept columns of the item, 0 .. 256 (0: a filler that rounds a range up to whole strips)
    int32_t sq;     // slab | column range << 8
};

// header of the workspace, written by the item kernel: items (a multiple of 16), strips
enum { kHdrItems = 0, kHdrStrips = 1 };

__host__ __device__ inline int64_t dv_max_items(int64_t B, int64_t N, int32_t R, int64_t capacity_cols) {
    const int64_t nslab = (R + 15) / 16, nr = (N + kDvRange - 1) / kDvRange;
    const int64_t n = nslab * (capacity_cols / kDvItemCols + nr * B) + 16 * nr;
    return (n + 15) / 16 * 16;
}
inline int64_t dv_max_units(int64_t max_items) { return max_items / 16 > kDvUnits ? max_items / 16 : kDvUnits; }

// LDS row of column c (local to its range) in the transposed tile: inside every 32 columns the four columns that
// one lane of the copy-in holds (c .. c + 3) lie 8 rows apart, so that the lanes of a wavefront, which hold
// consecutive column quads, write consecutive rows.
__device__ __forceinline__ uint32_t dv_row(uint32_t c) { return (c & ~31u) | ((c >> 2) & 7u) | ((c & 3u) << 3); }
// byte offset of tokens 8 kg .. 8 kg + 7 of column c: the four 16-byte pieces of a row rotate with bits 4 to 6 of the
// column, so that 16 consecutive lanes of the copy-in (16 consecutive column quads, one 8-byte store each) fall
// into 16 different 16-byte bank groups
__device__ __forceinline__ uint32_t dv_x_offset(uint32_t c, uint32_t kg) {
    const uint32_t sw = ((c >> 5) & 3u) ^ (((c >> 4) & 1u) << 1);
    return dv_row(c) * 64u + ((kg ^ sw) << 4);
}

// Bank group of column c: the 16 lanes of one pass of a 16-byte LDS read are conflict-free exactly when their
// columns differ in this number (row modulo 4, and the rotation of the row's pieces).
__device__ __forceinline__ uint32_t dv_class(uint32_t c) {
    const uint32_t sw = ((c >> 5) & 3u) ^ (((c >> 4) & 1u) << 1);
    return (((c >> 2) & 3u) << 2) | sw;
}
// some column of bank group k (for lanes without a column)
__device__ __forceinline__ uint32_t dv_class_column(uint32_t k) { return ((k >> 2) << 2) | ((k & 3u) << 5); }

__device__ __forceinline__ int dv_lower_bound(const int32_t *a, int n, int v) {  // first i with a[i] >= v
    int lo = 0, hi = n;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (a[mid] < v) lo = mid + 1;
        else hi = mid;
    }
    return lo;
}

// Lists the items: column ranges in turn, row-blocks ascending inside a range, every range rounded up to whole strips
// with fillers.  Every workgroup of the launch builds the whole list (the same values from every one of them: the
// list is short and a workgroup cannot wait for another), then the wavefronts of all workgroups share the second
// part, one item at a time.
__global__ __launch_bounds__(kDvThreads) void dvals_items_kernel(int64_t B, int32_t nslab, int32_t nr,
                                                                const int32_t *__restrict__ blk_cnt,
                                                                const int32_t *__restrict__ blk_ptr,
                                                                const int32_t *__restrict__ col_idx,
                                                                int32_t max_items, int32_t *__restrict__ hdr,
                                                                DvItem *__restrict__ items,
                                                                uint16_t *__restrict__ perm,
                                                                int32_t *__restrict__ groups) {
    __shared__ int s_scan[kDvThreads];
    __shared__ uint16_t s_perm[kDvThreads / kWave][kDvItemCols];
    const int tid = threadIdx.x;
    int run = 0;
    for (int q = 0; q < nr; ++q) {
        for (int64_t e0 = 0; e0 < B; e0 += kDvThreads) {
            const int64_t b = e0 + tid;
            int n = 0, first = 0, cnt = 0;
            if (b < B) {
                const int32_t base = blk_ptr[b];
                const int k = blk_cnt[b];
                const int lo = dv_lower_bound(col_idx + base, k, q * kDvRange);
                const int hi = dv_lower_bound(col_idx + base, k, (q + 1) * kDvRange);
                first = base + lo;
                cnt = hi - lo;
                n = nslab * ((cnt + kDvItemCols - 1) / kDvItemCols);
            }
            s_scan[tid] = n;
            __syncthreads();
            for (int o = 1; o < kDvThreads; o <<= 1) {
                const int add = tid >= o ? s_scan[tid - o] : 0;
                __syncthreads();
                s_scan[tid] += add;
                __syncthreads();
            }
            const int off = run + s_scan[tid] - n;
            for (int i = 0; i < n; ++i) {
                const int chunk = i / nslab, slab = i % nslab;
                const int left = cnt - kDvItemCols * chunk;
                if (off + i < max_items)
                    items[off + i] = DvItem{(int32_t)b, first + kDvItemCols * chunk, left < kDvItemCols ? left : kDvItemCols,
                                            slab | (q << 8)};
            }
            run += s_scan[kDvThreads - 1];
            __syncthreads();  // s_scan is rewritten by the next pass
        }
        const int padded = (run + 15) & ~15;
        for (int i = run + tid; i < padded && i < max_items; i += kDvThreads) items[i] = DvItem{0, 0, 0, q << 8};
        run = padded;
    }
    if (run > max_items) run = max_items;  // (cannot happen: max_items bounds the count)
    __syncthreads();  // the item records are complete (and visible to the whole workgroup)

    // Deal every item's columns to (group, lane) slots.  The first m groups take one column of every bank group, in
    // the lane of that number: their LDS reads are conflict-free.  Columns of bank groups that hold more than m fill
    // the groups behind them in any order.  m is the largest number for which one group more than the item's columns
    // need (16 at most) is enough.  perm[slot] = place of the column among the item's columns, 0xffff = none.
    {
        const int lane = tid & (kWave - 1), wave = tid / kWave;
        const uint64_t below = ((uint64_t)1 << lane) - 1;
        for (int it = blockIdx.x * (kDvThreads / kWave) + wave; it < run; it += gridDim.x * (kDvThreads / kWave)) {
            const DvItem item = items[it];
            if (item.ncols == 0) {  // a filler
#pragma unroll
                for (int e = 0; e < 4; ++e) perm[(int64_t)it * kDvItemCols + lane + kWave * e] = 0xffffu;
                if (lane == 0) groups[it] = 0;
                continue;
            }
            const int ncols = item.ncols, col0 = ((item.sq >> 8) & 0xffff) * kDvRange;
            int cls[4], rk[4] = {0, 0, 0, 0};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int j = lane + kWave * e;
                cls[e] = j < ncols ? (int)dv_class((uint32_t)(col_idx[item.pos0 + j] - col0)) : 16;
            }
            int mycnt = 0;  // lane k < 16: columns of bank group k
            for (int k = 0; k < 16; ++k) {
                int running = 0;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint64_t mask = __ballot(cls[e] == k);
                    if (cls[e] == k) rk[e] = running + __popcll(mask & below);
                    running += __popcll(mask);
                }
                if (lane == k) mycnt = running;
            }
            const int budget = min(16, (ncols + 15) / 16 + 1);
            int m = 16, tail = 0;
            for (; m >= 0; --m) {
                int over = lane < 16 ? max(0, mycnt - m) : 0;
#pragma unroll
                for (int o = 1; o < 16; o <<= 1) over += __shfl_xor(over, o, kWave);
                tail = over;  // (the same in lanes 0 .. 15; lane 0 decides)
                tail = __shfl(tail, 0, kWave);
                if (m + (tail + 15) / 16 <= budget) break;
            }
            if (m < 0) m = 0;  // (m = 0 always fits)
            int ovf = lane < 16 ? max(0, mycnt - m) : 0, pre = ovf;  // exclusive prefix of the overflow per bank group
#pragma unroll
            for (int o = 1; o < 16; o <<= 1) {
                const int up = __shfl_up(pre, o, kWave);
                if ((lane & 15) >= o) pre += up;
            }
            pre -= ovf;
            uint16_t *mine = s_perm[wave];
#pragma unroll
            for (int e = 0; e < 4; ++e) mine[lane + kWave * e] = 0xffffu;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int start = __shfl(pre, cls[e] & 15, kWave);
                if (cls[e] < 16) {
                    const int slot = rk[e] < m ? rk[e] * 16 + cls[e] : m * 16 + start + rk[e] - m;
                    mine[slot] = (uint16_t)(lane + kWave * e);
                }
            }
            // (one wavefront's LDS operations complete in order)
#pragma unroll
            for (int e = 0; e < 4; ++e) perm[(int64_t)it * kDvItemCols + lane + kWave * e] = mine[lane + kWave * e];
            if (lane == 0) groups[it] = m + (tail + 15) / 16;
        }
    }
    if (tid == 0 && blockIdx.x == 0) {
        hdr[kHdrItems] = run;
        hdr[kHdrStrips] = run / 16;
    }
}

// Token ranges of a call: as many as give about kDvUnits workgroups, whole tiles each.  tiles_per_range, ranges.
__device__ __forceinline__ void dv_ranges(int strips, int ntiles, int &tpu, int &S) {
    tpu = 1;
    S = 0;
    if (strips <= 0) return;
    int want = kDvUnits / strips;
    if (want < 1) want = 1;
    if (want > ntiles) want = ntiles;
    tpu = (ntiles + want - 1) / want;
    S = (ntiles + tpu - 1) / tpu;
}

template <int DT>
__global__ __launch_bounds__(kDvThreads) void dvals_partial_kernel(const uint16_t *__restrict__ X,
                                                                  const uint16_t *__restrict__ dY, int64_t T, int64_t M,
                                                                  int64_t N, int32_t R,
                                                                  const int32_t *__restrict__ col_idx,
                                                                  const int32_t *__restrict__ hdr,
                                                                  const DvItem *__restrict__ items,
                                                                  const uint16_t *__restrict__ perm,
                                                                  const int32_t *__restrict__ groups,
                                                                  float *__restrict__ partial) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, kg = lane >> 4, qd = (lane >> 2) & 3, p4 = lane & 3;
    const int strips = hdr[kHdrStrips];
    const int ntiles = (int)((T + kDvTok - 1) / kDvTok);
    int tpu, S;
    dv_ranges(strips, ntiles, tpu, S);
    uint8_t *xt = smem_x;
    uint8_t *yt = smem_x + kDvXBytes;
    // as a loader of X: kDvXUnits units of 4 columns x 4 tokens; as a loader of dY: half a token's 16 rows of each of
    // the wavefront's own slabs
    const int cq = tid & 255, tq0 = tid >> 8;
    const int y_tok = lane >> 1, y_half = lane & 1;
    // as a consumer: the lane's address inside a slab's dY rows for the transposing read (token 8 kg + qd, rows
    // 4 p4 .. 4 p4 + 3; the second read takes the token 4 further on)
    const uint32_t a_off = kDvXBytes + (uint32_t)(8 * kg + qd) * 32u + (uint32_t)p4 * 8u;

    // Workgroup ids go round the 8 XCDs (each with an L2 of its own): the units of one XCD are consecutive, so the
    // strips of one range of tokens, which read the same rows of X, mostly share an L2.
    const int total_units = strips * S, per_xcd = (total_units + 7) / 8;
    for (int u0 = blockIdx.x; u0 < per_xcd * 8; u0 += gridDim.x) {
        const int unit = (u0 & 7) * per_xcd + (u0 >> 3);
        if (unit >= total_units) continue;  // (the same for the whole workgroup)
        const int strip = unit % strips, s = unit / strips;
        int ncols[kDvPerWave], ng[kDvPerWave];
        int64_t row0[kDvPerWave];
        int col0 = 0;
        uint32_t xoff[kDvPerWave][kDvGroups / 2];  // LDS offsets of the lane's columns, two 16-bit halves per register
        f32x4 acc[kDvPerWave][kDvGroups];
#pragma unroll
        for (int i = 0; i < kDvPerWave; ++i) {
            const int64_t it = (int64_t)strip * kDvStrip + kDvPerWave * wave + i;
            const DvItem *mine = items + it;
            const int ib = __builtin_amdgcn_readfirstlane(mine->b);
            const int ipos = __builtin_amdgcn_readfirstlane(mine->pos0);
            const int isq = __builtin_amdgcn_readfirstlane(mine->sq);
            ncols[i] = __builtin_amdgcn_readfirstlane(mine->ncols);
            ng[i] = __builtin_amdgcn_readfirstlane(groups[it]);
            col0 = ((isq >> 8) & 0xffff) * kDvRange;  // the column range is the same for all items of a strip
            row0[i] = (int64_t)ib * R + 16 * (isq & 0xff);
#pragma unroll
            for (int g = 0; g < kDvGroups; ++g) {
                // the column dealt to this lane's slot; a lane without one reads a column of its own bank group
                const uint32_t pj = g < ng[i] ? perm[it * kDvItemCols + 16 * g + l16] : 0xffffu;
                const uint32_t c = pj != 0xffffu ? (uint32_t)(col_idx[ipos + (int)pj] - col0) : dv_class_column((uint32_t)l16);
                const uint32_t o = dv_x_offset(c, (uint32_t)kg);
                xoff[i][g >> 1] = (g & 1) ? (xoff[i][g >> 1] | (o << 16)) : o;
                acc[i][g] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
        }

        const int tile0 = s * tpu, tile1 = tile0 + tpu < ntiles ? tile0 + tpu : ntiles;
        uint2 xa[kDvXUnits][4];
        uint4 ya[kDvPerWave];
        // Addresses are a uniform base and a 32-bit byte offset per lane (32 rows of X or dY stay far below 4 GB).
        // Columns past N and, for R = 8, the upper half of the last row-block's slab are read from the nearest valid
        // place instead (nothing reads those LDS cells, or only into result rows that are not written); tokens
        // past T must be zeros in both operands: only the last tile can hold some and takes the guarded loads.
        const int cqc = col0 + 4 * cq + 4 <= N ? 4 * cq : (int)(N - col0 - 4);
        uint32_t xv[kDvXUnits], yv[kDvPerWave];
#pragma unroll
        for (int k = 0; k < kDvXUnits; ++k)
            xv[k] = 2u * ((uint32_t)(4 * (tq0 + (kDvThreads / 256) * k)) * (uint32_t)N + (uint32_t)cqc);
#pragma unroll
        for (int i = 0; i < kDvPerWave; ++i)
            yv[i] = 2u * ((uint32_t)y_tok * (uint32_t)M + (row0[i] + 8 * y_half + 8 <= M ? 8u * (uint32_t)y_half : 0u));
        auto issue = [&](int tile, auto full) {
            const int64_t t0 = (int64_t)tile * kDvTok;
            const int left = (int)(T - t0);  // tokens of this tile when it is the last one
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                int64_t xbase = 2 * ((t0 + i) * N + col0);
                asm volatile("" : "+s"(xbase));  // stays a scalar: the loads take X + xbase beside the lane's 32-bit offset
                const uint8_t *xrow = reinterpret_cast<const uint8_t *>(X) + xbase;
#pragma unroll
                for (int k = 0; k < kDvXUnits; ++k) {
                    const int t = 4 * (tq0 + (kDvThreads / 256) * k) + i;
                    xa[k][i] = (full.value || t < left) ? *reinterpret_cast<const uint2 *>(xrow + xv[k])
                                                        : make_uint2(0u, 0u);
                }
            }
#pragma unroll
            for (int i = 0; i < kDvPerWave; ++i) {
                int64_t ybase = 2 * (t0 * M + row0[i]);
                asm volatile("" : "+s"(ybase));
                const uint8_t *yrow = reinterpret_cast<const uint8_t *>(dY) + ybase;
                ya[i] = (full.value || y_tok < left) ? *reinterpret_cast<const uint4 *>(yrow + yv[i])
                                                     : make_uint4(0u, 0u, 0u, 0u);
            }
        };
        auto issue_tile = [&](int tile) {
            if ((int64_t)(tile + 1) * kDvTok <= T) issue(tile, std::true_type{});
            else issue(tile, std::false_type{});
        };
        auto commit = [&]() {
#pragma unroll
            for (int k = 0; k < kDvXUnits; ++k) {
                const uint32_t tq = (uint32_t)(tq0 + (kDvThreads / 256) * k);
                const uint32_t c = 4u * (uint32_t)cq;
                uint8_t *dst = xt + dv_x_offset(c, tq >> 1) + (tq & 1u) * 8u;  // columns c + 1 .. c + 3: 8, 16, 24 rows on
                uint2 w;
                w.x = (xa[k][0].x & 0xffffu) | (xa[k][1].x << 16);
                w.y = (xa[k][2].x & 0xffffu) | (xa[k][3].x << 16);
                *reinterpret_cast<uint2 *>(dst) = w;
                w.x = (xa[k][0].x >> 16) | (xa[k][1].x & 0xffff0000u);
                w.y = (xa[k][2].x >> 16) | (xa[k][3].x & 0xffff0000u);
                *reinterpret_cast<uint2 *>(dst + 8 * 64) = w;
                w.x = (xa[k][0].y & 0xffffu) | (xa[k][1].y << 16);
                w.y = (xa[k][2].y & 0xffffu) | (xa[k][3].y << 16);
                *reinterpret_cast<uint2 *>(dst + 16 * 64) = w;
                w.x = (xa[k][0].y >> 16) | (xa[k][1].y & 0xffff0000u);
                w.y = (xa[k][2].y >> 16) | (xa[k][3].y & 0xffff0000u);
                *reinterpret_cast<uint2 *>(dst + 24 * 64) = w;
            }
#pragma unroll
            for (int i = 0; i < kDvPerWave; ++i)
                *reinterpret_cast<uint4 *>(yt + (kDvPerWave * wave + i) * 1024 + y_tok * 32 + y_half * 16) = ya[i];
        };

        issue_tile(tile0);
        for (int tile = tile0; tile < tile1; ++tile) {
            commit();
            __syncthreads();
            if (tile + 1 < tile1) issue_tile(tile + 1);
            // The wavefront's groups go four at a time (a quad): the reads of the next quad are on their way while
            // the current one is multiplied; a group past the item's last one multiplies some column into an
            // accumulator that is never written out.
            uint4 a[kDvPerWave];
#pragma unroll
            for (int i = 0; i < kDvPerWave; ++i) {
                const uint32_t ao = a_off + (uint32_t)(kDvPerWave * wave + i) * 1024u;
                const uint2 lo = tr_read(smem_x, ao);
                const uint2 hi = tr_read(smem_x, ao + 4 * 32);
                a[i] = make_uint4(lo.x, lo.y, hi.x, hi.y);
            }
            uint4 bq[2][4];
            auto read_quad = [&](auto QD, uint4(&dst)[4]) {
                constexpr int I = QD.value / kDvQuads, Q = QD.value % kDvQuads;
                if (4 * Q < ng[I]) {
                    uint32_t w0 = xoff[I][2 * Q], w1 = xoff[I][2 * Q + 1];
                    asm volatile("" : "+v"(w0), "+v"(w1));  // (unpacked once before the loop they cost 32 registers)
                    dst[0] = *reinterpret_cast<const uint4 *>(xt + (w0 & 0xffffu));
                    dst[1] = *reinterpret_cast<const uint4 *>(xt + (w0 >> 16));
                    dst[2] = *reinterpret_cast<const uint4 *>(xt + (w1 & 0xffffu));
                    dst[3] = *reinterpret_cast<const uint4 *>(xt + (w1 >> 16));
                }
            };
            read_quad(std::integral_constant<int, 0>{}, bq[0]);
            static_for<0, kDvPerWave * kDvQuads>([&](auto QD) {
                constexpr int I = QD.value / kDvQuads, Q = QD.value % kDvQuads;
                if constexpr (QD.value + 1 < kDvPerWave * kDvQuads)
                    read_quad(std::integral_constant<int, QD.value + 1>{}, bq[(QD.value + 1) & 1]);
                if (4 * Q < ng[I]) {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        acc[I][4 * Q + j] = mfma16<DT>(a[I], bq[QD.value & 1][j], acc[I][4 * Q + j]);
                }
            });
            __syncthreads();  // every wavefront is done with the tile before the next one is written
        }
        static_for<0, kDvPerWave>([&](auto I) {
            float *dst = partial + ((int64_t)unit * kDvStrip + kDvPerWave * wave + I.value) * kDvItemFloats + lane * 4;
            static_for<0, kDvGroups>([&](auto G) {
                if (G.value < ng[I.value]) *reinterpret_cast<f32x4 *>(dst + G.value * 256) = acc[I.value][G.value];
            });
        });
    }
}

// Second pass: the partial sums of a group are added in the order of their token ranges, rounded once and written
// to their places in the panels; workgroups past the items clear the pad slots of one row-block each.
template <int GDT>
__global__ __launch_bounds__(kDvReduceThreads) void dvals_reduce_kernel(int64_t B, int32_t R,
                                                                 const int32_t *__restrict__ blk_cnt,
                                                                 const int32_t *__restrict__ blk_ptr,
                                                                 const int32_t *__restrict__ hdr,
                                                                 const DvItem *__restrict__ items,
                                                                 const uint16_t *__restrict__ perm,
                                                                 const int32_t *__restrict__ groups,
                                                                 const float *__restrict__ partial, int32_t max_items,
                                                                 int32_t ntiles, void *__restrict__ D) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l16 = lane & 15, kg = lane >> 4;
    const int64_t id = blockIdx.x;
    if (id >= max_items) {
        const int64_t b = id - max_items;
        if (b >= B) return;
        const int64_t base = blk_ptr[b];
        const int kp = blk_ptr[b + 1] - blk_ptr[b], k = blk_cnt[b], npad = kp - k;
        for (int i = tid; i < R * npad; i += kDvReduceThreads)
            elem<GDT>::store(D, (int64_t)R * base + (int64_t)(i / npad) * kp + k + i % npad, 0.0f);
        return;
    }
    if (id >= hdr[kHdrItems]) return;
    const int strips = hdr[kHdrStrips];
    int tpu, S;
    dv_ranges(strips, ntiles, tpu, S);
    const DvItem it = items[id];
    if (wave >= groups[id]) return;  // whole wavefronts leave: wavefront g adds group g
    const int64_t strip = id >> 4;
    const int w = (int)(id & 15);
    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < S; ++s) {
        const float *src = partial + ((s * strips + strip) * 16 + w) * kDvItemFloats + wave * 256 + lane * 4;
        const f32x4 v = *reinterpret_cast<const f32x4 *>(src);
        acc = s == 0 ? v : acc + v;
    }
    const int64_t base = blk_ptr[it.b];
    const int kp = blk_ptr[it.b + 1] - blk_ptr[it.b];
    const int slab = it.sq & 0xff;
    const uint32_t pj = perm[id * kDvItemCols + 16 * wave + l16];  // the column dealt to this lane's slot
    if (pj == 0xffffu) return;
    const int64_t cpos = it.pos0 - base + (int64_t)pj;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int r = 16 * slab + 4 * kg + j;
        if (r < R) elem<GDT>::store(D, (int64_t)R * base + (int64_t)r * kp + cpos, acc[j]);
    }
}

// Any dtype, any R: one output per thread, fp32 products added in the order of the tokens.
template <int XDT, int GDT>
__global__ __launch_bounds__(256) void dvals_plain_kernel(const void *__restrict__ X, const void *__restrict__ dY,
                                                          int64_t T, int64_t M, int64_t N, int32_t R,
                                                          const int32_t *__restrict__ blk_cnt,
                                                          const int32_t *__restrict__ blk_ptr,
                                                          const int32_t *__restrict__ col_idx, void *__restrict__ D) {
    const int64_t b = blockIdx.x;
    const int64_t base = blk_ptr[b];
    const int kp = blk_ptr[b + 1] - blk_ptr[b], k = blk_cnt[b];
    for (int i = blockIdx.y * 256 + threadIdx.x; i < R * kp; i += gridDim.y * 256) {
        const int r = i / kp, c = i % kp;
        float acc = 0.0f;
        if (c < k) {
            const int64_t j = col_idx[base + c];
            for (int64_t t = 0; t < T; ++t)
                acc = acc + elem<XDT>::load(dY, t * M + b * R + r) * elem<XDT>::load(X, t * N + j);
        }
        elem<GDT>::store(D, (int64_t)R * base + i, acc);
    }
}

struct DvLayout {
    int64_t max_items, max_units;
    size_t items_at, groups_at, perm_at, partial_at, total;
};
DvLayout dv_layout(int64_t M, int64_t N, int32_t R, int64_t capacity_cols) {
    DvLayout L;
    L.max_items = dv_max_items(M / R, N, R, capacity_cols);
    L.max_units = dv_max_units(L.max_items);
    L.items_at = kDvHeaderBytes;
    L.groups_at = (L.items_at + (size_t)L.max_items * sizeof(DvItem) + 255) / 256 * 256;
    L.perm_at = (L.groups_at + (size_t)L.max_items * sizeof(int32_t) + 255) / 256 * 256;
    L.partial_at = L.perm_at + (size_t)L.max_items * kDvItemCols * sizeof(uint16_t);
    L.total = L.partial_at + (size_t)L.max_units * 16 * kDvItemFloats * sizeof(float);
    return L;
}

template <typename K>
int dv_raise_lds(K kern, size_t lds) {
    static thread_local size_t configured = 0;  // per instantiation (K) and thread
    if (lds <= configured) return BSP_OK;
    hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) {
        set_last_hip_error((int)e);
        return BSP_ERR_HIP;
    }
    configured = lds;
    return BSP_OK;
}

template <int DT>
int launch_partial(hipStream_t s, const void *X, const void *dY, int64_t T, int64_t M, int64_t N, int32_t R,
                   const int32_t *col_idx, const int32_t *hdr, const DvItem *items, const uint16_t *perm,
                   const int32_t *groups, float *partial) {
    auto k = dvals_partial_kernel<DT>;
    const size_t lds = kDvXBytes + kDvYBytes;
    const int st = dv_raise_lds(k, lds);
    if (st != BSP_OK) return st;
    k<<<kDvUnits, kDvThreads, lds, s>>>((const uint16_t *)X, (const uint16_t *)dY, T, M, N, R, col_idx, hdr, items,
                                        perm, groups, partial);
    return BSP_OK;
}

}  // namespace
}  // namespace bsp

using namespace bsp;

extern "C" size_t bsp_linear_dvals_workspace_bytes(int64_t M, int64_t N, int32_t R, int64_t capacity_cols) {
    if (M <= 0 || N <= 0 || R < 1 || M % R != 0 || capacity_cols < 0) return 0;
    return dv_layout(M, N, R, capacity_cols).total;
}

extern "C" int bsp_linear_dvals(const void *X, const void *dY, int xdt, int64_t T, int64_t M, int64_t N, int32_t R,
                                int32_t k_align, const int32_t *blk_cnt, const int32_t *blk_ptr,
                                const int32_t *col_idx, int64_t capacity_cols, void *D, int gdt, void *ws,
                                size_t ws_bytes, int ws_state, void *stream) {
    if (!blk_cnt || !blk_ptr) return BSP_ERR_NULL;
    if (!valid_dtype(xdt) || !valid_dtype(gdt)) return BSP_ERR_DTYPE;
    if (T < 0 || M <= 0 || N <= 0 || R < 1 || M % R != 0 || capacity_cols < 0) return BSP_ERR_SHAPE;
    if (ws_state != BSP_DVALS_BUILD && ws_state != BSP_DVALS_REUSE) return BSP_ERR_SHAPE;
    if (!(k_align == 1 || k_align == 8 || k_align == 16 || k_align == 32 || k_align == 64)) return BSP_ERR_SHAPE;
    if (capacity_cols == 0) return BSP_OK;  // nothing kept: D is empty
    if (!D || !col_idx || (T > 0 && (!X || !dY))) return BSP_ERR_NULL;
    const int64_t B = M / R;
    if (B >= ((int64_t)1 << 31) - 65536 || (double)R * (double)capacity_cols >= 9.0e18) return BSP_ERR_SHAPE;
    hipStream_t s = (hipStream_t)stream;
    const int64_t ntiles = (T + kDvTok - 1) / kDvTok;
    const bool fast = xdt != BSP_F32 && T > 0 && R % 8 == 0 && R <= 64 && N % 4 == 0 && N < ((int64_t)1 << 22) &&
                      ntiles < ((int64_t)1 << 30) && capacity_cols < ((int64_t)1 << 31) && aligned(X, 8) &&
                      aligned(dY, 16) && ws && aligned(ws, 256);
    if (fast) {
        const DvLayout L = dv_layout(M, N, R, capacity_cols);
        if (L.max_items + B >= ((int64_t)1 << 31)) return BSP_ERR_SHAPE;
        if (ws_bytes < L.total) return BSP_ERR_CAPACITY;
        int32_t *hdr = (int32_t *)ws;
        DvItem *items = (DvItem *)((uint8_t *)ws + L.items_at);
        uint16_t *perm = (uint16_t *)((uint8_t *)ws + L.perm_at);
        int32_t *groups = (int32_t *)((uint8_t *)ws + L.groups_at);
        float *partial = (float *)((uint8_t *)ws + L.partial_at);
        const int32_t nslab = (R + 15) / 16, nr = (int32_t)((N + kDvRange - 1) / kDvRange);
        // a wavefront per item in the second part, in at most 64 workgroups
        int64_t lg = (L.max_items + kDvThreads / kWave - 1) / (kDvThreads / kWave);
        lg = lg < 1 ? 1 : (lg > 64 ? 64 : lg);
        if (ws_state == BSP_DVALS_BUILD)
            dvals_items_kernel<<<(unsigned)lg, kDvThreads, 0, s>>>(B, nslab, nr, blk_cnt, blk_ptr, col_idx,
                                                                   (int32_t)L.max_items, hdr, items, perm, groups);
        const int st = xdt == BSP_BF16 ? launch_partial<BSP_BF16>(s, X, dY, T, M, N, R, col_idx, hdr, items, perm, groups, partial)
                                       : launch_partial<BSP_F16>(s, X, dY, T, M, N, R, col_idx, hdr, items, perm, groups, partial);
        if (st != BSP_OK) return st;
        const unsigned grid = (unsigned)(L.max_items + B);
        BSP_DISPATCH_DTYPE(gdt, GDT, (dvals_reduce_kernel<GDT><<<grid, kDvReduceThreads, 0, s>>>(
                                         B, R, blk_cnt, blk_ptr, hdr, items, perm, groups, partial, (int32_t)L.max_items, (int32_t)ntiles, D)));
        return check_launch();
    }
    if (B > 0x7fffffff) return BSP_ERR_SHAPE;
    const dim3 grid((unsigned)B, 8);
    BSP_DISPATCH_DTYPE(xdt, XDT, BSP_DISPATCH_DTYPE(gdt, GDT, (dvals_plain_kernel<XDT, GDT><<<grid, 256, 0, s>>>(
                                                                  X, dY, T, M, N, R, blk_cnt, blk_ptr, col_idx, D))));
    return check_launch();
}
