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
// row-block form an item: what one wavefront accumulates (64 registers).  A strip is 12 consecutive items of one
// column range: what a workgroup accumulates while it walks a run of token tiles.  Per tile of 32 tokens the range's
// columns of X go into LDS transposed (64 bytes per column: a lane's operand, 8 consecutive tokens of its own kept
// column, is one 16-byte read) and the items' 16 columns of dY untransposed (the transposing LDS read delivers the
// other operand).
#include "bsp_common.h"
#include "bsp_mfma_device.h"

namespace bsp {
namespace {

constexpr int kDvTok = 32;               // tokens per tile: the contraction depth of one matrix instruction
constexpr int kDvRange = 1024;           // columns of X a tile holds
constexpr int kDvStrip = 12;             // items of a strip = of a workgroup: one per multiplying wavefront
constexpr int kDvLoadWaves = 4;          // wavefronts that copy the tiles in
constexpr int kDvWaves = kDvStrip + kDvLoadWaves;
constexpr int kDvThreads = kDvWaves * kWave;
constexpr int kDvLoadThreads = kDvLoadWaves * kWave;
static_assert(kDvLoadThreads == 256, "a copying thread owns 4 columns of the tile");
constexpr int kDvYPieces = kDvStrip * 64 / kDvLoadThreads;  // 16-byte pieces of dY a copying thread moves per tile
constexpr int kDvGroups = 16;            // groups of 16 kept columns per item
constexpr int kDvReduceThreads = kDvGroups * kWave;  // the second pass: one wavefront per group of an item
constexpr int kDvQuads = kDvGroups / 4;
constexpr int kDvItemCols = kDvGroups * 16;
constexpr int kDvItemFloats = kDvGroups * 256;
constexpr uint32_t kDvXBytes = kDvRange * 64;     // 64 KiB
constexpr uint32_t kDvYBytes = kDvStrip * 1024;   // 12 KiB: per item 32 tokens x 16 rows
constexpr int kDvUnits = 256;            // workgroups of the product: one per compute unit
constexpr size_t kDvHeaderBytes = 256;

struct DvItem {
    int32_t b;      // row-block
    int32_t pos0;   // index into col_idx of the item's first kept column
    int32_t ncols;  // kept columns of the item, 0 .. 256 (0: a filler that rounds a range up to whole strips)
    int32_t sq;     // slab | column range << 8
};

// header of the workspace, written by the item kernel: items (a multiple of kDvStrip), strips
enum { kHdrItems = 0, kHdrStrips = 1 };

__host__ __device__ inline int64_t dv_max_items(int64_t B, int64_t N, int32_t R, int64_t capacity_cols) {
    const int64_t nslab = (R + 15) / 16, nr = (N + kDvRange - 1) / kDvRange;
    const int64_t n = nslab * (capacity_cols / kDvItemCols + nr * B) + kDvStrip * nr;
    return (n + kDvStrip - 1) / kDvStrip * kDvStrip;
}
inline int64_t dv_max_units(int64_t max_items) {
    return max_items / kDvStrip > kDvUnits ? max_items / kDvStrip : kDvUnits;
}

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
                                                                uint16_t *__restrict__ slotcol,
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
        const int padded = (run + kDvStrip - 1) / kDvStrip * kDvStrip;
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
                for (int e = 0; e < 4; ++e) {
                    perm[(int64_t)it * kDvItemCols + lane + kWave * e] = 0xffffu;
                    slotcol[(int64_t)it * kDvItemCols + lane + kWave * e] = (uint16_t)dv_class_column((uint32_t)(lane & 15));
                }
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
            for (int e = 0; e < 4; ++e) {
                // slotcol: the slot's column inside the range -- what the product needs; a slot without a column
                // names a column of its lane's bank group, so that it does not disturb the others' reads
                const int sl = lane + kWave * e;
                const uint32_t pj = mine[sl];
                perm[(int64_t)it * kDvItemCols + sl] = (uint16_t)pj;
                slotcol[(int64_t)it * kDvItemCols + sl] =
                    (uint16_t)(pj != 0xffffu ? (uint32_t)(col_idx[item.pos0 + (int)pj] - col0) : dv_class_column((uint32_t)(sl & 15)));
            }
            if (lane == 0) groups[it] = m + (tail + 15) / 16;
        }
    }
    if (tid == 0 && blockIdx.x == 0) {
        hdr[kHdrItems] = run;
        hdr[kHdrStrips] = run / kDvStrip;
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

// Twelve wavefronts multiply (one item each), four copy the tiles in: a wavefront that issues a tile's loads is held
// for as long as the load path needs to deliver them (about 2000 clocks for a tile: 45 bytes per clock and compute
// unit), and a wavefront cannot multiply meanwhile, so the two kinds of work belong to different wavefronts.  Two tile
// buffers in LDS, one workgroup barrier per tile: while tile i is multiplied out of one buffer, the copying
// wavefronts write tile i + 1 into the other (every wavefront finished reading it before the barrier that ended
// tile i - 1) and then issue the loads of tile i + 2, which have a whole tile's time to arrive.
template <int DT>
__global__ __launch_bounds__(kDvThreads) void dvals_partial_kernel(const uint16_t *__restrict__ X,
                                                                  const uint16_t *__restrict__ dY, int64_t T, int64_t M,
                                                                  int64_t N, int32_t R,
                                                                  const int32_t *__restrict__ hdr,
                                                                  const DvItem *__restrict__ items,
                                                                  const uint16_t *__restrict__ slotcol,
                                                                  const int32_t *__restrict__ groups,
                                                                  float *__restrict__ partial) {
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, kg = lane >> 4, qd = (lane >> 2) & 3, p4 = lane & 3;
    const int strips = hdr[kHdrStrips];
    const int ntiles = (int)((T + kDvTok - 1) / kDvTok);
    int tpu, S;
    dv_ranges(strips, ntiles, tpu, S);
    constexpr uint32_t kBuf = kDvXBytes + kDvYBytes;
    const bool loader = wave >= kDvStrip;
    const int ltid = tid - kDvStrip * kWave;  // as a copying thread: columns 4 ltid .. 4 ltid + 3 of the tile

    // Workgroup ids go round the 8 XCDs (each with an L2 of its own): the units of one XCD are consecutive, so the
    // strips of one range of tokens, which read the same rows of X, mostly share an L2.
    // (one unit per workgroup: the launch has a workgroup for every unit a storage of this capacity can have)
    const int total_units = strips * S, per_xcd = (total_units + 7) / 8;
    {
        const int u0 = blockIdx.x;
        const int unit = (u0 & 7) * per_xcd + (u0 >> 3);
        if (u0 >= per_xcd * 8 || unit >= total_units) return;  // (the same for the whole workgroup, before any barrier)
        const int strip = unit % strips, s = unit / strips;
        const int tile0 = s * tpu, tile1 = tile0 + tpu < ntiles ? tile0 + tpu : ntiles;
        // the column range is the same for all items of a strip
        const int col0 = ((__builtin_amdgcn_readfirstlane(items[(int64_t)strip * kDvStrip].sq) >> 8) & 0xffff) * kDvRange;

        if (loader) {
            // ---------------------------------------------------------------- copying wavefronts
            // X: the thread's 4 columns x 32 tokens, one 8-byte load per token; columns past N are read from the last
            // valid place instead (nothing reads those LDS cells).  dY: kDvYPieces pieces of 8 rows of one token.
            // Tokens past T must be zeros in both operands (only the last tile can hold some).
            const int cqc = col0 + 4 * ltid + 4 <= N ? 4 * ltid : (int)(N - col0 - 4);
            uint32_t yoff[kDvYPieces];  // byte offset of the piece from the tile's first token row of dY
            uint32_t ydst[kDvYPieces];
#pragma unroll
            for (int e = 0; e < kDvYPieces; ++e) {
                const int pc = ltid + kDvLoadThreads * e, it = pc >> 6, tok = (pc & 63) >> 1, half = pc & 1;
                const DvItem *rec = items + (int64_t)strip * kDvStrip + it;
                const int64_t row0 = (int64_t)rec->b * R + 16 * (rec->sq & 0xff);
                // (for R = 8 the upper half of the last row-block's slab lies past M: its rows are never written out)
                const int64_t row = row0 + 8 * half + 8 <= M ? row0 + 8 * half : row0;
                yoff[e] = 2u * ((uint32_t)tok * (uint32_t)M + (uint32_t)row);
                ydst[e] = kDvXBytes + (uint32_t)it * 1024u + (uint32_t)tok * 32u + (uint32_t)half * 16u;
            }
            uint2 xa[kDvTok];
            uint4 ya[kDvYPieces];
            auto issue = [&](int tile) {
                const int64_t t0 = (int64_t)tile * kDvTok;
                const int left = (int)(T - t0 < kDvTok ? T - t0 : kDvTok);
                const uint8_t *xrow = reinterpret_cast<const uint8_t *>(X + t0 * N + col0) + 2 * cqc;
#pragma unroll
                for (int t = 0; t < kDvTok; ++t) {
                    xa[t] = t < left ? *reinterpret_cast<const uint2 *>(xrow) : make_uint2(0u, 0u);  // (t < left: uniform)
                    xrow += 2 * N;
                }
                const uint8_t *yrow = reinterpret_cast<const uint8_t *>(dY + t0 * M);
#pragma unroll
                for (int e = 0; e < kDvYPieces; ++e) {
                    const int tok = ((ltid + kDvLoadThreads * e) & 63) >> 1;
                    ya[e] = tok < left ? *reinterpret_cast<const uint4 *>(yrow + yoff[e]) : make_uint4(0u, 0u, 0u, 0u);
                }
            };
            auto commit = [&](uint32_t buf) {
                uint8_t *base = smem_x + buf * kBuf;
                // column c + j, tokens 8 g .. 8 g + 7: the j-th 16-bit field of eight consecutive loads
#pragma unroll
                for (int j = 0; j < 4; ++j) {
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        uint32_t w[4];
#pragma unroll
                        for (int h = 0; h < 4; ++h) {
                            const uint2 lo = xa[8 * g + 2 * h], hi = xa[8 * g + 2 * h + 1];
                            const uint32_t a = j < 2 ? lo.x : lo.y, bb = j < 2 ? hi.x : hi.y;
                            w[h] = (j & 1) ? ((a >> 16) | (bb & 0xffff0000u)) : ((a & 0xffffu) | (bb << 16));
                        }
                        *reinterpret_cast<uint4 *>(base + dv_x_offset(4u * (uint32_t)ltid + (uint32_t)j, (uint32_t)g)) =
                            make_uint4(w[0], w[1], w[2], w[3]);
                    }
                }
#pragma unroll
                for (int e = 0; e < kDvYPieces; ++e) *reinterpret_cast<uint4 *>(base + ydst[e]) = ya[e];
            };
            __syncthreads();
            issue(tile0);
            commit(0);
            if (tile0 + 1 < tile1) issue(tile0 + 1);
            __syncthreads();
            for (int tile = tile0; tile < tile1; ++tile) {
                const uint32_t cur = (uint32_t)(tile - tile0) & 1u;
                if (tile + 1 < tile1) {
                    commit(cur ^ 1u);
                    if (tile + 2 < tile1) issue(tile + 2);
                }
                __syncthreads();
            }
        } else {
            // ---------------------------------------------------------------- multiplying wavefronts
            const int64_t it = (int64_t)strip * kDvStrip + wave;
            const int ng = __builtin_amdgcn_readfirstlane(groups[it]);
            uint32_t xoff[kDvGroups / 2];  // LDS offsets of the lane's columns, two 16-bit halves per register
            f32x4 acc[kDvGroups];
#pragma unroll
            for (int g = 0; g < kDvGroups; ++g) {
                // the column dealt to this lane's slot (the list names one for empty slots too)
                const uint32_t c = g < ng ? (uint32_t)slotcol[it * kDvItemCols + 16 * g + l16] : dv_class_column((uint32_t)l16);
                const uint32_t o = dv_x_offset(c, (uint32_t)kg);
                xoff[g >> 1] = (g & 1) ? (xoff[g >> 1] | (o << 16)) : o;
                acc[g] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
            // the lane's address inside the item's dY rows for the transposing read (token 8 kg + qd, rows 4 p4 ..
            // 4 p4 + 3; the second read takes the token 4 further on)
            const uint32_t a_off = kDvXBytes + (uint32_t)wave * 1024u + (uint32_t)(8 * kg + qd) * 32u + (uint32_t)p4 * 8u;
            __syncthreads();
            __syncthreads();
            for (int tile = tile0; tile < tile1; ++tile) {
                const uint8_t *xt = smem_x + ((uint32_t)(tile - tile0) & 1u) * kBuf;
                // The item's groups go four at a time (a quad): the reads of the next quad are on their way while
                // the current one is multiplied; a group past the item's last one multiplies some column into an
                // accumulator that is never written out.
                const uint2 lo = tr_read(xt, a_off);
                const uint2 hi = tr_read(xt, a_off + 4 * 32);
                const uint4 a = make_uint4(lo.x, lo.y, hi.x, hi.y);
                uint4 bq[2][4];
                auto read_quad = [&](auto Q, uint4(&dst)[4]) {
                    if (4 * Q.value < ng) {
                        uint32_t w0 = xoff[2 * Q.value], w1 = xoff[2 * Q.value + 1];
                        asm volatile("" : "+v"(w0), "+v"(w1));  // (unpacked once before the loop they cost 16 registers)
                        dst[0] = *reinterpret_cast<const uint4 *>(xt + (w0 & 0xffffu));
                        dst[1] = *reinterpret_cast<const uint4 *>(xt + (w0 >> 16));
                        dst[2] = *reinterpret_cast<const uint4 *>(xt + (w1 & 0xffffu));
                        dst[3] = *reinterpret_cast<const uint4 *>(xt + (w1 >> 16));
                    }
                };
                read_quad(std::integral_constant<int, 0>{}, bq[0]);
                static_for<0, kDvQuads>([&](auto Q) {
                    if constexpr (Q.value + 1 < kDvQuads)
                        read_quad(std::integral_constant<int, Q.value + 1>{}, bq[(Q.value + 1) & 1]);
                    if (4 * Q.value < ng) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) acc[4 * Q.value + j] = mfma16<DT>(a, bq[Q.value & 1][j], acc[4 * Q.value + j]);
                    }
                });
                __syncthreads();
            }
            float *dst = partial + ((int64_t)unit * kDvStrip + wave) * kDvItemFloats + lane * 4;
            static_for<0, kDvGroups>([&](auto G) {
                if (G.value < ng) *reinterpret_cast<f32x4 *>(dst + G.value * 256) = acc[G.value];
            });
        }
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
    const int64_t strip = id / kDvStrip;
    const int w = (int)(id % kDvStrip);
    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < S; ++s) {
        const float *src = partial + ((s * strips + strip) * kDvStrip + w) * kDvItemFloats + wave * 256 + lane * 4;
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
    size_t items_at, groups_at, perm_at, slotcol_at, partial_at, total;
};
DvLayout dv_layout(int64_t M, int64_t N, int32_t R, int64_t capacity_cols) {
    DvLayout L;
    L.max_items = dv_max_items(M / R, N, R, capacity_cols);
    L.max_units = dv_max_units(L.max_items);
    L.items_at = kDvHeaderBytes;
    L.groups_at = (L.items_at + (size_t)L.max_items * sizeof(DvItem) + 255) / 256 * 256;
    L.perm_at = (L.groups_at + (size_t)L.max_items * sizeof(int32_t) + 255) / 256 * 256;
    L.slotcol_at = L.perm_at + (size_t)L.max_items * kDvItemCols * sizeof(uint16_t);
    L.partial_at = L.slotcol_at + (size_t)L.max_items * kDvItemCols * sizeof(uint16_t);
    L.total = L.partial_at + (size_t)L.max_units * kDvStrip * kDvItemFloats * sizeof(float);
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
                   const int32_t *hdr, const DvItem *items, const uint16_t *slotcol, const int32_t *groups,
                   float *partial, int64_t grid) {
    auto k = dvals_partial_kernel<DT>;
    const size_t lds = 2 * (size_t)(kDvXBytes + kDvYBytes);  // two tile buffers, 152 KiB
    const int st = dv_raise_lds(k, lds);
    if (st != BSP_OK) return st;
    k<<<(unsigned)grid, kDvThreads, lds, s>>>((const uint16_t *)X, (const uint16_t *)dY, T, M, N, R, hdr, items, slotcol,
                                        groups, partial);
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
        uint16_t *slotcol = (uint16_t *)((uint8_t *)ws + L.slotcol_at);
        int32_t *groups = (int32_t *)((uint8_t *)ws + L.groups_at);
        float *partial = (float *)((uint8_t *)ws + L.partial_at);
        const int32_t nslab = (R + 15) / 16, nr = (int32_t)((N + kDvRange - 1) / kDvRange);
        // a wavefront per item in the second part, in at most 64 workgroups
        int64_t lg = (L.max_items + kDvThreads / kWave - 1) / (kDvThreads / kWave);
        lg = lg < 1 ? 1 : (lg > 64 ? 64 : lg);
        if (ws_state == BSP_DVALS_BUILD)
            dvals_items_kernel<<<(unsigned)lg, kDvThreads, 0, s>>>(B, nslab, nr, blk_cnt, blk_ptr, col_idx,
                                                                   (int32_t)L.max_items, hdr, items, perm, slotcol, groups);
        const int64_t pgrid = (L.max_units + 7) / 8 * 8;  // whole rounds of the 8 XCDs
        const int st = xdt == BSP_BF16 ? launch_partial<BSP_BF16>(s, X, dY, T, M, N, R, hdr, items, slotcol, groups, partial, pgrid)
                                       : launch_partial<BSP_F16>(s, X, dY, T, M, N, R, hdr, items, slotcol, groups, partial, pgrid);
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
