// The transposed product of the block-structure-pruned layer:
//   Z[t, n] = bias[n] + sum over the kept columns (b, c) with col_idx[b, c] == n of
//             sum_r U[t, bR + r] * vals[b, r, c]
// With Y = X Wp^T + bias the layer of Sec. 3.1 (Wp: the matrix after Alg. 1), this is the
// gradient with respect to the layer's input (dX = dY Wp), and it is the layer itself when the
// pruned groups are row segments of column blocks (the other division of Alg. 1) and the
// matrix is stored transposed.
//
// Per row-block the product is a small dense one (tokens x R times R x kept columns) whose
// result is scattered to the kept columns' positions.  A workgroup owns a tile of tokens x a
// range of output columns as fp32 sums in LDS and walks the row-blocks; the kept columns of a
// row-block that fall into the range go through the matrix cores 16 at a time (contraction
// depth R), one such group and half of the tokens per wavefront, and the 16 x 16 results are
// added to the tile with a plain read, add and write: inside one row-block the kept columns
// are distinct, so no two wavefronts touch the same cell, and a workgroup barrier separates the
// additions of one row-block from those of the next.  (LDS floating-point atomics would allow
// any split of the work, but one ds_add_f32 of 64 lanes was measured at about 200 clocks here,
// twelve times the read, add and write.)  No sum leaves the compute unit before it is complete;
// the tile is rounded once on the way out.
#include "bsp_common.h"

namespace bsp {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int kTok = 64;            // tokens per workgroup: two halves of 32
constexpr int kCols = 256;          // output columns per workgroup
constexpr int kTileWords = (kCols + 1) * kTok;  // one row per column; row kCols is spare: lanes without a column add there
constexpr int kWaves = 8;           // wavefront w: token half w % 2, group w / 2 of the step's four groups
constexpr int kThreads = kWaves * kWave;
constexpr int kTable = 128;         // row-blocks per pass: one per thread (of the first 128) when the table is built
constexpr int kMaxSlots = (kCols + 3 + 63) / 64;  // slots of a row-block: 64 positions each, the first aligned down to 4
constexpr int kMaxSteps = kTable * kMaxSlots;
constexpr int kDepth = 4;           // steps whose operands are on their way from memory (even: LDS buffers alternate)
static_assert(kDepth % 2 == 0, "step k uses LDS buffer k % 2, and the unrolled loop starts at multiples of kDepth");

// LDS bytes of the matrix-core kernel for NK contraction chunks of 16: tile, table, step list, two operand buffers
constexpr int stage_pitch(int nk) { return 32 * nk + 8; }  // bytes per position / per token: 16 nk values and a pad
constexpr size_t stage_bytes(int nk) { return (size_t)2 * 64 * stage_pitch(nk); }  // value panel and U piece
constexpr size_t mfma_lds_bytes(int nk) {
    return sizeof(float) * kTileWords + 12 * kTable + 2 * kMaxSteps + 2 * stage_bytes(nk);
}

template <int DT>
struct mfma16;
template <>
struct mfma16<BSP_BF16> {
    static __device__ __forceinline__ f32x4 run(uint2 a, uint2 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, a), __builtin_bit_cast(s16x4, b), c,
                                                         0, 0, 0);
    }
};
template <>
struct mfma16<BSP_F16> {
    static __device__ __forceinline__ f32x4 run(uint2 a, uint2 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(f16x4, a), __builtin_bit_cast(f16x4, b), c, 0,
                                                     0, 0);
    }
};

// first position p in [0, n) with a[p] >= key (a ascending), n if none
__device__ __forceinline__ int lower_bound(const int32_t *__restrict__ a, int n, int key) {
    int lo = 0, hi = n;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (a[mid] < key) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// ---------------------------------------------------------------------------------------
// Matrix-core kernel.  16-bit values, R % 4 == 0, R <= 64, k_align % 8 == 0, U 4-byte aligned.
// One workgroup per (token tile, column range).  NK = contraction chunks of 16 (ceil(R / 16)).
//
// v_mfma_f32_16x16x16 with A = U (row = token, k = r) and B = the value panel (k = r, column =
// kept column): lane l supplies A[l % 16][4 (l / 16) ..+3] and B[4 (l / 16) ..+3][l % 16]; it
// receives D[4 (l / 16) + i][l % 16], i.e. four consecutive tokens of one kept column, which
// lie side by side in the tile (one row per column, rotated by 4 (column % 16) words so that
// the 16 columns of a group reach all banks): one 16-byte LDS read and one write add them.
//
// The work of a workgroup is a sequence of steps (row-block, slot), a slot being 64 positions
// of the row-block's kept columns in the range, i.e. four groups of 16: in a step wavefront w
// takes group w / 2 for its 32 tokens.  The sequence is written to LDS once per pass.  The
// operands of a step are fetched by the whole workgroup, 4 bytes per thread and operand with
// whole cache lines per instruction (the address unit, not the matrix cores, bounds this
// kernel): the R x 64 piece of the value panel and the 64 x R piece of U go kDepth steps ahead
// into registers, one step ahead into LDS (the panel transposed on the way), and from there
// every wavefront reads its operands with one 8-byte read each.  A barrier ends every step: it
// orders the additions of one row-block before those of the next and the LDS buffers' reuse.
// The loads of a step have no branches (a lane without work loads from clamped addresses and,
// inside a group, adds to the spare row of the tile); for R <= 16 a wavefront whose group lies
// past the row-block's range skips the products and the additions.
// ---------------------------------------------------------------------------------------
struct BlockEntry {  // one row-block as seen from a column range
    uint32_t lohi;   // positions [lo, hi) of its kept columns inside the range: lo | hi << 16
    uint32_t base;   // blk_ptr[b]
    uint32_t kp;     // padded number of kept columns: row pitch of the value panel
};

struct StepMeta {  // wave-uniform description of a step
    int lo, hi, gbase;  // the row-block's range and the first position of the slot
};

template <int DT, int NK, bool FULLK>  // FULLK: R == 16 NK, no row of the contraction is past R
__global__ __launch_bounds__(kThreads) void linear_t_mfma_kernel(const uint16_t *__restrict__ U, int64_t T, int64_t M,
                                                                 int64_t N, int64_t B, int32_t R,
                                                                 const int32_t *__restrict__ blk_cnt,
                                                                 const int32_t *__restrict__ blk_ptr,
                                                                 const int32_t *__restrict__ col_idx,
                                                                 const uint16_t *__restrict__ vals,
                                                                 const void *__restrict__ bias, void *__restrict__ Z) {
    constexpr int kSP = stage_pitch(NK);
    extern __shared__ __align__(16) unsigned char smem[];
    float *tile = reinterpret_cast<float *>(smem);  // cell of (column c, token t): c kTok + (t + 4 c) % kTok
    BlockEntry *table = reinterpret_cast<BlockEntry *>(smem + sizeof(float) * kTileWords);  // [kTable]
    uint16_t *steps = reinterpret_cast<uint16_t *>(table + kTable);  // [kMaxSteps]: block | slot << 9
    unsigned char *stage = reinterpret_cast<unsigned char *>(steps + kMaxSteps);
    // buffer p: value panel [64 positions][kSP] at stage + p stage_bytes, U piece [64 tokens][kSP] behind it
    __shared__ int wave_sum[kWaves];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, kg = lane >> 4;
    const int half = wave & 1, gsel = wave >> 1;
    // Workgroup ids go round the 8 XCDs (each with an L2 of its own): id % 8 names the XCD.  The column ranges of
    // one token tile take consecutive places on one XCD, so that they run at the same time and share the tile's
    // rows of U in that L2.
    const uint32_t nranges = (uint32_t)((N + kCols - 1) / kCols);
    const uint32_t place = blockIdx.x >> 3;
    const uint32_t tile_id = (place / nranges) * 8u + (blockIdx.x & 7u);
    const int64_t t0 = (int64_t)tile_id * kTok;
    if (t0 >= T) return;  // the grid is rounded up to whole rounds of the XCDs (uniform: before any barrier)
    const int cr0 = (int)(place % nranges) * kCols;

    for (int i = tid; i < kTileWords; i += kThreads) tile[i] = 0.0f;

    // as a loader: two positions of panel row 16 j + tid / 32, and two elements of token tid / 8
    const int ld_row = tid >> 5, ld_pos = (tid & 31) * 2;
    const int ld_tok = tid >> 3, ld_el = (tid & 7) * 2;
    const uint16_t *ld_urow = U + (t0 + ld_tok < T ? t0 + ld_tok : 0) * M;  // a token past T reads row 0
    // byte offsets inside a buffer.  Lanes l and l + 32 hold rows 2 wave and 2 wave + 1 of the same two positions:
    // they exchange halves, so that each writes one position's pair of rows as one word.
    const bool upper = lane >= 32;
    const uint32_t pair_sel = upper ? 0x07060302u : 0x05040100u;  // bytes of {row 2w + 1, row 2w}: the halves of one position
    const int st_v = (ld_pos + (upper ? 1 : 0)) * kSP + wave * 4;
    const int st_u = 64 * kSP + ld_tok * kSP + ld_el * 2;
    // as a consumer
    const int rd_b = (16 * gsel + l16) * kSP + kg * 8;
    const int rd_a = 64 * kSP + (32 * half + l16) * kSP + kg * 8;
    const int tcell = 32 * half + 4 * kg;  // the four tokens whose sums this lane receives

    for (int64_t bc = 0; bc < B; bc += kTable) {
        const int nb = (int)((B - bc) < kTable ? (B - bc) : kTable);
        __syncthreads();  // the tile is zeroed / the previous pass is done with the table and the buffers
        // Thread q describes the q-th row-block of this pass's order, which starts at another row-block for every
        // token tile: the workgroups resident at one time then do not all ask for the same value panels at once,
        // while the workgroups of one token tile (one per column range, on the same L2) walk the same rows of U in
        // the same order and share their fetches.
        const int rot = (int)((tile_id * 8u) % (unsigned)nb);
        int my_i = 0, my_slots = 0;
        if (tid < nb) {  // nb <= kTable
            my_i = tid + rot < nb ? tid + rot : tid + rot - nb;
            const int64_t b = bc + my_i;
            const int32_t base = blk_ptr[b];
            const int32_t *cols = col_idx + base;
            const int k = blk_cnt[b];
            const int lo = k ? lower_bound(cols, k, cr0) : 0;
            const int hi = k ? lower_bound(cols, k, cr0 + kCols) : 0;
            table[my_i].lohi = (uint32_t)lo | ((uint32_t)hi << 16);
            table[my_i].base = (uint32_t)base;
            table[my_i].kp = (uint32_t)(blk_ptr[b + 1] - base);
            my_slots = hi > lo ? (hi - (lo & ~3) + 63) >> 6 : 0;
        }
        // exclusive prefix sum of the slots over the threads: where each row-block's steps go
        int incl = my_slots;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int up = __shfl_up(incl, d, 64);
            if (lane >= d) incl += up;
        }
        if (lane == 63) wave_sum[wave] = incl;
        __syncthreads();
        int first = incl - my_slots, total = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const int ws = wave_sum[w];
            if (w < wave) first += ws;
            total += ws;
        }
        for (int sl = 0; sl < my_slots; ++sl) steps[first + sl] = (uint16_t)(my_i | (sl << 9));
        __syncthreads();
        if (total == 0) continue;  // uniform: nothing of this pass falls into the range

        // ring of loads on their way, slot s: the steps k with k % kDepth == s
        uint32_t rv[kDepth][NK], ru[kDepth][NK];  // this thread's pieces of the value panel and of U
        int rc[kDepth];                           // the kept column whose sums this lane receives
        StepMeta rm[kDepth];

        // The description of a step comes from LDS in two dependent reads (step list, then table); both are started
        // one call of issue() early, so that no call waits for a read of its own: pre_e is the table entry of the
        // step the next call loads (pre_i, pre_slot: its row-block and slot), pre_code the list entry after it.
        auto step_code = [&](int k) { return (uint32_t)steps[k < total ? k : total - 1]; };
        uint32_t pre_i, pre_slot, pre_code;
        BlockEntry pre_e;
        {
            const uint32_t c0 = __builtin_amdgcn_readfirstlane(step_code(0));
            pre_i = c0 & 511u;
            pre_slot = c0 >> 9;
            pre_e = table[pre_i];
            pre_code = step_code(1);
        }
        auto issue = [&](int s, int k) {  // the loads of step k (clamped to the last one); calls come with k ascending
            const uint32_t lohi = __builtin_amdgcn_readfirstlane(pre_e.lohi);
            const uint32_t base = __builtin_amdgcn_readfirstlane(pre_e.base);
            const uint32_t kp = __builtin_amdgcn_readfirstlane(pre_e.kp);
            const uint32_t i = pre_i;
            const int slot = (int)pre_slot;
            {  // the reads for the next calls
                const uint32_t c1 = __builtin_amdgcn_readfirstlane(pre_code);
                pre_i = c1 & 511u;
                pre_slot = c1 >> 9;
                pre_e = table[pre_i];
                pre_code = step_code(k + 2);
            }
            const int lo = (int)(lohi & 0xffffu), hi = (int)(lohi >> 16);
            const int gbase = (lo & ~3) + 64 * slot;
            rm[s].lo = lo;
            rm[s].hi = hi;
            rm[s].gbase = gbase;
            // every address is clamped into the row-block's own data; what a clamped lane loads is never used
            const uint32_t pv = (uint32_t)gbase + ld_pos < kp - 2 ? (uint32_t)gbase + ld_pos : kp - 2;  // even: 4-byte aligned
            const uint32_t uoff = ((uint32_t)bc + i) * (uint32_t)R;  // < M
#pragma unroll
            for (int j = 0; j < NK; ++j) {
                const uint32_t r = (FULLK || 16 * j + ld_row < R) ? 16 * j + ld_row : 0;
                rv[s][j] = *reinterpret_cast<const uint32_t *>(vals + ((uint32_t)R * base + r * kp + pv));
                const uint32_t el = (FULLK || 16 * j + ld_el < R) ? 16 * j + ld_el : 0;  // past R: the block's first
                ru[s][j] = *reinterpret_cast<const uint32_t *>(ld_urow + (uoff + el));
            }
            const int pa = gbase + 16 * gsel + l16;
            rc[s] = col_idx[base + (uint32_t)((pa >= lo && pa < hi) ? pa : lo)];
        };
        StepMeta cur;
        int cur_col;
        auto to_lds = [&](int s, int par) {  // step k's pieces into buffer par; its column and description to cur
            unsigned char *buf = stage + par * stage_bytes(NK);
#pragma unroll
            for (int j = 0; j < NK; ++j) {
                uint32_t u = ru[s][j];
                const u32x2 xy = __builtin_amdgcn_permlane32_swap(rv[s][j], rv[s][j], false, false);  // rows 2w, 2w + 1
                uint32_t v = __builtin_amdgcn_perm(xy.y, xy.x, pair_sel);  // low lanes: the first position, upper: the second
                if (!FULLK && !(16 * j + 2 * wave < R)) v = 0u;  // the contraction ends at R (a multiple of 4)
                if (!FULLK && !(16 * j + ld_el < R)) u = 0u;
                *reinterpret_cast<uint32_t *>(buf + st_v + 32 * j) = v;
                *reinterpret_cast<uint32_t *>(buf + st_u + 32 * j) = u;
            }
            cur = rm[s];
            cur_col = rc[s];
        };
        auto consume = [&](int par) {
            // wave-uniform: no group of this slot for this wavefront (measured: 0.20 -> 0.16 ms at 10x for R = 16, but
            // 9 % slower with the larger buffers of R >= 32, where one workgroup fills the compute unit)
            if (NK == 1 && cur.gbase + 16 * gsel >= cur.hi) return;
            const unsigned char *buf = stage + par * stage_bytes(NK);
            const int pa = cur.gbase + 16 * gsel + l16;
            // (the column test only matters for a malformed storage: it keeps every write inside the tile)
            const bool a_ok = pa >= cur.lo && pa < cur.hi && (unsigned)(cur_col - cr0) < (unsigned)kCols;
            // a lane without a column multiplies clamped loads; its sums go to the spare row
            const int c = a_ok ? cur_col - cr0 : kCols;
            static_assert((4 * kCols) % kTok == 0, "the spare row must not be rotated");
            const int rot = 4 * c;
            f32x4 *pa4 = reinterpret_cast<f32x4 *>(tile + c * kTok + ((tcell + rot) & (kTok - 1)));
            f32x4 *pb4 = reinterpret_cast<f32x4 *>(tile + c * kTok + ((tcell + 16 + rot) & (kTok - 1)));
            const f32x4 old_a = *pa4, old_b = *pb4;  // read beside the operands: the products need not wait for them
            f32x4 acc_a = {0.f, 0.f, 0.f, 0.f}, acc_b = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kc = 0; kc < NK; ++kc) {
                const uint2 bv = *reinterpret_cast<const uint2 *>(buf + rd_b + 32 * kc);
                const uint2 ua = *reinterpret_cast<const uint2 *>(buf + rd_a + 32 * kc);
                const uint2 ub = *reinterpret_cast<const uint2 *>(buf + rd_a + 16 * kSP + 32 * kc);
                acc_a = mfma16<DT>::run(ua, bv, acc_a);
                acc_b = mfma16<DT>::run(ub, bv, acc_b);
            }
            *pa4 = old_a + acc_a;  // the kept columns of a row-block are distinct: no other lane has this cell
            *pb4 = old_b + acc_b;
        };

#pragma unroll
        for (int s = 0; s < kDepth; ++s) issue(s, s);
        to_lds(0, 0);
        issue(0, kDepth);
        __syncthreads();
        // iteration k: step k + 1 goes to LDS, step k + 1 + kDepth is asked for, step k is computed
        int k0 = 0;
        for (; k0 + kDepth <= total; k0 += kDepth) {
#pragma unroll
            for (int j = 0; j < kDepth; ++j) {
                const int cons_par = j & 1;
                consume(cons_par);
                to_lds((j + 1) % kDepth, cons_par ^ 1);
                issue((j + 1) % kDepth, k0 + j + 1 + kDepth);
                __syncthreads();
            }
        }
#pragma unroll
        for (int j = 0; j < kDepth; ++j) {
            if (k0 + j < total) {  // uniform
                consume(j & 1);
                to_lds((j + 1) % kDepth, (j & 1) ^ 1);
                __syncthreads();
            }
        }
    }
    __syncthreads();

    // write the tile out: bias added in fp32, one rounding.  Consecutive lanes take consecutive tokens (consecutive
    // banks); a lane writes 8 columns of its token's row.
    const int ncol = (int)((N - cr0) < kCols ? (N - cr0) : kCols);
    auto cell_of = [&](int c, int tok) { return c * kTok + ((tok + 4 * c) & (kTok - 1)); };
    if (ncol == kCols && (N & 7) == 0 && (reinterpret_cast<uintptr_t>(Z) & 15) == 0) {
        for (int i = tid; i < kTok * (kCols / 8); i += kThreads) {
            const int tok = i % kTok, c8 = (i / kTok) * 8;
            const int64_t t = t0 + tok;
            if (t >= T) continue;
            uint32_t w[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float v0 = tile[cell_of(c8 + 2 * q, tok)], v1 = tile[cell_of(c8 + 2 * q + 1, tok)];
                if (bias) {
                    v0 += elem<DT>::load(bias, cr0 + c8 + 2 * q);
                    v1 += elem<DT>::load(bias, cr0 + c8 + 2 * q + 1);
                }
                w[q] = elem<DT>::bits(v0) | (elem<DT>::bits(v1) << 16);
            }
            *reinterpret_cast<uint4 *>((uint16_t *)Z + t * N + cr0 + c8) = make_uint4(w[0], w[1], w[2], w[3]);
        }
    } else {
        for (int i = tid; i < kTok * kCols; i += kThreads) {
            const int tok = i % kTok, c = i / kTok;
            const int64_t t = t0 + tok;
            if (t >= T || c >= ncol) continue;
            float v = tile[cell_of(c, tok)];
            if (bias) v += elem<DT>::load(bias, cr0 + c);
            elem<DT>::store(Z, t * N + cr0 + c, v);
        }
    }
}

// ---------------------------------------------------------------------------------------
// General kernel: any dtype, any R in [1, 64], any k_align.  Same tile, fp32 fused
// multiply-adds; a thread owns one kept column of the row-block at a time and walks the tokens.
// ---------------------------------------------------------------------------------------
constexpr int kGenTok = 32, kGenThreads = 256, kGenPitch = kCols + 1;

template <int DT>
__global__ __launch_bounds__(kGenThreads) void linear_t_general_kernel(const void *__restrict__ U, int64_t T, int64_t M,
                                                                      int64_t N, int64_t B, int32_t R,
                                                                      const int32_t *__restrict__ blk_cnt,
                                                                      const int32_t *__restrict__ blk_ptr,
                                                                      const int32_t *__restrict__ col_idx,
                                                                      const void *__restrict__ vals,
                                                                      const void *__restrict__ bias,
                                                                      void *__restrict__ Z) {
    __shared__ float tile[kGenTok][kGenPitch];
    __shared__ float us[kGenTok][64];
    const int tid = threadIdx.x;
    const int64_t t0 = (int64_t)blockIdx.x * kGenTok;
    const int cr0 = (int)blockIdx.y * kCols;
    for (int i = tid; i < kGenTok * kGenPitch; i += kGenThreads) (&tile[0][0])[i] = 0.0f;
    for (int64_t b = 0; b < B; ++b) {
        const int k = blk_cnt[b];
        if (k == 0) continue;  // uniform over the workgroup
        const int64_t base = blk_ptr[b];
        const int kp = blk_ptr[b + 1] - blk_ptr[b];
        __syncthreads();
        for (int i = tid; i < kGenTok * R; i += kGenThreads) {
            const int tok = i / R, r = i % R;
            const int64_t t = t0 + tok;
            us[tok][r] = t < T ? elem<DT>::load(U, t * M + b * R + r) : 0.0f;
        }
        __syncthreads();
        for (int p = tid; p < k; p += kGenThreads) {
            const int col = col_idx[base + p] - cr0;
            if (col < 0 || col >= kCols) continue;
            float acc[kGenTok];
#pragma unroll
            for (int tok = 0; tok < kGenTok; ++tok) acc[tok] = 0.0f;
            for (int r = 0; r < R; ++r) {
                const float w = elem<DT>::load(vals, (int64_t)R * base + (int64_t)r * kp + p);
#pragma unroll
                for (int tok = 0; tok < kGenTok; ++tok) acc[tok] = __builtin_fmaf(us[tok][r], w, acc[tok]);
            }
            // the kept columns of one row-block are distinct: no two threads share a cell
#pragma unroll
            for (int tok = 0; tok < kGenTok; ++tok) tile[tok][col] += acc[tok];
        }
    }
    __syncthreads();
    const int ncol = (int)((N - cr0) < kCols ? (N - cr0) : kCols);
    for (int i = tid; i < kGenTok * kCols; i += kGenThreads) {
        const int tok = i / kCols, c = i % kCols;
        const int64_t t = t0 + tok;
        if (t >= T || c >= ncol) continue;
        float v = tile[tok][c];
        if (bias) v += elem<DT>::load(bias, cr0 + c);
        elem<DT>::store(Z, t * N + cr0 + c, v);
    }
}

template <int DT, int NK, bool FULLK>
int launch_mfma_one(dim3 grid, size_t lds, hipStream_t s, const uint16_t *U, int64_t T, int64_t M, int64_t N,
                     int64_t B, int32_t R, const int32_t *blk_cnt, const int32_t *blk_ptr, const int32_t *col_idx,
                     const uint16_t *vals, const void *bias, void *Z) {
    auto k = linear_t_mfma_kernel<DT, NK, FULLK>;
    // per instantiation and thread: dynamic LDS above 64 KB must be asked for (repeating the call is harmless)
    static thread_local size_t configured = 0;
    if (lds > configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)lds);
        if (e != hipSuccess) {
            set_last_hip_error((int)e);
            return BSP_ERR_HIP;
        }
        configured = lds;
    }
    k<<<grid, kThreads, lds, s>>>(U, T, M, N, B, R, blk_cnt, blk_ptr, col_idx, vals, bias, Z);
    return BSP_OK;
}

template <int DT>
int launch_mfma(dim3 grid, size_t lds, hipStream_t s, const uint16_t *U, int64_t T, int64_t M, int64_t N, int64_t B,
                 int32_t R, const int32_t *blk_cnt, const int32_t *blk_ptr, const int32_t *col_idx,
                 const uint16_t *vals, const void *bias, void *Z) {
#define BSP_LT_ARGS grid, lds, s, U, T, M, N, B, R, blk_cnt, blk_ptr, col_idx, vals, bias, Z
    switch ((R + 15) / 16) {
        case 1: return R == 16 ? launch_mfma_one<DT, 1, true>(BSP_LT_ARGS) : launch_mfma_one<DT, 1, false>(BSP_LT_ARGS);
        case 2: return R == 32 ? launch_mfma_one<DT, 2, true>(BSP_LT_ARGS) : launch_mfma_one<DT, 2, false>(BSP_LT_ARGS);
        case 3: return R == 48 ? launch_mfma_one<DT, 3, true>(BSP_LT_ARGS) : launch_mfma_one<DT, 3, false>(BSP_LT_ARGS);
        default: return R == 64 ? launch_mfma_one<DT, 4, true>(BSP_LT_ARGS) : launch_mfma_one<DT, 4, false>(BSP_LT_ARGS);
    }
#undef BSP_LT_ARGS
}

}  // namespace
}  // namespace bsp

using namespace bsp;

extern "C" int bsp_linear_transposed(const void *U, int udt, int64_t T, int64_t M, int64_t N, int32_t R,
                                     int32_t k_align, const int32_t *blk_cnt, const int32_t *blk_ptr,
                                     const int32_t *col_idx, const void *vals, const void *bias, void *Z,
                                     void *stream) {
    if (!U || !blk_cnt || !blk_ptr || !Z) return BSP_ERR_NULL;
    if (!valid_dtype(udt)) return BSP_ERR_DTYPE;
    if (T < 0 || M <= 0 || N <= 0 || R < 1 || R > 64 || M % R != 0) return BSP_ERR_SHAPE;
    if (!(k_align == 1 || k_align == 8 || k_align == 16 || k_align == 32 || k_align == 64)) return BSP_ERR_SHAPE;
    if (T == 0) return BSP_OK;
    const int64_t B = M / R;
    const int64_t ranges = (N + kCols - 1) / kCols;
    if (ranges > 65535 || N > 65535) return BSP_ERR_SHAPE;  // kept-column positions travel as 16 bits
    hipStream_t s = (hipStream_t)stream;
    // the matrix-core kernel indexes the storage with 32 bits: at most M (N + k_align) values
    const bool mfma_ok = udt != BSP_F32 && R % 4 == 0 && k_align % 8 == 0 && col_idx && vals && aligned(U, 4) &&
                         aligned(vals, 4) && (double)M * (double)(N + 64) < 4.0e9;
    if (mfma_ok) {
        const int64_t tiles = (T + kTok - 1) / kTok;
        const int64_t wgs = (tiles + 7) / 8 * 8 * ranges;  // whole rounds of the 8 XCDs
        if (wgs >= ((int64_t)1 << 31)) return BSP_ERR_SHAPE;
        const dim3 grid((unsigned)wgs);
        const size_t lds = mfma_lds_bytes((R + 15) / 16);
        const int st = udt == BSP_BF16
                           ? launch_mfma<BSP_BF16>(grid, lds, s, (const uint16_t *)U, T, M, N, B, R, blk_cnt, blk_ptr,
                                                   col_idx, (const uint16_t *)vals, bias, Z)
                           : launch_mfma<BSP_F16>(grid, lds, s, (const uint16_t *)U, T, M, N, B, R, blk_cnt, blk_ptr,
                                                  col_idx, (const uint16_t *)vals, bias, Z);
        if (st != BSP_OK) return st;
    } else {
        const int64_t tiles = (T + kGenTok - 1) / kGenTok;
        if (tiles >= ((int64_t)1 << 31)) return BSP_ERR_SHAPE;
        const dim3 grid((unsigned)tiles, (unsigned)ranges);
        BSP_DISPATCH_DTYPE(udt, DT, {
            linear_t_general_kernel<DT><<<grid, kGenThreads, 0, s>>>(U, T, M, N, B, R, blk_cnt, blk_ptr, col_idx, vals,
                                                                     bias, Z);
        });
    }
    return check_launch();
}
