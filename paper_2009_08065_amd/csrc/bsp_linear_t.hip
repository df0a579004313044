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

constexpr int kTok = 64;            // tokens per workgroup: two halves of 32
constexpr int kCols = 256;          // output columns per workgroup
constexpr int kPitch = kTok + 4;    // tile pitch in words, one row per column: 16 columns at 4 tokens each reach all banks
constexpr int kTileWords = (kCols + 1) * kPitch;  // row kCols is spare: lanes without a column add there
constexpr int kWaves = 8;           // wavefront w: token half w % 2, group w / 2 of every four groups
constexpr int kThreads = kWaves * kWave;
constexpr int kTable = 256;         // row-blocks per pass: one per thread (of the first 256) when the table is built
constexpr int kMaxSlots = (kCols + 3 + 63) / 64;  // slots of a row-block: 64 positions each, the first aligned down to 4
constexpr int kMaxSteps = kTable * kMaxSlots;
constexpr int kDepth = 3;           // steps whose operands are in flight ahead of the one being computed

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
// Matrix-core kernel.  16-bit values, R % 4 == 0, R <= 64, k_align % 4 == 0, U 8-byte aligned.
// grid.x = token tiles, grid.y = column ranges.  NK = contraction chunks of 16 (ceil(R / 16)).
//
// v_mfma_f32_16x16x16 with A = U (row = token, k = r) and B = the value panel (k = r, column =
// kept column): lane l supplies A[l % 16][4 (l / 16) ..+3], four consecutive elements of a row
// of U, and B[4 (l / 16) ..+3][l % 16]; it receives D[4 (l / 16) + i][l % 16], i.e. four
// consecutive tokens of one kept column, which lie side by side in the tile (one row per
// column): one 16-byte LDS read and one write add them.
//
// The work of a workgroup is a sequence of steps (row-block, slot): in a step wavefront w takes
// group 4 slot + w / 2 of the row-block's groups of 16 kept columns (if there is one) for its
// 32 tokens.  The sequence is written to LDS once per pass, it is the same for all wavefronts,
// its loads are issued kDepth steps ahead into a ring of registers, and the barrier falls after
// the last slot of a row-block.  A step has no branches: a lane or a wavefront without work
// loads from clamped addresses, multiplies zeros and adds to a spare cell of its tile row.
// ---------------------------------------------------------------------------------------
struct BlockEntry {  // one row-block as seen from a column range
    uint32_t lohi;   // positions [lo, hi) of its kept columns inside the range: lo | hi << 16
    uint32_t base;   // blk_ptr[b]
    uint32_t kp;     // padded number of kept columns: row pitch of the value panel
};

template <int DT, int NK, bool FULLK>  // FULLK: R == 16 NK, no lane of the contraction is past R
__global__ __launch_bounds__(kThreads) void linear_t_mfma_kernel(const uint16_t *__restrict__ U, int64_t T, int64_t M,
                                                                 int64_t N, int64_t B, int32_t R,
                                                                 const int32_t *__restrict__ blk_cnt,
                                                                 const int32_t *__restrict__ blk_ptr,
                                                                 const int32_t *__restrict__ col_idx,
                                                                 const uint16_t *__restrict__ vals,
                                                                 const void *__restrict__ bias, void *__restrict__ Z) {
    extern __shared__ __align__(16) unsigned char smem[];
    float *tile = reinterpret_cast<float *>(smem);  // [kCols + 1][kPitch]: cell of (column c, token t) at c kPitch + t
    BlockEntry *table = reinterpret_cast<BlockEntry *>(smem + sizeof(float) * kTileWords);  // [kTable]
    uint16_t *steps = reinterpret_cast<uint16_t *>(table + kTable);  // [kMaxSteps]: block | slot << 9 | last << 12
    __shared__ int wave_sum[kWaves];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, kg = lane >> 4;
    const int half = wave & 1, gsel = wave >> 1;
    const int64_t t0 = (int64_t)blockIdx.x * kTok;
    const int cr0 = (int)blockIdx.y * kCols;

    for (int i = tid; i < kTileWords; i += kThreads) tile[i] = 0.0f;

    // this lane's two rows of U (A operands); a token past T reads row 0, and what it yields is never written out
    const int64_t ta = t0 + 32 * half + l16, tb = ta + 16;
    const uint16_t *urow_a = U + (ta < T ? ta : 0) * M;
    const uint16_t *urow_b = U + (tb < T ? tb : 0) * M;
    const int tcell = 32 * half + 4 * kg;  // the four tokens whose sums this lane receives, inside a tile row
    const int spare = kCols * kPitch + tcell;

    for (int64_t bc = 0; bc < B; bc += kTable) {
        const int nb = (int)((B - bc) < kTable ? (B - bc) : kTable);
        __syncthreads();  // the tile is zeroed / the previous pass is done with the table
        // Thread q describes the q-th row-block of this pass's order, which starts at another row-block in every
        // workgroup: the workgroups resident at one time then do not all ask for the same value panels and the
        // same column slice of U at once.
        const int rot = (int)(((blockIdx.x + 5u * blockIdx.y) * 8u) % (unsigned)nb);
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
        for (int sl = 0; sl < my_slots; ++sl)
            steps[first + sl] = (uint16_t)(my_i | (sl << 9) | ((sl + 1 == my_slots) << 12));
        __syncthreads();
        if (total == 0) continue;  // uniform: nothing of this pass falls into the range

        // ring of operands in flight
        uint32_t ra[kDepth][NK][4];  // four values of the panel, one per 16-bit load
        int rc[kDepth];              // the kept column whose sums this lane receives
        uint2 rua[kDepth][NK], rub[kDepth][NK];
        int s_lo[kDepth], s_hi[kDepth], s_g0[kDepth], s_last[kDepth];

        auto produce = [&](int st, int k) {
            const uint32_t code = __builtin_amdgcn_readfirstlane((uint32_t)steps[k < total ? k : total - 1]);
            const int i = (int)(code & 511u), slot = (int)((code >> 9) & 7u);
            const BlockEntry e = table[i];
            const uint32_t lohi = __builtin_amdgcn_readfirstlane(e.lohi);
            const uint32_t base = __builtin_amdgcn_readfirstlane(e.base);
            const uint32_t kp = __builtin_amdgcn_readfirstlane(e.kp);
            const int lo = (int)(lohi & 0xffffu), hi = (int)(lohi >> 16);
            const int g0 = (lo & ~3) + 16 * (4 * slot + gsel);
            s_lo[st] = lo;
            s_hi[st] = hi;
            s_g0[st] = g0;
            s_last[st] = (int)(code >> 12);
            // every address is clamped into the row-block's own data; what a clamped lane loads is never used
            const int gq = g0 < hi ? g0 : (lo & ~3);
            const int pa = gq + l16;
            const uint32_t pc = (uint32_t)((pa >= lo && pa < hi) ? pa : lo);
#pragma unroll
            for (int kc = 0; kc < NK; ++kc) {
                const uint32_t r = (FULLK || 16 * kc + 4 * kg < R) ? 16 * kc + 4 * kg : 0;
                const uint32_t q = (uint32_t)R * base + pc + r * kp;  // element index: fits (at most R * capacity)
                ra[st][kc][0] = vals[q];
                ra[st][kc][1] = vals[q + kp];
                ra[st][kc][2] = vals[q + 2 * kp];
                ra[st][kc][3] = vals[q + 3 * kp];
            }
            rc[st] = col_idx[base + pc];
            const uint32_t uoff = (uint32_t)(bc + i) * (uint32_t)R;  // < M
#pragma unroll
            for (int kc = 0; kc < NK; ++kc) {
                // a lane past R reads the row-block's first rows
                const uint32_t ko = (FULLK || 16 * kc + 4 * kg < R) ? 16 * kc + 4 * kg : 0;
                rua[st][kc] = *reinterpret_cast<const uint2 *>(urow_a + (uoff + ko));
                rub[st][kc] = *reinterpret_cast<const uint2 *>(urow_b + (uoff + ko));
            }
        };
        auto consume = [&](int st) {
            const int pa = s_g0[st] + l16;
            const bool a_ok = pa >= s_lo[st] && pa < s_hi[st];  // false in every lane of a wavefront without a group
            f32x4 acc_a = {0.f, 0.f, 0.f, 0.f}, acc_b = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kc = 0; kc < NK; ++kc) {
                uint2 bv = make_uint2(ra[st][kc][0] | (ra[st][kc][1] << 16), ra[st][kc][2] | (ra[st][kc][3] << 16));
                if (!FULLK && !(16 * kc + 4 * kg < R)) bv = make_uint2(0u, 0u);  // the contraction ends at R
                acc_a = mfma16<DT>::run(rua[st][kc], bv, acc_a);
                acc_b = mfma16<DT>::run(rub[st][kc], bv, acc_b);
            }
            // a lane without a column has multiplied clamped loads; its sums go to the spare row
            const int cell = a_ok ? (rc[st] - cr0) * kPitch + tcell : spare;
            f32x4 *pa4 = reinterpret_cast<f32x4 *>(tile + cell), *pb4 = reinterpret_cast<f32x4 *>(tile + cell + 16);
            const f32x4 old_a = *pa4, old_b = *pb4;
            *pa4 = old_a + acc_a;  // the kept columns of a row-block are distinct: no other lane has this cell
            *pb4 = old_b + acc_b;
            if (s_last[st]) __syncthreads();  // uniform; the next row-block may keep the same columns
        };

#pragma unroll
        for (int st = 0; st < kDepth; ++st) produce(st, st);
        int k0 = 0;
        for (; k0 + kDepth <= total; k0 += kDepth) {
#pragma unroll
            for (int st = 0; st < kDepth; ++st) {
                consume(st);
                produce(st, k0 + st + kDepth);
            }
        }
#pragma unroll
        for (int st = 0; st < kDepth; ++st)
            if (k0 + st < total) consume(st);
    }
    __syncthreads();

    // write the tile out: bias added in fp32, one rounding.  Consecutive lanes take consecutive tokens (consecutive
    // banks); a lane writes 8 columns of its token's row.
    const int ncol = (int)((N - cr0) < kCols ? (N - cr0) : kCols);
    if (ncol == kCols && (N & 7) == 0 && (reinterpret_cast<uintptr_t>(Z) & 15) == 0) {
        for (int i = tid; i < kTok * (kCols / 8); i += kThreads) {
            const int tok = i % kTok, c8 = (i / kTok) * 8;
            const int64_t t = t0 + tok;
            if (t >= T) continue;
            uint32_t w[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float v0 = tile[(c8 + 2 * q) * kPitch + tok], v1 = tile[(c8 + 2 * q + 1) * kPitch + tok];
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
            float v = tile[c * kPitch + tok];
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
void launch_mfma_one(dim3 grid, size_t lds, hipStream_t s, const uint16_t *U, int64_t T, int64_t M, int64_t N,
                     int64_t B, int32_t R, const int32_t *blk_cnt, const int32_t *blk_ptr, const int32_t *col_idx,
                     const uint16_t *vals, const void *bias, void *Z) {
    auto k = linear_t_mfma_kernel<DT, NK, FULLK>;
    static bool raised = false;  // per instantiation: dynamic LDS above 64 KB must be asked for once
    if (!raised) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)lds);
        raised = true;
    }
    k<<<grid, kThreads, lds, s>>>(U, T, M, N, B, R, blk_cnt, blk_ptr, col_idx, vals, bias, Z);
}

template <int DT>
void launch_mfma(dim3 grid, size_t lds, hipStream_t s, const uint16_t *U, int64_t T, int64_t M, int64_t N, int64_t B,
                 int32_t R, const int32_t *blk_cnt, const int32_t *blk_ptr, const int32_t *col_idx,
                 const uint16_t *vals, const void *bias, void *Z) {
#define BSP_LT_ARGS grid, lds, s, U, T, M, N, B, R, blk_cnt, blk_ptr, col_idx, vals, bias, Z
    switch ((R + 15) / 16) {
        case 1: R == 16 ? launch_mfma_one<DT, 1, true>(BSP_LT_ARGS) : launch_mfma_one<DT, 1, false>(BSP_LT_ARGS); break;
        case 2: R == 32 ? launch_mfma_one<DT, 2, true>(BSP_LT_ARGS) : launch_mfma_one<DT, 2, false>(BSP_LT_ARGS); break;
        case 3: R == 48 ? launch_mfma_one<DT, 3, true>(BSP_LT_ARGS) : launch_mfma_one<DT, 3, false>(BSP_LT_ARGS); break;
        default: R == 64 ? launch_mfma_one<DT, 4, true>(BSP_LT_ARGS) : launch_mfma_one<DT, 4, false>(BSP_LT_ARGS); break;
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
    const bool mfma_ok = udt != BSP_F32 && R % 4 == 0 && k_align % 4 == 0 && col_idx && vals && aligned(U, 8) &&
                         aligned(col_idx, 16) && (double)M * (double)(N + 64) < 4.0e9;
    if (mfma_ok) {
        const int64_t tiles = (T + kTok - 1) / kTok;
        if (tiles >= ((int64_t)1 << 31)) return BSP_ERR_SHAPE;
        const dim3 grid((unsigned)tiles, (unsigned)ranges);
        const size_t lds = sizeof(float) * kTileWords + sizeof(BlockEntry) * kTable + sizeof(uint16_t) * kMaxSteps;
        if (udt == BSP_BF16)
            launch_mfma<BSP_BF16>(grid, lds, s, (const uint16_t *)U, T, M, N, B, R, blk_cnt, blk_ptr, col_idx,
                                  (const uint16_t *)vals, bias, Z);
        else
            launch_mfma<BSP_F16>(grid, lds, s, (const uint16_t *)U, T, M, N, B, R, blk_cnt, blk_ptr, col_idx,
                                 (const uint16_t *)vals, bias, Z);
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
