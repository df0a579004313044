// The layer kernel for row-blocks of 16 rows and layers of more than 1024 input columns (Sec. 3.1, Sec. 4.4),
// bf16 / fp16 on gfx950: the X tile streams through LDS in chunks of 512 columns while the products run.
//
// A workgroup owns 64 tokens and 32 row-blocks (a group of the plan).  Eight wavefronts compute: each keeps the
// accumulators of four consecutive row-blocks (128 bytes of a token's output row) across all column chunks and
// walks, chunk by chunk, the steps of its blocks inside the chunk -- the step loop of the kernel for narrow layers
// (assembly: operand ring of four steps, hand-counted waits, X fragments of the next step requested between the
// matrix instructions of this one), once per accumulator set.  Eight more wavefronts do nothing but copy X: while
// the products of chunk q run out of one half of the 128 KiB tile, they write chunk q + 1 (64 tokens x 512
// columns, transposed to [column][16 tokens]) into the other half, with the loads of the chunks after it already
// in flight.  One barrier per chunk hands a filled half over and frees the other one.  Wavefronts that only load
// and wavefronts that only multiply keep separate load counters, so neither ever waits for the other's memory
// latency -- with the copy inside the multiplying wavefronts every wait for an operand would also be a wait for
// the chunk's loads, which are issued earlier and complete in order.  (Measured on the BERT-large down-projection:
// the products alone take 2.0 us per chunk, and a chunk of X that comes from HBM adds about 1.4 us during which the
// operand streams -- loads that hit in the L2 -- do not advance: the compute unit's loads return in order.  Eight
// copying wavefronts keep enough loads in flight to bring X in at the rate HBM gives, four did not.)
//
// The plan of such a layer is cut into chunks of 512 columns (plan_chunks), has 8 streams and runs of 4 row-blocks
// and gives every (row-block, chunk) at least one step, so a run never has zero steps.  Output once at the end:
// bias added, rounded, the lanes re-dealt so that every store instruction writes 8 token rows x 128 bytes.
#include "bsp_common.h"
#include "bsp_linear_internal.h"
#include "bsp_mfma_device.h"
#include "bsp_tile_device.h"

namespace bsp {
namespace {

constexpr int kStComputeWaves = 8;
constexpr int kStLoadWaves = 8;
constexpr int kStThreads = (kStComputeWaves + kStLoadWaves) * 64;
constexpr int kStNacc = 4;
constexpr int kStChunk = 512;  // columns

// Registers of the loop (fixed, listed as clobbers; the accumulators are operands):
//   v64-79 panel fragments of four steps, v80-83 offset words of four steps, v84-99 / v100-115 X fragments of an
//   even / odd step, v116-118 LDS addresses and scratch, v119 lane * 16, v120 (lane / 4) * 4, v121 token-quad mask,
//   v122 = 3.  s[40:41] fragment pointer, s[42:43] offset pointer (both four steps ahead), s44 steps left in the
//   run of the current row-block - 1, s45 chunks left - 1, s46 the step counts of the current chunk's four runs
//   (8 bits each, the current run's lowest), s47-53 those of the chunks to come, s59 scratch
#define ST_W(J) "v[64+4*" #J ":67+4*" #J "]"
#define ST_O(J) "v[80+" #J "]"
#define ST_XP(P, U, H) "v[84+16*" #P "+4*" #U "+2*" #H ":85+16*" #P "+4*" #U "+2*" #H "]"
#define ST_XQ(P, U) "v[84+16*" #P "+4*" #U ":87+16*" #P "+4*" #U "]"
#define ST_LOAD(J)                                                        \
    "global_load_dword " ST_O(J) ", v120, s[42:43] offset:64*" #J "\n"      \
    "global_load_dwordx4 " ST_W(J) ", v119, s[40:41] offset:1024*" #J "\n"
#define ST_ADVANCE                                         \
    "s_add_u32 s40, s40, 4096\n s_addc_u32 s41, s41, 0\n"  \
    "s_add_u32 s42, s42, 256\n s_addc_u32 s43, s43, 0\n"
#define ST_ADDR(JN)                                                                                            \
    "v_xor_b32 v118, " ST_O(JN) ", v121\n"                                                                     \
    "v_lshlrev_b32_sdwa v116, v122, v118 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_0\n" \
    "v_lshlrev_b32_sdwa v117, v122, v118 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1\n"
#define ST_RD(PN, U, OFF)                                              \
    "ds_read_b64_tr_b16 " ST_XP(PN, U, 0) ", v116 offset:" #OFF "\n"     \
    "ds_read_b64_tr_b16 " ST_XP(PN, U, 1) ", v117 offset:" #OFF "\n"
#define ST_READS(JN, PN) ST_ADDR(JN) ST_RD(PN, 0, 0) ST_RD(PN, 1, 16384) ST_RD(PN, 2, 32768) ST_RD(PN, 3, 49152)
#define ST_MF(MFMA, A, J, P, U) MFMA " %[a" #A #U "], " ST_W(J) ", " ST_XQ(P, U) ", %[a" #A #U "]\n"
// One step of accumulator set A at ring slot J (see the kernel for narrow layers: the same step).
#define ST_STEP(MFMA, A, J, JN, P, PN)                      \
    "s_waitcnt vmcnt(5)\n"                                  \
    ST_ADDR(JN)                                             \
    "s_waitcnt lgkmcnt(0)\n"                                \
    ST_MF(MFMA, A, J, P, 0) ST_RD(PN, 0, 0)                 \
    ST_MF(MFMA, A, J, P, 1) ST_RD(PN, 1, 16384)             \
    ST_MF(MFMA, A, J, P, 2) ST_RD(PN, 2, 32768)             \
    ST_MF(MFMA, A, J, P, 3) ST_RD(PN, 3, 49152)             \
    ST_LOAD(J)                                              \
    "s_sub_u32 s44, s44, 1\n"                               \
    "s_cbranch_scc1 Lend" #A "_" #J "_%=\n"                 \
    "Lres" #A "_" #J "_%=:\n"
#define ST_SET(MFMA, A)                                                                                   \
    "Ltop" #A "_%=:\n"                                                                                    \
    ST_STEP(MFMA, A, 0, 1, 0, 1) ST_STEP(MFMA, A, 1, 2, 1, 0) ST_STEP(MFMA, A, 2, 3, 0, 1) ST_STEP(MFMA, A, 3, 0, 1, 0) \
    ST_ADVANCE                                                                                            \
    "s_branch Ltop" #A "_%=\n"
// The run of set A has ended behind ring slot J: on with the next row-block's run, one slot further.
#define ST_NEXT_RUN(A, AN, J)                                                                  \
    "Lend" #A "_" #J "_%=:\n"                                                                  \
    "s_lshr_b32 s46, s46, 8\n s_and_b32 s44, s46, 0xff\n s_sub_u32 s44, s44, 1\n"              \
    "s_branch Lres" #AN "_" #J "_%=\n"
// The chunk has ended behind ring slot J.  The X fragments the last step requested for its successor came out of
// the half of the tile that was still being filled; they are requested again behind the barrier.
#define ST_NEXT_CHUNK(J, JN, PN)                                                               \
    "Lend3_" #J "_%=:\n"                                                                       \
    "s_sub_u32 s45, s45, 1\n"                                                                  \
    "s_cbranch_scc1 Ldone%=\n"                                                                 \
    "s_mov_b32 s46, s47\n s_mov_b32 s47, s48\n s_mov_b32 s48, s49\n s_mov_b32 s49, s50\n"      \
    "s_mov_b32 s50, s51\n s_mov_b32 s51, s52\n s_mov_b32 s52, s53\n"                           \
    "s_and_b32 s44, s46, 0xff\n s_sub_u32 s44, s44, 1\n"                                       \
    "s_waitcnt lgkmcnt(0)\n"                                                                   \
    "s_barrier\n"                                                                              \
    ST_READS(JN, PN)                                                                           \
    "s_branch Lres0_" #J "_%=\n"

#define ST_CLOBBERS                                                                                                    \
    "v64", "v65", "v66", "v67", "v68", "v69", "v70", "v71", "v72", "v73", "v74", "v75", "v76", "v77", "v78", "v79",    \
        "v80", "v81", "v82", "v83", "v84", "v85", "v86", "v87", "v88", "v89", "v90", "v91", "v92", "v93", "v94",       \
        "v95", "v96", "v97", "v98", "v99", "v100", "v101", "v102", "v103", "v104", "v105", "v106", "v107", "v108",     \
        "v109", "v110", "v111", "v112", "v113", "v114", "v115", "v116", "v117", "v118", "v119", "v120", "v121",        \
        "v122", "s40", "s41", "s42", "s43", "s44", "s45", "s46", "s47", "s48", "s49", "s50", "s51", "s52", "s53",      \
        "s59", "scc", "memory"

#define ST_ACC_OPERANDS                                                                                              \
    [a00] "+v"(acc[0][0]), [a01] "+v"(acc[0][1]), [a02] "+v"(acc[0][2]), [a03] "+v"(acc[0][3]), [a10] "+v"(acc[1][0]), \
        [a11] "+v"(acc[1][1]), [a12] "+v"(acc[1][2]), [a13] "+v"(acc[1][3]), [a20] "+v"(acc[2][0]),                  \
        [a21] "+v"(acc[2][1]), [a22] "+v"(acc[2][2]), [a23] "+v"(acc[2][3]), [a30] "+v"(acc[3][0]),                  \
        [a31] "+v"(acc[3][1]), [a32] "+v"(acc[3][2]), [a33] "+v"(acc[3][3])

// The whole walk of a wavefront: all chunks, four runs each.
#define ST_WALK(MFMA)                                                                                             \
    asm volatile(                                                                                                 \
        "s_mov_b64 s[40:41], %[wb]\n s_mov_b64 s[42:43], %[ob]\n s_sub_u32 s45, %[nq], 1\n"                       \
        "s_mov_b64 s[46:47], %[c01]\n s_mov_b64 s[48:49], %[c23]\n s_mov_b64 s[50:51], %[c45]\n"                  \
        "s_mov_b64 s[52:53], %[c67]\n"                                                                            \
        "v_mbcnt_lo_u32_b32 v118, -1, 0\n v_mbcnt_hi_u32_b32 v118, -1, v118\n"                                    \
        "v_lshlrev_b32 v119, 4, v118\n v_and_b32 v120, 0xfc, v118\n"                                              \
        "v_and_b32 v121, 3, v118\n v_lshl_or_b32 v121, v121, 16, v121\n v_mov_b32 v122, 3\n"                      \
        ST_LOAD(0) ST_LOAD(1) ST_LOAD(2) ST_LOAD(3) ST_ADVANCE                                                    \
        "s_and_b32 s44, s46, 0xff\n s_sub_u32 s44, s44, 1\n"                                                      \
        "s_barrier\n" /* the first chunk is there */                                                              \
        "s_waitcnt vmcnt(7)\n"                                                                                    \
        ST_READS(0, 0)                                                                                            \
        ST_SET(MFMA, 0) ST_SET(MFMA, 1) ST_SET(MFMA, 2) ST_SET(MFMA, 3)                                           \
        ST_NEXT_RUN(0, 1, 0) ST_NEXT_RUN(0, 1, 1) ST_NEXT_RUN(0, 1, 2) ST_NEXT_RUN(0, 1, 3)                       \
        ST_NEXT_RUN(1, 2, 0) ST_NEXT_RUN(1, 2, 1) ST_NEXT_RUN(1, 2, 2) ST_NEXT_RUN(1, 2, 3)                       \
        ST_NEXT_RUN(2, 3, 0) ST_NEXT_RUN(2, 3, 1) ST_NEXT_RUN(2, 3, 2) ST_NEXT_RUN(2, 3, 3)                       \
        ST_NEXT_CHUNK(0, 1, 1) ST_NEXT_CHUNK(1, 2, 0) ST_NEXT_CHUNK(2, 3, 1) ST_NEXT_CHUNK(3, 0, 0)               \
        "Ldone%=:\n"                                                                                              \
        "s_waitcnt vmcnt(0) lgkmcnt(0)\n"                                                                         \
        "s_nop 15\n s_nop 7\n" /* the last matrix instruction has written its result */                           \
        : ST_ACC_OPERANDS                                                                                         \
        : [wb] "s"(wb), [ob] "s"(ob), [nq] "s"(nq), [c01] "s"(cnt[0]), [c23] "s"(cnt[1]), [c45] "s"(cnt[2]),      \
          [c67] "s"(cnt[3])                                                                                       \
        : ST_CLOBBERS)

// Loads of one chunk of X by the copying wavefronts: thread j of 256 takes units j, j + 256, ... (a unit = 4 columns
// x 4 tokens); the values wait in registers until the half of the tile they go to is free.
constexpr int kStUnits = 4;  // per thread: 64 tokens x 512 columns / 16 / 512
struct ChunkRegs {
    uint2 a[kStUnits][4];
};
__device__ __forceinline__ void chunk_issue(ChunkRegs &r, const uint16_t *__restrict__ X, int64_t T, int64_t N,
                                            int32_t col0, int32_t width, int64_t t0, int j) {
    const int cquads = width >> 2;
    const int units = cquads * 16;
#pragma unroll
    for (int k = 0; k < kStUnits; ++k) {
        const int u = j + k * (kStLoadWaves * 64);
        const int cq = u % cquads, tq = u / cquads;
        const int c = cq << 2;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t t = t0 + 4 * tq + i;
            r.a[k][i] = (u < units && t < T && col0 + c < N) ? *reinterpret_cast<const uint2 *>(X + t * N + col0 + c)
                                                             : make_uint2(0u, 0u);
        }
    }
}
__device__ __forceinline__ void chunk_commit(const ChunkRegs &r, int32_t width, uint32_t half, int j) {
    const int cquads = width >> 2;
    const int units = cquads * 16;
#pragma unroll
    for (int k = 0; k < kStUnits; ++k) {
        const int u = j + k * (kStLoadWaves * 64);
        if (u >= units) break;
        const int cq = u % cquads, tq = u / cquads;
        const int c = cq << 2;
        const uint32_t sub = (uint32_t)(tq >> 2), pq = (uint32_t)(tq & 3);
        uint8_t *dst = smem_x + sub * kSubStride4 + lds_col_offset4(half * kStChunk + (uint32_t)c, pq);
        uint2 w;  // columns c+1 .. c+3 lie 8, 16, 24 LDS rows further on
        w.x = (r.a[k][0].x & 0xffffu) | (r.a[k][1].x << 16);
        w.y = (r.a[k][2].x & 0xffffu) | (r.a[k][3].x << 16);
        *reinterpret_cast<uint2 *>(dst) = w;
        w.x = (r.a[k][0].x >> 16) | (r.a[k][1].x & 0xffff0000u);
        w.y = (r.a[k][2].x >> 16) | (r.a[k][3].x & 0xffff0000u);
        *reinterpret_cast<uint2 *>(dst + 8 * 32) = w;
        w.x = (r.a[k][0].y & 0xffffu) | (r.a[k][1].y << 16);
        w.y = (r.a[k][2].y & 0xffffu) | (r.a[k][3].y << 16);
        *reinterpret_cast<uint2 *>(dst + 16 * 32) = w;
        w.x = (r.a[k][0].y >> 16) | (r.a[k][1].y & 0xffff0000u);
        w.y = (r.a[k][2].y >> 16) | (r.a[k][3].y & 0xffff0000u);
        *reinterpret_cast<uint2 *>(dst + 24 * 32) = w;
    }
}

// The same for a whole tile (64 token rows inside X) of a layer whose rows are whole 16-byte pieces: copying
// wavefront w takes the token quads w and w + 8 and its lanes the 64 eight-column pieces of the chunk's 512 columns
// (1 KiB of a row per load instruction).  Four 16-byte loads per quad, 16 byte-permutes, eight 8-byte LDS stores at
// one address plus constant offsets (the 8 columns share their 32-column group; columns 0 - 3 lie 8 LDS rows apart,
// columns 4 - 7 one row behind them); no bounds tests, no divisions.  The copying wavefronts share their SIMDs'
// issue slots with the multiplying ones, so what they do not execute the others can.
struct ChunkRegs16 {
    uint4 a[2][4];
};
__device__ __forceinline__ void chunk_issue(ChunkRegs16 &r, const uint16_t *__restrict__ X, int64_t T, int64_t N,
                                            int32_t col0, int32_t width, int64_t t0, int j) {
    const int lane = j & 63, wl = j >> 6;
    const int64_t c = (int64_t)col0 + 8 * lane;
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const uint16_t *row = X + (t0 + 4 * (wl + kStLoadWaves * k)) * N + c;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            r.a[k][i] = c < N ? *reinterpret_cast<const uint4 *>(row + i * N) : make_uint4(0u, 0u, 0u, 0u);
    }
}
__device__ __forceinline__ void chunk_commit(const ChunkRegs16 &r, int32_t width, uint32_t half, int j) {
    const int lane = j & 63, wl = j >> 6;
    if (8 * lane >= width) return;
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const uint32_t tq = (uint32_t)(wl + kStLoadWaves * k);
        uint8_t *dst = smem_x + (tq >> 2) * kSubStride4 + lds_col_offset4(half * kStChunk + 8u * (uint32_t)lane, tq & 3u);
        const uint32_t w[4][4] = {{r.a[k][0].x, r.a[k][1].x, r.a[k][2].x, r.a[k][3].x},
                                  {r.a[k][0].y, r.a[k][1].y, r.a[k][2].y, r.a[k][3].y},
                                  {r.a[k][0].z, r.a[k][1].z, r.a[k][2].z, r.a[k][3].z},
                                  {r.a[k][0].w, r.a[k][1].w, r.a[k][2].w, r.a[k][3].w}};
#pragma unroll
        for (int j2 = 0; j2 < 4; ++j2) {  // the column pair 2 j2, 2 j2 + 1 of the piece
            uint2 lo, hi;
            lo.x = __builtin_amdgcn_perm(w[j2][1], w[j2][0], 0x05040100u);
            lo.y = __builtin_amdgcn_perm(w[j2][3], w[j2][2], 0x05040100u);
            hi.x = __builtin_amdgcn_perm(w[j2][1], w[j2][0], 0x07060302u);
            hi.y = __builtin_amdgcn_perm(w[j2][3], w[j2][2], 0x07060302u);
            const uint32_t at = (uint32_t)(j2 >> 1) * 32u + (uint32_t)(j2 & 1) * (16u * 32u);
            *reinterpret_cast<uint2 *>(dst + at) = lo;
            *reinterpret_cast<uint2 *>(dst + at + 8u * 32u) = hi;
        }
    }
}

// The copying wavefronts' loop.  Two register sets: the loads of chunks k + 1 and k + 2 travel while chunk k is
// written and handed over (with one set a chunk's loads would be requested only after the previous chunk's had
// arrived).
template <typename Regs>
__device__ __forceinline__ void copy_chunks(const uint16_t *__restrict__ X, int64_t T, int64_t N, int32_t npad,
                                            int32_t nq, int64_t t0, int j) {
    Regs ra, rb;
    auto width_of = [&](int k) { return min(kStChunk, npad - k * kStChunk); };
    chunk_issue(ra, X, T, N, 0, width_of(0), t0, j);
    if (nq > 1) chunk_issue(rb, X, T, N, kStChunk, width_of(1), t0, j);
    for (int k = 0; k < nq; k += 2) {
        chunk_commit(ra, width_of(k), 0u, j);
        __syncthreads();  // barrier k: chunk k is written; the multiplying wavefronts are done with chunk k - 1
        if (k + 1 < nq) {
            chunk_commit(rb, width_of(k + 1), 1u, j);
            // the loads of the next two chunks leave together: while loads that miss the L2 are under way, the
            // compute unit's later loads (the operand streams of the multiplying wavefronts, which hit) wait
            // behind them, so there are as few such episodes as the registers allow
            if (k + 2 < nq) chunk_issue(ra, X, T, N, (k + 2) * kStChunk, width_of(k + 2), t0, j);
            if (k + 3 < nq) chunk_issue(rb, X, T, N, (k + 3) * kStChunk, width_of(k + 3), t0, j);
            __syncthreads();  // barrier k + 1
        }
    }
}

template <int DT>
__global__ __launch_bounds__(kStThreads) void linear_stream16_kernel(
    const uint16_t *__restrict__ X, int64_t T, int64_t M, int64_t N, int32_t npad, const int32_t *__restrict__ wptr,
    const uint8_t *__restrict__ wfrag, const uint8_t *__restrict__ xoff, const void *__restrict__ bias,
    void *__restrict__ Y, int32_t ntiles, int32_t NG, int32_t B, int32_t nq, int32_t max_step, int32_t act,
    const uint16_t *__restrict__ residual) {
    const int tile = blockIdx.x % ntiles, g = blockIdx.x / ntiles;
    const int64_t t0 = (int64_t)tile * 64;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));

    if (wave >= kStComputeWaves) {
        // ---- the copying wavefronts: chunk k into half k % 2, handed over by barrier k ----
        const int j = (int)threadIdx.x - kStComputeWaves * 64;
        // whole tiles of layers whose rows are whole 16-byte pieces take the copy without bounds tests (uniform)
        if (t0 + 64 <= T && (N & 7) == 0) copy_chunks<ChunkRegs16>(X, T, N, npad, nq, t0, j);
        else copy_chunks<ChunkRegs>(X, T, N, npad, nq, t0, j);
        return;
    }

    // ---- the multiplying wavefronts ----
    const int l16 = lane & 15, G = lane >> 4;
    const int64_t b0 = ((int64_t)g * kStComputeWaves + wave) * kStNacc;  // first row-block of the wavefront's run
    // step counts of the wavefront's runs, chunk by chunk, kept inside the plan whatever it holds; a run has
    // at least one step (runs of row-blocks past the end of the layer too: their products are never stored)
    // (a stream holds a group's runs chunk after chunk, then the next group's: entry (g * nq + q) * 4 + i)
    const int32_t *my = wptr + (int64_t)wave * ((int64_t)nq * NG * kStNacc + 1) + (int64_t)g * nq * kStNacc;
    uint64_t cnt[4] = {0, 0, 0, 0};
    const int first = min(max(my[0], 0), max_step);
    int cur = first;
    for (int q = 0; q < nq; ++q) {
        uint32_t packed = 0;
        const int32_t *ent = my + q * kStNacc;
        for (int i = 0; i < kStNacc; ++i) {
            const int nxt = min(max(ent[i + 1], cur), max_step);
            const int c = min(max(nxt - cur, 1), 64);
            packed |= (uint32_t)c << (8 * i);
            cur += c;
        }
        packed = __builtin_amdgcn_readfirstlane(packed);
        cnt[q >> 1] |= (uint64_t)packed << (32 * (q & 1));
    }
    const uint8_t *wb = wfrag + (int64_t)first * 1024;
    const uint8_t *ob = xoff + (int64_t)first * 64;
    f32x4 acc[kStNacc][4];
#pragma unroll
    for (int a = 0; a < kStNacc; ++a)
#pragma unroll
        for (int u = 0; u < 4; ++u) acc[a][u] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < 4; ++i)
        cnt[i] = (uint64_t)__builtin_amdgcn_readfirstlane((uint32_t)cnt[i]) |
                 ((uint64_t)__builtin_amdgcn_readfirstlane((uint32_t)(cnt[i] >> 32)) << 32);
    if constexpr (DT == BSP_BF16) ST_WALK("v_mfma_f32_16x16x32_bf16");
    else ST_WALK("v_mfma_f32_16x16x32_f16");

    // ---- output: bias, activation, residual, rounding, lane re-deal, whole lines ----
    if (b0 >= B) return;
    uint2 half[kStNacc][4];  // rounded: block a, sub-tile u: columns 4 G .. 4 G + 3 of token 16 u + l16
#pragma unroll
    for (int a = 0; a < kStNacc; ++a) {
        float bv[4] = {0.f, 0.f, 0.f, 0.f};
        if (bias && b0 + a < B) {
#pragma unroll
            for (int v = 0; v < 4; ++v) bv[v] = elem<DT>::load(bias, (b0 + a) * 16 + 4 * G + v);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            float y[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                y[v] = acc[a][u][v] + bv[v];
                if (act == BSP_ACT_GELU) y[v] = 0.5f * y[v] * (1.0f + erff(y[v] * 0.70710678118654752f));
            }
            const int64_t t = t0 + 16 * u + l16;
            if (residual && t < T && b0 + a < B) {  // the lane's 4 columns of token t: 8 bytes
                const uint2 rw = *reinterpret_cast<const uint2 *>(residual + t * M + (b0 + a) * 16 + 4 * G);
                const uint32_t h[4] = {rw.x & 0xffffu, rw.x >> 16, rw.y & 0xffffu, rw.y >> 16};
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    if constexpr (DT == BSP_BF16) y[v] += __uint_as_float(h[v] << 16);
                    else y[v] += (float)__builtin_bit_cast(_Float16, (uint16_t)h[v]);
                }
            }
            half[a][u].x = cvt_pk<DT>(y[0], y[1]);
            half[a][u].y = cvt_pk<DT>(y[2], y[3]);
        }
    }
    uint8_t *Yq = reinterpret_cast<uint8_t *>(Y) + t0 * M * 2 + b0 * 32;  // the quad's 128 bytes of the tile's first row
    const int nblk = (int)min((int64_t)kStNacc, B - b0);                    // row-blocks of the run inside the layer
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        // pairs of blocks: after the two swaps a lane holds 16 contiguous bytes (bytes 16 G ..) of token l16's 64
        uint4 pr[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const u32x2 px = __builtin_amdgcn_permlane32_swap(half[2 * h][u].x, half[2 * h + 1][u].x, false, false);
            const u32x2 py = __builtin_amdgcn_permlane32_swap(half[2 * h][u].y, half[2 * h + 1][u].y, false, false);
            const u32x2 qx = __builtin_amdgcn_permlane16_swap(px[0], px[1], false, false);
            const u32x2 qy = __builtin_amdgcn_permlane16_swap(py[0], py[1], false, false);
            pr[h] = make_uint4(qx[0], qy[0], qx[1], qy[1]);
        }
        if (nblk == kStNacc) {
            // the pairs trade lanes 8-15 / 0-7 of every 16-lane row: then the lanes of a row hold the whole 128 bytes
            // of token rows 0-7 (first) or 8-15 (second) of the sub-tile, and a store writes 8 whole lines
            uint4 lo, hi;
            auto trade_lo = [](uint32_t a, uint32_t b) {
                return (uint32_t)__builtin_amdgcn_update_dpp((int)a, (int)b, 0x128, 0xf, 0xc, false);
            };
            auto trade_hi = [](uint32_t a, uint32_t b) {
                return (uint32_t)__builtin_amdgcn_update_dpp((int)b, (int)a, 0x128, 0xf, 0x3, false);
            };
            lo = make_uint4(trade_lo(pr[0].x, pr[1].x), trade_lo(pr[0].y, pr[1].y), trade_lo(pr[0].z, pr[1].z),
                            trade_lo(pr[0].w, pr[1].w));
            hi = make_uint4(trade_hi(pr[0].x, pr[1].x), trade_hi(pr[0].y, pr[1].y), trade_hi(pr[0].z, pr[1].z),
                            trade_hi(pr[0].w, pr[1].w));
            const int row = 16 * u + (l16 & 7);
            uint8_t *dst = Yq + (int64_t)row * M * 2 + 64 * (l16 >> 3) + 16 * G;
            if (t0 + row < T) store_y16(dst, lo);
            if (t0 + row + 8 < T) store_y16(dst + 8 * M * 2, hi);
        } else {
            // a run that reaches past the layer's last row-block: pair by pair, a single block as its 32 bytes
            const int row = 16 * u + l16;
            uint8_t *dst = Yq + (int64_t)row * M * 2 + 16 * G;
            if (t0 + row < T) {
                if (nblk >= 2 || G < 2) store_y16(dst, pr[0]);
                if (nblk == 3 && G < 2) store_y16(dst + 64, pr[1]);
            }
        }
    }
}

}  // namespace

// Launch for R = 16, 1024 < npad <= 4096, a plan of 8 streams cut into chunks of 512 columns, Y aligned to 16 bytes.
int launch_linear_stream16(const TiledArgs &a, int64_t max_step, hipStream_t s) {
    const PlanChunks ch = plan_chunks(a.N, a.R, a.M);
    const int64_t NG = plan_groups(a.B, kStComputeWaves, kStNacc, false);
    const int64_t ntiles = (a.T + 63) / 64;
    if (ntiles * NG >= ((int64_t)1 << 31) || ch.n > kPlanMaxChunks) return BSP_ERR_SHAPE;
    if (a.act != BSP_ACT_NONE && a.act != BSP_ACT_GELU) return BSP_ERR_SHAPE;
    if (a.residual && !aligned(a.residual, 8)) return BSP_ERR_SHAPE;
    const size_t lds = kXTileBytes;
    auto go = [&](auto kern, size_t &configured) {
        int st = raise_lds_limit(kern, lds, configured);
        if (st != BSP_OK) return st;
        kern<<<dim3((unsigned)(ntiles * NG)), dim3(kStThreads), lds, s>>>(
            a.X, a.T, a.M, a.N, a.npad, a.wptr, (const uint8_t *)a.wfrag, (const uint8_t *)a.xoff, a.bias, a.Y,
            (int32_t)ntiles, (int32_t)NG, (int32_t)a.B, ch.n, (int32_t)max_step, (int32_t)a.act,
            (const uint16_t *)a.residual);
        return check_launch();
    };
    if (a.xdt == BSP_BF16) {
        static thread_local size_t configured = 0;
        return go(linear_stream16_kernel<BSP_BF16>, configured);
    }
    static thread_local size_t configured = 0;
    return go(linear_stream16_kernel<BSP_F16>, configured);
}

}  // namespace bsp
