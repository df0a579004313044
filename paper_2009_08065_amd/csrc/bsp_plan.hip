// Derived operand buffer ("plan") for the tiled layer kernel, built from the compact storage.
//
// The contraction order inside a row-block is free, so the kept columns are re-ordered for
// the LDS gather: the tiled kernel fetches an X fragment with two transposing reads, and in
// each of them a half-wavefront touches 8 columns (8 rows of 32 bytes = all 64 LDS banks when
// the rows fall into 8 different bank groups).  The kept columns of a row-block are dealt into
// sets of 8, one column per bank group where the counts allow; columns of over-full groups and
// zero-weight pads fill the gaps.  Per 32-column step the plan stores, ready to load per lane,
// the value-panel fragments (16 rows x 32 columns, 16 bytes per lane) and the two 16-bit LDS
// byte offsets of the lane's transposing reads.
//
// Order of the steps: a wavefront of the layer kernel owns "quads" of nacc = 4 / nfrag consecutive
// row-blocks (quad w of every group of `waves` quads), so the plan keeps the steps of wavefront w
// contiguous, stream after stream, in the order it walks them: chunk by chunk (layers of more than
// 1024 input columns are cut into chunks of 1024), group by group, block by block.
// wptr[w][(g * chunks + q) * nacc + i] is the step where block (g * waves + w) * nacc + i starts in
// chunk q (a stream holds a group's runs chunk after chunk, then the next group's); the last entry of a row is
// where stream w ends.
//
// Buffer layout (bytes): wptr int32 [waves][chunks * NG * nacc + 1], padded to 256 | fragments
// [steps][nfrag][64] lanes x 16 bytes (a lane's 8 values of its row) | offsets uint32 [steps][16] (one word per 4 lanes: the lanes
// of a column differ by their token quad only), with steps = capacity_cols / 32
// + 3 per row-block (every chunk pads its columns to a multiple of 32 on its own) + read-ahead slack.
// Integer work only; deterministic.
#include "bsp_common.h"
#include "bsp_linear_internal.h"

namespace bsp {
namespace {

constexpr int kThreads = 256;
constexpr int kMaxKp = 4096 + 32;
constexpr int kMaxChunk = 1024 + 32;  // kept columns of one row-block inside one column chunk, padded

__device__ __forceinline__ int slot_index(int set, int group) {
    // sets 4s .. 4s+3 of step s are what {first, second} read x {lower, upper} half-wavefront touch
    return 32 * (set >> 2) + ((set >> 1) & 1) * 16 + (set & 1) * 4 + (group >> 2) * 8 + (group & 3);
}

// Steps of every (row-block of the plan, column chunk): ceil(kept columns of the block inside the chunk / 32).
// One workgroup per block; the result goes to steps_bq[b * kPlanMaxChunks + q].  virt: the plan's block b is made
// of the stored row-blocks 2 b and 2 b + 1 (8 rows each) and keeps the union of their columns; split > 1: the
// plan's block b is a 16-row slab of the stored row-block b / split.
__global__ __launch_bounds__(kThreads) void plan_count_kernel(const int32_t *__restrict__ blk_cnt,
                                                              const int32_t *__restrict__ blk_ptr,
                                                              const int32_t *__restrict__ col_idx,
                                                              int64_t capacity_cols, int32_t chunk_shift,
                                                              int32_t nchunks, int32_t virt, int32_t split,
                                                              int32_t *__restrict__ steps_bq) {
    __shared__ int cnt[kPlanMaxChunks];
    __shared__ uint32_t seen[(kMaxKp + 31) / 32];  // columns of the first stored block (virt)
    const int64_t b = blockIdx.x;
    if (threadIdx.x < kPlanMaxChunks) cnt[threadIdx.x] = 0;
    for (int i = threadIdx.x; i < (kMaxKp + 31) / 32; i += kThreads) seen[i] = 0u;
    __syncthreads();
    for (int j = 0; j < (virt ? 2 : 1); ++j) {
        const int64_t sb = virt ? 2 * b + j : b / split;
        const int base = blk_ptr[sb];
        const int kp = blk_ptr[sb + 1] - base;
        const int kb = blk_cnt[sb];
        const bool ok = kp > 0 && kp <= kMaxKp && kb >= 0 && kb <= kp && base >= 0 && (int64_t)base + kp <= capacity_cols;
        if (ok)
            for (int i = threadIdx.x; i < kb; i += kThreads) {
                const int c = col_idx[base + i];
                const int q = c >> chunk_shift;
                if (c < 0 || c >= kMaxKp || q >= nchunks) continue;
                if (!virt) {
                    atomicAdd(&cnt[q], 1);
                } else if (j == 0) {
                    atomicOr(&seen[c >> 5], 1u << (c & 31));
                    atomicAdd(&cnt[q], 1);
                } else if (!((seen[c >> 5] >> (c & 31)) & 1u)) {
                    atomicAdd(&cnt[q], 1);
                }
            }
        __syncthreads();
    }
    if (threadIdx.x < kPlanMaxChunks) {
        steps_bq[b * kPlanMaxChunks + threadIdx.x] = (cnt[threadIdx.x] + 31) >> 5;
    }
}

// What fixes the order and the sizes of a plan's streams.
struct PlanShape {
    const int32_t *steps_bq;  // steps per (block of the plan, chunk) where a count launch made them (chunked plans,
                              // plans of paired 8-row blocks), else nullptr
    const int32_t *blk_cnt, *blk_ptr;
    int64_t capacity_cols;
    int32_t B, NG, nacc, nchunks, paired, min_one, virt, split, waves;
    __device__ bool chunked() const { return nchunks > 1; }
    __device__ int entries() const { return nchunks * NG * nacc; }  // of a stream: (group g, chunk q, block i of the run)
};

// Steps of entry e of stream w.  Stream order: group by group, inside a group chunk by chunk, inside a chunk the
// run's blocks.
__device__ inline int plan_entry_steps(const PlanShape &P, int w, int e) {
    const int eg = e / (P.nchunks * P.nacc), q = (e / P.nacc) % P.nchunks;
    const int64_t b = plan_block(eg, w, e % P.nacc, P.waves, P.nacc, P.paired != 0);
    // (chunked plans that give every run a step give one to the runs past the layer's last row-block too, so
    // that all streams of a group have the same shape; their step of zero weights is written by the scan)
    if (b >= P.B) return (P.chunked() && P.min_one) ? 1 : 0;
    // steps of a stored row-block (zero for an empty or malformed one: the same validity test as the count
    // and fill kernels make)
    auto stored_steps = [&](int64_t sb) {
        if (P.steps_bq) return P.steps_bq[sb * kPlanMaxChunks + q];
        const int base = P.blk_ptr[sb], kp = P.blk_ptr[sb + 1] - base, kb = P.blk_cnt[sb];
        const bool ok = kp > 0 && kp <= kMaxKp && kb >= 0 && kb <= kp && base >= 0 &&
                        (int64_t)base + kp <= P.capacity_cols;
        return ok && kb > 0 ? (kb + 31) >> 5 : 0;
    };
    // (virt: B counts blocks of 16 rows, each the union of the stored row-blocks 2 b and 2 b + 1: always counted;
    // split: the slabs of a stored row-block have its steps)
    int st = stored_steps(P.steps_bq ? b : b / P.split);
    // plans that give every run a step: an empty (or malformed) block gets a step of zero weights, so that
    // a wavefront's step loop never meets a block without steps
    if (P.min_one && st == 0) st = 1;
    return st;
}

// The step where entry `ee` of stream `ew` starts: the steps of all streams before it and of the entries before it in
// its own stream, added up by the whole workgroup (every thread must call; the plan's streams hold a few hundred
// entries in all).  The workgroups that fill the plan find their places this way instead of waiting for the table.
__device__ inline int plan_start(const PlanShape &P, int ew, int ee) {
    __shared__ int s_part[kThreads / 64];
    const int E = P.entries();
    int acc = 0;
    for (int idx = threadIdx.x; idx < ew * E + ee; idx += blockDim.x) acc += plan_entry_steps(P, idx / E, idx % E);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
    __syncthreads();  // (s_part may still be read from an earlier call)
    if ((threadIdx.x & 63) == 0) s_part[threadIdx.x >> 6] = acc;
    __syncthreads();
    int total = 0;
    for (int k = 0; k < (int)(blockDim.x >> 6); ++k) total += s_part[k];
    return total;
}

// The table of the streams, by one workgroup (its wavefronts take the streams in turn): wptr[w][e] = first step of
// entry e of stream w, wptr[w][E] = end of stream w; the zero steps of runs past the layer's end; valid offsets for
// the steps a layer kernel reads past the end of the last stream.
__device__ inline void plan_write_table(const PlanShape &P, int32_t nfrag, int64_t cap_steps, int32_t slack_steps,
                                        int32_t *__restrict__ wptr, uint32_t *__restrict__ wfrag,
                                        uint32_t *__restrict__ xoff) {
    __shared__ int totals[kPlanWavesWide];
    const int waves = P.waves, nw = blockDim.x >> 6;  // streams of the plan, wavefronts of this workgroup
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int E = P.entries();
    for (int w = wv; w < waves; w += nw) {
        int32_t *mine = wptr + (int64_t)w * (E + 1);
        int carry = 0;
        for (int ebase = 0; ebase < E; ebase += 64) {
            const int e = ebase + lane;
            const int st = e < E ? plan_entry_steps(P, w, e) : 0;
            int incl = st;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int up = __shfl_up(incl, o, 64);
                if (lane >= o) incl += up;
            }
            if (e < E) mine[e] = carry + incl - st;
            carry += __shfl(incl, 63, 64);
        }
        if (lane == 0) {
            mine[E] = carry;
            totals[w] = carry;
        }
    }
    __syncthreads();  // (the stores above are visible to the whole workgroup now)
    for (int w = wv; w < waves; w += nw) {
        int32_t *mine = wptr + (int64_t)w * (E + 1);
        int wbase = 0;
        for (int k = 0; k < w; ++k) wbase += totals[k];
        for (int e = lane; e <= E; e += 64) mine[e] += wbase;
        if (P.chunked() && P.min_one) {
            // (runs past the layer's end can only be in the last group: its entries close the stream)
            for (int e = max(0, E - P.nchunks * P.nacc); e < E; ++e) {  // uniform over the wavefront
                const int eg = e / (P.nchunks * P.nacc);
                if (plan_block(eg, w, e % P.nacc, waves, P.nacc, P.paired != 0) < P.B) continue;
                // where the entry starts: the stream's base and the steps of its entries before it (a handful)
                int64_t gs = wbase;
                for (int k = 0; k < e; ++k) gs += plan_entry_steps(P, w, k);
                if (gs < 0 || gs + 1 > cap_steps) continue;
                for (int f = 0; f < nfrag; ++f)
                    *reinterpret_cast<uint4 *>(wfrag + (gs * nfrag + f) * 256 + lane * 4) = make_uint4(0u, 0u, 0u, 0u);
                if (lane < 16) xoff[gs * 16 + lane] = 0u;
            }
        }
        // the layer kernel reads a few steps past the end of the last stream: give those steps the
        // LDS offset 0 (their values are never used, but the addresses must be valid)
        if (w == waves - 1) {
            const int64_t total = (int64_t)wbase + totals[w];
            if (total + slack_steps <= cap_steps)
                for (int i = lane; i < slack_steps * 16; i += 64) xoff[total * 16 + i] = 0u;
        }
    }
}

// One workgroup per (block of the plan, column chunk): order the chunk's kept columns and write its steps; one more
// workgroup behind them writes the table of the streams.  virt: the block is made of two stored row-blocks of 8 rows;
// its kept columns are the union of theirs, and a step's fragment holds the first one's weights in rows 0-7 and the
// second one's in rows 8-15 (zeros where only the other one keeps the column).  split > 1: the block is a 16-row slab
// of the stored row-block pb / split: that block's columns, the slab's rows of its panel.
__global__ __launch_bounds__(kThreads) void plan_fill_kernel(int32_t R, int32_t nfrag, int32_t NG, int32_t nacc,
                                                             int32_t chunk_shift,
                                                             int32_t nchunks, const int32_t *__restrict__ blk_cnt,
                                                             const int32_t *__restrict__ blk_ptr,
                                                             const int32_t *__restrict__ col_idx,
                                                             const uint16_t *__restrict__ vals, int64_t capacity_cols,
                                                             int64_t cap_steps, int32_t *__restrict__ wptr,
                                                             uint32_t *__restrict__ wfrag, uint32_t *__restrict__ xoff,
                                                             int32_t cols_cap, int32_t waves, int32_t paired,
                                                             int32_t min_one, int32_t virt, int32_t split, int32_t B,
                                                             const int32_t *__restrict__ steps_bq,
                                                             int32_t slack_steps) {
    // columns and canonical positions are below 4096 + 32: 16 bits each; 0xffff marks "none".  The lists of the
    // stored blocks' kept columns are sized by the launch for the layer's width (cols_cap entries each).
    extern __shared__ __attribute__((aligned(16))) uint16_t cols[];  // [1 or 2][cols_cap]
    __shared__ uint16_t slotcol[kMaxChunk], slotsrc[kMaxChunk], ovfcol[kMaxChunk], ovfsrc[kMaxChunk];
    // the chunk's kept columns (virt: the union, ascending): column inside the chunk, place in either block's panel
    __shared__ uint16_t ucol[kMaxChunk], usrc[2][kMaxChunk];
    __shared__ uint16_t mark[2][1024];  // virt: per column of the chunk its place in either block's panel
    __shared__ int s_filled[8], s_hp[9], s_novf, s_cnt[2][kPlanMaxChunks], s_wcnt[kThreads / 64];
    PlanShape P;
    P.steps_bq = steps_bq; P.blk_cnt = blk_cnt; P.blk_ptr = blk_ptr; P.capacity_cols = capacity_cols;
    P.B = B; P.NG = NG; P.nacc = nacc; P.nchunks = nchunks; P.paired = paired; P.min_one = min_one; P.virt = virt;
    P.split = split;
    P.waves = waves;
    if (blockIdx.x == gridDim.x - 1) {  // the workgroup behind the row-blocks writes the table of the streams
        if (blockIdx.y == 0) plan_write_table(P, nfrag, cap_steps, slack_steps, wptr, wfrag, xoff);
        return;
    }
    const int64_t pb = blockIdx.x;  // the plan's block
    const int q = blockIdx.y;
    const int nsrc = virt ? 2 : 1;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l16 = lane & 15, G = lane >> 4, qd = (lane >> 2) & 3, p = lane & 3;
    // the step where this (block, chunk) starts in its stream
    int64_t my_eg;
    int my_ew, my_ei;
    plan_entry(pb, waves, nacc, paired != 0, my_eg, my_ew, my_ei);
    const int64_t start = plan_start(P, my_ew, (int)((my_eg * nchunks + q) * nacc + my_ei));
    // the stored blocks (a malformed one counts as empty)
    int base[2] = {0, 0}, kp[2] = {0, 0}, kb[2] = {0, 0};
    bool ok[2] = {false, false};
    for (int j = 0; j < nsrc; ++j) {
        const int64_t sb = virt ? 2 * pb + j : pb / split;
        base[j] = blk_ptr[sb];
        kp[j] = blk_ptr[sb + 1] - base[j];
        kb[j] = blk_cnt[sb];
        ok[j] = kp[j] > 0 && kb[j] > 0 && kp[j] <= cols_cap && kb[j] <= kp[j] && base[j] >= 0 &&
                (int64_t)base[j] + kp[j] <= capacity_cols;
    }
    // the single step of an empty (block, chunk) of a plan that gives each of them one: zero weights, LDS offset 0
    auto zero_step = [&]() {
        if (!min_one || wave != 0) return;
        if (start >= 0 && start + 1 <= cap_steps) {
            for (int f = 0; f < nfrag; ++f)
                *reinterpret_cast<uint4 *>(wfrag + (start * nfrag + f) * 256 + lane * 4) = make_uint4(0u, 0u, 0u, 0u);
            if (lane < 16) xoff[start * 16 + lane] = 0u;
        }
    };
    if (!ok[0] && !ok[1]) {
        zero_step();
        return;
    }
    // the blocks' kept columns, fetched once with coalesced loads, and their counts per chunk
    if (threadIdx.x < 2 * kPlanMaxChunks) s_cnt[threadIdx.x / kPlanMaxChunks][threadIdx.x % kPlanMaxChunks] = 0;
    __syncthreads();
    for (int j = 0; j < nsrc; ++j) {
        if (!ok[j]) continue;
        for (int i = threadIdx.x; i < kb[j]; i += kThreads) {
            const int c = col_idx[base[j] + i];
            cols[j * cols_cap + i] = (uint16_t)c;
            const int cq = c >> chunk_shift;
            if (cq >= 0 && cq < nchunks) atomicAdd(&s_cnt[j][cq], 1);
        }
    }
    __syncthreads();
    const int col0 = q << chunk_shift;
    int lo[2] = {0, 0}, cqj[2] = {0, 0};  // canonical position of the chunk's first kept column (columns ascend, so
                                          // chunks are runs), and the run's length
    for (int j = 0; j < nsrc; ++j) {
        for (int k = 0; k < q; ++k) lo[j] += s_cnt[j][k];
        cqj[j] = ok[j] ? s_cnt[j][q] : 0;
        if (cqj[j] > 1024) cqj[j] = 0;  // (more than 1024: malformed storage, duplicate columns)
    }
    int cq = 0;  // kept columns of the plan's block inside the chunk
    if (!virt) {
        cq = cqj[0];
        for (int i = threadIdx.x; i < cq; i += kThreads) {
            ucol[i] = (uint16_t)((int)cols[lo[0] + i] - col0);
            usrc[0][i] = (uint16_t)(lo[0] + i);
        }
    } else {
        for (int i = threadIdx.x; i < 2 * 1024; i += kThreads) mark[i >> 10][i & 1023] = 0xffffu;
        __syncthreads();
        for (int j = 0; j < 2; ++j)
            for (int i = threadIdx.x; i < cqj[j]; i += kThreads) {
                const int c = (int)cols[j * cols_cap + lo[j] + i] - col0;
                if (c >= 0 && c < 1024) mark[j][c] = (uint16_t)(lo[j] + i);
            }
        __syncthreads();
        const uint64_t lt = (1ull << lane) - 1ull;
        for (int c0 = 0; c0 < 1024; c0 += kThreads) {  // the union in ascending order
            const int c = c0 + threadIdx.x;
            const uint16_t ma = mark[0][c], mb = mark[1][c];
            const bool present = ma != 0xffffu || mb != 0xffffu;
            const uint64_t m = __ballot(present);
            if (lane == 0) s_wcnt[wave] = __popcll(m);
            __syncthreads();
            int at = cq;
            for (int w = 0; w < wave; ++w) at += s_wcnt[w];
            if (present) {
                at += __popcll(m & lt);
                ucol[at] = (uint16_t)c;
                usrc[0][at] = ma;
                usrc[1][at] = mb;
            }
            for (int w = 0; w < kThreads / 64; ++w) cq += s_wcnt[w];
            __syncthreads();
        }
    }
    __syncthreads();
    if (cq <= 0) {  // uniform
        zero_step();
        return;
    }
    const int nsteps = (cq + 31) >> 5;
    const int S = nsteps * 4;  // sets of 8 columns
    if (wave == 0) {
        int cnt[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        int novf = 0;
        const uint64_t lt = (1ull << lane) - 1ull;
        for (int i0 = 0; i0 < cq; i0 += 64) {
            const int i = i0 + lane;
            const bool valid = i < cq;
            const int col = valid ? (int)ucol[i] : 0;  // column inside the chunk
            const int g = (int)lds_bank_group((uint32_t)col);
            int rank = 0;
#pragma unroll
            for (int gg = 0; gg < 8; ++gg) {
                const uint64_t m = __ballot(valid && g == gg);
                if (g == gg) rank = cnt[gg] + __popcll(m & lt);
                cnt[gg] += __popcll(m);
            }
            const bool over = valid && rank >= S;
            const uint64_t mo = __ballot(over);
            if (valid && !over) {
                const int slot = slot_index(rank, g);
                slotcol[slot] = (uint16_t)col;
                slotsrc[slot] = (uint16_t)i;
            } else if (over) {
                const int oi = novf + __popcll(mo & lt);
                ovfcol[oi] = (uint16_t)col;
                ovfsrc[oi] = (uint16_t)i;
            }
            novf += __popcll(mo);
        }
        if (lane == 0) {
            int run = 0;
            for (int g = 0; g < 8; ++g) {
                const int f = cnt[g] < S ? cnt[g] : S;
                s_filled[g] = f;
                s_hp[g] = run;
                run += S - f;
            }
            s_hp[8] = run;
            s_novf = novf;
        }
    }
    __syncthreads();
    // gaps: group g lacks a column in sets filled[g] .. S-1; gap e takes overflow column e, else a zero pad
    const int H = s_hp[8], novf = s_novf;
    for (int e = threadIdx.x; e < H; e += kThreads) {
        int g = 0;
#pragma unroll
        for (int gg = 1; gg < 8; ++gg)
            if (s_hp[gg] <= e) g = gg;
        const int set = s_filled[g] + (e - s_hp[g]);
        const int slot = slot_index(set, g);
        if (e < novf) {
            slotcol[slot] = ovfcol[e];
            slotsrc[slot] = ovfsrc[e];
        } else {
            slotcol[slot] = (uint16_t)(g << 2);  // any column of bank group g; its weight is zero
            slotsrc[slot] = 0xffffu;
        }
    }
    __syncthreads();
    // per-lane operands of the chunk's steps
    const int64_t gs0 = start;
    if (gs0 < 0 || gs0 + nsteps > cap_steps) return;
    for (int s = wave; s < nsteps; s += kThreads / 64) {
        const int s1 = 32 * s + 8 * G + qd;
        // (chunks of 512 columns alternate between the two halves of the tile)
        const uint32_t half = chunk_shift == 9 ? (uint32_t)(q & 1) * 512u : 0u;
        const uint32_t o1 = lds_col_offset4(half + (uint32_t)slotcol[s1], (uint32_t)p);
        const uint32_t o2 = lds_col_offset4(half + (uint32_t)slotcol[s1 + 4], (uint32_t)p);
        // offsets are multiples of 8 bytes; the 4 lanes of a column (token quads p = 0 .. 3) differ by
        // p in both halves (the swizzle is an exclusive-or on those bits), so p = 0 stands for all four
        if (p == 0) xoff[(gs0 + s) * 16 + (lane >> 2)] = (o1 >> 3) | ((o2 >> 3) << 16);
        for (int f = 0; f < nfrag; ++f) {
            // the fragment row's stored block and its row there
            const int fr = f * 16 + l16;
            // (split: the plan's block is the slab pb % split of its stored block)
            const int j = virt ? fr >> 3 : 0, r = virt ? fr & 7 : 16 * (int)(pb % split) + fr;
            uint32_t w[4] = {0u, 0u, 0u, 0u};
            if (r < R && j < nsrc && ok[j]) {
                const uint16_t *row = vals + (int64_t)R * base[j] + (int64_t)r * kp[j];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const uint32_t u = slotsrc[32 * s + 8 * G + i];
                    const uint32_t src = u != 0xffffu ? (uint32_t)usrc[j][u] : 0xffffu;
                    const uint32_t v = src != 0xffffu ? (uint32_t)row[src] : 0u;
                    w[i >> 1] |= v << (16 * (i & 1));
                }
            }
            *reinterpret_cast<uint4 *>(wfrag + ((gs0 + s) * nfrag + f) * 256 + lane * 4) = make_uint4(w[0], w[1], w[2], w[3]);
        }
    }
}

inline int nfrag_of(int32_t R) { return R <= 16 ? 1 : (R <= 32 ? 2 : 4); }

struct PlanLayout {
    int64_t NG;
    size_t steps, wptr_bytes, wfrag_bytes, xoff_bytes, cnt_bytes;
    size_t total() const { return wptr_bytes + wfrag_bytes + xoff_bytes + cnt_bytes; }
};
// Sized for the worst case of kPlanMaxChunks column chunks, so that the size does not depend on N:
// every (row-block, chunk) pads its columns to a multiple of 32 on its own.
// The buffer is sized for the finest grouping (nacc = 1) and the most chunks, so that its size does not
// depend on N; NG is the number of groups for the grouping the layer's width selects.
inline PlanLayout plan_layout(int64_t M, int64_t N, int32_t R, int64_t capacity_cols) {
    PlanLayout L;
    const int64_t B = M / R;  // stored row-blocks
    const int32_t Re = plan_block_rows(R, M);  // block height the plan is laid out for
    const int64_t Bp = M / Re;                 // blocks of the plan
    const int64_t Bm = B > Bp ? B : Bp;
    const int split = plan_split16(R);
    const bool chunked = plan_chunks(N, Re, M).n > 1;
    L.NG = plan_groups(Bp, plan_waves(N, Re, M), plan_nacc(nfrag_of(Re), chunked, Re), plan_paired(Re, chunked));
    // every (stored row-block, chunk) pads its columns to a multiple of 32 on its own and has a step even when it is
    // empty; the slabs of a split row-block repeat its steps
    // (+ a step per run of a last group that reaches past the layer, for the plans that give every run one)
    L.steps = (size_t)split * ((size_t)((capacity_cols + 31) / 32) + (size_t)B * kPlanMaxChunks) +
              (size_t)kPlanWaves * 4 * kPlanMaxChunks + (size_t)plan_slack_steps();
    // entries per stream <= chunks * (blocks rounded up to whole groups) / streams, groups of at most 32 blocks
    // (16 streams of a one-chunk layer need less than the 8 streams of a chunked one)
    L.wptr_bytes = ((size_t)kPlanWavesWide * (size_t)(kPlanMaxChunks * ((Bm + 31) / 32 * 4) + 1) * sizeof(int32_t) + 255) /
                   256 * 256;
    L.wfrag_bytes = L.steps * (size_t)nfrag_of(Re) * 1024;
    L.xoff_bytes = L.steps * 64;
    // step counts per (block of the plan, chunk) where a launch counts them: read by the workgroups that fill the plan
    L.cnt_bytes = ((size_t)Bm * kPlanMaxChunks * sizeof(int32_t) + 255) / 256 * 256;
    return L;
}

}  // namespace
}  // namespace bsp

using namespace bsp;

extern "C" int bsp_linear_plan_supported(int xdt, int64_t N, int32_t k_align) {
    return tiled_supported(xdt, N, k_align) ? 1 : 0;
}

extern "C" size_t bsp_linear_plan_bytes(int64_t M, int32_t R, int64_t capacity_cols) {
    if (R < 1 || R > 64 || M <= 0 || M % R != 0 || capacity_cols < 0) return 0;
    return plan_layout(M, 1, R, capacity_cols).total();
}

extern "C" int bsp_linear_plan(int vdt, int64_t M, int64_t N, int32_t R, int32_t k_align, const int32_t *blk_cnt,
                               const int32_t *blk_ptr, const int32_t *col_idx, const void *vals,
                               int64_t capacity_cols, void *plan, size_t plan_bytes, void *stream) {
    if (!blk_cnt || !blk_ptr || !plan) return BSP_ERR_NULL;
    if (M <= 0 || N <= 0 || R < 1 || R > 64 || M % R != 0 || M / R > 65535) return BSP_ERR_SHAPE;
    if (!tiled_supported(vdt, N, k_align)) return BSP_ERR_SHAPE;
    if (capacity_cols < 0) return BSP_ERR_CAPACITY;
    if (capacity_cols > 0 && (!col_idx || !vals)) return BSP_ERR_NULL;
    const PlanLayout L = plan_layout(M, N, R, capacity_cols);
    if (plan_bytes < L.total() || !aligned(plan, 16)) return BSP_ERR_CAPACITY;
    const bool virt = plan_virtual16(R, M);
    const int split = plan_split16(R);
    const int32_t Re = plan_block_rows(R, M);  // block height of the plan
    const int64_t B = M / Re;           // the plan's row-blocks
    const int nf = nfrag_of(Re);
    int32_t *wptr = (int32_t *)plan;
    uint32_t *wfrag = (uint32_t *)((uint8_t *)plan + L.wptr_bytes);
    uint32_t *xoff = (uint32_t *)((uint8_t *)plan + L.wptr_bytes + L.wfrag_bytes);
    hipStream_t s = (hipStream_t)stream;
    const PlanChunks ch = plan_chunks(N, Re, M);
    const int32_t min_one = plan_min_one_step(Re, ch.n > 1) ? 1 : 0;
    const int32_t paired = plan_paired(Re, ch.n > 1) ? 1 : 0;
    int32_t *steps_bq = (int32_t *)((uint8_t *)plan + L.wptr_bytes + L.wfrag_bytes + L.xoff_bytes);
    // a layer of one chunk needs no count (its steps per row-block follow from blk_cnt) unless its blocks are unions
    const bool counted = ch.n > 1 || virt;
    if (counted)
        plan_count_kernel<<<(unsigned)B, kThreads, 0, s>>>(blk_cnt, blk_ptr, col_idx, capacity_cols, ch.shift, ch.n,
                                                           virt ? 1 : 0, split, steps_bq);
    const int32_t nacc = plan_nacc(nf, ch.n > 1, Re);
    const int waves = plan_waves(N, Re, M);
    // One launch fills the plan: a workgroup per (block of the plan, chunk), each finding its place in its stream by
    // adding up the step counts before it, and one more that writes the table of the streams.
    // a row-block keeps at most N columns, padded to the alignment (at most 64)
    const int32_t cols_cap = (int32_t)(N + 64 < kMaxKp ? (N + 64 + 7) / 8 * 8 : kMaxKp);
    plan_fill_kernel<<<dim3((unsigned)B + 1, (unsigned)ch.n), kThreads, (size_t)cols_cap * 2 * (virt ? 2 : 1), s>>>(
        R, nf, (int32_t)L.NG, nacc, ch.shift, ch.n, blk_cnt, blk_ptr, col_idx, (const uint16_t *)vals, capacity_cols,
        (int64_t)L.steps, wptr, wfrag, xoff, cols_cap, waves, paired, min_one, virt ? 1 : 0, split, (int32_t)B,
        counted ? steps_bq : nullptr, plan_slack_steps());
    return check_launch();
}

extern "C" int bsp_linear_planned(const void *X, int xdt, int64_t T, int64_t M, int64_t N, int32_t R, int32_t k_align,
                                  const void *plan, int64_t capacity_cols, const void *bias, void *Y, void *stream) {
    return bsp_linear_planned_fused(X, xdt, T, M, N, R, k_align, plan, capacity_cols, bias, BSP_ACT_NONE, nullptr, Y,
                                    stream);
}

extern "C" int bsp_linear_planned_fused(const void *X, int xdt, int64_t T, int64_t M, int64_t N, int32_t R,
                                        int32_t k_align, const void *plan, int64_t capacity_cols, const void *bias,
                                        int act, const void *residual, void *Y, void *stream) {
    if (!X || !plan || !Y) return BSP_ERR_NULL;
    if (act != BSP_ACT_NONE && act != BSP_ACT_GELU) return BSP_ERR_SHAPE;
    if (residual && !aligned(residual, 8)) return BSP_ERR_SHAPE;
    if (T < 0 || M <= 0 || N <= 0 || R < 1 || R > 64 || M % R != 0 || M / R > 65535) return BSP_ERR_SHAPE;
    if (!tiled_supported(xdt, N, k_align)) return BSP_ERR_SHAPE;
    if (capacity_cols < 0) return BSP_ERR_CAPACITY;
    if (!aligned(X, 16) || !aligned(Y, 16) || !aligned(plan, 16)) return BSP_ERR_SHAPE;
    if (T == 0) return BSP_OK;
    const PlanLayout L = plan_layout(M, N, R, capacity_cols);
    TiledArgs a{};
    a.xdt = xdt;
    a.X = (const uint16_t *)X;
    // (pairs of 8-row blocks, slabs of 32-, 48- and 64-row blocks: the plan is the one of blocks of 16 rows)
    const int32_t Re = plan_block_rows(R, M);
    a.T = T; a.M = M; a.N = N; a.B = M / Re; a.R = Re;
    a.wptr = (const int32_t *)plan;
    a.wfrag = (const uint8_t *)plan + L.wptr_bytes;
    a.xoff = (const uint32_t *)((const uint8_t *)plan + L.wptr_bytes + L.wfrag_bytes);
    a.plan_steps = (int64_t)L.steps;
    a.capacity_cols = capacity_cols;
    a.bias = bias;
    a.Y = Y;
    a.act = act;
    a.residual = residual;
    if (act != BSP_ACT_NONE || residual) {
        // fused by the two kernels of 16-row blocks only; the residual by the one that writes its output at its end
        if (Re != 16) return BSP_ERR_SHAPE;
        if (residual && plan_chunks(N, Re, M).n <= 1) return BSP_ERR_SHAPE;
    }
    return launch_linear_tiled(a, true, (hipStream_t)stream);
}
