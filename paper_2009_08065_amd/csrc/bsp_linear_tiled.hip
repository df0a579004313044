// Tiled matrix-core kernels of the block-structure-pruned linear layer (Sec. 3.1, Sec. 4.4)
// for bf16 / fp16 on gfx950.
//
// A workgroup owns a tile of 16*NSUB tokens and a strip of row-blocks.  It copies its X tile
// from HBM into LDS once, with full-row coalesced loads, transposed to [column][16 tokens] so
// that the 16 tokens of one X column are 32 contiguous bytes.  Every wavefront then takes a
// contiguous run of the strip's row-blocks holding an equal share of the strip's kept columns
// (uneven kept counts balance).  It walks its kept columns 32 at a time ("step"): the value
// panel fragment (16 rows x 32 kept columns) comes straight from global memory / L2 and is
// reused for all NSUB token sub-tiles; the matching X fragment (32 kept columns x 16 tokens)
// is gathered out of LDS by two transposing reads (ds_read_b64_tr_b16), in which every lane
// supplies the address of its own column, so the per-row-block gather costs no extra
// instructions.  One v_mfma_f32_16x16x32 per (32 kept columns, 16 tokens, 16 rows).
//
// LDS placement of column c of a sub-tile (swizzled so that the transposing 8-byte stores of
// the copy-in are bank-conflict free): see lds_col_offset().
//
// Two kernels, one per source of the per-step operands:
//   canonical  the compact storage itself (col_idx / vals);
//   planned    a derived buffer built by bsp_linear_plan, where the kept columns of a row-block
//              are re-ordered so that the 8 columns one half-wavefront reads in one LDS
//              instruction fall into 8 different bank groups, and where the panel fragment
//              and the two LDS offsets of every lane are stored ready to load.  Its inner loop
//              is written to keep vector-ALU work per step minimal (on CDNA a 64-lane VALU
//              instruction occupies the SIMD for 4 cycles, a 16x16x32 MFMA for 16): operand
//              addresses advance by constants, operands of the next kRing steps are in flight,
//              and the LDS reads of step s+1 are issued before the MFMAs of step s.
#include "bsp_common.h"
#include "bsp_linear_internal.h"
#include "bsp_mfma_device.h"
#include "bsp_tile_device.h"

namespace bsp {
namespace {

constexpr int kMaxStripBlocks = 1024;  // row-blocks per strip (their blk_ptr slice is cached in LDS)
constexpr int kRing = 4;               // steps of operands in flight per wavefront, canonical kernel
constexpr int kPlanRing = 8;           // the same for the planned kernels with 8 wavefronts, divided by the fragments per
                                       // step (with 16 wavefronts: 2 steps).  Deeper rings were measured slower (4 to 8
                                       // steps are equal, 16 is 10 % slower): latency is covered, and more requests in
                                       // flight only queue up

// This wavefront's share of the strip: a contiguous run [b_lo, b_hi) of row-blocks holding about
// 1 / nwaves of the strip's padded kept columns (lower bounds on the cached blk_ptr slice).
__device__ __forceinline__ void wave_share(const int *s_ptr, int nrb, int wave, int nwaves, int &b_lo, int &b_hi) {
    auto first_block_at = [&](int64_t target_cols) {
        int lo = 0, hi = nrb;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (s_ptr[mid] < target_cols) lo = mid + 1; else hi = mid;
        }
        return lo;
    };
    const int64_t c_begin = s_ptr[0], c_total = (int64_t)s_ptr[nrb] - s_ptr[0];
    b_lo = wave == 0 ? 0 : first_block_at(c_begin + c_total * wave / nwaves);
    b_hi = wave == nwaves - 1 ? nrb : first_block_at(c_begin + c_total * (wave + 1) / nwaves);
    b_lo = __builtin_amdgcn_readfirstlane(b_lo);
    b_hi = __builtin_amdgcn_readfirstlane(b_hi);
}

// Per-lane output state of a wavefront: where its accumulators go and the bias of the
// current row-block.  acc[f][u][v] = Y[t0 + 16u + l16, bR + 16f + 4G + v] before the bias.
template <int DT, int NFRAG, int NSUB>
struct Epilogue {
    uint16_t *yrow[NSUB];  // Y + token row of sub-tile u + 4G
    uint32_t tok_ok;       // bit u: the lane's token of sub-tile u is inside T
    const void *bias;
    int64_t M;
    int32_t R, G;
    bool vec4;             // 4 consecutive outputs can go out as one 8-byte store
    float bv[NFRAG][4];

    __device__ __forceinline__ void init(void *Y, const void *bias_, int64_t T, int64_t M_, int32_t R_, int64_t t0,
                                         int l16, int G_) {
        bias = bias_; M = M_; R = R_; G = G_;
        vec4 = (R & 3) == 0 && (M & 3) == 0 && (reinterpret_cast<uintptr_t>(bias) & 7) == 0;
        tok_ok = 0;
#pragma unroll
        for (int u = 0; u < NSUB; ++u) {
            const int64_t t = t0 + 16 * u + l16;
            if (t < T) tok_ok |= 1u << u;
            yrow[u] = (uint16_t *)Y + (t < T ? t : 0) * M + 4 * G;
        }
#pragma unroll
        for (int f = 0; f < NFRAG; ++f)
#pragma unroll
            for (int v = 0; v < 4; ++v) bv[f][v] = 0.0f;
    }
    // Issued when a row-block starts and used when it ends; unconditional loads on clamped rows,
    // so nothing waits on them before the use.
    __device__ __forceinline__ void load_bias(int64_t b) {
        if (!bias) return;
#pragma unroll
        for (int f = 0; f < NFRAG; ++f) {
            const int r0 = f * 16 + 4 * G;
            if (vec4) {
                const int rr = r0 < R ? r0 : 0;
                const uint2 w = *reinterpret_cast<const uint2 *>((const uint16_t *)bias + b * R + rr);
                const uint32_t h[4] = {w.x & 0xffffu, w.x >> 16, w.y & 0xffffu, w.y >> 16};
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    if constexpr (DT == BSP_BF16) bv[f][v] = __uint_as_float(h[v] << 16);
                    else bv[f][v] = (float)__builtin_bit_cast(_Float16, (uint16_t)h[v]);
                }
            } else {
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int rr = r0 + v < R ? r0 + v : R - 1;
                    bv[f][v] = elem<DT>::load(bias, b * R + rr);
                }
            }
        }
    }
    __device__ __forceinline__ void write_block(int64_t b, const f32x4 (&acc)[NFRAG][NSUB]) {
#pragma unroll
        for (int f = 0; f < NFRAG; ++f) {
            const int r0 = f * 16 + 4 * G;
            if (r0 >= R) continue;
            const int64_t mcol = b * R + f * 16;  // + 4G is already in yrow
#pragma unroll
            for (int u = 0; u < NSUB; ++u) {
                if (!((tok_ok >> u) & 1u)) continue;
                if (vec4) {
                    uint2 o;
                    o.x = cvt_pk<DT>(acc[f][u][0] + bv[f][0], acc[f][u][1] + bv[f][1]);
                    o.y = cvt_pk<DT>(acc[f][u][2] + bv[f][2], acc[f][u][3] + bv[f][3]);
                    *reinterpret_cast<uint2 *>(yrow[u] + mcol) = o;
                } else {
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        if (r0 + v < R) elem<DT>::store(yrow[u], mcol + v, acc[f][u][v] + bv[f][v]);
                }
            }
        }
    }
};

template <int NFRAG, int NSUB>
__device__ __forceinline__ void clear_acc(f32x4 (&acc)[NFRAG][NSUB]) {
#pragma unroll
    for (int f = 0; f < NFRAG; ++f)
#pragma unroll
        for (int u = 0; u < NSUB; ++u) acc[f][u] = f32x4{0.f, 0.f, 0.f, 0.f};
}

// ---------------------------------------------------------------------------------------------
// canonical operands
// ---------------------------------------------------------------------------------------------
template <int NFRAG>
struct StepOps {       // one lane's operands of one step, as loaded (nothing is derived from the
    uint4 a[NFRAG];    // loaded words at fetch time: a use would stall the stream on the load)
    uint32_t c1, c2;   // the lane's two columns
};

template <int DT, int NFRAG, int NSUB>
__global__ __launch_bounds__(1024) void linear_tiled_canonical_kernel(
    const uint16_t *__restrict__ X, int64_t T, int64_t M, int64_t N, int32_t R, int32_t npad,
    const int32_t *__restrict__ blk_ptr, const int32_t *__restrict__ col_idx, const uint16_t *__restrict__ vals,
    const void *__restrict__ bias, void *__restrict__ Y, int32_t ntiles, int32_t rb_per_strip, int32_t B) {
    __shared__ int s_ptr[kMaxStripBlocks + 1];
    const int tile = blockIdx.x % ntiles, strip = blockIdx.x / ntiles;
    const int64_t t0 = (int64_t)tile * (16 * NSUB);
    const int rb0 = strip * rb_per_strip;
    const int nrb = min(rb_per_strip, B - rb0);
    for (int i = threadIdx.x; i <= nrb; i += blockDim.x) s_ptr[i] = blk_ptr[rb0 + i];
    stage_x_tile<NSUB>(X, T, N, npad, t0);
    __syncthreads();

    const int lane = threadIdx.x & 63;
    const int l16 = lane & 15, G = lane >> 4, q = (lane >> 2) & 3, p = lane & 3;
    int b_lo, b_hi;
    wave_share(s_ptr, nrb, __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)), blockDim.x >> 6, b_lo, b_hi);
    if (b_lo >= b_hi) return;
    const int gs_lo = s_ptr[b_lo] >> 5, gs_hi = s_ptr[b_hi] >> 5;

    // cursor of the operand stream (which row-block the next fetched step belongs to)
    int f_blk = b_lo, f_base = s_ptr[b_lo], f_end = s_ptr[b_lo + 1];
    auto fetch = [&](int gs, StepOps<NFRAG> &o) {
        while ((gs << 5) >= f_end && f_blk + 1 < nrb) {
            ++f_blk;
            f_base = f_end;
            f_end = s_ptr[f_blk + 1];
        }
        const int kp = f_end - f_base, cpos = (gs << 5) - f_base;
#pragma unroll
        for (int f = 0; f < NFRAG; ++f) {
            const int r = f * 16 + l16;
            o.a[f] = (r < R) ? *reinterpret_cast<const uint4 *>(vals + (int64_t)R * f_base + (int64_t)r * kp + cpos + 8 * G)
                             : make_uint4(0u, 0u, 0u, 0u);
        }
        o.c1 = (uint32_t)col_idx[f_base + cpos + 8 * G + q];
        o.c2 = (uint32_t)col_idx[f_base + cpos + 8 * G + 4 + q];
    };

    Epilogue<DT, NFRAG, NSUB> ep;
    ep.init(Y, bias, T, M, R, t0, l16, G);
    f32x4 acc[NFRAG][NSUB];
    clear_acc(acc);
    ep.load_bias(rb0 + b_lo);
    int blk = b_lo;
    int blk_end = s_ptr[blk + 1] >> 5;  // first step index past the current row-block
    int gs = gs_lo;
    // finished (possibly empty) row-blocks are written as soon as the stream has passed them
    auto pass_boundaries = [&]() {
        while (blk < b_hi && blk_end <= gs) {
            ep.write_block(rb0 + blk, acc);
            clear_acc(acc);
            ++blk;
            blk_end = blk < b_hi ? (s_ptr[blk + 1] >> 5) : -1;
            if (blk < b_hi) ep.load_bias(rb0 + blk);
        }
    };
    pass_boundaries();

    StepOps<NFRAG> ring[kRing];
#pragma unroll
    for (int j = 0; j < kRing; ++j)
        if (gs + j < gs_hi) fetch(gs + j, ring[j]);
    while (gs < gs_hi) {
#pragma unroll
        for (int j = 0; j < kRing; ++j) {
            if (gs < gs_hi) {
                const StepOps<NFRAG> cur = ring[j];
                if (gs + kRing < gs_hi) fetch(gs + kRing, ring[j]);
                const uint32_t o1 = tile_col_offset<NSUB>(cur.c1, (uint32_t)p), o2 = tile_col_offset<NSUB>(cur.c2, (uint32_t)p);
                uint4 xb[NSUB];
#pragma unroll
                for (int u = 0; u < NSUB; ++u) {
                    const uint2 lo = tr_read(smem_x + u * sub_stride<NSUB>(), o1);
                    const uint2 hi = tr_read(smem_x + u * sub_stride<NSUB>(), o2);
                    xb[u] = make_uint4(lo.x, lo.y, hi.x, hi.y);
                }
#pragma unroll
                for (int u = 0; u < NSUB; ++u)
#pragma unroll
                    for (int f = 0; f < NFRAG; ++f) acc[f][u] = mfma16<DT>(cur.a[f], xb[u], acc[f][u]);
                ++gs;
                pass_boundaries();
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// planned operands
// ---------------------------------------------------------------------------------------------
// A wavefront owns NACC consecutive row-blocks at a time (a run: 64 or 128 bytes of consecutive output
// columns, see plan_nacc) and, in the column-chunked kernel, keeps all their accumulators, so that it can
// write whole lines of Y: group g of a layer = `waves` runs = blocks [g * waves * NACC, (g + 1) * waves * NACC),
// run w of the group belongs to wavefront w (waves = 8 or 16, see plan_waves).  The plan stores the steps in
// exactly the order a wavefront walks them (its run of group 0 block by block, then group 1, ...; chunk-major
// for layers cut into column chunks), so a wavefront streams its operands with constant address increments.
// wptr[w][(g * chunks + q) * NACC + i] = first step of block (g * waves + w) * NACC + i inside chunk q.

constexpr int kOutPitch = 144;  // bytes per token row of a wavefront's output staging (128 + pad)

// Output of one quad.  The accumulators hold, per lane, 4 consecutive output columns of one token
// (the MFMA result layout); written as they are, a store instruction would touch 16 token rows with
// 32 bytes each.  They go through a small per-wavefront LDS buffer instead, so that 8 lanes write one
// whole 128-byte line of a token row.
template <int DT, int NFRAG, int NSUB, int NACC>
struct QuadEpilogue {
    uint16_t *Y;
    const void *bias;
    int64_t T, M, t0;
    int32_t R, B, l16, G, lane;
    bool fast;       // R == 16 * NFRAG or R == 8: a quad is NACC * R contiguous output columns, a multiple of 64 bytes
    uint8_t *stage;  // this wavefront's LDS staging, 16 rows of kOutPitch bytes
    uint2 bv[NACC][NFRAG];  // bias of the lane's 4 output columns per (block, fragment), as stored (16-bit floats)

    __device__ __forceinline__ void init(void *Y_, const void *bias_, int64_t T_, int64_t M_, int32_t R_, int32_t B_,
                                         int64_t t0_, int lane_, uint8_t *stage_, bool fast_) {
        Y = (uint16_t *)Y_; bias = bias_; T = T_; M = M_; R = R_; B = B_; t0 = t0_;
        lane = lane_; l16 = lane_ & 15; G = lane_ >> 4; stage = stage_; fast = fast_;
#pragma unroll
        for (int k = 0; k < NACC; ++k)
#pragma unroll
            for (int f = 0; f < NFRAG; ++f) bv[k][f] = make_uint2(0u, 0u);  // +0 in both formats
    }
    // Bias of the quad whose first row-block is b0; issued early, used by convert().  Unconditional loads
    // on clamped addresses, so nothing waits on them before the use.
    __device__ __forceinline__ void load_bias(int64_t b0) {
        if (!bias) return;
#pragma unroll
        for (int k = 0; k < NACC; ++k) {
            const int64_t b = b0 + k < B ? b0 + k : B - 1;
#pragma unroll
            for (int f = 0; f < NFRAG; ++f) {
                const int r0 = f * 16 + 4 * G;
                if (fast) {
                    // (R = 8: the lanes of the unused upper half of the fragment read the lower half's bias)
                    bv[k][f] = *reinterpret_cast<const uint2 *>((const uint16_t *)bias + b * R + (r0 < R ? r0 : r0 - 8));
                } else {
                    uint32_t h[4];
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int rr = r0 + v < R ? r0 + v : R - 1;
                        h[v] = ((const uint16_t *)bias)[b * R + rr];
                    }
                    bv[k][f] = make_uint2(h[0] | (h[1] << 16), h[2] | (h[3] << 16));
                }
            }
        }
    }
    __device__ __forceinline__ static float widen(uint32_t h) {
        if constexpr (DT == BSP_BF16) return __uint_as_float(h << 16);
        else return (float)__builtin_bit_cast(_Float16, (uint16_t)h);
    }
    // Bias added, rounded to the output type: the form in which a finished quad waits for its store.
    typedef uint2 Packed[NACC][NFRAG][NSUB];
    __device__ __forceinline__ void convert(const f32x4 (&acc)[NACC][NFRAG][NSUB], Packed &out) const {
#pragma unroll
        for (int k = 0; k < NACC; ++k)
#pragma unroll
            for (int f = 0; f < NFRAG; ++f)
#pragma unroll
                for (int u = 0; u < NSUB; ++u) {
                    const float b0 = widen(bv[k][f].x & 0xffffu), b1 = widen(bv[k][f].x >> 16);
                    const float b2 = widen(bv[k][f].y & 0xffffu), b3 = widen(bv[k][f].y >> 16);
                    out[k][f][u].x = cvt_pk<DT>(acc[k][f][u][0] + b0, acc[k][f][u][1] + b1);
                    out[k][f][u].y = cvt_pk<DT>(acc[k][f][u][2] + b2, acc[k][f][u][3] + b3);
                }
    }
    // Store the quad whose first row-block is b0.  out[k][f][u] = 4 consecutive output columns
    // (16 f + 4 G ..) of block b0 + k for token 16 u + l16 of the tile.
    __device__ __forceinline__ void flush(int64_t b0, const Packed &out) {
        if (b0 >= B) return;  // uniform
        if (fast) {
            // a token row of the quad is 64 or 128 contiguous bytes (32 per fragment, 16 when R = 8 leaves the
            // upper half of the fragment unused): lpr lanes x 16 bytes write one row
            const int bpf = NFRAG == 1 ? 2 * R : 32;
            const int lpr = NACC * NFRAG * bpf / 16, rpi = 64 / lpr;  // lanes per row, rows per store instruction
            const int row = lane / lpr, piece = lane % lpr;
            // the 16-byte piece covers 8 output columns, all inside one row-block
            const bool blk_ok = b0 + (piece * 8) / R < B;
            uint16_t *dst = Y + b0 * R + piece * 8;
#pragma unroll
            for (int u = 0; u < NSUB; ++u) {
                if (8 * G < bpf) {
#pragma unroll
                    for (int k = 0; k < NACC; ++k)
#pragma unroll
                        for (int f = 0; f < NFRAG; ++f)
                            *reinterpret_cast<uint2 *>(stage + l16 * kOutPitch + (k * NFRAG + f) * bpf + 8 * G) = out[k][f][u];
                }
                // same wavefront writes and reads: LDS operations of a wavefront complete in order
                for (int i = 0; i < 16 / rpi; ++i) {
                    const uint4 o = *reinterpret_cast<const uint4 *>(stage + (row + rpi * i) * kOutPitch + piece * 16);
                    const int64_t t = t0 + 16 * u + rpi * i + row;
                    if (t < T && blk_ok) store_y16(dst + t * M, o);
                }
            }
        } else {
#pragma unroll
            for (int k = 0; k < NACC; ++k) {
                if (b0 + k >= B) continue;
#pragma unroll
                for (int f = 0; f < NFRAG; ++f) {
                    const int r0 = f * 16 + 4 * G;
#pragma unroll
                    for (int u = 0; u < NSUB; ++u) {
                        const int64_t t = t0 + 16 * u + l16;
                        if (t >= T) continue;
                        const uint32_t h[4] = {out[k][f][u].x & 0xffffu, out[k][f][u].x >> 16, out[k][f][u].y & 0xffffu,
                                               out[k][f][u].y >> 16};
#pragma unroll
                        for (int v = 0; v < 4; ++v)
                            if (r0 + v < R) Y[t * M + (b0 + k) * R + r0 + v] = (uint16_t)h[v];
                    }
                }
            }
        }
    }
};

// The MFMAs of one step go to the accumulators of the row-block the step belongs to; `which` is
// uniform over the wavefront, so this is a scalar branch.
template <int DT, int NFRAG, int NSUB, int NACC>
__device__ __forceinline__ void step_mfma(f32x4 (&acc)[NACC][NFRAG][NSUB], int which, const uint4 (&a)[NFRAG],
                                          const uint4 (&xb)[NSUB]) {
    auto into = [&](f32x4 (&c)[NFRAG][NSUB]) {
#pragma unroll
        for (int u = 0; u < NSUB; ++u)
#pragma unroll
            for (int f = 0; f < NFRAG; ++f) c[f][u] = mfma16<DT>(a[f], xb[u], c[f][u]);
    };
    if constexpr (NACC == 1) {
        into(acc[0]);
    } else if constexpr (NACC == 2) {
        if (which == 0) into(acc[0]); else into(acc[1]);
    } else {
        static_assert(NACC == 4, "accumulator sets per wavefront");
        if (which < 2) {
            if (which == 0) into(acc[0]); else into(acc[1]);
        } else {
            if (which == 2) into(acc[2]); else into(acc[3]);
        }
    }
}

template <int NACC, int NFRAG, int NSUB>
__device__ __forceinline__ void clear_quad(f32x4 (&acc)[NACC][NFRAG][NSUB]) {
#pragma unroll
    for (int k = 0; k < NACC; ++k) clear_acc(acc[k]);
}

// Layers of up to 1024 input columns: the whole 64-token X tile stays in LDS while the workgroup
// walks the groups of its strip.
//
// Output path.  The MFMA result layout gives a lane 4 consecutive output columns of one token, so a
// store straight from the accumulators touches 16 token rows with 32 bytes each.  OUT says how the output
// leaves instead.  A template parameter, because the output code is inlined at every slot of the unrolled
// operand ring: it has to be small, and its constants known.
// kOutSwap (R == 16 * NFRAG): a pair of finished 16-row fragments (two row-blocks for R = 16, the two halves of
// one for R = 32) is rounded to 8 bytes per lane each and re-dealt among the four 16-lane rows of the wavefront
// with two lane-swap instructions per dword, after which every lane holds 16 contiguous bytes of a token's
// 64-byte run and the wavefront stores 16 token rows x 64 bytes per instruction.  The bias of the strip's rows
// waits in LDS as fp32 (behind the X tile) and is what an accumulator starts from.
// kOutStaged8 (R == 8, NFRAG = 1, half fragments of 16 bytes, runs of 4 row-blocks): a finished fragment is
// rounded (bias added) and parked in a per-wavefront LDS buffer of 64 token rows x 64 bytes; once the buffer holds
// 32 consecutive output columns of all 64 tokens it is written with 16-byte lanes, 64 contiguous bytes per token
// row.  The LDS operations of a wavefront complete in order, so the buffer needs no barrier.  (In the read,
// row = 16 i + lane / 4, so row / 4 % 4 is the lane's G.)
// kOutElements: any other R (or an output that cannot be written in 16-byte pieces), outputs stored one by one,
// and kOutElements8 the same for R == 8, whose plan deals the row-blocks in runs of 4.
constexpr int kLeanGroup = 3;                // steps per operand group of the 16-wavefront kernels
constexpr uint32_t kOutStageBytes = 4096;    // per wavefront: 64 token rows x 64 bytes
enum { kOutElements = 0, kOutStaged8 = 2, kOutElements8 = 3, kOutSwap = 4 };
constexpr uint32_t kBiasTableBytes = 32768;  // at most: 8192 rows of a strip
template <int DT, int NFRAG, int OUT, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void linear_tiled_planned_kernel(
    const uint16_t *__restrict__ X, int64_t T, int64_t M, int64_t N, int32_t R, int32_t npad,
    const int32_t *__restrict__ wptr, const uint32_t *__restrict__ wfrag, const uint32_t *__restrict__ xoff,
    const void *__restrict__ bias, void *__restrict__ Y, int32_t ntiles, int32_t groups_per_strip, int32_t NG,
    int32_t B, int32_t max_step) {
    constexpr int NSUB = 4;
    constexpr bool FAST = OUT == kOutStaged8;
    constexpr bool SWAP = OUT == kOutSwap;
    // row-blocks of a wavefront's run: together 64 bytes per token row
    constexpr int NACC = plan_nacc(NFRAG, false, (OUT == kOutStaged8 || OUT == kOutElements8) ? 8 : 0);
    constexpr int nacc_shift = NACC == 4 ? 2 : (NACC == 2 ? 1 : 0);
    // 8 wavefronts: the same bytes in flight for every fragment count, and the X fragments of the next step are read
    // from LDS while this step's MFMAs run (two register sets).  16 wavefronts: a ring of 2 steps and one register
    // set -- four wavefronts per SIMD cover for each other (measured as fast as a 4-step ring with two sets), and
    // the kernel then needs under 96 registers, which leaves a quarter of the register file to other kernels.
    constexpr bool LEAN = WAVES == kPlanWavesWide;
    // 16 wavefronts: the operands travel in two groups of kLeanGroup steps.  A group is requested as a whole, right
    // after the wavefront has made sure that the other group has arrived, and used one group of products later: the
    // only wait for operands is then one with nothing else in flight, the form the compiler's conservative wait
    // insertion (a wait for all loads at every loop head) costs nothing in.  With a slot refilled right behind its
    // products, as before, every step waited for the loads of the step before it: one L2 round trip per step.
    constexpr int RING = LEAN ? 2 * kLeanGroup : kPlanRing / NFRAG;
    static_assert(RING % 2 == 0, "the X fragment ping-pong needs an even ring");
    const int tile = blockIdx.x % ntiles, strip = blockIdx.x / ntiles;
    const int64_t t0 = (int64_t)tile * (16 * NSUB);
    const int g0 = strip * groups_per_strip;
    const int ng = min(groups_per_strip, NG - g0);
    // The X tile is copied in by the first use (below): a wavefront first requests the operands of its
    // first RING steps, so that they travel while the tile is copied.  Every wavefront passes the barrier once.
    bool staged = false;
    // kOutSwap: the bias of the strip's rows as fp32, behind the X tile (zeros without a bias and past row M)
    float *btab = reinterpret_cast<float *>(smem_x + kXTileBytes);
    const int64_t strip_row0 = (int64_t)g0 * (WAVES * NACC) * R;
    auto stage_once = [&]() {
        if (staged) return;
        stage_x_tile<NSUB>(X, T, N, npad, t0);
        if constexpr (SWAP) {
            const int rows = ng * (WAVES * NACC) * R;
            for (int i = threadIdx.x; i < rows; i += WAVES * 64) {
                const int64_t r = strip_row0 + i;
                btab[i] = (bias && r < M) ? elem<DT>::load(bias, r) : 0.0f;
            }
        }
        __syncthreads();
        staged = true;
    };

    const int lane = threadIdx.x & 63;
    const int l16 = lane & 15, G = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    // this wavefront's row of step pointers, from the strip's first entry on (uniform: scalar loads)
    const int32_t *my = wptr + (int64_t)wave * ((int64_t)NG * NACC + 1) + (int64_t)g0 * NACC;
    uint8_t *stg = smem_x + kXTileBytes + wave * kOutStageBytes;
    // 16-byte pieces of a staging row are stored at piece ^ (row / 4 % 4): with a pitch of 64 bytes both the
    // 8-byte writes (16 token rows per half-wavefront) and the 16-byte reads (4 rows per 16 lanes) then
    // spread over all LDS banks; unswizzled, the writes are a 4-way bank conflict
    const int swz = (l16 >> 2) & 3;
    uint16_t *Yh = (uint16_t *)Y;

    f32x4 acc[NFRAG][NSUB];
    uint32_t bs[NFRAG][8];  // bias of the current block as stored, 16 values per fragment (uniform)
    // kOutSwap: the rounded fragment of the even row-block of a pair (R = 16) until the odd one is finished; the
    // bias the next accumulator starts from (read one row-block ahead); the lane's place in a token's 64-byte
    // run after the swap (row G of the wavefront takes bytes 16 G .. 16 G + 15), relative to the sub-tile's first row
    uint2 hold[NSUB];
    f32x4 bnxt[NFRAG];
    bool tok[NSUB];
    uint8_t *Ytile = reinterpret_cast<uint8_t *>(Y) + t0 * M * 2;
    const uint32_t yoff = (uint32_t)(l16 * M * 2 + 16 * G);  // sub-tile u adds 16 u rows (uniform)
#pragma unroll
    for (int u = 0; u < NSUB; ++u) {
        hold[u] = make_uint2(0u, 0u);
        tok[u] = t0 + 16 * u + l16 < T;
    }
    auto fetch_bias = [&](int64_t b) {  // of row-block b of this strip, from the LDS table
        const int at = (int)(b * R - strip_row0) + 4 * G;
#pragma unroll
        for (int f = 0; f < NFRAG; ++f) bnxt[f] = *reinterpret_cast<const f32x4 *>(btab + at + 16 * f);
    };
    auto start_acc = [&]() {
#pragma unroll
        for (int f = 0; f < NFRAG; ++f)
#pragma unroll
            for (int u = 0; u < NSUB; ++u) acc[f][u] = bnxt[f];
    };
    uint4 ra[RING][NFRAG];
    uint32_t rx[RING];
    uint4 xb[2][NSUB];  // X fragments of the current step (even / odd ping-pong, resolved by the unrolling)
    const uint32_t pmask = (uint32_t)(lane & 3) * 0x10001u;
    auto issue_reads = [&](uint32_t w, uint4 (&dst)[NSUB]) {
        w ^= pmask;  // the stored word is the one of token quad 0
        const uint32_t o1 = (w & 0xffffu) << 3, o2 = (w >> 13) & 0x7fff8u;  // packed in units of 8 bytes
#pragma unroll
        for (int u = 0; u < NSUB; ++u) {
            const uint2 lo = tr_read(smem_x + u * sub_stride<NSUB>(), o1);
            const uint2 hi = tr_read(smem_x + u * sub_stride<NSUB>(), o2);
            dst[u] = make_uint4(lo.x, lo.y, hi.x, hi.y);
        }
    };
    auto load_frag = [&](const uint32_t *q) { return *reinterpret_cast<const uint4 *>(q); };
    auto block_of = [&](int e) {
        return ((((int64_t)(g0 + (e >> nacc_shift)) * WAVES + wave)) << nacc_shift) + (e & (NACC - 1));
    };
    auto widen = [](uint32_t h) {
        if constexpr (DT == BSP_BF16) return __uint_as_float(h << 16);
        else return (float)__builtin_bit_cast(_Float16, (uint16_t)h);
    };
    // Issued when a row-block starts, used when it ends.  The address is uniform, so these are scalar
    // loads: a vector load here would put a "wait for (nearly) all vector loads" in front of the use,
    // because vector loads complete in order, and drain the operand ring at every row-block.
    const uint32_t *bias32 = (const uint32_t *)bias;
    const uint32_t gm[4] = {G == 0 ? ~0u : 0u, G == 1 ? ~0u : 0u, G == 2 ? ~0u : 0u, G == 3 ? ~0u : 0u};
    auto load_bias = [&](int64_t b) {
#pragma unroll
        for (int f = 0; f < NFRAG; ++f)
#pragma unroll
            for (int i = 0; i < 8; ++i) bs[f][i] = 0u;  // +0 in both formats
        if (!SWAP && FAST && bias && b < B) {
#pragma unroll
            for (int f = 0; f < NFRAG; ++f)
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    if (OUT != kOutStaged8 || i < 4) bs[f][i] = bias32[(b * R + f * 16) / 2 + i];
        }
    };
    // Output of the finished row-block b (the accumulators hold it).
    auto finish_block = [&](int64_t b) __attribute__((always_inline)) {
        if (b >= B) return;  // uniform
        if constexpr (SWAP) {
#pragma unroll
            for (int f = 0; f < NFRAG; f += (NFRAG == 1 ? 1 : 2)) {
                uint2 lo[NSUB], hi[NSUB];  // the 16-row fragments of output columns c0 .. c0 + 15 and c0 + 16 .. c0 + 31
                bool lone = false;
                int64_t c0;
                if constexpr (NFRAG == 1) {
                    if ((b & 1) == 0) {  // uniform
#pragma unroll
                        for (int u = 0; u < NSUB; ++u) {
                            hold[u].x = cvt_pk<DT>(acc[0][u][0], acc[0][u][1]);
                            hold[u].y = cvt_pk<DT>(acc[0][u][2], acc[0][u][3]);
                        }
                        if (b + 1 < B) return;
                        lone = true;  // the last row-block of a layer with an odd number of them leaves alone
                    }
                    c0 = (b & ~(int64_t)1) * 16;
#pragma unroll
                    for (int u = 0; u < NSUB; ++u) {
                        lo[u] = hold[u];
                        hi[u].x = cvt_pk<DT>(acc[0][u][0], acc[0][u][1]);
                        hi[u].y = cvt_pk<DT>(acc[0][u][2], acc[0][u][3]);
                    }
                } else {
                    c0 = b * R + f * 16;
#pragma unroll
                    for (int u = 0; u < NSUB; ++u) {
                        lo[u].x = cvt_pk<DT>(acc[f][u][0], acc[f][u][1]);
                        lo[u].y = cvt_pk<DT>(acc[f][u][2], acc[f][u][3]);
                        hi[u].x = cvt_pk<DT>(acc[f + 1][u][0], acc[f + 1][u][1]);
                        hi[u].y = cvt_pk<DT>(acc[f + 1][u][2], acc[f + 1][u][3]);
                    }
                }
                uint8_t *dst = Ytile + c0 * 2;  // uniform
#pragma unroll
                for (int u = 0; u < NSUB; ++u) {
                    // rows of 16 lanes, before: lo = [a0 a1 a2 a3], hi = [b0 b1 b2 b3] (a_g = columns 4 g .. 4 g + 3 of
                    // the first fragment); after the two swaps: first = [a0 a2 b0 b2], second = [a1 a3 b1 b3]
                    const u32x2 px = __builtin_amdgcn_permlane32_swap(lo[u].x, hi[u].x, false, false);
                    const u32x2 py = __builtin_amdgcn_permlane32_swap(lo[u].y, hi[u].y, false, false);
                    const u32x2 qx = __builtin_amdgcn_permlane16_swap(px[0], px[1], false, false);
                    const u32x2 qy = __builtin_amdgcn_permlane16_swap(py[0], py[1], false, false);
                    if (tok[u] && !(lone && G >= 2))
                        store_y16(dst + (int64_t)u * (32 * M) + yoff, make_uint4(qx[0], qy[0], qx[1], qy[1]));
                }
            }
        } else if constexpr (FAST) {
#pragma unroll
            for (int f = 0; f < NFRAG; ++f) {
                // A fragment of this block fills bpf bytes of a token row (32; 16 when R = 8 leaves the upper half
                // of the fragment unused); `slot` is its place in the 64-byte staging row.
                constexpr int bpf = OUT == kOutStaged8 ? 16 : 32;
                constexpr int last_slot = 64 / bpf - 1;
                const int slot = NFRAG == 1 ? (int)(b & last_slot) : (f & 1);
                // the lane's 4 columns 4 G .. 4 G + 3 are words 2 G and 2 G + 1 of the fragment's 8
                // (picked with lane masks: and / or of uniform words, no indexing)
                const uint32_t w0 = (bs[f][0] & gm[0]) | (bs[f][2] & gm[1]) | (bs[f][4] & gm[2]) | (bs[f][6] & gm[3]);
                const uint32_t w1 = (bs[f][1] & gm[0]) | (bs[f][3] & gm[1]) | (bs[f][5] & gm[2]) | (bs[f][7] & gm[3]);
                const float b0 = widen(w0 & 0xffffu), b1 = widen(w0 >> 16);
                const float b2 = widen(w1 & 0xffffu), b3 = widen(w1 >> 16);
                const int byte = slot * bpf + 8 * G;  // of the row; its 16-byte piece is swizzled
                if (8 * G < bpf) {
#pragma unroll
                    for (int u = 0; u < NSUB; ++u) {
                        uint2 o;
                        o.x = cvt_pk<DT>(acc[f][u][0] + b0, acc[f][u][1] + b1);
                        o.y = cvt_pk<DT>(acc[f][u][2] + b2, acc[f][u][3] + b3);
                        *reinterpret_cast<uint2 *>(stg + (16 * u + l16) * 64 + (((byte >> 4) ^ swz) << 4) + (byte & 8)) = o;
                    }
                }
                // The staging rows are complete after the last slot; the last row-block of a layer whose
                // block count is not a multiple of the run leaves with the slots filled so far.
                const bool lone = NFRAG == 1 && slot != last_slot && b + 1 >= B;
                if (slot == last_slot || lone) {
                    const int piece = lane & 3;  // 16-byte piece of the 64-byte row
                    const int64_t col0 = b * R + f * 16 - slot * (bpf >> 1);
                    if (piece * 16 < (slot + 1) * bpf) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int row = 16 * i + (lane >> 2);
                            const uint4 o = *reinterpret_cast<const uint4 *>(stg + row * 64 + ((piece ^ G) << 4));
                            if (t0 + row < T) store_y16(Yh + (t0 + row) * M + col0 + piece * 8, o);
                        }
                    }
                }
            }
        } else {
#pragma unroll
            for (int f = 0; f < NFRAG; ++f)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int r = f * 16 + 4 * G + v;
                    if (r >= R) continue;
                    const float bb = bias ? elem<DT>::load(bias, b * R + r) : 0.0f;
#pragma unroll
                    for (int u = 0; u < NSUB; ++u) {
                        const int64_t t = t0 + 16 * u + l16;
                        if (t < T) elem<DT>::store(Y, t * M + b * R + r, acc[f][u][v] + bb);
                    }
                }
        }
    };

    // Workgroups that share an L2 (blockIdx.x mod 8 picks the XCD) walk the strip's groups from
    // different starting points, so that they do not all pull the same plan lines at the same time:
    // groups [rot, ng) first, then [0, rot).
    const int rot = ng > 1 ? ((tile >> 3) + strip) % ng : 0;
    for (int seg = 0; seg < 2; ++seg) {
        const int ea = (seg == 0 ? rot : 0) << nacc_shift, eb = (seg == 0 ? ng : rot) << nacc_shift;
        if (ea >= eb) continue;
        // (the clamps keep a malformed plan from driving the operand pointers out of the buffer)
        const int gs_hi = min(my[eb], max_step);
        int gs = min(max(my[ea], 0), gs_hi);
        int e = ea;                             // current entry, row-block block_of(e)
        int blk_end = min(my[ea + 1], gs_hi);   // first step past the current block
        int nxt_end = my[min(ea + 2, eb)];      // the same for the block after it, fetched one block ahead

        // Per-lane operand pointers, advanced by a constant per RING steps.  The stream is read up
        // to RING steps past the segment's last step: those loads stay inside the plan buffer (its
        // size includes that slack) and their values are never used.
        // A fragment is stored lane by lane, 16 bytes each: one load instruction per fragment.
        // The first RING steps are requested before anything else, so that they travel while the X tile and
        // the bias are copied in.
        const uint32_t *wp = wfrag + (int64_t)gs * (NFRAG * 256) + lane * 4;
        const uint32_t *xp = xoff + (int64_t)gs * 16 + (lane >> 2);
#pragma unroll
        for (int j = 0; j < (LEAN ? kLeanGroup : RING); ++j) {
#pragma unroll
            for (int f = 0; f < NFRAG; ++f) ra[j][f] = load_frag(wp + (j * NFRAG + f) * 256);
            rx[j] = xp[j * 16];
            // keep the order of the step loop (fragment, then offsets, slot by slot): the waits the compiler puts
            // in front of each step count the loads issued after the wanted one on every path into the loop, and
            // a different order here would make them wait for (nearly) everything
            __builtin_amdgcn_sched_barrier(0);
        }
        stage_once();
        if constexpr (SWAP) {
            fetch_bias(block_of(e));
            start_acc();
            fetch_bias(block_of(min(e + 1, eb - 1)));
        } else {
            clear_acc(acc);
            load_bias(block_of(e));
        }
        // finished (possibly empty) row-blocks leave as soon as the stream has passed them
        auto pass_boundaries = [&]() __attribute__((always_inline)) {
            while (e < eb && blk_end <= gs) {
                finish_block(block_of(e));
                ++e;
                blk_end = e < eb ? min(nxt_end, gs_hi) : 0x7fffffff;
                nxt_end = my[min(e + 2, eb)];
                if constexpr (SWAP) {
                    start_acc();  // with the bias of block e, fetched one block ago
                    fetch_bias(block_of(min(e + 1, eb - 1)));
                    // The scalar load above must not stay outstanding into the step loop: scalar loads return out
                    // of order, and with one in flight every wait for an LDS read becomes a wait for all of them,
                    // which undoes the one-step lead of the X fragment reads.  It has had the whole block end to
                    // arrive; take it here.
                    asm volatile("" : "+s"(nxt_end));
                } else {
                    clear_acc(acc);
                    if (e < eb) load_bias(block_of(e));
                }
            }
        };
        pass_boundaries();
        if (gs >= gs_hi) continue;  // then e == eb: every block of the segment has been written
        bool done = false;
        if constexpr (LEAN) {
            while (!done) {
                static_for<0, 2>([&](auto hc) __attribute__((always_inline)) {
                    constexpr int h = decltype(hc)::value;
                    if (done) return;  // uniform
                    // this group must have arrived before the other one is requested again
#pragma unroll
                    for (int j = 0; j < kLeanGroup; ++j) {
#pragma unroll
                        for (int f = 0; f < NFRAG; ++f)
                            asm volatile("" ::"v"(ra[h * kLeanGroup + j][f].x), "v"(ra[h * kLeanGroup + j][f].y),
                                         "v"(ra[h * kLeanGroup + j][f].z), "v"(ra[h * kLeanGroup + j][f].w));
                        asm volatile("" ::"v"(rx[h * kLeanGroup + j]));
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int j = 0; j < kLeanGroup; ++j) {
#pragma unroll
                        for (int f = 0; f < NFRAG; ++f)
                            ra[(1 - h) * kLeanGroup + j][f] = load_frag(wp + ((kLeanGroup + j) * NFRAG + f) * 256);
                        rx[(1 - h) * kLeanGroup + j] = xp[(kLeanGroup + j) * 16];
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int j = 0; j < kLeanGroup; ++j) {
                        if (done) break;  // uniform
                        issue_reads(rx[h * kLeanGroup + j], xb[0]);
                        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                        for (int u = 0; u < NSUB; ++u)
#pragma unroll
                            for (int f = 0; f < NFRAG; ++f)
                                acc[f][u] = mfma16<DT>(ra[h * kLeanGroup + j][f], xb[0][u], acc[f][u]);
                        __builtin_amdgcn_sched_barrier(0);
                        ++gs;
                        if (gs >= blk_end) {  // uniform
                            pass_boundaries();
                            if (e >= eb) done = true;
                        }
                    }
                    wp += kLeanGroup * NFRAG * 256;
                    xp += kLeanGroup * 16;
                });
            }
            continue;
        }
        if constexpr (!LEAN) issue_reads(rx[0], xb[0]);
        while (!done) {
#pragma unroll
            for (int j = 0; j < RING; ++j) {
                // the LDS reads of the next step go out before this step's MFMAs (the scheduler
                // would otherwise sink them below the MFMAs); with one register set, this step's own reads
                if constexpr (LEAN) issue_reads(rx[j], xb[0]);
                else issue_reads(rx[(j + 1) % RING], xb[(j + 1) & 1]);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int u = 0; u < NSUB; ++u)
#pragma unroll
                    for (int f = 0; f < NFRAG; ++f) acc[f][u] = mfma16<DT>(ra[j][f], xb[LEAN ? 0 : (j & 1)][u], acc[f][u]);
                __builtin_amdgcn_sched_barrier(0);
                // refill this ring slot with step gs + RING
#pragma unroll
                for (int f = 0; f < NFRAG; ++f) ra[j][f] = load_frag(wp + ((RING + j) * NFRAG + f) * 256);
                rx[j] = xp[(RING + j) * 16];  // its old value went into the previous sub-iteration's reads
                ++gs;
                if (gs >= blk_end) {  // uniform
                    pass_boundaries();
                    if (e >= eb) {
                        done = true;
                        break;
                    }
                }
            }
            wp += RING * NFRAG * 256;
            xp += RING * 16;
        }
    }
    stage_once();  // a wavefront without steps still takes part in the copy and its barrier
}

// Layers wider than one LDS tile (more than 1024 input columns): the workgroup keeps the 64-token
// tile, walks the input columns chunk by chunk (1024 columns of X in LDS at a time) and carries the
// accumulators of its quads across the chunks, so the operand stream is read once per 64 tokens
// whatever the layer width.  One group (a quad per wavefront) per workgroup.
template <int DT, int NFRAG, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void linear_tiled_chunked_kernel(
    const uint16_t *__restrict__ X, int64_t T, int64_t M, int64_t N, int32_t R, int32_t npad,
    const int32_t *__restrict__ wptr, const uint32_t *__restrict__ wfrag, const uint32_t *__restrict__ xoff,
    const void *__restrict__ bias, void *__restrict__ Y, int32_t ntiles, int32_t NG, int32_t B, int32_t nchunks,
    int32_t max_step, int32_t fast_store) {
    constexpr int NSUB = 4;
    // 8 wavefronts: runs of 4 / NFRAG row-blocks (R = 8 and the odd sizes, NFRAG = 1, have 4 too); 16 wavefronts
    // (R = 16, 32): runs of 2 / NFRAG, a 2-step ring and one set of X fragment registers, as in the kernel above
    constexpr bool LEAN = WAVES == kPlanWavesWide;
    constexpr int NACC = LEAN ? 2 / NFRAG : (4 / NFRAG > 0 ? 4 / NFRAG : 1);
    static_assert(!LEAN || NFRAG <= 2, "16 wavefronts: R = 16 or 32");
    constexpr int RING = LEAN ? 2 : kPlanRing / NFRAG;
    static_assert(RING % 2 == 0, "the X fragment ping-pong needs an even ring");
    const int tile = blockIdx.x % ntiles, g = blockIdx.x / ntiles;
    const int64_t t0 = (int64_t)tile * (16 * NSUB);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int32_t *my = wptr + (int64_t)wave * ((int64_t)nchunks * NG * NACC + 1);

    f32x4 acc[NACC][NFRAG][NSUB];
    clear_quad(acc);
    uint4 ra[RING][NFRAG];
    uint32_t rx[RING];
    uint4 xb[2][NSUB];
    const uint32_t pmask = (uint32_t)(lane & 3) * 0x10001u;
    auto issue_reads = [&](uint32_t w, uint4 (&dst)[NSUB]) {
        w ^= pmask;  // the stored word is the one of token quad 0
        const uint32_t o1 = (w & 0xffffu) << 3, o2 = (w >> 13) & 0x7fff8u;  // packed in units of 8 bytes
#pragma unroll
        for (int u = 0; u < NSUB; ++u) {
            const uint2 lo = tr_read(smem_x + u * sub_stride<NSUB>(), o1);
            const uint2 hi = tr_read(smem_x + u * sub_stride<NSUB>(), o2);
            dst[u] = make_uint4(lo.x, lo.y, hi.x, hi.y);
        }
    };
    auto load_frag = [&](const uint32_t *q) { return *reinterpret_cast<const uint4 *>(q); };

    for (int q = 0; q < nchunks; ++q) {
        // the wavefront's step range of this chunk and where each of its row-blocks ends
        const int32_t *ent = my + ((int64_t)g * nchunks + q) * NACC;
        int gs = __builtin_amdgcn_readfirstlane(ent[0]);
        int ends[NACC];
#pragma unroll
        for (int k = 0; k < NACC; ++k) ends[k] = __builtin_amdgcn_readfirstlane(ent[k + 1]);
        int gs_hi = ends[NACC - 1];
        // a malformed plan must not drive the operand pointers out of the buffer
        gs = max(gs, 0);
        gs_hi = min(gs_hi, max_step);
        const bool work = gs < gs_hi;
        const uint32_t *wp = wfrag + (int64_t)gs * (NFRAG * 256) + lane * 4;
        const uint32_t *xp = xoff + (int64_t)gs * 16 + (lane >> 2);
        if (work) {  // operands of the first RING steps travel while the chunk of X is copied in
#pragma unroll
            for (int j = 0; j < RING; ++j) {
#pragma unroll
                for (int f = 0; f < NFRAG; ++f) ra[j][f] = load_frag(wp + (j * NFRAG + f) * 256);
                rx[j] = xp[j * 16];
            }
        }
        __syncthreads();  // every wavefront is done with the previous chunk of X
        stage_x_chunk<NSUB>(X, T, N, q << 10, min(1024, npad - (q << 10)), t0);
        __syncthreads();
        if (!work) continue;  // no barrier below this line inside the chunk

        if constexpr (LEAN) {
            // The loop over the wavefront's row-blocks is unrolled, so that each block's products go to its own
            // accumulator registers by name (chosen at run time, the sets are merged after every step: 16 register
            // moves per step, on hardware whose vector ALU does not run beside the matrix cores).  The operand ring
            // runs on across the block ends: `par` is the ring slot of the next step.
            int par = 0;
            static_for<0, NACC>([&](auto kc) __attribute__((always_inline)) {
                constexpr int k = decltype(kc)::value;
                const int end_k = min(ends[k], gs_hi);
                auto step = [&](auto jc) __attribute__((always_inline)) {
                    constexpr int j = decltype(jc)::value;
                    issue_reads(rx[j], xb[0]);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int u = 0; u < NSUB; ++u)
#pragma unroll
                        for (int f = 0; f < NFRAG; ++f) acc[k][f][u] = mfma16<DT>(ra[j][f], xb[0][u], acc[k][f][u]);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int f = 0; f < NFRAG; ++f) ra[j][f] = load_frag(wp + ((RING + j) * NFRAG + f) * 256);
                    rx[j] = xp[(RING + j) * 16];
                    ++gs;
                };
                for (;;) {
                    if (par == 0) {
                        if (gs >= end_k) break;
                        step(std::integral_constant<int, 0>{});
                        par = 1;
                    }
                    if (gs >= end_k) break;
                    step(std::integral_constant<int, 1>{});
                    par = 0;
                    wp += RING * NFRAG * 256;
                    xp += RING * 16;
                }
            });
            continue;
        }
        int cur = 0;
        auto end_of = [&](int k) {
            int v = ends[0];
#pragma unroll
            for (int i = 1; i < NACC; ++i) v = k == i ? ends[i] : v;
            return v;
        };
        int blk_end = ends[0];
        while (blk_end <= gs && cur < NACC - 1) blk_end = end_of(++cur);
        if constexpr (!LEAN) issue_reads(rx[0], xb[0]);
        bool done = false;
        while (!done) {
#pragma unroll
            for (int j = 0; j < RING; ++j) {
                if constexpr (LEAN) issue_reads(rx[j], xb[0]);
                else issue_reads(rx[(j + 1) % RING], xb[(j + 1) & 1]);
                __builtin_amdgcn_sched_barrier(0);
                step_mfma<DT, NFRAG, NSUB, NACC>(acc, cur, ra[j], xb[LEAN ? 0 : (j & 1)]);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int f = 0; f < NFRAG; ++f) ra[j][f] = load_frag(wp + ((RING + j) * NFRAG + f) * 256);
                rx[j] = xp[(RING + j) * 16];
                ++gs;
                if (gs >= blk_end) {  // uniform
                    if (gs >= gs_hi) {
                        done = true;
                        break;
                    }
                    while (blk_end <= gs && cur < NACC - 1) blk_end = end_of(++cur);
                }
            }
            wp += RING * NFRAG * 256;
            xp += RING * 16;
        }
    }

    // The output staging of a wavefront (16 rows of kOutPitch bytes) takes the place of the X chunk once every
    // wavefront is done with it: the kernel then holds 128 KiB of LDS and leaves the rest of the compute unit's
    // to small kernels of other streams.
    __syncthreads();
    typedef QuadEpilogue<DT, NFRAG, NSUB, NACC> Ep;
    Ep ep;
    ep.init(Y, bias, T, M, R, B, t0, lane, smem_x + wave * (16 * kOutPitch), fast_store != 0);
    const int64_t b0 = ((int64_t)g * WAVES + wave) * NACC;
    if (b0 < B) {
        typename Ep::Packed out;
        ep.load_bias(b0);
        ep.convert(acc, out);
        ep.flush(b0, out);
    }
}

template <int DT, int NFRAG, int NSUB>
int launch_canonical(const TiledArgs &a, int waves, hipStream_t s) {
    const size_t lds = tile_bytes<NSUB>(a.npad);
    static thread_local size_t configured = 0;  // per instantiation and thread
    const int64_t ntiles = (a.T + 16 * NSUB - 1) / (16 * NSUB);
    int64_t nstrips = (256 + ntiles - 1) / ntiles;  // enough strips to give every compute unit a workgroup
    if (nstrips < 1) nstrips = 1;
    auto kern = linear_tiled_canonical_kernel<DT, NFRAG, NSUB>;
    int st = raise_lds_limit(kern, lds, configured);
    if (st != BSP_OK) return st;
    const int64_t max_strips = (a.B + 3) / 4;  // never fewer than 4 row-blocks per strip
    if (nstrips > max_strips) nstrips = max_strips;
    int64_t rb_per_strip = (a.B + nstrips - 1) / nstrips;
    if (rb_per_strip > kMaxStripBlocks) rb_per_strip = kMaxStripBlocks;
    nstrips = (a.B + rb_per_strip - 1) / rb_per_strip;
    if (ntiles * nstrips >= ((int64_t)1 << 31)) return BSP_ERR_SHAPE;
    kern<<<dim3((unsigned)(ntiles * nstrips)), dim3((unsigned)(waves * 64)), lds, s>>>(
        a.X, a.T, a.M, a.N, a.R, a.npad, a.blk_ptr, a.col_idx, a.vals, a.bias, a.Y, (int32_t)ntiles,
        (int32_t)rb_per_strip, (int32_t)a.B);
    return check_launch();
}

template <int DT, int NFRAG, int OUT, int WAVES>
int launch_planned_1024(const TiledArgs &a, int64_t ntiles, int64_t NG, int64_t max_step, hipStream_t s);

template <int DT, int NFRAG>
int launch_planned(const TiledArgs &a, hipStream_t s) {
    const bool chunked = plan_chunks(a.N, a.R, a.M).n > 1;
    const int NACC = plan_nacc(NFRAG, chunked, a.R);
    const size_t lds = kXTileBytes;  // 64 tokens x 1024 columns
    const int64_t ntiles = (a.T + 63) / 64;
    const int waves = plan_waves(a.N, a.R, a.M);  // as the plan was built
    const int64_t NG = (a.B + waves * NACC - 1) / (waves * NACC);
    // the staged store path: full fragments, and a bias that can be read in 4-byte words
    const int32_t fast = ((a.R == 16 * NFRAG || a.R == 8) && (reinterpret_cast<uintptr_t>(a.bias) & 3) == 0 &&
                          (reinterpret_cast<uintptr_t>(a.Y) & 15) == 0)
                             ? 1
                             : 0;
    const int64_t max_step = a.plan_steps - plan_slack_steps();
    if (max_step < 0 || max_step > INT32_MAX) return BSP_ERR_CAPACITY;
    if (chunked) {
        if constexpr (NFRAG == 1) {  // R = 16: the kernel that streams X through LDS beside the products
            if (a.R == 16) return launch_linear_stream16(a, max_step, s);
        }
        if (ntiles * NG >= ((int64_t)1 << 31)) return BSP_ERR_SHAPE;
        const PlanChunks ch = plan_chunks(a.N, a.R, a.M);
        auto go = [&](auto kern, size_t &configured, int w) {
            int st = raise_lds_limit(kern, lds, configured);
            if (st != BSP_OK) return st;
            kern<<<dim3((unsigned)(ntiles * NG)), dim3(w * 64), lds, s>>>(
                a.X, a.T, a.M, a.N, a.R, a.npad, a.wptr, (const uint32_t *)a.wfrag, a.xoff, a.bias, a.Y, (int32_t)ntiles,
                (int32_t)NG, (int32_t)a.B, ch.n, (int32_t)max_step, fast);
            return check_launch();
        };
        if constexpr (NFRAG <= 2) {
            if (waves == kPlanWavesWide) {  // R = 16, 32
                static thread_local size_t configured = 0;
                return go(linear_tiled_chunked_kernel<DT, NFRAG, kPlanWavesWide>, configured, kPlanWavesWide);
            }
        }
        if (waves != kPlanWaves) return BSP_ERR_SHAPE;
        static thread_local size_t configured8 = 0;
        return go(linear_tiled_chunked_kernel<DT, NFRAG, kPlanWaves>, configured8, kPlanWaves);
    }
    if constexpr (NFRAG == 1) {
        if (a.R == 8 && fast) return launch_planned_1024<DT, NFRAG, kOutStaged8, kPlanWaves>(a, ntiles, NG, max_step, s);
        if (a.R == 8) return launch_planned_1024<DT, NFRAG, kOutElements8, kPlanWaves>(a, ntiles, NG, max_step, s);
    }
    // full fragments and 16-byte stores: the lane-swap output path (any bias address: it is read element by element)
    if (a.R == 16 * NFRAG && (reinterpret_cast<uintptr_t>(a.Y) & 15) == 0) {
        // R = 16 and 32: 16 wavefronts (the plan has 16 streams); R = 64: 8
        constexpr int WAVES = NFRAG <= 2 ? kPlanWavesWide : kPlanWaves;
        if constexpr (NFRAG == 1) {  // R = 16: the kernel whose step loop is written in assembly (its plans are paired)
            if (waves == kPlanWaves16) return launch_linear_steploop16(a, max_step, s);
            return BSP_ERR_SHAPE;
        } else {
            if (waves == WAVES) return launch_planned_1024<DT, NFRAG, kOutSwap, WAVES>(a, ntiles, NG, max_step, s);
        }
    }
    if (waves != kPlanWaves) return BSP_ERR_SHAPE;  // (a plan of 16 streams is only consumed by the path above)
    return launch_planned_1024<DT, NFRAG, kOutElements, kPlanWaves>(a, ntiles, NG, max_step, s);
}

template <int DT, int NFRAG, int OUT, int WAVES>
int launch_planned_1024(const TiledArgs &a, int64_t ntiles, int64_t NG, int64_t max_step, hipStream_t s) {
    static thread_local size_t configured = 0;
    auto kern = linear_tiled_planned_kernel<DT, NFRAG, OUT, WAVES>;
    int64_t nstrips = (256 + ntiles - 1) / ntiles;  // enough strips to give every compute unit a workgroup
    if (nstrips > NG) nstrips = NG;
    if (nstrips < 1) nstrips = 1;
    int64_t gps = (NG + nstrips - 1) / nstrips;
    // behind the X tile: the per-wavefront staging buffers, or (lane-swap output) the fp32 bias of a strip's rows
    size_t lds_planned = kXTileBytes + (size_t)WAVES * kOutStageBytes;  // all 160 KiB of a compute unit
    if constexpr (OUT == kOutSwap) {
        const int64_t rows_per_group = (int64_t)WAVES * plan_nacc(NFRAG, false, 16 * NFRAG) * 16 * NFRAG;
        const int64_t max_gps = kBiasTableBytes / (4 * rows_per_group);  // >= 8
        if (gps > max_gps) gps = max_gps;
        lds_planned = kXTileBytes + (size_t)(gps * rows_per_group * 4);
    }
    nstrips = (NG + gps - 1) / gps;
    int st = raise_lds_limit(kern, lds_planned, configured);
    if (st != BSP_OK) return st;
    if (ntiles * nstrips >= ((int64_t)1 << 31)) return BSP_ERR_SHAPE;
    kern<<<dim3((unsigned)(ntiles * nstrips)), dim3(WAVES * 64), lds_planned, s>>>(
        a.X, a.T, a.M, a.N, a.R, a.npad, a.wptr, (const uint32_t *)a.wfrag, a.xoff, a.bias, a.Y, (int32_t)ntiles,
        (int32_t)gps, (int32_t)NG, (int32_t)a.B, (int32_t)max_step);
    return check_launch();
}

template <int DT, int NFRAG, bool PLAN>
int launch_nsub(const TiledArgs &a, int waves, hipStream_t s) {
    if constexpr (PLAN) return launch_planned<DT, NFRAG>(a, s);
    // the X tile must fit the 160 KiB of LDS: 64 tokens up to 1024 columns, 32 up to 2048, 16 up to 4096
    if (a.npad <= 1024) return launch_canonical<DT, NFRAG, 4>(a, waves, s);
    if (a.npad <= 2048) return launch_canonical<DT, NFRAG, 2>(a, waves, s);
    return launch_canonical<DT, NFRAG, 1>(a, waves, s);
}

template <int DT, bool PLAN>
int launch_nfrag(const TiledArgs &a, int waves, hipStream_t s) {
    if (a.R <= 16) return launch_nsub<DT, 1, PLAN>(a, waves, s);
    if (a.R <= 32) return launch_nsub<DT, 2, PLAN>(a, waves, s);
    return launch_nsub<DT, 4, PLAN>(a, waves, s);
}

}  // namespace

constexpr int kCanonicalWaves = 16;  // wavefronts per workgroup of the kernel on the compact storage

int plan_slack_steps() { return 16; }  // covers the read-ahead of every kernel that consumes a plan

bool tiled_supported(int xdt, int64_t N, int32_t k_align) {
    if (xdt != BSP_BF16 && xdt != BSP_F16) return false;
    if (k_align % 32 != 0 || N < 32 || N % 8 != 0) return false;
    const int64_t npad = (N + 255) / 256 * 256;
    return npad <= 4096;  // a 16-token sub-tile of 4096 columns fills 128 KiB of LDS
}

int launch_linear_tiled(const TiledArgs &args, bool plan, hipStream_t s) {
    TiledArgs a = args;
    a.npad = (int32_t)((a.N + 255) / 256 * 256);
    if (a.xdt == BSP_BF16)
        return plan ? launch_nfrag<BSP_BF16, true>(a, kCanonicalWaves, s) : launch_nfrag<BSP_BF16, false>(a, kCanonicalWaves, s);
    return plan ? launch_nfrag<BSP_F16, true>(a, kCanonicalWaves, s) : launch_nfrag<BSP_F16, false>(a, kCanonicalWaves, s);
}

}  // namespace bsp
