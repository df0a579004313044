// Internal interface between the layer's entry points and its tiled matrix-core kernel.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bsp {

constexpr int kPlanWaves = 8;       // wavefronts per workgroup of a planned kernel = streams of a plan ...
constexpr int kPlanWavesWide = 16;  // ... and where the registers allow it: see plan_waves()
#define kPlanWaves16 16             // ... of the kernel for R = 16 and narrow layers (a macro: its assembly needs the literal)

struct TiledArgs {
    int xdt;
    const uint16_t *X;
    int64_t T, M, N, B;
    int32_t R;
    int32_t npad;             // filled by the launcher: N rounded up to 256 columns
    const int32_t *blk_ptr;
    const int32_t *col_idx;   // canonical source
    const uint16_t *vals;     // canonical source
    const int32_t *wptr;      // planned source: [waves][chunks * NG * nacc + 1] first step of (chunk q, block (g * waves + w) * nacc + i) at [w][(g * chunks + q) * nacc + i]
    const void *wfrag;        // planned source: [step][fragment][lane] 16-byte panel fragments
    const uint32_t *xoff;     // planned source: [step][lane] two 16-bit LDS byte offsets
    int64_t plan_steps;       // planned source: steps the fragment / offset regions hold (slack included)
    int64_t capacity_cols;    // planned source: the caller's bound on the padded kept columns of the storage
    const void *bias;
    void *Y;
    int act;                  // bsp_activation applied to the sums before they are rounded (the planned kernels of R = 16)
    const void *residual;     // [T, M], type of X, added after the activation (only the kernel that streams X), or null
};

// True when the tiled kernel can take this layer (16-bit floats, kp_b % 32 == 0, X tile fits in LDS).
bool tiled_supported(int xdt, int64_t N, int32_t k_align);
int launch_linear_tiled(const TiledArgs &args, bool plan, hipStream_t s);
// The planned kernel for R = 16 and layers of up to 1024 input columns (16-bit floats, a plan of 16 streams, Y
// aligned to 16 bytes); NG = groups of the plan, max_step = steps the plan holds without its read-ahead slack.
int launch_linear_steploop16(const TiledArgs &args, int64_t max_step, hipStream_t s);
// The same for R = 16 and wider layers (up to 4096 input columns), whose plans are cut into chunks of 512 columns.
int launch_linear_stream16(const TiledArgs &args, int64_t max_step, hipStream_t s);
// Column chunks of a plan: layers with more than 1024 (padded) input columns are cut into chunks of
// 1024 columns, the width of X that fits in LDS next to 64 tokens; narrower layers are one chunk.
// R = 16: chunks of 512 columns, two of which are in LDS at a time -- one being used, one being filled.  Layers of
// R = 16 with few row-blocks (up to 64: the attention output projection) are planned that way from 513 columns
// on: with so few blocks the kernel for narrow layers would give a wavefront one or two pairs of row-blocks per
// workgroup, and the kernel that streams X runs them as fast and writes its output once, at its end -- which is
// where a residual can be added without a load in the step loop.
constexpr int kPlanMaxChunks = 8;
struct PlanChunks {
    int32_t n;      // number of chunks
    int32_t shift;  // column >> shift = chunk
};
inline PlanChunks plan_chunks(int64_t N, int32_t R, int64_t M) {
    const int64_t npad = (N + 255) / 256 * 256;
    if (R == 16 && (npad > 1024 || (npad > 512 && M / 16 <= 64))) return PlanChunks{(int32_t)((npad + 511) / 512), 9};
    if (npad <= 1024) return PlanChunks{1, 30};
    return PlanChunks{(int32_t)((npad + 1023) / 1024), 10};
}
// Row-blocks of 8 rows ride the kernels written for 16 when the layer's height allows it: two neighbouring row-blocks
// form one block of 16 rows that keeps the union of their columns; a step's fragment holds the first one's weights in
// rows 0-7 and the second one's in rows 8-15, with zeros where only the other one keeps the column.  Every plan
// parameter is then the one of R = 16.
inline bool plan_virtual16(int32_t R, int64_t M) { return R == 8 && M % 16 == 0; }
// Row-blocks of 32, 48 or 64 rows ride them too: a block of the plan is one 16-row slab of a stored row-block (the
// stored block's kept columns, the slab's rows of its panel), so such a layer runs as the layer of 16-row blocks with
// the same kept columns does.  (The slabs of a block gather the same columns of X from LDS once each; a kernel that
// shared the gather would need a step loop of its own per block height.)
inline int plan_split16(int32_t R) { return (R > 16 && R % 16 == 0) ? R / 16 : 1; }
// Height of the blocks a layer's plan is made of.
inline int32_t plan_block_rows(int32_t R, int64_t M) { return (plan_virtual16(R, M) || plan_split16(R) > 1) ? 16 : R; }
// Chunked plans of R = 16 give every (row-block, chunk) at least one step (of zero weights where the block keeps
// no column of the chunk), as one-chunk plans give every row-block: the assembly loops never meet an empty run.
inline bool plan_min_one_step(int32_t R, bool chunked) { return !chunked || R == 16; }
// A wavefront of the planned kernels works on runs of nacc consecutive row-blocks, so that it can write 64
// or 128 contiguous bytes per token row: 4 sixteen-row fragments' worth in the column-chunked kernel with 8
// wavefronts (which holds all their accumulators and writes once, at the end), 2 with 16 wavefronts (R = 16, 32:
// see plan_waves) and in the kernel for layers of up to 1024 columns (64 bytes per row are enough there).
// R = 8 fills half a fragment, so 4 of its row-blocks make 64 bytes.
constexpr int plan_nacc(int nfrag, bool chunked, int R) {
    if (R == 8) return 4;
    if (R == 16 && chunked) return 4;  // (8 wavefronts that hold the accumulators of 4 row-blocks each)
    const int frags = (chunked && R != 16 && R != 32) ? 4 : 2;
    return frags / nfrag > 0 ? frags / nfrag : 1;
}
// Streams of a plan = wavefronts of the workgroup that consumes it.  Layers with R = 16 or 32 run 16
// wavefronts (4 per SIMD) on a short operand ring: their kernels stay within 128 registers, and the
// per-wavefront chains of dependent instructions overlap better (measured 10-14 % faster than 8 wavefronts).
// The other R do not fit (R = 64: four fragments of accumulators; R = 8 and odd sizes: their output paths).
inline int plan_waves(int64_t N, int32_t R, int64_t M) {
    if (R == 16 && plan_chunks(N, R, M).n > 1) return kPlanWaves;  // beside them run the wavefronts that copy X in
    if (R == 16) return kPlanWaves16;
    return R == 32 ? kPlanWavesWide : kPlanWaves;
}
// Which row-block a plan's entry (group g, wavefront w, place i in the run) stands for, and back.  Plain plans deal
// runs of nacc blocks round robin: block (g * waves + w) * nacc + i.  Paired plans (R = 16, one column chunk: the
// kernel with the assembly loop) deal runs of 2 blocks so that the runs of one wavefront in groups 2 s and 2 s + 1 are
// neighbours -- four consecutive row-blocks, 128 bytes of a token's output row, which that kernel stores together as
// whole lines whenever both groups fall into its strip -- while the unit that balances the wavefronts stays a run.
inline bool plan_paired(int32_t R, bool chunked) { return R == 16 && !chunked; }
__host__ __device__ inline int64_t plan_block(int64_t g, int w, int i, int waves, int nacc, bool paired) {
    if (paired) return (g >> 1) * (4 * waves) + 4 * w + 2 * (int)(g & 1) + i;
    return (g * waves + w) * nacc + i;
}
__host__ __device__ inline void plan_entry(int64_t b, int waves, int nacc, bool paired, int64_t &g, int &w, int &i) {
    if (paired) {
        const int r = (int)(b % (4 * waves));
        g = 2 * (b / (4 * waves)) + ((r >> 1) & 1);
        w = r >> 2;
        i = r & 1;
    } else {
        const int64_t run = b / nacc;
        g = run / waves;
        w = (int)(run % waves);
        i = (int)(b % nacc);
    }
}
// Groups of a plan.
inline int64_t plan_groups(int64_t B, int waves, int nacc, bool paired) {
    if (paired) return 2 * ((B + 4 * waves - 1) / (4 * waves));
    return (B + (int64_t)waves * nacc - 1) / ((int64_t)waves * nacc);
}
// Steps the planned kernel may read past the last step of the storage (values unused).
int plan_slack_steps();

// Placement of X column c inside a 16-token sub-tile held in LDS, shared by the copy-in of the
// tiled kernels and by the plan builder: byte offset of token quad p (tokens 4p .. 4p+3).
__host__ __device__ inline uint32_t lds_col_offset(uint32_t c, uint32_t p) {
    const uint32_t row = (c & ~31u) | ((c >> 2) & 7u) | ((c & 3u) << 3);
    return row * 32u + ((p ^ ((c >> 5) & 3u)) << 3);
}
// The same for the 64-token tiles (four sub-tiles, up to 1024 columns) of the planned kernels: columns 0 .. 511
// fill the first 64 KiB of the tile and columns 512 .. 1023 the second, and sub-tile u of either half lies
// u * kSubStride4 bytes further on -- all four sub-tiles of a column are then within the 64 KiB that the immediate
// offset of an LDS instruction reaches, so one address register per column serves the whole tile.
constexpr uint32_t kSubStride4 = 16384u;
__host__ __device__ inline uint32_t lds_col_offset4(uint32_t c, uint32_t p) {
    return (c >> 9) * 65536u + lds_col_offset(c & 511u, p);
}
// LDS bank group (8 banks of 4 bytes = one 32-byte row) that column c lands in.
__host__ __device__ inline uint32_t lds_bank_group(uint32_t c) { return (c >> 2) & 7u; }

}  // namespace bsp
