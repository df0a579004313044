/*
 * bsp.h -- C ABI of the block-structured-pruning library for AMD CDNA4 (gfx950).
 *
 * The operations are those of "Efficient Transformer-based Large Scale Language
 * Representations using Hardware-friendly Block Structured Pruning" (arXiv 2009.08065):
 * group l2 norms and reweighting factors (Sec. 3.2, Eq. 3), the prune decision of
 * Alg. 1 by threshold or percentile (Sec. 3.1), the compact storage in which only the
 * kept columns of a block are indexed (Sec. 3.1), and the pruned linear layer the
 * storage exists for (Sec. 3.1, Sec. 4.4).
 *
 * Conventions
 *   W      weight, row-major [M, N] = [out_features, in_features];  Y = X W^T + bias.
 *   R      rows per row-block ("block column size" d_n of Eq. 3);  B = M / R row-blocks.
 *   group  g = (b, j): the R weights W[bR .. bR+R-1, j].
 *   Every data pointer is a DEVICE pointer owned by the caller unless marked "host".
 *   The library allocates nothing and keeps no state between calls; scratch memory is
 *   passed in by the caller (see the *_workspace_bytes queries).  The two exceptions are
 *   bsp_prune_mask_static, whose scratch is a device array inside the library, and
 *   bsp_linear_transposed_dense, which hands a dense product to rocBLAS.
 *   Every call validates its arguments on the host, then enqueues its kernels on
 *   `stream` (a hipStream_t passed as void*; NULL = the default stream) and returns
 *   without waiting.  Return value: a bsp_status; nothing is launched unless it is BSP_OK.
 *   Inputs are assumed finite.
 */
#ifndef BSP_H
#define BSP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    BSP_OK = 0,
    BSP_ERR_NULL = 1,     /* a required pointer is NULL */
    BSP_ERR_SHAPE = 2,    /* a dimension is <= 0, M % R != 0, R outside [1, 64], sizes overflow int32 where one is used */
    BSP_ERR_DTYPE = 3,    /* dtype / enum value not supported by this call */
    BSP_ERR_CAPACITY = 4, /* an output or workspace buffer is too small */
    BSP_ERR_FORMAT = 5,   /* compact storage is malformed (bsp_packed_validate only) */
    BSP_ERR_HIP = 6       /* a HIP call failed; see bsp_last_hip_error() */
} bsp_status;

typedef enum { BSP_F32 = 0, BSP_BF16 = 1, BSP_F16 = 2 } bsp_dtype;

/* Reweighting factor of a group with sum of squares s (Sec. 3.2, update rule under Eq. 3):
 * BSP_ALPHA_NORM   1 / (sqrt(s) + eps)   the form printed in the paper
 * BSP_ALPHA_SQNORM 1 / (s + eps)         squared-norm form (its gradient alpha*W equals the
 *                                        paper's gamma * W / ||W|| at the moment of a refresh) */
typedef enum { BSP_ALPHA_SQNORM = 0, BSP_ALPHA_NORM = 1 } bsp_alpha_mode;

/* What a percentile ranks over: each row of the [B, N] group array on its own (one
 * row-block), or all B*N groups together (one matrix, or several matrices with equal R
 * whose group arrays lie end to end). */
typedef enum { BSP_SCOPE_BLOCK = 0, BSP_SCOPE_MATRIX = 1 } bsp_scope;
/* What a layer does to its sums before it rounds them (bsp_linear_planned_fused):
 * BSP_ACT_GELU  y = 0.5 y (1 + erf(y / sqrt 2)), the exact form (BERT's) */
typedef enum { BSP_ACT_NONE = 0, BSP_ACT_GELU = 1 } bsp_activation;

/* ---- group norms and reweighting factors (Sec. 3.2, Eq. 3; Alg. 1 norm step) ---------
 * For every group: sumsq = sum_r W[bR+r, j]^2 accumulated in fp32 with one fused
 * multiply-add per row, rows ascending; norm = sqrt(sumsq); alpha per `mode`, each step
 * one IEEE fp32 operation.
 * W: [M, N] of dtype wdt.  sumsq, norm, alpha: [B, N] fp32, each may be NULL (not written). */
int bsp_group_norms(const void *W, int wdt, int64_t M, int64_t N, int32_t R, float eps, int mode,
                    float *sumsq, float *norm, float *alpha, void *stream);

/* ---- gradient of the regulariser with fixed reweighting factors (Eq. 3; Alg. 2 loop) --
 * coef_g = lambda * alpha_g                     (BSP_ALPHA_SQNORM)
 *        = lambda * alpha_g / sqrt(sumsq_g)     (BSP_ALPHA_NORM; 0 for an all-zero group)
 * grad[m, j] = coef_g * W[m, j], or fma(coef_g, W[m, j], grad[m, j]) when accumulate != 0,
 * rounded to wdt.  sumsq_g is recomputed from W as in bsp_group_norms.
 * grad: [M, N] of dtype wdt.  penalty: optional device double receiving the value of the
 * regulariser, lambda * sum_g alpha_g ||W_g|| (NORM) or (lambda/2) * sum_g alpha_g ||W_g||^2
 * (SQNORM); it is summed in a fixed order, so repeated calls give identical bits.
 * ws: scratch of at least bsp_penalty_grad_workspace_bytes(M, N, R) bytes; only needed
 * (may be NULL) when penalty != NULL. */
int bsp_penalty_grad(const void *W, int wdt, int64_t M, int64_t N, int32_t R, const float *alpha,
                     float lambda, int mode, int accumulate, void *grad, double *penalty, void *ws,
                     size_t ws_bytes, void *stream);
size_t bsp_penalty_grad_workspace_bytes(int64_t M, int64_t N, int32_t R);

/* ---- prune decision (Alg. 1: a group with norm <= t_b is removed; Sec. 3.1 percentile) -
 * sumsq: [B, N] fp32 as written by bsp_group_norms.  keep: [B, N] uint8, 1 = kept.
 * n_keep < 0  threshold form: keep = (sumsq > t*t), compared exactly; t < 0 keeps all.
 * n_keep >= 0 percentile form: in every scope of n groups, P = n - n_keep groups are to be
 *             pruned; the threshold is the P-th smallest sumsq of the scope (none when
 *             P <= 0) and keep = (sumsq > threshold): ties at the cut are pruned, so at
 *             most n_keep groups survive.  `t` is ignored.
 * t_used: optional, one fp32 per scope (B for BSP_SCOPE_BLOCK, 1 for BSP_SCOPE_MATRIX):
 *         the threshold applied, in the squared domain (-inf when nothing was pruned).
 *         Written by the percentile form only.
 * ws: scratch of at least bsp_prune_mask_workspace_bytes(B, N, scope) bytes (percentile
 *     form only).  B*N must be below 2^31. */
int bsp_prune_mask(const float *sumsq, int64_t B, int64_t N, float t, int64_t n_keep, int scope,
                   uint8_t *keep, float *t_used, void *ws, size_t ws_bytes, void *stream);
size_t bsp_prune_mask_workspace_bytes(int64_t B, int64_t N, int scope);

/* ---- the same call for callers that cannot allocate (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc) ------------------------------------------
 * bsp_prune_mask with its scratch taken from a device array inside the library instead of a
 * workspace argument: same arguments otherwise, same kernels, same results bit for bit.  The
 * call allocates and frees nothing.  The array (about 4.1 MiB, held on every GPU the library
 * runs on until the process ends) serves every size the workspace form accepts: B*N < 2^31;
 * larger inputs return BSP_ERR_SHAPE, a workspace need above the array BSP_ERR_CAPACITY.
 * The array's device address is looked up on the first call on a device (make that call
 * outside a graph capture).  All calls on one GPU share the array, whatever their stream:
 * calls that overlap on one GPU race; order them on one stream or with events.  Nothing has
 * to be cleared between calls (every launch overwrites what the next one reads). */
int bsp_prune_mask_static(const float *sumsq, int64_t B, int64_t N, float t, int64_t n_keep, int scope,
                          uint8_t *keep, float *t_used, void *stream);

/* ---- refresh and gradient in one pass (Alg. 2 at a milestone: "update gamma", then the
 * regulariser term of the next step's gradient with the new factors) --------------------
 * Exactly bsp_group_norms followed by bsp_penalty_grad with the alpha just computed, bit for
 * bit, but W is read once.  sumsq, norm, alpha may be NULL; grad must not. */
int bsp_group_norms_grad(const void *W, int wdt, int64_t M, int64_t N, int32_t R, float eps, int mode,
                         float lambda, int accumulate, float *sumsq, float *norm, float *alpha, void *grad,
                         void *stream);

/* ---- masked weights (Alg. 1: a pruned group is set to zero; Alg. 2: W = W * Mask after every
 * retraining update) ---------------------------------------------------------------------
 * In place: every weight of a group with keep[b, j] == 0 becomes +0; the weights of kept
 * groups keep their bits.  W: [M, N] row-major of dtype wdt; keep: [M / R, N] uint8. */
int bsp_mask_weights(void *W, int wdt, int64_t M, int64_t N, int32_t R, const uint8_t *keep, void *stream);

/* ---- whole-block pruning (the "block sparse" comparison of Sec. 4.4 / Table 4: a block is kept
 * or removed as a whole) ----------------------------------------------------------------------
 * A tile is the R rows of a row-block times C consecutive columns (N % C == 0).  bsp_tile_sumsq
 * adds the C column-group sums of every tile in fp32, columns ascending, starting from +0:
 * sumsq [B, N] (as written by bsp_group_norms) -> tile_sumsq [B, N / C].  The decision is then
 * bsp_prune_mask on tile_sumsq (threshold or percentile, any scope), and bsp_expand_tile_mask
 * spreads it over the columns: keep[b, j] = tile_keep[b, j / C] != 0, the mask bsp_pack and the
 * layer take.  C = 1 is the column-granular method itself. */
int bsp_tile_sumsq(const float *sumsq, int64_t B, int64_t N, int32_t C, float *tile_sumsq, void *stream);
int bsp_expand_tile_mask(const uint8_t *tile_keep, int64_t B, int64_t N, int32_t C, uint8_t *keep, void *stream);

/* ---- the other division (Sec. 3.2, Eq. 2; Alg. 1 as printed: column blocks of C columns, a group
 * is a row of a block) on the matrix as it is stored ---------------------------------------------
 * bsp_rowseg_norms: for every row segment sumsq[m, q] = sum_c W[m, qC + c]^2 in fp32, one fused
 * multiply-add per element, columns ascending (bit for bit what bsp_group_norms gives for the
 * transposed matrix with R = C); norm and alpha as in bsp_group_norms.  Outputs [M, N / C] fp32,
 * each may be NULL.  1 <= C <= 64, N % C == 0.  The decision is bsp_prune_mask on sumsq
 * (B = M, N = N / C).  bsp_mask_weights_rowseg zeroes the pruned segments in place
 * (keep_seg [M, N / C], 1 = kept); applied together with bsp_mask_weights it leaves the matrix
 * pruned by both divisions at once (Sec. 3.1: "row pruning and column pruning on each block"),
 * which bsp_pack then stores by its kept column groups. */
int bsp_rowseg_norms(const void *W, int wdt, int64_t M, int64_t N, int32_t C, float eps, int mode, float *sumsq,
                     float *norm, float *alpha, void *stream);
int bsp_mask_weights_rowseg(void *W, int wdt, int64_t M, int64_t N, int32_t C, const uint8_t *keep_seg,
                            void *stream);

/* ---- one weight update (Alg. 2: "update W ... using Adam"; in the retraining loop followed
 * by W = W * Mask) ---------------------------------------------------------------------
 * Adam as published (Kingma & Ba, Algorithm 1) on fp32 master weights W [M,N] with fp32
 * moments m, v of the same shape, all updated in place; G [M,N] (dtype gdt) is the gradient
 * of the prediction loss and is only read.  t >= 1 is the step count (bias corrections
 * 1 - beta^t).  All arithmetic is fp32, one rounding per operation:
 *   g <- fma(coef, w, g)   if alpha != NULL: the gradient of the regulariser (Eq. 3) with the
 *                          factors alpha [B,N] fixed, coef as in bsp_penalty_grad (mode, lambda):
 *                          Adam then minimises the mixed loss of the reweighted-training loop;
 *   m <- beta1*m + (1-beta1)*g;   v <- beta2*v + ((1-beta2)*g)*g;
 *   w <- w - (lr*(m/c1)) / (sqrt(v/c2) + eps);
 *   w <- +0                if keep != NULL and keep[b][j] == 0 (the retraining loop's mask);
 * the moments of a pruned weight keep evolving (the algorithm masks W only).
 * B = M/R <= 65535.  Errors: NULL W/G/m/v, bad dtype or mode, M % R != 0, t < 1. */
int bsp_adam_step(float *W, const void *G, int gdt, float *m, float *v, int64_t M, int64_t N, int32_t R,
                  const float *alpha, float lambda, int mode, const uint8_t *keep, float lr, float beta1,
                  float beta2, float eps, int64_t t, void *stream);

/* ---- compact storage (Sec. 3.1: only the kept columns of a block are indexed) ----------
 * Layout.  For block b: cols_b = ascending j with keep[b, j] != 0; k_b = |cols_b| =
 * blk_cnt[b]; kp_b = k_b rounded up to a multiple of k_align (0 stays 0);
 * blk_ptr[0] = 0, blk_ptr[b+1] = blk_ptr[b] + kp_b.
 *   col_idx[blk_ptr[b] + c]               = cols_b[c]          c < k_b
 *                                         = cols_b[k_b - 1]    k_b <= c < kp_b   (pad)
 *   vals[R*blk_ptr[b] + r*kp_b + c]       = W[bR + r, cols_b[c]] converted to vdt (RNE)
 *                                         = +0                 pad
 * Two phases because the size depends on the mask: bsp_pack_count fills blk_cnt [B] and
 * blk_ptr [B+1]; the caller reads blk_ptr[B], allocates col_idx (that many int32) and vals
 * (R times that many elements of vdt), and calls bsp_pack with capacity_cols = the number
 * of columns the two buffers can hold.  A block whose range would exceed capacity_cols is
 * left unwritten (nothing is written out of bounds).  k_align in {1, 8, 16, 32, 64}. */
int bsp_pack_count(const uint8_t *keep, int64_t B, int64_t N, int32_t k_align, int32_t *blk_cnt,
                   int32_t *blk_ptr, void *stream);
int bsp_pack(const void *W, int wdt, int64_t M, int64_t N, int32_t R, const uint8_t *keep,
             int32_t k_align, const int32_t *blk_cnt, const int32_t *blk_ptr, int64_t capacity_cols,
             int32_t *col_idx, void *vals, int vdt, void *stream);

/* The prune decision (Alg. 1, Sec. 3.1 percentile) and the sizes of its compact storage
 * (Sec. 3.1) in one call: keep, t_used as bsp_prune_mask writes them for the same
 * (sumsq, t, n_keep, scope), blk_cnt and blk_ptr as bsp_pack_count writes them for that keep
 * and k_align -- the same integers.  For the matrix-scope percentile the launch that writes
 * the mask also counts each row's kept groups and its last workgroup adds the counts up: two
 * launches fewer than the two calls, which is what matters on the small arrays of one weight
 * matrix.  The other forms run the two stages one after the other.  Arguments, workspace and
 * errors as in the two calls; all buffers are the caller's (device memory). */
int bsp_prune_mask_count(const float *sumsq, int64_t B, int64_t N, float t, int64_t n_keep, int scope,
                         uint8_t *keep, float *t_used, int32_t k_align, int32_t *blk_cnt,
                         int32_t *blk_ptr, void *ws, size_t ws_bytes, void *stream);

/* Debug check of a compact storage: blk_ptr starts at 0 and grows by kp_b, indices in
 * [0, N), strictly ascending over the first k_b slots, pads as specified.  Synchronises
 * the stream.  Returns BSP_OK or BSP_ERR_FORMAT.  flag: device int32 scratch (1 element). */
int bsp_packed_validate(int64_t M, int64_t N, int32_t R, int32_t k_align, const int32_t *blk_cnt,
                        const int32_t *blk_ptr, const int32_t *col_idx, int64_t capacity_cols,
                        int32_t *flag, void *stream);

/* ---- the pruned linear layer (Sec. 3.1; Sec. 4.4) ---------------------------------------
 *   Y[t, bR + r] = bias[bR + r] + sum_{c < kp_b} X[t, col_idx[blk_ptr[b] + c]] * vals[b, r, c]
 * X: [T, N], Y: [T, M], row-major contiguous, dtype xdt; vals and bias have dtype xdt too;
 * bias may be NULL.  Products are accumulated in fp32 (matrix cores for bf16 / fp16), the
 * bias is added in fp32, and the sum is rounded once to xdt (RNE).  The order of the
 * additions is unspecified.  The storage must be well formed (bsp_packed_validate).
 * X and vals must be 16-byte aligned. */
int bsp_linear(const void *X, int xdt, int64_t T, int64_t M, int64_t N, int32_t R, int32_t k_align,
               const int32_t *blk_cnt, const int32_t *blk_ptr, const int32_t *col_idx, const void *vals,
               const void *bias, void *Y, void *stream);

/* ---- the transposed product of the pruned layer (Sec. 3.1: with Wp the matrix after Alg. 1
 * the layer is Y = X Wp^T + bias, so the gradient with respect to its input is dX = dY Wp;
 * the same product is the layer itself when the pruned groups are row segments of column
 * blocks, the other division of Alg. 1 and the second regulariser of Sec. 3.2, and the matrix
 * is stored transposed) ------------------------------------------------------------------
 *   Z[t, n] = bias[n] + sum_{b, c < k_b : col_idx[blk_ptr[b] + c] == n}
 *                       sum_{r < R} U[t, bR + r] * vals[b, r, c]
 * U: [T, M], Z: [T, N], row-major contiguous, dtype udt; vals and bias (length N, may be
 * NULL) have dtype udt too.  The compact storage is the one bsp_pack writes; pad slots
 * (c >= k_b) are not part of the matrix and add nothing, whatever U holds.  A column that no
 * row-block keeps receives the bias alone.  Products are accumulated in fp32 (matrix cores
 * for bf16 / fp16 when R % 4 == 0, k_align >= 8, U and vals 4-byte aligned and
 * M * (N + 64) < 4e9; fp32 multiply-adds otherwise), the bias is added in fp32 and the sum
 * is rounded once to udt (RNE).  The order of the additions is unspecified but fixed for
 * given arguments: two calls give the same bits.  The storage must be well formed
 * (bsp_packed_validate); a malformed one gives unspecified values in Z but no access
 * outside the buffers as long as blk_ptr and blk_cnt are consistent with their sizes.
 * N <= 65535.  Errors: NULL U / blk_cnt / blk_ptr / Z, bad dtype, M % R != 0, R > 64. */
int bsp_linear_transposed(const void *U, int udt, int64_t T, int64_t M, int64_t N, int32_t R, int32_t k_align,
                          const int32_t *blk_cnt, const int32_t *blk_ptr, const int32_t *col_idx,
                          const void *vals, const void *bias, void *Z, void *stream);

/* The same product from the masked dense matrix instead of the compact storage (Sec. 3.1: dX = dY Wp
 * with Wp the matrix after Alg. 1, i.e. W after bsp_mask_weights):
 *   Z[t, n] = bias[n] + sum_m U[t, m] * Wm[m, n]      U: [T, M], Wm: [M, N], Z: [T, N], one dtype udt
 * It multiplies the pruned zeros too (1 / density times the work) but as one plain dense product,
 * which is handed to rocBLAS (fp32 accumulation, bias added in fp32, one rounding): up to about
 * 16x compression that is the faster way on this machine.  rocBLAS is loaded on the first call (the
 * other entry points do not need it) and, unlike them, allocates device memory of its own and keeps
 * a handle per device; calls are serialised per process.  Returns BSP_ERR_HIP when rocBLAS cannot
 * be loaded or fails; BSP_ERR_NULL, BSP_ERR_DTYPE, BSP_ERR_SHAPE (a size of 2^31 or more). */
int bsp_linear_transposed_dense(const void *U, int udt, int64_t T, int64_t M, int64_t N, const void *Wm,
                                const void *bias, void *Z, void *stream);

/* ---- gradient with respect to the kept weights (Alg. 2 updates W from the gradient of the
 * loss; for the layer Y = X Wp^T + bias of Sec. 3.1 the chain rule gives
 * dW[m, j] = sum_t dY[t, m] X[t, j], and only the kept groups need it) --------------------------
 *   D[R*blk_ptr[b] + r*kp_b + c] = sum_t dY[t, b*R + r] * X[t, col_idx[b, c]]   c < k_b
 *                                = +0                                            pad slots
 * in the layout of the value panels (kp_b = blk_ptr[b+1] - blk_ptr[b]), so that an optimiser can
 * walk vals and D side by side.  All pointers are device pointers.  X: [T, N], dY: [T, M],
 * row-major contiguous, dtype xdt; D: R * blk_ptr[B] elements of dtype gdt (at most
 * R * capacity_cols; the caller owns it, every element is written).  bf16 / fp16 inputs with
 * R % 8 == 0, R <= 64, N % 4 == 0, X 8-byte and dY 16-byte aligned go through the matrix cores:
 * products exact, sums in fp32 (per tile of 32 tokens inside the matrix instruction, tiles in
 * ascending order inside a range of tokens, then the ranges in ascending order), rounded once to
 * gdt (RNE); two calls with the same arguments give the same bits.  That path needs ws: device
 * scratch of at least bsp_linear_dvals_workspace_bytes(M, N, R, capacity_cols) bytes, 256-byte
 * aligned.  Its head holds a work list derived from the storage alone (not from X, dY or T):
 * ws_state = BSP_DVALS_BUILD builds it (one more launch, 10 to 30 us), BSP_DVALS_REUSE states
 * that the last call with this ws had the same storage and M, N, R, capacity_cols and reuses it
 * -- the case of Alg. 2's retraining, where the mask is fixed while W is updated step after step.
 * The rest of ws is undefined before and after.  Other arguments (fp32 inputs, other R, ws ==
 * NULL) take a plain kernel that adds fp32 products token by token.  T == 0 gives zeros.
 * Returns BSP_OK, BSP_ERR_NULL, BSP_ERR_DTYPE, BSP_ERR_SHAPE (M % R != 0, bad k_align, sizes
 * past 32-bit indices), BSP_ERR_CAPACITY (ws_bytes too small) or BSP_ERR_HIP.  The storage must
 * be well formed (bsp_packed_validate) with ascending columns inside a row-block. */
typedef enum { BSP_DVALS_BUILD = 0, BSP_DVALS_REUSE = 1 } bsp_dvals_ws_state;
size_t bsp_linear_dvals_workspace_bytes(int64_t M, int64_t N, int32_t R, int64_t capacity_cols);
int bsp_linear_dvals(const void *X, const void *dY, int xdt, int64_t T, int64_t M, int64_t N, int32_t R,
                     int32_t k_align, const int32_t *blk_cnt, const int32_t *blk_ptr, const int32_t *col_idx,
                     int64_t capacity_cols, void *D, int gdt, void *ws, size_t ws_bytes, int ws_state, void *stream);

/* ---- derived operand buffer for the layer (Sec. 4.4 names "matrix reorder and compact model
 * storage" as what makes the pruned model fast; the order of the kept columns inside a
 * row-block is free, so it is chosen for the hardware) ---------------------------------------
 * bsp_linear_plan builds, from a compact storage with k_align = 32 or 64 and 16-bit values, a
 * buffer in which the kept columns of each row-block are re-ordered for conflict-free LDS
 * gathers, the row-blocks are laid out in the order the kernel's wavefronts visit them, and
 * every lane's matrix-core operands lie ready to load.  bsp_linear_planned computes exactly
 * what bsp_linear computes (same sums, different order of the additions) from that buffer
 * alone; it needs neither blk_ptr, col_idx nor vals.
 * bsp_linear_plan_supported: 1 when (xdt, N, k_align) can be planned (bf16 / fp16,
 * 32 <= N <= 4096, N % 8 == 0, k_align % 32 == 0), else 0; the other calls return
 * BSP_ERR_SHAPE for an unsupported layer and the caller stays with bsp_linear.
 * plan: device buffer of at least bsp_linear_plan_bytes(M, R, capacity_cols) bytes, 16-byte
 * aligned, where capacity_cols >= blk_ptr[B] is the same value in all three calls.
 * bsp_linear_planned wants X and Y 16-byte aligned too (BSP_ERR_SHAPE otherwise; bias: any
 * address). */
int bsp_linear_plan_supported(int xdt, int64_t N, int32_t k_align);
size_t bsp_linear_plan_bytes(int64_t M, int32_t R, int64_t capacity_cols);
int bsp_linear_plan(int vdt, int64_t M, int64_t N, int32_t R, int32_t k_align, const int32_t *blk_cnt,
                    const int32_t *blk_ptr, const int32_t *col_idx, const void *vals, int64_t capacity_cols,
                    void *plan, size_t plan_bytes, void *stream);
int bsp_linear_planned(const void *X, int xdt, int64_t T, int64_t M, int64_t N, int32_t R, int32_t k_align,
                       const void *plan, int64_t capacity_cols, const void *bias, void *Y, void *stream);

/* ---- the layer with its epilogue: Sec. 4.4 (what a deployed layer fuses), Sec. 4.2 (the networks) --------
 * Y = round(act(X Wp^T + bias) + residual): the Transformer blocks the paper prunes follow the FFN up-projection
 * with GELU and the attention-output and FFN down-projections with a residual addition; done inside the layer
 * kernel, on the fp32 sums and before the one rounding, either saves a pass over Y (one read and one write of
 * T x M values; a residual: two reads and a write).
 * Arguments as bsp_linear_planned, plus: act a bsp_activation; residual: device pointer [T, M] row-major of the
 * type of X, 8-byte aligned, or NULL.  Fused are: the activation for the row-blocks that run in the kernels of
 * 16-row blocks -- R = 16, 32, 48, 64, and R = 8 when M % 16 == 0 -- at any planned width; the residual for those
 * of them whose kernel writes its output once, at its end: more than 1024 input columns, or more than 512 input
 * columns and M <= 1024.  Any other request returns BSP_ERR_SHAPE and writes nothing: the caller runs
 * bsp_linear_planned and its own element-wise pass. */
int bsp_linear_planned_fused(const void *X, int xdt, int64_t T, int64_t M, int64_t N, int32_t R, int32_t k_align,
                             const void *plan, int64_t capacity_cols, const void *bias, int act,
                             const void *residual, void *Y, void *stream);

/* ---- helpers (host only) -------------------------------------------------------------- */
/* dense parameters / kept parameters = M*N / (R * kept_cols_total) (Sec. 4.4: 1.428x <=> 30 % sparsity) */
double bsp_compression_rate(int64_t M, int64_t N, int32_t R, int64_t kept_cols_total);
const char *bsp_status_string(int status);
int bsp_last_hip_error(void); /* hipError_t of the last failing HIP call on this thread, 0 if none */
const char *bsp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* BSP_H */
