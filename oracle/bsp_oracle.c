/*
 * bsp_oracle.c -- plain CPU oracle for block-structured-pruned linear layers.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct definition that the
 * GPU library is compared against.  It shares no code, headers, tables or helpers with the
 * HIP kernels and must never be called from the product path.
 *
 * What it computes follows "Efficient Transformer-based Large Scale Language Representations
 * using Hardware-friendly Block Structured Pruning" (arXiv 2009.08065):
 *   - Sec. 3.1 / Alg. 1: a weight matrix is divided into blocks; inside each block a group of
 *     weights (here: one column segment of a row-block, the "column division" form that
 *     Eq. 3 of Sec. 3.2 writes out) is removed when its l2 norm is <= a threshold t_b, the
 *     threshold being pre-set or a percentile.
 *   - Sec. 3.2, Eq. 3: the reweighted group-Lasso term  lambda * sum_g gamma_g * ||W_g||_2
 *     with gamma_g = 1 / (||W_g||_2 + eps), refreshed at milestones (Alg. 2).
 *   - Sec. 3.1 (storage remark) and Sec. 4.4: only the kept groups and one index per kept
 *     group need to be stored; the layer is then a smaller dense product.
 *   - The same layer read backwards: its input gradient dX = dY Wp (chain rule), which is
 *     also the layer of Alg. 1's other division (row segments of column blocks) when the
 *     matrix is kept transposed.
 *
 * Conventions.  W is row-major [M, N] = [out_features, in_features]; Y = X W^T + bias.
 * A row-block b holds rows bR .. bR+R-1; group g = (b, j) is the R weights W[bR+r, j].
 * All arrays are host arrays.  Low-precision tensors (bf16 / fp16) are passed as float
 * arrays whose values are exactly representable in that type; results that the method
 * rounds to a low-precision type are rounded here (round-to-nearest-even) and returned
 * as floats holding the rounded value.
 *
 * Build: gcc -O2 -std=c11 -ffp-contract=off -fopenmp -shared -fPIC (see build.py).
 * -ffp-contract=off keeps every float operation individually rounded; the only fused
 * operation is the explicit fmaf() in the canonical sum of squares.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORC_F32 = 0, ORC_BF16 = 1, ORC_F16 = 2 };
enum { ORC_ALPHA_SQNORM = 0, ORC_ALPHA_NORM = 1 };
enum { ORC_SCOPE_BLOCK = 0, ORC_SCOPE_MATRIX = 1 };

/* ------------------------------------------------------------------------------------ */
/* Rounding of a real value to a binary floating-point format, round-to-nearest-even.    */
/* p = significand bits including the implicit one, emin = exponent of the smallest       */
/* normal, maxv = largest finite value.  The quotient v/q is exact (q is a power of two), */
/* rint() rounds to nearest even in the default rounding mode.                            */
/* ------------------------------------------------------------------------------------ */
static double round_to_format(double v, int p, int emin, double maxv)
{
    if (v == 0.0 || isnan(v) || isinf(v)) return v;
    int e = ilogb(v);
    if (e < emin) e = emin;
    double q = ldexp(1.0, e - (p - 1));
    double r = rint(v / q) * q;
    if (fabs(r) > maxv) r = (r > 0) ? INFINITY : -INFINITY;
    return r;
}

double orc_round(double v, int dtype)
{
    switch (dtype) {
    case ORC_BF16: return round_to_format(v, 8, -126, 0x1.FEp127);
    case ORC_F16:  return round_to_format(v, 11, -14, 65504.0);
    default:       return (double)(float)v;   /* C conversion double->float is RNE */
    }
}

/* ------------------------------------------------------------------------------------ */
/* Group sums of squares: inner sum of Eq. 3 (Sec. 3.2); Alg. 1 computes its root.        */
/* Canonical fp32 form: one fused multiply-add per row of the group, rows ascending.      */
/* s is [B, N] with B = M / R.                                                            */
/* ------------------------------------------------------------------------------------ */
void orc_sumsq(const float *W, int64_t M, int64_t N, int32_t R, float *s)
{
    int64_t B = M / R;
    for (int64_t b = 0; b < B; ++b)
        for (int64_t j = 0; j < N; ++j) {
            float acc = 0.0f;
            for (int32_t r = 0; r < R; ++r) {
                float w = W[(b * R + r) * N + j];
                acc = fmaf(w, w, acc);
            }
            s[b * N + j] = acc;
        }
}

/* The same sum in double: every fp32 square is exact in double, so this is the true      */
/* value up to R-1 double roundings.  Used to bound the error of the canonical fp32 sum.  */
void orc_sumsq_exact(const float *W, int64_t M, int64_t N, int32_t R, double *s)
{
    int64_t B = M / R;
    for (int64_t b = 0; b < B; ++b)
        for (int64_t j = 0; j < N; ++j) {
            double acc = 0.0;
            for (int32_t r = 0; r < R; ++r) {
                double w = (double)W[(b * R + r) * N + j];
                acc += w * w;
            }
            s[b * N + j] = acc;
        }
}

/* ------------------------------------------------------------------------------------ */
/* Group norm and reweighting factor (Sec. 3.2, the update rule printed under Eq. 3):     */
/*   NORM   : gamma = 1 / (sqrt(s) + eps)        -- the paper's form                      */
/*   SQNORM : alpha = 1 / (s + eps)              -- squared-norm form                     */
/* Each operation is one IEEE fp32 operation.  norm / alpha may be NULL.                  */
/* ------------------------------------------------------------------------------------ */
void orc_norm_alpha(const float *s, int64_t n, float eps, int32_t mode, float *norm, float *alpha)
{
    for (int64_t i = 0; i < n; ++i) {
        float root = sqrtf(s[i]);
        if (norm) norm[i] = root;
        if (alpha) {
            float den = (mode == ORC_ALPHA_NORM) ? (root + eps) : (s[i] + eps);
            alpha[i] = 1.0f / den;
        }
    }
}

/* ------------------------------------------------------------------------------------ */
/* Gradient of the regulariser of Eq. 3 with the reweighting factors held fixed, as the   */
/* optimiser of Alg. 2 sees it between milestones.                                        */
/*   SQNORM : d/dw [ (lambda/2) alpha_g ||W_g||^2 ] = (lambda alpha_g) w                  */
/*   NORM   : d/dw [ lambda gamma_g ||W_g||_2 ]     = (lambda gamma_g / ||W_g||_2) w,     */
/*            taken as 0 for an all-zero group (the subgradient 0).                       */
/* coef is built from fp32 operations, each rounded: la = lambda*alpha; NORM divides la   */
/* by sqrtf(s) with s the canonical fp32 sum of squares of the same W.                    */
/* G = coef*w (one rounding) or, when accumulate != 0, fmaf(coef, w, G) (one rounding);   */
/* the result is then rounded to dtype gdt.  *penalty (may be NULL) receives the value of */
/* the regulariser itself, in double from the exact sums of squares.                      */
/* ------------------------------------------------------------------------------------ */
void orc_penalty_grad(const float *W, int64_t M, int64_t N, int32_t R, const float *alpha,
                      float lambda, int32_t mode, int32_t accumulate, int32_t gdt, float *G,
                      double *penalty)
{
    int64_t B = M / R;
    double pen = 0.0;
    for (int64_t b = 0; b < B; ++b)
        for (int64_t j = 0; j < N; ++j) {
            float s = 0.0f;
            double sd = 0.0;
            for (int32_t r = 0; r < R; ++r) {
                float w = W[(b * R + r) * N + j];
                s = fmaf(w, w, s);
                sd += (double)w * (double)w;
            }
            float a = alpha[b * N + j];
            float coef = lambda * a;
            if (mode == ORC_ALPHA_NORM) {
                coef = (s > 0.0f) ? coef / sqrtf(s) : 0.0f;
                pen += (double)lambda * (double)a * sqrt(sd);
            } else {
                pen += 0.5 * (double)lambda * (double)a * sd;
            }
            for (int32_t r = 0; r < R; ++r) {
                int64_t idx = (b * R + r) * N + j;
                float w = W[idx];
                float g = accumulate ? fmaf(coef, w, G[idx]) : coef * w;
                G[idx] = (float)orc_round((double)g, gdt);
            }
        }
    if (penalty) *penalty = pen;
}

/* ------------------------------------------------------------------------------------ */
/* Keep-mask, threshold form (Alg. 1: a group whose norm is <= t_b is zeroed, so a group  */
/* is kept iff its norm is strictly greater).  The test ||W_g|| > t is made on the sum of */
/* squares, exactly: s > t*t evaluated in double (both sides exact).  t < 0 keeps all.    */
/* ------------------------------------------------------------------------------------ */
void orc_mask_threshold(const float *s, int64_t n, float t, uint8_t *keep)
{
    double t2 = (double)t * (double)t;
    for (int64_t i = 0; i < n; ++i)
        keep[i] = (t < 0.0f) ? 1 : (uint8_t)((double)s[i] > t2);
}

static int cmp_float(const void *a, const void *b)
{
    float x = *(const float *)a, y = *(const float *)b;
    return (x > y) - (x < y);
}

/* ------------------------------------------------------------------------------------ */
/* Keep-mask, percentile form (Sec. 3.1: "threshold or percentile"; the appendix chooses  */
/* a compression ratio per layer).  A scope is one row of the [B, N] array (BLOCK) or the */
/* whole array (MATRIX).  With n groups in the scope and P = n - n_keep to be pruned:     */
/* P <= 0 keeps everything (threshold reported as -inf); otherwise the threshold is the   */
/* P-th smallest sum of squares of the scope and Alg. 1's rule applies: keep iff s is     */
/* strictly greater, so ties at the cut are pruned and at most n_keep groups survive.     */
/* t_used (may be NULL) receives one threshold per scope, in the squared domain.          */
/* ------------------------------------------------------------------------------------ */
void orc_mask_rank(const float *s, int64_t B, int64_t N, int64_t n_keep, int32_t scope,
                   uint8_t *keep, float *t_used)
{
    int64_t n_scopes = (scope == ORC_SCOPE_BLOCK) ? B : 1;
    int64_t n = (scope == ORC_SCOPE_BLOCK) ? N : B * N;
    float *tmp = (float *)malloc((size_t)(n > 0 ? n : 1) * sizeof(float));
    for (int64_t sc = 0; sc < n_scopes; ++sc) {
        const float *v = s + sc * n;
        uint8_t *k = keep + sc * n;
        int64_t P = n - n_keep;
        float thr;
        if (P <= 0) {
            thr = -INFINITY;
        } else {
            memcpy(tmp, v, (size_t)n * sizeof(float));
            qsort(tmp, (size_t)n, sizeof(float), cmp_float);
            thr = tmp[(P > n ? n : P) - 1];
        }
        for (int64_t i = 0; i < n; ++i) k[i] = (uint8_t)(v[i] > thr);
        if (t_used) t_used[sc] = thr;
    }
    free(tmp);
}

/* ------------------------------------------------------------------------------------ */
/* Compact storage (Sec. 3.1: only the non-zero columns of a block are indexed).          */
/* For block b: cols_b = ascending j with keep[b, j] != 0, k_b = |cols_b|,                */
/* kp_b = k_b rounded up to a multiple of k_align (0 stays 0), blk_ptr = exclusive scan   */
/* of kp_b with blk_ptr[B] = total.                                                       */
/* ------------------------------------------------------------------------------------ */
void orc_pack_count(const uint8_t *keep, int64_t B, int64_t N, int32_t k_align,
                    int32_t *blk_cnt, int32_t *blk_ptr)
{
    int32_t run = 0;
    for (int64_t b = 0; b < B; ++b) {
        int32_t k = 0;
        for (int64_t j = 0; j < N; ++j) k += keep[b * N + j] != 0;
        blk_cnt[b] = k;
        blk_ptr[b] = run;
        run += ((k + k_align - 1) / k_align) * k_align;
    }
    blk_ptr[B] = run;
}

/* col_idx[blk_ptr[b] + c] = cols_b[c] (c < k_b), pad slots repeat the last kept column.  */
/* vals[R*blk_ptr[b] + r*kp_b + c] = W[bR + r, cols_b[c]] rounded to vdt, pad slots +0.   */
void orc_pack(const float *W, int64_t M, int64_t N, int32_t R, const uint8_t *keep,
              int32_t k_align, const int32_t *blk_cnt, const int32_t *blk_ptr, int32_t vdt,
              int32_t *col_idx, float *vals)
{
    int64_t B = M / R;
    (void)k_align;
    for (int64_t b = 0; b < B; ++b) {
        int32_t kb = blk_cnt[b];
        int32_t kp = blk_ptr[b + 1] - blk_ptr[b];
        int64_t base = blk_ptr[b];
        int32_t c = 0;
        for (int64_t j = 0; j < N; ++j)
            if (keep[b * N + j]) {
                col_idx[base + c] = (int32_t)j;
                for (int32_t r = 0; r < R; ++r)
                    vals[R * base + (int64_t)r * kp + c] =
                        (float)orc_round((double)W[(b * R + r) * N + j], vdt);
                ++c;
            }
        for (; c < kp; ++c) {
            col_idx[base + c] = col_idx[base + kb - 1];
            for (int32_t r = 0; r < R; ++r) vals[R * base + (int64_t)r * kp + c] = 0.0f;
        }
    }
}

/* ------------------------------------------------------------------------------------ */
/* The layer, brute force: the dense product with pruned entries zeroed.                  */
/*   Y[t, m] = bias[m] + sum_{j ascending} X[t, j] * (keep[m / R, j] ? W[m, j] : 0)        */
/* accumulated in double (each product of two floats is exact), then rounded to ydt.      */
/* Y (floats holding the rounded value) and Yd (the double before rounding) may be NULL.  */
/* ------------------------------------------------------------------------------------ */
void orc_linear_dense(const float *X, const float *W, const uint8_t *keep, const float *bias,
                      int64_t T, int64_t M, int64_t N, int32_t R, int32_t ydt, float *Y,
                      double *Yd)
{
    for (int64_t t = 0; t < T; ++t)
        for (int64_t m = 0; m < M; ++m) {
            double acc = bias ? (double)bias[m] : 0.0;
            for (int64_t j = 0; j < N; ++j) {
                double w = keep[(m / R) * N + j] ? (double)W[m * N + j] : 0.0;
                acc += (double)X[t * N + j] * w;
            }
            if (Yd) Yd[t * M + m] = acc;
            if (Y) Y[t * M + m] = (float)orc_round(acc, ydt);
        }
}

/* The same sum taken through the compact storage, kept columns ascending (pad slots hold */
/* zero values and contribute exact zeros).  Rows of X from t0 to t1-1 only, so a caller  */
/* can evaluate a sample of a large problem; Y / Yd are indexed by the full t.            */
void orc_linear_packed(const float *X, int64_t t0, int64_t t1, int64_t M, int64_t N, int32_t R,
                       const int32_t *blk_cnt, const int32_t *blk_ptr, const int32_t *col_idx,
                       const float *vals, const float *bias, int32_t ydt, float *Y, double *Yd,
                       int32_t n_threads)
{
    int64_t B = M / R;
    (void)blk_cnt;
    if (n_threads < 1) n_threads = 1;
#pragma omp parallel for num_threads(n_threads) schedule(static)
    for (int64_t b = 0; b < B; ++b) {
        int64_t base = blk_ptr[b];
        int32_t kp = blk_ptr[b + 1] - blk_ptr[b];
        for (int64_t t = t0; t < t1; ++t)
            for (int32_t r = 0; r < R; ++r) {
                int64_t m = b * R + r;
                double acc = bias ? (double)bias[m] : 0.0;
                for (int32_t c = 0; c < kp; ++c)
                    acc += (double)X[t * N + col_idx[base + c]] *
                           (double)vals[R * base + (int64_t)r * kp + c];
                if (Yd) Yd[t * M + m] = acc;
                if (Y) Y[t * M + m] = (float)orc_round(acc, ydt);
            }
    }
}

/* ------------------------------------------------------------------------------------ */
/* The transposed product of the pruned layer.  With Wp the weight matrix with its pruned */
/* groups zeroed (Alg. 1), the layer of Sec. 3.1 is Y = X Wp^T + bias; the chain rule     */
/* gives the gradient with respect to its input as dX = dY Wp, and the same product is    */
/* the layer itself when the groups are row segments of column blocks (the other division */
/* of Alg. 1, the second regulariser of Sec. 3.2) and the matrix is kept transposed:      */
/*   Z[t, j] = bias[j] + sum_{m ascending} U[t, m] * (keep[m / R, j] ? W[m, j] : 0)        */
/* U: [T, M], Z: [T, N]; accumulated in double, then rounded to zdt.                      */
/* ------------------------------------------------------------------------------------ */
void orc_linear_t_dense(const float *U, const float *W, const uint8_t *keep, const float *bias,
                        int64_t T, int64_t M, int64_t N, int32_t R, int32_t zdt, float *Z,
                        double *Zd)
{
    for (int64_t t = 0; t < T; ++t)
        for (int64_t j = 0; j < N; ++j) {
            double acc = bias ? (double)bias[j] : 0.0;
            for (int64_t m = 0; m < M; ++m) {
                double w = keep[(m / R) * N + j] ? (double)W[m * N + j] : 0.0;
                acc += (double)U[t * M + m] * w;
            }
            if (Zd) Zd[t * N + j] = acc;
            if (Z) Z[t * N + j] = (float)orc_round(acc, zdt);
        }
}

/* The same sum taken through the compact storage: the kept column c of row-block b adds  */
/* sum_r U[t, bR + r] * vals[b, r, c] to Z[t, col_idx[b, c]]; row-blocks ascending, rows   */
/* ascending, so every Z[t, j] is summed over m ascending as above.  Pad slots (c >= k_b)  */
/* are not part of the matrix and are skipped.  Rows t0 .. t1-1 of U only.                */
void orc_linear_t_packed(const float *U, int64_t t0, int64_t t1, int64_t M, int64_t N, int32_t R,
                         const int32_t *blk_cnt, const int32_t *blk_ptr, const int32_t *col_idx,
                         const float *vals, const float *bias, int32_t zdt, float *Z, double *Zd,
                         int32_t n_threads)
{
    int64_t B = M / R;
    if (n_threads < 1) n_threads = 1;
#pragma omp parallel for num_threads(n_threads) schedule(static)
    for (int64_t t = t0; t < t1; ++t) {
        double *acc = (double *)malloc(sizeof(double) * (size_t)N);
        for (int64_t j = 0; j < N; ++j) acc[j] = bias ? (double)bias[j] : 0.0;
        for (int64_t b = 0; b < B; ++b) {
            int64_t base = blk_ptr[b];
            int32_t kp = blk_ptr[b + 1] - blk_ptr[b];
            for (int32_t r = 0; r < R; ++r) {
                double u = (double)U[t * M + b * R + r];
                for (int32_t c = 0; c < blk_cnt[b]; ++c)
                    acc[col_idx[base + c]] += u * (double)vals[R * base + (int64_t)r * kp + c];
            }
        }
        for (int64_t j = 0; j < N; ++j) {
            if (Zd) Zd[t * N + j] = acc[j];
            if (Z) Z[t * N + j] = (float)orc_round(acc[j], zdt);
        }
        free(acc);
    }
}

/* ------------------------------------------------------------------------------------ */
/* Alg. 1's effect on the stored weights ("the group is set to zero") and the retraining  */
/* step of Alg. 2 (W = W * Mask after every update): every weight of a pruned group       */
/* becomes +0, every weight of a kept group is left as it is (bit for bit).  The mask is  */
/* the group mask keep[B, N] (Alg. 2 builds an element mask from W != 0 after pruning:    */
/* the same thing except for a kept weight that happens to be exactly 0).                 */
/* ------------------------------------------------------------------------------------ */
void orc_mask_weights(float *W, int64_t M, int64_t N, int32_t R, const uint8_t *keep)
{
    for (int64_t m = 0; m < M; ++m)
        for (int64_t j = 0; j < N; ++j)
            if (!keep[(m / R) * N + j]) W[m * N + j] = 0.0f;
}

/* ------------------------------------------------------------------------------------ */
/* One weight update of Alg. 2: "update W to minimise the loss using Adam", where the     */
/* loss is the mixed loss during reweighted training (gradient of the prediction loss G   */
/* plus the gradient of the regulariser with the factors alpha held fixed, Eq. 3) and the */
/* prediction loss alone during retraining, followed there by W = W * Mask.               */
/* Adam as published (Kingma & Ba, Algorithm 1), all in fp32, every operation rounded     */
/* once, in this order, per element (w, g, m, v):                                         */
/*   g  <- fmaf(coef, w, g)              only when alpha != NULL (coef as orc_penalty_grad)*/
/*   m  <- beta1*m + (1 - beta1)*g                                                        */
/*   v  <- beta2*v + ((1 - beta2)*g)*g                                                    */
/*   w  <- w - (lr * (m / c1)) / (sqrtf(v / c2) + eps),   c_i = 1 - beta_i^t              */
/*   w  <- +0                             only when keep != NULL and the group is pruned   */
/* c1, c2 are formed in double (pow) and rounded to fp32; 1 - beta_i is an fp32           */
/* subtraction.  The moments of a pruned weight keep evolving: Alg. 2 masks W only.       */
/* ------------------------------------------------------------------------------------ */
void orc_adam_step(float *W, const float *G, float *m, float *v, int64_t M, int64_t N, int32_t R,
                   const float *alpha, float lambda, int32_t mode, const uint8_t *keep, float lr,
                   float beta1, float beta2, float eps, int64_t t)
{
    float c1 = (float)(1.0 - pow((double)beta1, (double)t));
    float c2 = (float)(1.0 - pow((double)beta2, (double)t));
    float omb1 = 1.0f - beta1, omb2 = 1.0f - beta2;
    int64_t B = M / R;
    for (int64_t b = 0; b < B; ++b)
        for (int64_t j = 0; j < N; ++j) {
            float coef = 0.0f;
            if (alpha) {
                float s = 0.0f;
                for (int32_t r = 0; r < R; ++r) {
                    float w = W[(b * R + r) * N + j];
                    s = fmaf(w, w, s);
                }
                coef = lambda * alpha[b * N + j];
                if (mode == ORC_ALPHA_NORM) coef = (s > 0.0f) ? coef / sqrtf(s) : 0.0f;
            }
            for (int32_t r = 0; r < R; ++r) {
                int64_t i = (b * R + r) * N + j;
                float w = W[i], g = G[i];
                if (alpha) g = fmaf(coef, w, g);
                float t1 = beta1 * m[i];
                float t2 = omb1 * g;
                float mn = t1 + t2;
                float t3 = beta2 * v[i];
                float t4 = omb2 * g;
                t4 = t4 * g;
                float vn = t3 + t4;
                float mh = mn / c1;
                float vh = vn / c2;
                float num = lr * mh;
                float den = sqrtf(vh) + eps;
                float q = num / den;
                float wn = w - q;
                if (keep && !keep[b * N + j]) wn = 0.0f;
                W[i] = wn;
                m[i] = mn;
                v[i] = vn;
            }
        }
}

/* Compression rate as the paper counts it (Sec. 4.4: 1.428x <=> 30 % sparsity):          */
/* dense parameters over kept parameters.                                                 */
double orc_compression_rate(int64_t M, int64_t N, int32_t R, int64_t kept_cols_total)
{
    if (kept_cols_total <= 0) return INFINITY;
    return ((double)M * (double)N) / ((double)R * (double)kept_cols_total);
}

/* ------------------------------------------------------------------------------------ */
/* Epilogue of a layer (Sec. 4.4 names the operations around the pruned product as what  */
/* a deployed layer fuses; the Transformer blocks of Sec. 4.2 follow the FFN              */
/* up-projection with GELU and the attention-output and FFN down-projections with a       */
/* residual addition).  Element-wise, on the unrounded sums Yd (bias already added):      */
/*   y = Yd;  act == 1: y = 0.5 y (1 + erf(y / sqrt 2))  (the exact GELU, BERT's form);    */
/*   residual != NULL: y += residual;  then one rounding to ydt.                          */
/* ------------------------------------------------------------------------------------ */
void orc_epilogue(const double *Yd, const float *residual, int64_t n, int32_t act, int32_t ydt,
                  float *Y, double *Ye)
{
    for (int64_t i = 0; i < n; ++i) {
        double y = Yd[i];
        if (act == 1) y = 0.5 * y * (1.0 + erf(y / sqrt(2.0)));
        if (residual) y += (double)residual[i];
        if (Ye) Ye[i] = y;
        if (Y) Y[i] = (float)orc_round(y, ydt);
    }
}

/* ------------------------------------------------------------------------------------ */
/* Gradient of the layer with respect to its kept weights (Alg. 2 updates W from the      */
/* gradient of the loss; for Y = X Wp^T + bias of Sec. 3.1 the chain rule gives           */
/* dW[m, j] = sum_t dY[t, m] X[t, j], needed on kept groups only), in the layout of the   */
/* value panels:                                                                          */
/*   dvals[R*blk_ptr[b] + r*kp_b + c] = sum_{t ascending} dY[t, bR + r] * X[t, col_idx[b, c]]  c < k_b */
/*                                    = +0                                                   pad  */
/* accumulated in double, then rounded to gdt.  Dd (double, same layout) is optional.     */
/* ------------------------------------------------------------------------------------ */
void orc_linear_dvals(const float *X, const float *dY, int64_t T, int64_t M, int64_t N, int32_t R,
                      const int32_t *blk_cnt, const int32_t *blk_ptr, const int32_t *col_idx,
                      int32_t gdt, float *D, double *Dd, int32_t n_threads)
{
    int64_t B = M / R;
    if (n_threads < 1) n_threads = 1;
#pragma omp parallel for num_threads(n_threads) schedule(dynamic, 1)
    for (int64_t b = 0; b < B; ++b) {
        int64_t base = blk_ptr[b];
        int32_t kp = blk_ptr[b + 1] - blk_ptr[b], kb = blk_cnt[b];
        for (int32_t r = 0; r < R; ++r)
            for (int32_t c = 0; c < kp; ++c) {
                double acc = 0.0;
                if (c < kb) {
                    int64_t j = col_idx[base + c];
                    for (int64_t t = 0; t < T; ++t)
                        acc += (double)dY[t * M + b * R + r] * (double)X[t * N + j];
                }
                int64_t at = R * base + (int64_t)r * kp + c;
                if (Dd) Dd[at] = acc;
                if (D) D[at] = (c < kb) ? (float)orc_round(acc, gdt) : 0.0f;
            }
    }
}

/* ------------------------------------------------------------------------------------ */
/* Whole-block pruning, the comparison of Sec. 4.4 / Table 4 ("block sparse": a block is  */
/* kept or removed as a whole).  A tile = the R rows of row-block b times the C columns   */
/* jC .. jC + C - 1.  Its sum of squares is the sum of its C column-group sums, added in  */
/* fp32, columns ascending, starting from +0 (the group sums s[b, j] are those of          */
/* orc_sumsq, so both sides build on bit-identical inputs).  N % C == 0.                   */
/*   ts[b, jt] = (((s[b, jtC] + s[b, jtC+1]) + ...) + s[b, jtC + C - 1])                    */
/* The decision (threshold or percentile) is then Alg. 1's, taken on ts by the functions  */
/* above, and orc_expand_tile_mask spreads a tile's decision over its C columns.          */
/* ------------------------------------------------------------------------------------ */
void orc_tile_sumsq(const float *s, int64_t B, int64_t N, int32_t C, float *ts)
{
    int64_t NT = N / C;
    for (int64_t b = 0; b < B; ++b)
        for (int64_t jt = 0; jt < NT; ++jt) {
            float acc = 0.0f;
            for (int32_t c = 0; c < C; ++c) acc = acc + s[b * N + jt * C + c];
            ts[b * NT + jt] = acc;
        }
}

void orc_expand_tile_mask(const uint8_t *tkeep, int64_t B, int64_t N, int32_t C, uint8_t *keep)
{
    int64_t NT = N / C;
    for (int64_t b = 0; b < B; ++b)
        for (int64_t j = 0; j < N; ++j) keep[b * N + j] = tkeep[b * NT + j / C] ? 1 : 0;
}

/* ------------------------------------------------------------------------------------ */
/* Group sums of the other division (Eq. 2; Alg. 1 as printed: the matrix is cut into     */
/* column blocks of C columns and the norm is taken over each row of a block), on the     */
/* matrix as it is stored:  s[m, q] = sum_{c ascending} W[m, qC + c]^2, fp32, one fused    */
/* multiply-add per element, starting from +0: the same canonical chain as orc_sumsq,     */
/* along a row segment instead of a column segment.  W: [M, N], N % C == 0; s: [M, N/C].   */
/* ------------------------------------------------------------------------------------ */
void orc_rowseg_sumsq(const float *W, int64_t M, int64_t N, int32_t C, float *s)
{
    int64_t Q = N / C;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t q = 0; q < Q; ++q) {
            float acc = 0.0f;
            for (int32_t c = 0; c < C; ++c) {
                float w = W[m * N + q * C + c];
                acc = fmaf(w, w, acc);
            }
            s[m * Q + q] = acc;
        }
}
