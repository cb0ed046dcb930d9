/*
 * TEST INFRASTRUCTURE -- not part of the product.
 *
 * CPU oracle for the FastGS rasterizer hot path (projection, Gaussian-tile pairs, depth
 * order, alpha compositing and its gradient, L1 term, error mask, per-Gaussian count of
 * high-error pixels).  Plain C, single-threaded, written from the paper's equations; see
 * fastgs_oracle_impl.h for the floating-point body, which is instantiated here for float
 * (suffix _f32, the pinned-operation-order build used for parity with the GPU) and double
 * (suffix _f64, used for finite differences and closed-form checks).
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math -shared -fPIC [-mfma] fastgs_oracle.c -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------------------- */
/* exp(x) for x <= 0 in the pinned fp32 form shared (as a specification, not as code) with
 * the GPU kernels:  t = x*log2(e) (clamped below at -125);  n = rint(t);  r = t - n;
 * p = degree-5 polynomial for 2^r on [-1/2,1/2] by Horner with fused multiply-adds;
 * result = p * 2^n.  Maximum relative error about 5e-7.                                   */
static float exp_neg_f32(float x)
{
    float t = x * 0x1.715476p+0f;
    if (t < -125.0f) t = -125.0f;
    float n = rintf(t);
    float r = t - n;
    float p = 0x1.5bba14p-10f;
    p = fmaf(p, r, 0x1.3cea88p-7f);
    p = fmaf(p, r, 0x1.c6b752p-5f);
    p = fmaf(p, r, 0x1.ebf9bcp-3f);
    p = fmaf(p, r, 0x1.62e42ap-1f);
    p = fmaf(p, r, 1.0f);
    return ldexpf(p, (int)n);
}

/* ln(x), x > 0, in a pinned fp32 form (used once per Gaussian by the Compact Box threshold):
 * x = m 2^e with m in [sqrt(1/2), sqrt(2)); s = (m-1)/(m+1); z = s*s;
 * ln m = 2 s (1 + z/3 + z^2/5 + z^3/7 + z^4/9) by Horner with fused multiply-adds; result = fma(e, ln2, ln m). */
static float log_c_f32(float x)
{
    int e;
    float m = frexpf(x, &e);                    /* m in [0.5, 1) */
    if (m < 0x1.6a09e6p-1f) { m = m + m; e = e - 1; }
    float s = (m - 1.0f) / (m + 1.0f);
    float z = s * s;
    float p = 0x1.c71c72p-4f;                   /* 1/9 */
    p = fmaf(p, z, 0x1.24924ap-3f);             /* 1/7 */
    p = fmaf(p, z, 0x1.99999ap-3f);             /* 1/5 */
    p = fmaf(p, z, 0x1.555556p-2f);             /* 1/3 */
    p = fmaf(p, z, 1.0f);
    float lnm = (s + s) * p;
    return fmaf((float)e, 0x1.62e43p-1f, lnm);
}
float orc_log_c_f32(float x) { return log_c_f32(x); }

#define REAL float
#define FN(name) name##_f32
#define SQRT sqrtf
#define CEIL ceilf
#define FLOOR floorf
#define FABS fabsf
#define FMIN fminf
#define FMAX fmaxf
#define FMA fmaf
#define EXPNEG exp_neg_f32
#define LOGC log_c_f32
#include "fastgs_oracle_impl.h"
#undef REAL
#undef FN
#undef SQRT
#undef CEIL
#undef FLOOR
#undef FABS
#undef FMIN
#undef FMAX
#undef FMA
#undef EXPNEG
#undef LOGC

#define REAL double
#define FN(name) name##_f64
#define SQRT sqrt
#define CEIL ceil
#define FLOOR floor
#define FABS fabs
#define FMIN fmin
#define FMAX fmax
#define FMA(a, b, c) ((a) * (b) + (c))
#define EXPNEG exp
#define LOGC log
#include "fastgs_oracle_impl.h"

/* exposed so a test can compare the pinned fp32 exponential with the library's */
float orc_exp_neg_f32(float x) { return exp_neg_f32(x); }

/* ------------------------------------------------------------------------------------- */
/* Integer part of the path: Gaussian-tile pairs, their order, per-tile ranges.           */

/* Step a2: exclusive prefix sum of tiles_touched; returns the total P.                   */
uint64_t orc_exclusive_scan(int64_t n, const uint32_t *touched, uint64_t *offsets)
{
    uint64_t run = 0;
    for (int64_t i = 0; i < n; i++) { offsets[i] = run; run += touched[i]; }
    return run;
}

/* Step a3: one (key, Gaussian) entry per tile of each Gaussian's rectangle, emitted in
 * Gaussian order, rows then columns.  key = tile_id << 32 | bit pattern of the fp32 depth
 * (depth > 0, so the unsigned bit pattern orders like the value); tile_id = ty*TX + tx.   */
uint64_t orc_emit_pairs(int64_t n, const int32_t *rect, const float *depth, int TX,
                        uint64_t *keys, uint32_t *vals)
{
    uint64_t p = 0;
    for (int64_t i = 0; i < n; i++) {
        uint32_t dbits;
        memcpy(&dbits, &depth[i], 4);
        for (int ty = rect[4 * i + 1]; ty < rect[4 * i + 3]; ty++)
            for (int tx = rect[4 * i + 0]; tx < rect[4 * i + 2]; tx++) {
                if (keys) {
                    keys[p] = ((uint64_t)(uint32_t)(ty * TX + tx) << 32) | dbits;
                    vals[p] = (uint32_t)i;
                }
                p++;
            }
    }
    return p;
}

/* Brute-force statement of which pairs exist: Gaussian i meets tile (tx,ty) iff the closed
 * square [mx-r, mx+r] x [my-r, my+r] intersects [tile*tx, tile*tx+tile) x [tile*ty, ...).
 * Evaluated in double on the stored fp32 values; used to pin the rectangle rounding.      */
uint64_t orc_pairs_bruteforce(int64_t n, const float *mean2d, const int32_t *radius, int width, int height,
                              int tile, uint8_t *hit /* [n, TY*TX] */)
{
    int TX = (width + tile - 1) / tile, TY = (height + tile - 1) / tile;
    uint64_t total = 0;
    for (int64_t i = 0; i < n; i++)
        for (int ty = 0; ty < TY; ty++)
            for (int tx = 0; tx < TX; tx++) {
                int h = 0;
                if (radius[i] > 0) {
                    double x0 = (double)mean2d[2 * i] - radius[i], x1 = (double)mean2d[2 * i] + radius[i];
                    double y0 = (double)mean2d[2 * i + 1] - radius[i], y1 = (double)mean2d[2 * i + 1] + radius[i];
                    h = x1 >= (double)tile * tx && x0 < (double)tile * (tx + 1) &&
                        y1 >= (double)tile * ty && y0 < (double)tile * (ty + 1);
                }
                hit[(size_t)i * TX * TY + (size_t)ty * TX + tx] = (uint8_t)h;
                total += h;
            }
    return total;
}

struct kv { uint64_t key; uint32_t val; };
static int kv_cmp(const void *pa, const void *pb)
{
    const struct kv *a = pa, *b = pb;
    if (a->key != b->key) return a->key < b->key ? -1 : 1;
    if (a->val != b->val) return a->val < b->val ? -1 : 1;
    return 0;
}

/* Steps a4: order the pairs by (tile, depth), ties by Gaussian index -- the C library sort. */
void orc_sort_pairs(uint64_t P, uint64_t *keys, uint32_t *vals)
{
    struct kv *a = malloc((P ? P : 1) * sizeof(*a));
    for (uint64_t i = 0; i < P; i++) { a[i].key = keys[i]; a[i].val = vals[i]; }
    qsort(a, P, sizeof(*a), kv_cmp);
    for (uint64_t i = 0; i < P; i++) { keys[i] = a[i].key; vals[i] = a[i].val; }
    free(a);
}

/* Step a5: ranges[t] = [first, last) positions of tile t in the ordered list (0,0 if empty). */
void orc_tile_ranges(uint64_t P, const uint64_t *keys_sorted, int num_tiles, uint32_t *ranges)
{
    memset(ranges, 0, (size_t)num_tiles * 2 * sizeof(uint32_t));
    for (uint64_t i = 0; i < P; i++) {
        uint32_t t = (uint32_t)(keys_sorted[i] >> 32);
        if (i == 0 || (uint32_t)(keys_sorted[i - 1] >> 32) != t) ranges[2 * t] = (uint32_t)i;
        if (i + 1 == P || (uint32_t)(keys_sorted[i + 1] >> 32) != t) ranges[2 * t + 1] = (uint32_t)(i + 1);
    }
}

/* ------------------------------------------------------------------------------------- */
/* Photometric loss of Sec. 4.3 / Sec. 4.5:  E = (1 - lambda) L1 + lambda (1 - SSIM).
 * The paper cites the structural-similarity index without restating it; the reading taken is
 * the usual one for Gaussian-splatting losses: per channel, local statistics under an 11x11
 * Gaussian window (standard deviation 1.5 px, normalised to sum 1, the outer product of two
 * 11-tap windows), the image continued by zeros outside its border, C1 = 0.01^2, C2 = 0.03^2
 * (dynamic range 1), and the mean of the SSIM map over all channels and pixels.
 * Everything here is double precision and written as the plain 121-tap definition.            */

#define SSIM_R 5
static void ssim_window(double w[2 * SSIM_R + 1])
{
    double s = 0;
    for (int k = -SSIM_R; k <= SSIM_R; k++) { w[k + SSIM_R] = exp(-(double)(k * k) / (2.0 * 1.5 * 1.5)); s += w[k + SSIM_R]; }
    for (int k = 0; k <= 2 * SSIM_R; k++) w[k] /= s;
}

/* out(v,u) = sum_{i,j} w_i w_j in(v+i, u+j), terms outside the plane dropped */
static void window_sum(int H, int W, const double *in, const double w[2 * SSIM_R + 1], double *out)
{
    for (int v = 0; v < H; v++)
        for (int u = 0; u < W; u++) {
            double s = 0;
            for (int i = -SSIM_R; i <= SSIM_R; i++) {
                if (v + i < 0 || v + i >= H) continue;
                for (int j = -SSIM_R; j <= SSIM_R; j++) {
                    if (u + j < 0 || u + j >= W) continue;
                    s += w[i + SSIM_R] * w[j + SSIM_R] * in[(size_t)(v + i) * W + (u + j)];
                }
            }
            out[(size_t)v * W + u] = s;
        }
}

/* SSIM map [C,H,W] of x against y, its mean, and (if grad != NULL) d mean / d x.
 * With mu1 = <x>, mu2 = <y>, e11 = <x^2>, e22 = <y^2>, e12 = <x y> (window sums):
 *   s1 = e11 - mu1^2, s2 = e22 - mu2^2, s12 = e12 - mu1 mu2,
 *   ssim = (2 mu1 mu2 + C1)(2 s12 + C2) / ((mu1^2 + mu2^2 + C1)(s1 + s2 + C2)).
 * The gradient follows from the chain rule through (mu1, e11, e12), each a window sum of x, x^2, x y. */
double orc_ssim(int C, int H, int W, const double *x, const double *y, double *map, double *grad)
{
    const double C1 = 0.01 * 0.01, C2 = 0.03 * 0.03;
    double w[2 * SSIM_R + 1];
    ssim_window(w);
    size_t n = (size_t)H * W;
    double *t = malloc(sizeof(double) * n * 9);
    double *xx = t, *yy = t + n, *xy = t + 2 * n, *mu1 = t + 3 * n, *mu2 = t + 4 * n, *e11 = t + 5 * n,
           *e22 = t + 6 * n, *e12 = t + 7 * n, *tmp = t + 8 * n;
    double total = 0;
    for (int c = 0; c < C; c++) {
        const double *xc = x + c * n, *yc = y + c * n;
        for (size_t p = 0; p < n; p++) { xx[p] = xc[p] * xc[p]; yy[p] = yc[p] * yc[p]; xy[p] = xc[p] * yc[p]; }
        window_sum(H, W, xc, w, mu1);
        window_sum(H, W, yc, w, mu2);
        window_sum(H, W, xx, w, e11);
        window_sum(H, W, yy, w, e22);
        window_sum(H, W, xy, w, e12);
        /* reuse xx, yy, xy for the three derivative maps */
        for (size_t p = 0; p < n; p++) {
            double m1 = mu1[p], m2 = mu2[p];
            double s1 = e11[p] - m1 * m1, s2 = e22[p] - m2 * m2, s12 = e12[p] - m1 * m2;
            double A = 2 * m1 * m2 + C1, B = 2 * s12 + C2, Cq = m1 * m1 + m2 * m2 + C1, D = s1 + s2 + C2;
            double s = (A * B) / (Cq * D);
            if (map) map[c * n + p] = s;
            total += s;
            /* d ssim / d mu1, / d e11, / d e12 with the other window sums held fixed */
            xx[p] = (2 * m2 * (B - A) - s * 2 * m1 * (D - Cq)) / (Cq * D);
            yy[p] = -s / D;
            xy[p] = 2 * A / (Cq * D);
        }
        if (grad) {
            double inv = 1.0 / ((double)C * (double)n);
            window_sum(H, W, xx, w, tmp);
            for (size_t p = 0; p < n; p++) grad[c * n + p] = tmp[p] * inv;
            window_sum(H, W, yy, w, tmp);
            for (size_t p = 0; p < n; p++) grad[c * n + p] += 2 * xc[p] * tmp[p] * inv;
            window_sum(H, W, xy, w, tmp);
            for (size_t p = 0; p < n; p++) grad[c * n + p] += yc[p] * tmp[p] * inv;
        }
    }
    free(t);
    return total / ((double)C * (double)n);
}

/* VCP pruning score (Sec. 4.3): s_p = N( sum_j count_i^j * E_photo^j ), N = min-max normalisation
 * over the Gaussians (all zeros when every sum is equal).  counts: [K,n] row-major.            */
void orc_prune_score(int K, int64_t n, const int32_t *counts, const double *E, double *raw, double *score)
{
    double lo = 0, hi = 0;
    for (int64_t i = 0; i < n; i++) {
        double s = 0;
        for (int j = 0; j < K; j++) s += (double)counts[(size_t)j * n + i] * E[j];
        raw[i] = s;
        if (i == 0 || s < lo) lo = s;
        if (i == 0 || s > hi) hi = s;
    }
    for (int64_t i = 0; i < n; i++) score[i] = hi > lo ? (raw[i] - lo) / (hi - lo) : 0.0;
}
