// Internal declarations shared by the HIP translation units of libfastgs_hip (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fastgs.h"

namespace fs {

constexpr int TILE = 16;           // pixels per tile edge (the binning unit of the ABI)
constexpr int TILE_PIX = TILE * TILE;

// Camera and conventions as passed by value to kernels.
struct CamDev {
    int width, height;
    float fx, fy, cx, cy;
    float R[9];
    float t[3];
    int tiles_x, tiles_y;
};

struct CfgDev {
    float z_near, lowpass, alpha_min, alpha_max, T_min;
    float bg[3];
    float jclamp;
    float power_min;  // exponents below this cannot reach alpha_min for opacity <= 1 (conservative)
    int score_mode;
    int compact_box;  // pairs from the ellipse-tile test instead of the 3-sigma square
    float cb_beta;
};

// ---- Compact Box (FastGS Sec. 4.4 and its supplement) ------------------------------------------
// Support of a Gaussian: (p - mu_2D)^T Sigma_2D^-1 (p - mu_2D) <= Q, Q = beta * 2 ln(sigma / tau_alpha)
// with tau_alpha = alpha_min.  These three functions decide integers (pair counts, which keys exist),
// so their fp32 operation order is fixed: plain IEEE operations as written, fused multiply-adds only
// where spelled out.

// ln(x) for x > 0: x = m 2^e, m in [sqrt(1/2), sqrt(2)); s = (m-1)/(m+1); z = s^2;
// ln m = 2 s (1 + z/3 + z^2/5 + z^3/7 + z^4/9) by Horner with fmaf; ln x = fmaf(e, ln 2, ln m).
__device__ __forceinline__ float log_c(float x)
{
    int e;
    float m = frexpf(x, &e);
    if (m < 0x1.6a09e6p-1f) { m = m + m; e = e - 1; }
    const float s = (m - 1.0f) / (m + 1.0f);
    const float z = s * s;
    float p = 0x1.c71c72p-4f;
    p = __builtin_fmaf(p, z, 0x1.24924ap-3f);
    p = __builtin_fmaf(p, z, 0x1.99999ap-3f);
    p = __builtin_fmaf(p, z, 0x1.555556p-2f);
    p = __builtin_fmaf(p, z, 1.0f);
    const float lnm = (s + s) * p;
    return __builtin_fmaf((float)e, 0x1.62e43p-1f, lnm);
}

// Q of a Gaussian of opacity sigma; 0 when it can never reach alpha_min.
__device__ __forceinline__ float cb_threshold(float sigma, const CfgDev& cfg)
{
    const float ratio = sigma / cfg.alpha_min;
    if (!(ratio > 1.0f)) return 0.0f;
    return cfg.cb_beta * (2.0f * log_c(ratio));
}

// Does the closed rectangle of tile (tx, ty) meet the ellipse?  The quadratic form is convex with its
// minimum at mu_2D: the minimum over the rectangle is 0 when mu_2D is inside, and otherwise lies on the
// vertical and/or horizontal edge that faces mu_2D, where it is a 1-D quadratic with a clamped minimiser.
__device__ __forceinline__ bool cb_tile_hit(float mx, float my, float A, float B, float C, float Q, int tx, int ty)
{
    const float X0 = (float)(tx * TILE), X1 = (float)(tx * TILE + TILE);
    const float Y0 = (float)(ty * TILE), Y1 = (float)(ty * TILE + TILE);
    const float dxl = X0 - mx, dxr = X1 - mx, dyt = Y0 - my, dyb = Y1 - my;
    const bool in_x = dxl <= 0.0f && dxr >= 0.0f;
    const bool in_y = dyt <= 0.0f && dyb >= 0.0f;
    if (in_x && in_y) return true;
    const float B2 = B + B;
    bool have = false;
    float qmin = 0.0f;
    if (!in_x) {
        const float ex = dxl > 0.0f ? dxl : dxr;
        float dys = -(B * ex) / C;
        dys = fminf(fmaxf(dys, dyt), dyb);
        qmin = __builtin_fmaf(ex, __builtin_fmaf(B2, dys, A * ex), (C * dys) * dys);
        have = true;
    }
    if (!in_y) {
        const float ey = dyt > 0.0f ? dyt : dyb;
        float dxs = -(B * ey) / A;
        dxs = fminf(fmaxf(dxs, dxl), dxr);
        const float q = __builtin_fmaf(dxs, __builtin_fmaf(B2, ey, A * dxs), (C * ey) * ey);
        if (!have || q < qmin) qmin = q;
    }
    return qmin <= Q;
}

// ---- workgroup reductions in double precision (fixed tree: results do not depend on scheduling) ----------
constexpr int RED_BLOCKS = 1024;  // partial sums per reduction (a multiple of RED_THREADS)
constexpr int RED_THREADS = 256;

__device__ __forceinline__ double shfl_down_f64(double v, int d)
{
    const long long b = __double_as_longlong(v);
    const int lo = __shfl_down((int)(b & 0xffffffffll), d, 64);
    const int hi = __shfl_down((int)(b >> 32), d, 64);
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}

enum RedOp { RED_SUM, RED_MIN, RED_MAX };

template <RedOp OP>
__device__ __forceinline__ double red_combine(double a, double b)
{
    if (OP == RED_SUM) return a + b;
    if (OP == RED_MIN) return a < b ? a : b;
    return a > b ? a : b;
}

// Reduces one value per thread over the workgroup; the result is valid in thread 0.
template <RedOp OP>
__device__ __forceinline__ double block_reduce(double v, double* smem /*[4]*/)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v = red_combine<OP>(v, shfl_down_f64(v, d));
    __syncthreads();
    if ((threadIdx.x & 63) == 0) smem[threadIdx.x >> 6] = v;
    __syncthreads();
    if (threadIdx.x == 0) v = red_combine<OP>(red_combine<OP>(smem[0], smem[1]), red_combine<OP>(smem[2], smem[3]));
    return v;
}

template <RedOp OP>
__device__ __forceinline__ double red_identity()
{
    if (OP == RED_SUM) return 0.0;
    if (OP == RED_MIN) return 1.0e300;
    return -1.0e300;
}

// ---- launchers (each enqueues on `st` and returns hipGetLastError()) ------------------------
hipError_t launch_preprocess(hipStream_t st, int64_t n, int deg, const fs_gaussians& g, const CamDev& cam,
                             const CfgDev& cfg, const fs_projected& out);
// pair_grad: records of PAIR_REC floats (see render.hip); Gaussian i owns records
// [rec_offsets[i], rec_offsets[i] + rec_counts[i]); touched as in fs_projected (0 = not visible)
constexpr int PAIR_REC = 12;
hipError_t launch_preprocess_bwd(hipStream_t st, int64_t n, int deg, const fs_gaussians& g, const CamDev& cam,
                                 const CfgDev& cfg, const uint8_t* clamped, const uint32_t* touched,
                                 const uint32_t* rec_counts, const uint32_t* rec_offsets, const float* pair_grad, uint8_t* rec_valid,
                                 const fs_grads& out);

// exclusive scan of n uint32 values; total (uint64) written to *total_dev. tmp: >= scan_tmp_bytes(n).
size_t scan_tmp_bytes(int64_t n);
hipError_t launch_exclusive_scan(hipStream_t st, const uint32_t* in, uint32_t* out, int64_t n, void* tmp,
                                 uint64_t* total_dev);

// Splat record (SPLAT_REC floats = 64 bytes, one per Gaussian): mx my a b | c sigma r g | b offset rect01 rect23 | unused
constexpr int SPLAT_REC = 16;
hipError_t launch_emit_pairs(hipStream_t st, int64_t n, const fs_projected& proj, const uint32_t* offsets,
                             int tiles_x, uint64_t* keys, uint32_t* vals, float* splats);
// Compact Box: rec_counts[i] = tiles in Gaussian i's box (the candidates of the ellipse test)
hipError_t launch_rect_area(hipStream_t st, int64_t n, const uint16_t* rect, uint32_t* rec_counts);
// Compact Box emission: one key per candidate tile that meets the ellipse, at offsets[i] + its rank among
// the Gaussian's hits; the gradient record of every candidate that misses (rec_offsets[i] + row-major
// place in the box) is zeroed, since no render workgroup will ever write it.
hipError_t launch_emit_pairs_cb(hipStream_t st, int64_t n, const fs_projected& proj, const CfgDev& cfg,
                                const uint32_t* offsets, const uint32_t* rec_offsets, int tiles_x, int64_t P,
                                uint64_t* keys, uint32_t* vals, float* splats, float* pair_grad);

// Tile-bucketed ordering (used when no tile's list is longer than TILE_SORT_HUGE; otherwise the global
// radix sort below): per-tile counts and ranges, then placement into the tiles' segments and an LDS sort
// of every segment.  ranges/tile_order/tile_total: [num_tiles]; tile_count: [TILE_COPIES, num_tiles], turned by
// launch_tile_count into each copy's start within its tile (the `cursor` of launch_tile_scatter_sort).
// launch_tile_count also gives every Gaussian the place of its backward records (rec_offsets [n]: disjoint,
// contiguous per Gaussian, not ordered by index; rec_counts [n], may be null: the area of its rectangle) from
// `counters` (two uint64 that are zero at the start and are left zero), and writes
// totals [4] = {sum of proj.tiles_touched, records handed out, pairs counted per tile, longest list}.
constexpr int TILE_COPIES = 256;        // workgroups of the counting / placement kernels, each with its own counters (a multiple of 64)
constexpr int TILE_PAIR_THREADS = 1024;
constexpr int TILE_LDS_MAX_TILES = 15360;  // their per-tile counters live in LDS (60 KB)
constexpr int TILE_SORT_GROUP16_FROM = 1024;  // padded list length from which a thread merges 16 words in registers, not 8
constexpr int TILE_SORT_SMALL = 2048;  // longest list one workgroup sorts with 20 KB of LDS (256 threads)
constexpr int TILE_SORT_MID = 4096;    // ... with 40 KB (512 threads: four such workgroups fit a compute unit, two of the next)
constexpr int TILE_SORT_MAX = 8192;    // ... with 80 KB (1024 threads)
constexpr int TILE_SORT_HUGE = 16384;  // ... with 144 KB (a compute unit of this chip has 160 KB): the longest list of the
                                       // per-tile ordering; anything longer takes the radix path
hipError_t launch_tile_count(hipStream_t st, int64_t n, const fs_projected& proj, const CfgDev& cfg, int tiles_x,
                             int num_tiles, uint32_t* tile_count, uint32_t* tile_total, uint2* ranges,
                             uint32_t* tile_order, uint64_t* totals, uint32_t* rec_offsets, uint32_t* rec_counts,
                             uint64_t* counters);
// Placement and the per-tile sorts.  pair_limit / rec_limit: how many words / gradient records the buffers hold; the
// kernels write nothing at or beyond them and leave alone a segment that reaches beyond pair_limit, so they may be
// enqueued before the host knows the totals.
hipError_t launch_tile_scatter(hipStream_t st, int64_t n, const fs_projected& proj, const CfgDev& cfg,
                               const uint32_t* rec_offsets, int tiles_x, int num_tiles, uint32_t pair_limit,
                               uint32_t rec_limit, const uint2* ranges, uint32_t* cursor, uint64_t* bucket, float* splats,
                               float* pair_grad);
// The sort launches, by the list lengths they take: (0, SMALL], (SMALL, MID], (MID, MAX], (MAX, HUGE], and
// (SMALL, MAX] in one launch (TS_MIDMAX, instead of TS_MID and TS_MAX).  The lists between SMALL and MID get a launch of
// their own (four of its workgroups fit a compute unit, two of the MAX kind) when the lists are long throughout
// (`long_lists`: there are then enough of them to fill the chip); when only a few tiles are that long, every launch is
// a chain of steps that nothing overlaps with, and one launch fewer is the better deal.
// tile_sort_variants: the launches still needed for lists of up to max_len entries when those in `have` are enqueued.
enum { TS_SMALL = 1, TS_MID = 2, TS_MAX = 4, TS_HUGE = 8, TS_MIDMAX = 16 };
int tile_sort_variants(int64_t max_len, bool long_lists, int have);
hipError_t launch_tile_sorts(hipStream_t st, int num_tiles, int variants, uint32_t pair_limit, const uint2* ranges,
                             const uint32_t* tile_order, const uint64_t* bucket, uint64_t* keys_out, uint32_t* vals_out);

constexpr int RADIX_BLOCK_KEYS = 2048;  // keys ranked by one workgroup per pass
constexpr int RADIX_BITS = 9;            // widest digit
constexpr int RADIX_DIGITS = 1 << RADIX_BITS;
inline int64_t radix_num_blocks(int64_t P) { return (P + RADIX_BLOCK_KEYS - 1) / RADIX_BLOCK_KEYS; }
// Stable LSD sort of P (key,val) pairs on key bits [0,total_bits). Result ends in *keys_out/*vals_out,
// which point into one of the two ping-pong buffers. hist: RADIX_DIGITS*radix_num_blocks(P) uint32.
hipError_t launch_radix_sort(hipStream_t st, int64_t P, int total_bits, uint64_t* keys[2], uint32_t* vals[2],
                             uint32_t* hist, void* scan_tmp, uint64_t* scan_total_dev, int* result_index);

// ranges [num_tiles,2] and tile_order [num_tiles] (tiles by decreasing list length)
hipError_t launch_tile_ranges(hipStream_t st, int64_t P, const uint64_t* keys_sorted, int num_tiles,
                              uint32_t* ranges, uint32_t* tile_order);

// The threshold of the mask from the error map's statistics (Sec. 4.2, second and third equations): mean + k * std
// with the population variance taken as mean(e^2) - mean(e)^2 in double precision (e lies in [0, 1] and the sums
// are exact to about 1e-13, far below what the single-precision threshold resolves), or min + k * (max - min).
__device__ __forceinline__ float threshold_from_stats(double sum, double lo, double hi, double sumsq, int64_t pixels,
                                                      int rule, float k)
{
    if (rule == FS_MASK_MEAN_STD) {
        const double mean = sum / (double)pixels;
        double var = sumsq / (double)pixels - mean * mean;
        var = var > 0.0 ? var : 0.0;
        return (float)(mean + (double)k * sqrt(var));
    }
    const float l = (float)lo, h = (float)hi;
    return l + k * (h - l);
}

// The record a forward pass leaves for the count pass (see k_score_bits).  For every pair that the multi-view score
// counts at one or more pixels of its tile: a row of PAIR_BITS_BYTES (which pixels) and the pair's Gaussian.  The rows of
// a tile sit together at the start of the tile's segment of the pair arrays, [ranges[tile].x, + tile_rows[tile]), in no
// particular order; pairs that are counted nowhere leave nothing.  rows == null: no record.
constexpr int PAIR_BITS_BYTES = 32;
struct ScoreRecord {
    uint4* rows;           // [P, 2]
    uint32_t* row_gauss;   // [P]
    int32_t* tile_rows;    // [tiles]
};
inline size_t score_record_bytes(int64_t num_pairs, int tiles)
{
    return (size_t)num_pairs * (PAIR_BITS_BYTES + sizeof(uint32_t)) + (size_t)tiles * sizeof(int32_t);
}
inline ScoreRecord score_record_at(void* base, int64_t num_pairs)
{
    unsigned char* b = static_cast<unsigned char*>(base);
    ScoreRecord r;
    r.rows = reinterpret_cast<uint4*>(b);
    r.row_gauss = reinterpret_cast<uint32_t*>(b + (size_t)num_pairs * PAIR_BITS_BYTES);
    r.tile_rows = reinterpret_cast<int32_t*>(b + (size_t)num_pairs * (PAIR_BITS_BYTES + sizeof(uint32_t)));
    return r;
}
hipError_t launch_render_fwd(hipStream_t st, const CamDev& cam, const CfgDev& cfg, const uint32_t* ranges,
                             const uint32_t* tile_order, const uint32_t* gauss_sorted, const float* splats, float* image, float* final_T,
                             uint32_t* n_contrib, const ScoreRecord& record);

// forward pass with the L1 term and the error map fused into its epilogue (see k_render_fwd);
// tile_partial: 5 * tiles doubles, err: H*W floats, dL may be null; record as for launch_render_fwd
hipError_t launch_render_fwd_fused(hipStream_t st, const CamDev& cam, const CfgDev& cfg, const uint32_t* ranges,
                                   const uint32_t* tile_order, const uint32_t* gauss_sorted, const float* splats,
                                   float* image, float* final_T, uint32_t* n_contrib, const float* target, float* dL,
                                   float* err, double* tile_partial, const ScoreRecord& record);
// the count pass from that record: counts[g] += |bits(row) & mask(tile)| over the rows of every tile
// (longest_list: an upper bound of the rows of any tile, 0 if not known)
hipError_t launch_score_bits(hipStream_t st, const CamDev& cam, const uint32_t* ranges, const ScoreRecord& record,
                             const uint8_t* mask, int32_t* counts, int64_t longest_list);
// the same with the mask made on the way: mask[p] <- err[p] > threshold(stats, rule, k) for every pixel (stats: the four
// doubles {sum, min, max, sum of squares} of the error map), *thr_out <- the threshold, then the count as above
hipError_t launch_mask_score_bits(hipStream_t st, const CamDev& cam, const uint32_t* ranges, const ScoreRecord& record,
                                  const float* err, const double* stats, int rule, float k, uint8_t* mask, float* thr_out,
                                  int32_t* counts, int64_t longest_list);
// rows[tile] <- the record's number of rows of the tile
hipError_t launch_record_rows(hipStream_t st, int tiles, const ScoreRecord& record, int32_t* rows);
// stats: >= fused_partials() doubles: {sum, min, max, sum of squares} of the error map
int fused_partials();
hipError_t launch_fold_tile_partials(hipStream_t st, const double* tile_partial, int tiles, int64_t count,
                                     double* stats, double* loss_out);
hipError_t launch_error_mask_from_map(hipStream_t st, int64_t pixels, int rule, float k, const float* err,
                                      const double* stats, uint8_t* mask, float* thr);

hipError_t launch_render_bwd(hipStream_t st, const CamDev& cam, const CfgDev& cfg, const uint32_t* ranges,
                             const uint32_t* tile_order, const uint32_t* gauss_sorted, const float* splats, const float* final_T,
                             const uint32_t* n_contrib, const float* dL_dimage, float* pair_grad, uint8_t* rec_valid,
                             bool abs_grad, bool per_splat);

hipError_t launch_score(hipStream_t st, const CamDev& cam, const CfgDev& cfg, const uint32_t* ranges,
                        const uint32_t* tile_order, const uint32_t* gauss_sorted, const float* splats, const uint32_t* n_contrib,
                        const uint8_t* mask, int32_t* counts);

hipError_t launch_l1_grad(hipStream_t st, const float* image, const float* target, int64_t count,
                          float* dL, double* partial /* >= l1_partials() doubles */, double* loss_out);
int l1_partials();

// err: [H*W] floats, partial: >= 4*mask_partials() doubles
hipError_t launch_error_mask(hipStream_t st, const float* image, const float* target, int64_t pixels, int rule,
                             float k, float* err, double* partial, uint8_t* mask, float* thr_out);
int mask_partials();

// Photometric loss (1-lambda) L1 + lambda (1 - SSIM).  dmaps: 3 * 3*H*W floats (only touched when dL != null);
// partial: >= 2 * photo_blocks(H, W) doubles; dL (may be null): dE/d image; out3 (may be null): {L1, SSIM, E}.
int photo_blocks(int H, int W);
hipError_t launch_photo_loss(hipStream_t st, const float* image, const float* target, int H, int W, float lambda,
                             float* dmaps, double* partial, float* dL, double* out3);
// acc[i] += counts[i] * *E;  then out = min-max normalised acc (partial: >= 2*mask_partials() + 2 doubles)
hipError_t launch_prune_accumulate(hipStream_t st, const int32_t* counts, int64_t n, const double* E, double* acc);
hipError_t launch_prune_normalize(hipStream_t st, const double* acc, int64_t n, double* partial, float* out);

// densification / pruning decisions and index plumbing (densify.hip)
hipError_t launch_densify_accumulate(hipStream_t st, int64_t n, const float* dmean2d, const float* dabs,
                                     const uint32_t* touched, float* grad_accum, float* abs_accum, uint32_t* denom);
hipError_t launch_select(hipStream_t st, int64_t n, const float* grad_accum, const float* abs_accum,
                         const uint32_t* denom, const int32_t* counts, const float* scales, const float* opac,
                         const float* s_p, const fs_select_params& prm, uint8_t* clone, uint8_t* split, uint8_t* prune);
// positions: uint32 [n] scratch; total_dev receives the number of selected elements
hipError_t launch_compact(hipStream_t st, int64_t n, const uint8_t* mask, uint32_t* positions, void* scan_tmp,
                          uint64_t* total_dev, uint32_t* indices);
hipError_t launch_gather_rows(hipStream_t st, const float* src, int row_floats, const uint32_t* indices,
                              int64_t count, float* dst);

hipError_t launch_combine_masks(hipStream_t st, int64_t n, const uint8_t* clone, const uint8_t* split,
                                const uint8_t* prune, uint8_t* keep, uint8_t* clone_eff, uint8_t* split_eff);
hipError_t launch_counts_add(hipStream_t st, int64_t n, int32_t* total, const int32_t* view);
// children of m split parents: rows c*m + r of child_means / child_scales [2m,3]; normals [m,2,3]
hipError_t launch_split_children(hipStream_t st, int64_t m, const float* means, const float* scales, const float* quats,
                                 const uint32_t* parents, const float* normals, float phi, float* child_means,
                                 float* child_scales);
// keys[j] = bits(exponentials[i] / scores[i]) << 32 | i, vals[j] = i for the m listed candidates i = cand_idx[j]
hipError_t launch_sample_keys(hipStream_t st, int64_t m, const uint32_t* cand_idx, const float* scores,
                              const float* exponentials, uint64_t* keys, uint32_t* vals);
// mask[0..n) = 0, then mask[idx[j]] = 1 for j < k
hipError_t launch_mark_indices(hipStream_t st, int64_t n, int64_t k, const uint32_t* idx, uint8_t* mask);

// optimiser and activations (optimizer.hip)
hipError_t launch_adam(hipStream_t st, float* p, float* g, float* m, float* v, int64_t count, float lr, float beta1,
                       float beta2, float eps, int step, float grad_scale, bool zero_grad);
hipError_t launch_grad_accumulate(hipStream_t st, float* acc, const float* g, int64_t count);
hipError_t launch_activate(hipStream_t st, int64_t n, const float* raw_s, const float* raw_q, const float* raw_o,
                           float* s, float* q, float* o);
hipError_t launch_activate_bwd(hipStream_t st, int64_t n, const float* raw_s, const float* raw_q, const float* raw_o,
                               const float* d_s, const float* d_q, const float* d_o, float* d_raw_s, float* d_raw_q,
                               float* d_raw_o);
hipError_t launch_activate_inv(hipStream_t st, int64_t n, const float* s, const float* o, float lo, float hi,
                               float* raw_s, float* raw_o);

// reference measurements: streaming copy of `bytes` (multiple of 16), and 8 fma chains x iters per lane on
// blocks x 256 lanes (out: blocks * 256 floats)
hipError_t launch_copy(hipStream_t st, const void* src, void* dst, int64_t bytes);
hipError_t launch_fma_chain(hipStream_t st, float* out, int blocks, int iters);

hipError_t launch_fill_u32(hipStream_t st, uint32_t* p, uint32_t v, int64_t count);

}  // namespace fs
