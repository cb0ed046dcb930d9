/*
 * fastgs.h -- C ABI of the MI355X (gfx950) FastGS rasterizer hot path.
 *
 * What it computes (paper: FastGS, Sec. 3 "Background: 3D Gaussian Splatting", Sec. 4.2
 * "Multi-view Consistent Densification", Sec. 4.3 "Multi-view Consistent Pruning", Sec. 4.4 "Compact Box",
 * Sec. 4.5 "Optimization", and the supplement's "Details of Compact Box" and "Implementation Details"):
 *   fs_preprocess        projection of every Gaussian to a screen-space splat   (Eqs. (2), (3))
 *   fs_bin_sort          Gaussian-tile pairs, ordered by (tile, depth)          (Sec. 3, "sorted by depth")
 *   fs_render_fwd        front-to-back alpha compositing                        (Eqs. (4), (5))
 *   fs_l1_grad           L1 term of the training loss and dL/dC                 (Sec. 4.5)
 *   fs_render_fwd_loss / fs_error_mask_fused
 *                        the forward pass with the L1 term and the error map fused into it
 *   fs_render_bwd        gradient of a loss w.r.t. every Gaussian parameter     (chain rule of Eqs. (2)-(5))
 *   fs_set_backward_mode per-pixel (default) or per-splat-parallel mapping of it (Sec. 5.3: the baseline's backward)
 *   fs_set_record_mode   dense or sparse per-pair gradient records between its two kernels
 *   fs_error_mask        per-pixel L1 error map and high-error mask             (Sec. 4.2, first three equations)
 *   fs_score_accumulate  per-Gaussian count of high-error pixels it contributes to,
 *                        one view per call                                      (Sec. 4.2, Eq. for s_d)
 *   fs_set_score_record  whether the forward passes keep the per-pair record that this count is taken from
 *   fs_mask_score_fused  fs_error_mask_fused + fs_score_accumulate as one call (one kernel launch with the record)
 *   fs_score_record_rows how many pairs of every tile that record holds a row for (a diagnostic)
 *   fs_photo_loss        E = (1-lambda) L1 + lambda (1 - SSIM) and dE/dC        (Sec. 4.3 E_photo; Sec. 4.5 Eq. for L)
 *   fs_prune_score_accumulate / fs_prune_score_normalize
 *                        s_p = N(sum over views of count * E_photo)             (Sec. 4.3, Eq. for s_p)
 *   fs_adam_step / fs_grad_accumulate / fs_adam_interval / fs_activate / fs_activate_bwd
 *                        fused Adam update with the 32/64 schedule, parameter activations
 *                                                                               (Sec. 5.1, supplement)
 *   fs_densify_accumulate / fs_select / fs_combine_masks / fs_compact / fs_gather_rows
 *                        gradient statistics, clone / split / prune masks, index lists and row copies
 *                                                                               (Sec. 4.2, 4.3, supplement)
 *   fs_split_children / fs_sample_by_score / fs_counts_add / fs_activate_inv
 *                        the children of split Gaussians, the early-phase sampling of half the pruning
 *                        candidates by score, per-view count sums, stored parameters from used ones
 *                                                                               (supplement, "Implementation Details")
 *
 * General rules
 *   - Every pointer inside the structs below is a DEVICE pointer (HIP, the ctx's device) owned
 *     by the caller unless marked "ctx-owned"; structs themselves live in host memory.
 *   - Arrays are dense, row-major, 4-byte aligned (16-byte for [n,4] float arrays); fp32 unless
 *     stated.  Nothing is freed or reallocated on the caller's behalf.
 *   - Work is enqueued on the stream given to fs_create, and a call may return with its work still in
 *     flight there: the arrays it was given must stay valid, and must only be touched by work ordered
 *     after it on that stream, until then.  fs_compact reads 8 bytes back (the count), fs_sample_by_score
 *     8, and fs_measure_peaks / fs_profile_read wait for their measurements: these synchronise the
 *     stream.  fs_bin_sort reads 32 bytes back (the pair count and what it needs to choose its path) and
 *     waits for the kernels that make them, but may return with its last kernels still running.
 *   - Every call returns FS_OK (0) or a negative fs_status and never throws or aborts;
 *     fs_last_error gives a message for the last failure on that ctx.
 *   - n = 0 Gaussians and P = 0 pairs are valid (the image is the background).
 *   - A ctx must not be used from two threads at once.
 */
#ifndef FASTGS_H
#define FASTGS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FS_OK = 0,
    FS_EINVAL = -1,    /* null pointer, bad shape / degree / size                     */
    FS_ENOMEM = -2,    /* growing the ctx's scratch memory failed                      */
    FS_EHIP = -3,      /* a HIP runtime call failed (message has the HIP error name)  */
    FS_ECAPACITY = -4  /* a count (Gaussians, pairs, candidate tiles) reaches 2^31      */
} fs_status;

enum { FS_SCORE_WEIGHT = 0, FS_SCORE_ALPHA = 1 };
enum { FS_MASK_MEAN_STD = 0, FS_MASK_MINMAX_TAU = 1 };
enum { FS_SORT_AUTO = 0, FS_SORT_RADIX = 1 };

/* Conventions the paper leaves open; fs_default_config fills in the documented defaults. */
typedef struct {
    int32_t tile;       /* tile edge in pixels; only 16 is supported                                  */
    float z_near;       /* Gaussians with camera depth <= z_near are culled (0.2)                     */
    float lowpass;      /* added to both diagonal entries of Sigma_2D, in px^2 (0.3)                  */
    float alpha_min;    /* alphas below it are not blended (1/255)                                    */
    float alpha_max;    /* alpha cap (0.99)                                                           */
    float T_min;        /* a pixel stops before its transmittance would fall below this (1e-4)        */
    float bg[3];        /* background colour                                                          */
    float jclamp;       /* t_x/t_z, t_y/t_z used inside J are limited to jclamp*tan(fov/2); <=0: off (1.3) */
    int32_t score_mode; /* FS_SCORE_WEIGHT: count where alpha*T > alpha_min; FS_SCORE_ALPHA: where blended */
    int32_t compact_box; /* 0: pairs from the 3-sigma square; 1: Compact Box (Sec. 4.4): a (Gaussian, tile) pair
                            exists iff the tile's closed rectangle meets the ellipse
                            (p-mu_2D)^T Sigma_2D^-1 (p-mu_2D) <= cb_beta * 2 ln(sigma / alpha_min)  (0)          */
    float cb_beta;       /* Compact Box threshold scale beta in (0, 1]; 1 keeps every pixel with alpha >= alpha_min (1) */
    int32_t sort_mode;   /* how fs_bin_sort orders the pairs; the result is the same either way.  FS_SORT_AUTO: per-tile
                            segments sorted in LDS while no tile's list exceeds 16384 entries, else the global radix sort;
                            FS_SORT_RADIX: always the global stable LSD radix sort on tile << 32 | depth bits (0)   */
} fs_config;

/* Pinhole camera: x_cam = R x_world + t (the paper's viewing transformation W);
 * pixel = (fx x/z + cx, fy y/z + cy); pixel (u,v) is sampled at (u+0.5, v+0.5). Host struct. */
typedef struct {
    int32_t width, height;
    float fx, fy, cx, cy;
    float R[9]; /* row-major */
    float t[3];
} fs_camera;

/* The scene (Sec. 3): mean mu, scale s, rotation r, opacity sigma, SH colour coefficients c. */
typedef struct {
    int64_t n;
    int32_t sh_degree;      /* 0..3, (sh_degree+1)^2 coefficients per channel                */
    const float *means;     /* [n,3] world space                                             */
    const float *scales;    /* [n,3] activated (> 0)                                         */
    const float *quats;     /* [n,4] (w,x,y,z), unit length (not re-normalised)              */
    const float *opacities; /* [n]   activated, in (0,1]                                     */
    const float *sh;        /* [n,(sh_degree+1)^2,3]                                         */
} fs_gaussians;

/* Output of fs_preprocess, caller-owned.  Culled Gaussians get zeros everywhere. */
typedef struct {
    float *mean2d;           /* [n,2] mu_2D in pixels                                         */
    float *depth;            /* [n]   camera-space z                                          */
    float *conic_opacity;    /* [n,4] Sigma_2D^-1 as (a, b, c) with q = a dx^2 + 2 b dx dy + c dy^2, then sigma */
    float *rgb;              /* [n,3] view-dependent colour max(0, 0.5 + SH)                  */
    uint16_t *rect;          /* [n,4] tile rectangle x0,y0,x1,y1, half-open (Compact Box: the tiles met by the
                                      ellipse's axis-aligned bounding box)                              */
    uint32_t *tiles_touched; /* [n]   number of pairs: (x1-x0)*(y1-y0), or with the Compact Box the tiles
                                      of rect that meet the ellipse; 0 = culled                         */
    uint8_t *clamped;        /* [n,3] 1 where the colour channel was clamped at 0             */
} fs_projected;

/* Output of fs_bin_sort.  Arrays are ctx-owned and stay valid until the next fs_bin_sort or
 * fs_destroy on the same ctx: no other call writes to them.  A later call that is handed the fs_bins
 * of an earlier fs_bin_sort (or of another ctx) returns FS_EINVAL (see `generation`). */
typedef struct {
    int64_t num_pairs;            /* P, host-visible on return                                        */
    const uint64_t *keys_sorted;  /* [P] tile_id << 32 | bits(depth), ascending; ties by Gaussian index */
    const uint32_t *gauss_sorted; /* [P] Gaussian index of each entry                                 */
    const uint32_t *tile_ranges;  /* [tiles,2] first,last(+1) entry of each tile; 0,0 if empty; tile_id = ty*TX+tx */
    const uint32_t *pair_offsets; /* radix ordering: [n] exclusive prefix sum of tiles_touched (Gaussian i's pairs were
                                     emitted from pair_offsets[i] on, rows then columns of rect, before the sort);
                                     NULL when the pairs were ordered per tile, which emits nothing in index order */
    int64_t num_records;          /* backward scratch records: P, or with the Compact Box the sum of rect areas  */
    const uint32_t *record_offsets; /* [n] Gaussian i's backward records start here; the record of tile (tx,ty) is
                                     record_offsets[i] + (ty - y0)*(x1 - x0) + (tx - x0).  The places of different
                                     Gaussians are disjoint and lie within num_records; they are in index order
                                     only after the radix ordering (then equal to pair_offsets without the Compact
                                     Box), and may differ from call to call otherwise.                          */
    const uint32_t *record_counts;  /* [n] records per Gaussian (rect area); NULL = proj->tiles_touched           */
    const uint32_t *tile_order;   /* [tiles] the tiles by decreasing list length: the order the render kernels take them in */
    const void *splats;           /* [n] 64-byte records (opaque): fs_bin_sort's copy of mean2d, conic_opacity, rgb,
                                     rect and record_offsets of every visible Gaussian, one cache line per gather.
                                     The render, backward and score calls read the splats from here.             */
    uint64_t generation;          /* which fs_bin_sort of the ctx filled this struct (set by the library; 0 = none)   */
} fs_bins;

/* Output of fs_render_bwd, caller-owned, OVERWRITTEN (not accumulated). dconic and drgb may be
 * NULL (the ctx then keeps them in its own scratch). */
typedef struct {
    float *dmeans;     /* [n,3]              */
    float *dscales;    /* [n,3]              */
    float *dquats;     /* [n,4]              */
    float *dopacities; /* [n]                */
    float *dsh;        /* [n,(deg+1)^2,3]    */
    float *dmean2d;    /* [n,2] dL/dmu_2D (the screen-space positional gradient used by densification) */
    float *dconic;     /* [n,3] dL/d(a,b,c) of conic_opacity, b counted with its factor 2; may be NULL */
    float *drgb;       /* [n,3] dL/d rgb; may be NULL                                                   */
    float *dmean2d_abs; /* [n,2] absolute positional gradient: sum over pixels of |that pixel's contribution to
                          dL/dmu_2D|, component-wise (the quantity FastGS thresholds for splitting; supplement,
                          "Implementation Details").  May be NULL: then it is not computed.                    */
} fs_grads;

typedef struct fs_ctx fs_ctx;

/* Fills *cfg with the defaults listed in fs_config. */
void fs_default_config(fs_config *cfg);

/* Creates a context bound to HIP device `device` and stream `hip_stream` (a hipStream_t, NULL =
 * the default stream).  cfg may be NULL (defaults).  The ctx owns scratch device memory that
 * grows on demand and is released by fs_destroy.  Errors: FS_EINVAL (bad cfg: tile != 16,
 * alpha_min <= 0, ...), FS_EHIP. */
int fs_create(fs_ctx **out, int device, void *hip_stream, const fs_config *cfg);
void fs_destroy(fs_ctx *ctx);
const char *fs_last_error(const fs_ctx *ctx);

/* Step a1 (Eqs. (2),(3); 3-sigma rule): camera-space mean, Sigma_3D = R S S^T R^T,
 * Sigma_2D = upper-left 2x2 of J W Sigma_3D W^T J^T (+ low-pass), its inverse, mu_2D,
 * radius ceil(3 sqrt(lambda_max)), tile rectangle, SH colour.  Errors: FS_EINVAL, FS_EHIP. */
int fs_preprocess(fs_ctx *ctx, const fs_gaussians *g, const fs_camera *cam, fs_projected *out);

/* Steps a2-a5: one 64-bit key tile_id << 32 | bits(depth) per (Gaussian, tile) pair, the keys in ascending order
 * (ties by Gaussian index: the order a stable sort of index-ordered keys gives) and the per-tile ranges.
 * Default path (FS_SORT_AUTO, while no tile's list exceeds 16384 entries and the image has at most 15360
 * tiles): the pairs are counted per tile, the ranges follow from an exclusive scan over the TILES, every pair is
 * placed into its tile's segment and each segment is sorted in LDS; no prefix sum over the Gaussians is made and
 * bins->pair_offsets is NULL.  Otherwise (FS_SORT_RADIX, or as the fall-back): exclusive scan of tiles_touched
 * (bins->pair_offsets), keys emitted in index order, a global stable LSD radix sort, ranges from the sorted keys.
 * Both give bit-identical keys, order and ranges.  n = number of Gaussians in `proj`.  Also packs the projected
 * splats into bins->splats and gives every pair the place of its backward record (bins->record_offsets); later
 * calls that take `bins` must be given the same `proj`.  Reads 32 bytes back (the host waits for the counting
 * kernels, not for the whole stream: from a context's second per-tile ordering on, placement and sorts are enqueued
 * ahead of that wait, bounded by what the context's buffers hold, and repeated if the totals say they did not fit).
 * Errors: FS_EINVAL, FS_ENOMEM, FS_EHIP, FS_ECAPACITY (n, P or the candidate tile count >= 2^31). */
int fs_bin_sort(fs_ctx *ctx, const fs_projected *proj, const fs_camera *cam, int64_t n, fs_bins *out);

/* Step a6 (Eqs. (4),(5)): image [3,H,W] planar, final_T [H,W] (transmittance left at each pixel),
 * n_contrib [H,W] (1-based position, in the pixel's tile list, of the last Gaussian blended).
 * All three are fully overwritten. */
int fs_render_fwd(fs_ctx *ctx, const fs_projected *proj, const fs_bins *bins, const fs_camera *cam,
                  float *image, float *final_T, uint32_t *n_contrib);

/* Steps a6 + a7 in one pass, and the first pass of a10: fs_render_fwd with, fused into the epilogue of its kernel,
 * dL_dimage = sign(image - target) / (3 H W) (may be NULL), the L1 loss (loss_out: device pointer to one double, may be
 * NULL) and the per-pixel error map of fs_error_mask, which the ctx keeps for a following fs_error_mask_fused.
 * Saves reading the finished image twice more.  Same outputs as the separate calls (the two fp64 sums are formed in
 * a different order).  target: [3,H,W]. */
int fs_render_fwd_loss(fs_ctx *ctx, const fs_projected *proj, const fs_bins *bins, const fs_camera *cam,
                       const float *target, float *image, float *final_T, uint32_t *n_contrib, float *dL_dimage,
                       double *loss_out);

/* Step a10 from the error map that the last fs_render_fwd_loss on this ctx left behind (same rule / k / outputs as
 * fs_error_mask).  FS_EINVAL if no such map of H x W pixels is pending: fs_l1_grad, fs_error_mask, fs_photo_loss,
 * fs_prune_score_normalize and fs_measure_peaks reuse that scratch and discard it; it may be used any number of
 * times until then. */
int fs_error_mask_fused(fs_ctx *ctx, int32_t height, int32_t width, int32_t rule, float k, uint8_t *mask,
                        float *threshold_out);

/* Whether the forward passes (fs_render_fwd, fs_render_fwd_loss) also record, for every pair, at which pixels of its
 * tile the multi-view score (Sec. 4.2) counts the pair's Gaussian: up to 36 bytes per pair of ctx scratch (pairs that are
 * counted nowhere leave nothing).  On by default.
 * When the latest forward pass on the ctx over `bins` made such a record, fs_score_accumulate takes its counts from it
 * (one population count per pair against the tile's mask) instead of walking the tile lists a second time; it then
 * reads neither final_T nor n_contrib, and the counts are the same.  The record costs the forward kernel some time
 * (about a tenth): turn it off for forward passes that no count pass follows (plain training iterations). */
int fs_set_score_record(fs_ctx *ctx, int32_t on);

/* Step a7: loss = mean |image - target| over 3*H*W values; dL_dimage = sign(image-target)/(3HW).
 * loss_out (device pointer to one double) may be NULL. */
int fs_l1_grad(fs_ctx *ctx, const float *image, const float *target, int32_t height, int32_t width,
               float *dL_dimage, double *loss_out);

/* Steps a8+a9: back-to-front gradient of the compositing, reduced per Gaussian, then chained
 * through the projection to the scene parameters.  final_T / n_contrib are fs_render_fwd's; bins
 * must be the result of the latest fs_bin_sort on this ctx for the same proj: every (Gaussian, tile) pair
 * owns one record of partial sums in ctx scratch, at bins->record_offsets[i] + the tile's place in the
 * Gaussian's rectangle, which the tile's workgroup stores once (see fs_set_record_mode for when a pair that received
 * nothing stores none); the projection's backward kernel then adds up each Gaussian's contiguous records.  No global
 * atomics.  Errors: FS_EINVAL (also: stale bins), FS_ENOMEM, FS_EHIP. */
int fs_render_bwd(fs_ctx *ctx, const fs_gaussians *g, const fs_camera *cam, const fs_projected *proj,
                  const fs_bins *bins, const float *final_T, const uint32_t *n_contrib,
                  const float *dL_dimage, fs_grads *out);

/* How fs_render_bwd maps the backward of the compositing onto the GPU (same inputs, outputs and tolerances):
 * FS_BWD_PER_PIXEL (default): a lane per pixel walks its sub-tile's list back to front; a Gaussian's sums over the
 *   pixels are reduced across lanes.
 * FS_BWD_PER_SPLAT: a lane per list entry, the pixels of an 8x8 block pass by one after the other; the quantities
 *   carried along a pixel's list become scans over the lanes, the sums need no reduction.  This is the mapping of
 *   the paper's baseline (Sec. 5.3 and the supplement: per-splat parallel backpropagation); on this chip and on
 *   lists as sparse as the benchmark's it is the slower of the two, and it is kept for comparison. */
enum { FS_BWD_PER_PIXEL = 0, FS_BWD_PER_SPLAT = 1 };
int fs_set_backward_mode(fs_ctx *ctx, int32_t mode);

/* How fs_render_bwd hands the per-pair gradients of the compositing (step a8) to the per-Gaussian sums (step a9);
 * same results either way:
 * FS_RECORDS_DENSE: every pair gets a 48-byte record, zeros where it received nothing; the sums read them all.
 * FS_RECORDS_SPARSE: only pairs that received something (blended at some pixel of their tile) get a record and a
 *   flag byte; the sums read the flags and the flagged records.  Pays where most pairs receive nothing -- deep,
 *   opaque scenes whose lists are long and mostly end behind the pixels' last blended Gaussian -- and costs a few
 *   microseconds otherwise (one more scattered byte per record, one more dependent load per chunk of records).
 * FS_RECORDS_AUTO (default): sparse when the tile lists hold 320 pairs or more on average. */
enum { FS_RECORDS_AUTO = 0, FS_RECORDS_DENSE = 1, FS_RECORDS_SPARSE = 2 };
int fs_set_record_mode(fs_ctx *ctx, int32_t mode);

/* Step a10: e = mean over channels of |image - target|; threshold t = mean(e) + k*std(e)
 * (FS_MASK_MEAN_STD; population std, fp64 accumulation) or min(e) + k*(max(e)-min(e))
 * (FS_MASK_MINMAX_TAU, i.e. min-max normalised e > k); mask = e > t (uint8 0/1, [H,W]).
 * threshold_out (device pointer to one float) may be NULL. */
int fs_error_mask(fs_ctx *ctx, const float *image, const float *target, int32_t height, int32_t width,
                  int32_t rule, float k, uint8_t *mask, float *threshold_out);

/* fs_error_mask for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): same arguments, outputs and arithmetic, but the error map and the
 * reduction partials live in a static device array of the library (about 16.8 MB on every GPU a context has
 * been created on, held until the process ends) instead of growable ctx scratch.  The call allocates and frees
 * nothing.  Images of more than FS_NOALLOC_MAX_PIXELS pixels are refused with FS_ECAPACITY (and a message);
 * FS_EINVAL as for fs_error_mask.  All contexts on one GPU share the array: calls that may overlap on one GPU
 * (different streams) race and must be ordered by the caller; consecutive calls on one stream are safe, and no
 * call depends on what an earlier one left in the array. */
#define FS_NOALLOC_MAX_PIXELS (4 * 1024 * 1024)
int fs_error_mask_noalloc(fs_ctx *ctx, const float *image, const float *target, int32_t height, int32_t width,
                          int32_t rule, float k, uint8_t *mask, float *threshold_out);

/* Step a11: for one view, counts[i] += number of pixels p with mask[p] = 1 at which Gaussian i
 * is blended by the forward pass (and, in FS_SCORE_WEIGHT mode, with alpha_i T_i > alpha_min).
 * counts [n] int32 is ACCUMULATED: zero it before the first view; s_d = counts / K.
 * final_T / n_contrib: those of the latest forward pass over `bins` (see fs_set_score_record for when they are not
 * read). */
int fs_score_accumulate(fs_ctx *ctx, const fs_projected *proj, const fs_bins *bins, const fs_camera *cam,
                        const float *final_T, const uint32_t *n_contrib, const uint8_t *mask,
                        int32_t *counts);

/* fs_error_mask_fused followed by fs_score_accumulate, as one call: mask [H,W] (OVERWRITTEN) and *threshold_out (may
 * be NULL) from the error map that the latest fs_render_fwd_loss on the ctx left, then counts [n] += the view's counts
 * under that mask (steps a10 + a11, Sec. 4.2).  Same results as the two calls.  When the forward pass left its record
 * (fs_set_score_record) this is a single kernel launch: the count pass builds each tile's part of the mask on its
 * way; otherwise the two kernels of the separate calls run, and n_contrib (of that forward pass) is read.
 * Errors: FS_EINVAL (no pending error map of the camera's size, bins of another fs_bin_sort, null arrays), FS_EHIP. */
int fs_mask_score_fused(fs_ctx *ctx, const fs_projected *proj, const fs_bins *bins, const fs_camera *cam,
                        const uint32_t *n_contrib, int32_t rule, float k, uint8_t *mask, float *threshold_out,
                        int32_t *counts);

/* The size of the record behind fs_set_score_record, per tile: rows_per_tile [tiles_y * tiles_x] int32 (device,
 * OVERWRITTEN) receives, for every tile, how many pairs of its list the score of Sec. 4.2 counts at one or more of the
 * tile's pixels under the all-ones mask -- the pairs the record keeps a row of 32 + 4 bytes for, and all that a count
 * pass from the record reads.  A diagnostic (bench.py prices the count pass with it); nothing on the path needs it.
 * Errors: FS_EINVAL when the latest forward pass on the ctx left no record for `bins` (record switched off, no
 * pairs, other bins); FS_EHIP. */
int fs_score_record_rows(fs_ctx *ctx, const fs_bins *bins, const fs_camera *cam, int32_t *rows_per_tile);

/* Photometric loss of one view (Sec. 4.3: E_photo; Sec. 4.5: the training loss has the same form):
 *   E = (1 - lambda) * L1 + lambda * (1 - SSIM),  L1 = mean |image - target| over the 3*H*W values.
 * SSIM (the paper cites the index without restating it): per channel, local means / variances /
 * covariance under an 11x11 Gaussian window (standard deviation 1.5 px, normalised to sum 1), the
 * images continued by zeros beyond their border, C1 = 0.01^2, C2 = 0.03^2; mean of the SSIM map over
 * channels and pixels.  image, target: [3,H,W] planar.  dL_dimage [3,H,W] (may be NULL) receives
 * dE/d image, OVERWRITTEN.  out3 (device pointer to three doubles, may be NULL) receives
 * {L1, SSIM, E}.  The ctx keeps 9*H*W floats of scratch when the gradient is requested.
 * Errors: FS_EINVAL, FS_ENOMEM, FS_EHIP. */
int fs_photo_loss(fs_ctx *ctx, const float *image, const float *target, int32_t height, int32_t width,
                  float lambda, float *dL_dimage, double *out3);

/* Pruning score (Sec. 4.3, Eq. for s_p).  Per view j, after fs_score_accumulate has filled that view's
 * own counts_view [n] (zeroed before the call) and fs_photo_loss has left E^j on the device:
 *   acc[i] += counts_view[i] * (*E)          acc: [n] doubles, caller-owned, zeroed before the first view.
 * E points at ONE device double (e.g. out3 + 2 of fs_photo_loss). */
int fs_prune_score_accumulate(fs_ctx *ctx, const int32_t *counts_view, int64_t n, const double *E, double *acc);

/* s_p[i] = (acc[i] - min acc) / (max acc - min acc): the min-max normalisation N over the Gaussians;
 * all zeros when max = min.  s_p: [n] floats. */
int fs_prune_score_normalize(fs_ctx *ctx, const double *acc, int64_t n, float *s_p);

/* ---- densification / pruning decisions (Sec. 4.2 VCD, Sec. 4.3 VCP, supplement "Implementation Details") ----
 * The paper keeps the gradient tests of vanilla 3DGS (plain positional gradient for cloning, the absolute
 * one for splitting) and adds: densify only where s_d = counts / K exceeds tau_d (5 in the paper); prune
 * where opacity < 0.1 or s_p > 0.9.  The gradient thresholds and the size limit are the caller's.        */
typedef struct {
    float tau_grad;    /* clone: mean over iterations of |dL/dmu_2D| (Euclidean norm, pixels) >= tau_grad     */
    float tau_abs;     /* split: the same mean of the absolute positional gradient >= tau_abs                 */
    float tau_d;       /* both: s_d = counts / K > tau_d                                                      */
    float size_limit;  /* clone if the largest scale <= size_limit, split if it is larger                     */
    float min_opacity; /* prune if opacity < min_opacity                                                      */
    float tau_p;       /* prune if s_p > tau_p                                                                */
    int32_t K;         /* number of views behind `counts`                                                     */
} fs_select_params;

/* After each fs_render_bwd of a training view: for every Gaussian visible in that view (tiles_touched > 0)
 *   grad_accum[i] += |dmean2d[i]|,  abs_accum[i] += |dmean2d_abs[i]|,  denom[i] += 1.
 * dmean2d_abs and abs_accum may both be NULL.  Accumulators are caller-owned and zeroed by the caller. */
int fs_densify_accumulate(fs_ctx *ctx, const float *dmean2d, const float *dmean2d_abs, const uint32_t *tiles_touched,
                          int64_t n, float *grad_accum, float *abs_accum, uint32_t *denom);

/* The three masks ([n] uint8, 0/1).  abs_accum may be NULL (then nothing is split); s_p may be NULL (then
 * only the opacity test prunes).  scales [n,3], opacities [n]: the scene's activated values.
 * Divisions and comparisons are fp32: mean = accum / max(denom, 1), s_d = counts / K. */
int fs_select(fs_ctx *ctx, int64_t n, const float *grad_accum, const float *abs_accum, const uint32_t *denom,
              const int32_t *counts, const float *scales, const float *opacities, const float *s_p,
              const fs_select_params *params, uint8_t *clone, uint8_t *split, uint8_t *prune);

/* Stream compaction: indices[0..count) = ascending positions i with mask[i] != 0.  indices needs room for n
 * entries.  *count_host (host pointer) is set on return; the call synchronises the stream for that.  Uses
 * scratch of its own: it may be called between fs_bin_sort and the calls that consume its fs_bins. */
int fs_compact(fs_ctx *ctx, const uint8_t *mask, int64_t n, uint32_t *indices, int64_t *count_host);

/* dst[r, 0..row_floats) = src[indices[r], 0..row_floats) for r < count: the copy that clone / prune-keep /
 * split-parent selection apply to each per-Gaussian array.  src and dst must not overlap. */
int fs_gather_rows(fs_ctx *ctx, const float *src, int64_t row_floats, const uint32_t *indices, int64_t count,
                   float *dst);

/* The three decisions applied together ([n] uint8 each): keep = not pruned and not split (a split parent is
 * replaced by its children), clone_eff = clone and not pruned, split_eff = split and not pruned. */
int fs_combine_masks(fs_ctx *ctx, int64_t n, const uint8_t *clone, const uint8_t *split, const uint8_t *prune,
                     uint8_t *keep, uint8_t *clone_eff, uint8_t *split_eff);

/* total[i] += view[i] (int32, n entries): the sum over the K views of the per-view counts that
 * fs_prune_score_accumulate also needs one view at a time. */
int fs_counts_add(fs_ctx *ctx, int32_t *total, const int32_t *view, int64_t n);

/* Splitting (supplement, "Implementation Details": densification as in vanilla 3DGS, selected by the absolute
 * gradient).  Each of the m parents p = parents[r] gets two children: child c sits at
 *   mu_p + R(q_p) (s_p * xi[r,c,:])       xi: the CALLER's standard normal draws, normals [m,2,3],
 * a sample of the parent's own density N(mu_p, Sigma_3D), and has scales s_p / phi (phi = 1.6 in vanilla 3DGS:
 * 0.8 x the number of children).  means [n,3], scales [n,3] (activated), quats [n,4] (unit, 16-byte aligned).
 * child_means, child_scales: [2m,3], row c*m + r.  Rotation, opacity and colour of a child are its parent's
 * (fs_gather_rows with `parents`); removing the parents is a compaction (fs_combine_masks' keep).
 * Errors: FS_EINVAL, FS_ECAPACITY (m >= 2^30), FS_EHIP. */
int fs_split_children(fs_ctx *ctx, const float *means, const float *scales, const float *quats,
                      const uint32_t *parents, int64_t m, const float *normals, float phi, float *child_means,
                      float *child_scales);

/* "Sampling half of the candidate Gaussians according to their pruning scores" (supplement, "Implementation
 * Details": pruning before iteration 15 000), read as weighted sampling without replacement: of the m Gaussians
 * with candidates[i] != 0, floor(m / 2) are drawn one after the other, each time with probability proportional
 * to scores[i] (the pruning score s_p) among those left.  The random stream is the CALLER's: exponentials [n]
 * holds one Exp(1) variate per Gaussian; the sample is the floor(m / 2) candidates with the smallest
 * exponentials[i] / scores[i] (fp32 division; +inf for a score <= 0; equal values go to the lower index), which
 * is that process exactly.  sample [n] uint8 is overwritten with the 0/1 mask of the drawn candidates;
 * *sampled_host (host pointer, may be NULL) receives their number.  Reads 8 bytes back (synchronises the stream).
 * Errors: FS_EINVAL, FS_ENOMEM, FS_ECAPACITY, FS_EHIP. */
int fs_sample_by_score(fs_ctx *ctx, const uint8_t *candidates, const float *scores, const float *exponentials,
                       int64_t n, uint8_t *sample, int64_t *sampled_host);

/* ---- optimiser (Sec. 5.1: all methods train with Adam; supplement "Implementation Details": the update
 * schedule of the accelerated baseline) ---------------------------------------------------------------- */

/* One Adam update (Kingma & Ba, Algorithm 1, with bias correction) of `count` parameters, in place:
 *   g = grad_scale * grad;  m = beta1 m + (1-beta1) g;  v = beta2 v + (1-beta2) g^2;
 *   param -= lr * (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps),   step >= 1.
 * If zero_grad != 0 the gradient array is cleared in the same pass.  All four arrays: `count` floats,
 * 16-byte aligned (FS_EINVAL otherwise). */
int fs_adam_step(fs_ctx *ctx, float *param, float *grad, float *m, float *v, int64_t count, float lr, float beta1,
                 float beta2, float eps, int32_t step, float grad_scale, int32_t zero_grad);

/* acc += grad (count floats, 16-byte aligned): the sum of the gradients of the iterations between two
 * optimiser updates. */
int fs_grad_accumulate(fs_ctx *ctx, float *acc, const float *grad, int64_t count);

/* Iterations between optimiser updates at training iteration `iteration`: 1 before 15 000, 32 from 15 000
 * to 20 000, 64 afterwards.  Host-only helper. */
int32_t fs_adam_interval(int32_t iteration);

/* Stored -> used parameters of vanilla 3DGS (which the paper's pipeline keeps): scale = exp(raw),
 * quaternion = raw / |raw|, opacity = 1 / (1 + exp(-raw)).  raw_quats and quats 16-byte aligned. */
int fs_activate(fs_ctx *ctx, int64_t n, const float *raw_scales, const float *raw_quats, const float *raw_opacities,
                float *scales, float *quats, float *opacities);

/* Chain rule through fs_activate: gradients w.r.t. the used parameters -> w.r.t. the stored ones.  The outputs
 * may alias the corresponding inputs (d_raw_scales == d_scales, ...). */
int fs_activate_bwd(fs_ctx *ctx, int64_t n, const float *raw_scales, const float *raw_quats,
                    const float *raw_opacities, const float *d_scales, const float *d_quats, const float *d_opacities,
                    float *d_raw_scales, float *d_raw_quats, float *d_raw_opacities);

/* Used -> stored parameters, the inverse of fs_activate for scale and opacity: raw_scale = ln(scale),
 * raw_opacity = ln(o / (1 - o)) with o = the opacity limited to [lo, hi], 0 < lo <= hi < 1 (an opacity of exactly
 * 0 or 1 has no finite stored value).  A unit quaternion is its own stored value. */
int fs_activate_inv(fs_ctx *ctx, int64_t n, const float *scales, const float *opacities, float lo, float hi,
                    float *raw_scales, float *raw_opacities);

/* ---- measurement helpers (no part of the method) ------------------------------------------
 * Per-kernel timing with HIP events recorded on the ctx stream around the launches of the
 * selected kernel groups.  fs_profile_enable(mask) clears the accumulated times and selects the
 * groups (bit k = group k below; 0 switches timing off).  fs_profile_read synchronises the
 * stream and returns the accumulated duration and the number of timed launches of one group.
 * Errors: FS_EINVAL (bad group), FS_EHIP. */
enum {
    FS_K_PREPROCESS = 0, /* k_preprocess                                  */
    FS_K_SCAN,           /* the three kernels of the tiles_touched scan   */
    FS_K_EMIT,           /* k_emit_pairs, or the per-tile counting kernels */
    FS_K_ORDER,          /* the ordering: placement + per-tile LDS sort, or the radix passes */
    FS_K_RANGES,         /* k_tile_ranges + k_tile_order (radix mode only) */
    FS_K_RENDER_FWD,     /* k_render_fwd                                  */
    FS_K_L1,             /* k_l1_grad (+ final reduction)                 */
    FS_K_PHOTO,          /* the kernels of fs_photo_loss                  */
    FS_K_RENDER_BWD,     /* k_render_bwd                                  */
    FS_K_PREPROCESS_BWD, /* k_preprocess_bwd                              */
    FS_K_ERR_MASK,       /* the kernels of fs_error_mask                  */
    FS_K_SCORE,          /* k_score                                       */
    FS_K_COUNT
};
int fs_profile_enable(fs_ctx *ctx, uint32_t group_mask);
int fs_profile_read(fs_ctx *ctx, int32_t group, const char **name, double *total_ms, int64_t *launches);

/* Two reference measurements on the ctx's device and stream, for the roofline figures: a streaming copy of
 * `copy_bytes` (device scratch, read + written once: *copy_gbs = 2 * copy_bytes / time) and chains of
 * independent fp32 fused multiply-adds, 2 flops each, without packed-fp32 instructions (*fma_tflops).
 * Either output may be NULL.  Synchronises the stream.  Errors: FS_EINVAL, FS_ENOMEM, FS_EHIP. */
int fs_measure_peaks(fs_ctx *ctx, int64_t copy_bytes, double *copy_gbs, double *fma_tflops);

#ifdef __cplusplus
}
#endif
#endif /* FASTGS_H */
