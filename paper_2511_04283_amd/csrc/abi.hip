// C ABI of libfastgs_hip: argument checks, scratch memory, and the order of kernel launches for
// each entry point of fastgs.h.  No arithmetic of the method lives here.
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <new>
#include <utility>
#include <vector>

#include "common.hpp"

using namespace fs;

// A device buffer that only ever grows (capacity doubling), owned by the ctx.
struct ScratchBuf {
    void* ptr = nullptr;
    size_t cap = 0;
};

struct fs_ctx {
    int device = 0;
    hipStream_t stream = nullptr;
    fs_config cfg;
    char err[256];

    ScratchBuf offsets;       // uint32 [n]
    ScratchBuf scan_tmp;      // uint64 block sums for the scans
    ScratchBuf keys[2];       // uint64 [P]: final keys and the tiles' unsorted segments, or the radix ping-pong pair
    ScratchBuf vals[2];       // uint32 [P] ping-pong
    ScratchBuf hist;          // uint32 [RADIX_DIGITS * radix blocks] (radix mode)
    ScratchBuf ranges;        // uint32: ranges [T,2] | tile order [T] | tile totals [T] | counters [TILE_COPIES,T]
    ScratchBuf pair_grad;     // float  [P, PAIR_REC] per-pair partial gradients of the backward pass
    ScratchBuf splats;        // float  [n, SPLAT_REC] packed projected splats (written by fs_bin_sort)
    ScratchBuf rec_counts;    // uint32 [n] Compact Box: tiles in each Gaussian's box
    ScratchBuf rec_offsets;   // uint32 [n] Compact Box: exclusive prefix sum of rec_counts
    ScratchBuf err_map;       // float  [H*W]
    ScratchBuf ssim_maps;     // float  [3, 3*H*W] derivative maps of the SSIM term
    ScratchBuf partial;       // double reduction partials
    ScratchBuf compact_pos;   // uint32 [n] fs_compact / fs_sample_by_score: positions of the selected elements
    ScratchBuf compact_scan;  // ... and the block sums of their scan
    ScratchBuf sel_keys[2];   // uint64 [m] fs_sample_by_score: arrival-time keys, ping-pong for the radix sort
    ScratchBuf sel_vals[2];   // uint32 [m] candidate indices, ping-pong
    ScratchBuf sel_hist;      // uint32 radix histograms of that sort
    uint64_t generation = 0;  // bumped by every fs_bin_sort; fs_bins of an earlier one are refused
    hipEvent_t totals_event = nullptr;   // recorded behind the read-back of fs_bin_sort's totals
    int spec_set = 0;                    // the sort launches (TS_*) the previous per-tile ordering on this ctx would have
                                         // chosen (0: none): what fs_bin_sort enqueues ahead of its read-back
    uint64_t* total_dev = nullptr;   // device: totals [4]: pairs, backward records, pairs counted per tile, longest tile list
    uint64_t* total_host = nullptr;  // pinned host block of four totals (copied from total_dev, or written by k_tile_scan)
    uint64_t* alloc_dev = nullptr;   // device: the two counters of the counting kernel (zero between calls)
    bool alloc_dirty = false;        // a call failed between the kernel that adds to them and the one that clears them
    ScratchBuf tile_partial;         // double [5, tiles]: per-tile sums of the fused forward pass
    ScratchBuf pair_bits;            // the record of the forward passes for the count pass (score_record_at)
    ScratchBuf rec_valid;            // uint8 [records]: 1 where k_render_bwd left a gradient record; k_preprocess_bwd puts
                                     // every flag it finds back to 0, so the array is all zeros between calls
    size_t rec_valid_zeroed = 0;     // the capacity of rec_valid that has been zeroed since its allocation
    bool rec_valid_dirty = false;    // a call ended between the kernel that sets flags and the one that clears them
    bool per_splat_bwd = false;      // fs_set_backward_mode
    int record_mode = FS_RECORDS_AUTO;   // fs_set_record_mode
    bool record_bits = true;         // the forward passes fill pair_bits (fs_set_score_record)
    int64_t bits_pairs = -1;         // pair_bits describe the latest forward pass over the bins of this many pairs,
    const void* bits_order = nullptr;  // ... with this gauss_sorted, on this many tiles; -1: they describe nothing
    int bits_tiles = 0;
    int64_t longest_list = 0;        // longest tile list of the latest fs_bin_sort (0: not known, the radix ordering)
    int64_t fused_pixels = 0;        // > 0: err_map / partial hold the error map of the last fs_render_fwd_loss

    // per-group event timing (measurement only)
    uint32_t prof_mask = 0;
    std::vector<std::pair<hipEvent_t, hipEvent_t>> prof_pending[FS_K_COUNT];
    std::vector<hipEvent_t> prof_free;
    double prof_ms[FS_K_COUNT] = {};
    int64_t prof_launches[FS_K_COUNT] = {};
};

// ---- scratch of the entry point that allocates nothing (fs_error_mask_noalloc) ---------------------------------
// One file-scope device array per GPU the library runs on, held until the process ends: the error map of up to
// FS_NOALLOC_MAX_PIXELS pixels, one float for the threshold, and the reduction partials.  In host code the array's
// name is only a handle: its device address is looked up once per device (noalloc_setup, called by fs_create with
// that device current) and kernels are handed that address.
constexpr size_t NOALLOC_ERR_BYTES = ((size_t)FS_NOALLOC_MAX_PIXELS + 64) * sizeof(float);   // (+ the threshold slot)
constexpr size_t NOALLOC_PARTIAL_BYTES = (size_t)4 * RED_BLOCKS * sizeof(double);
static __device__ __align__(256) unsigned char scratch[NOALLOC_ERR_BYTES + NOALLOC_PARTIAL_BYTES];
constexpr int NOALLOC_MAX_DEVICES = 64;
static void* g_noalloc_ptr[NOALLOC_MAX_DEVICES] = {};

namespace {

// `device` must be current.  Returns hipSuccess when the address is (already) known.
hipError_t noalloc_setup(int device)
{
    if (device < 0 || device >= NOALLOC_MAX_DEVICES) return hipErrorInvalidDevice;
    if (g_noalloc_ptr[device]) return hipSuccess;
    void* ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    g_noalloc_ptr[device] = ptr;
    return hipSuccess;
}

int fail(fs_ctx* c, int code, const char* fmt, const char* a = "")
{
    if (c) snprintf(c->err, sizeof(c->err), fmt, a);
    return code;
}

int hip_fail(fs_ctx* c, hipError_t e, const char* where)
{
    if (c) snprintf(c->err, sizeof(c->err), "%s: %s", where, hipGetErrorString(e));
    return FS_EHIP;
}

#define FS_HIP(call, where)                                   \
    do {                                                      \
        hipError_t e_ = (call);                               \
        if (e_ != hipSuccess) return hip_fail(ctx, e_, where); \
    } while (0)

int ensure(fs_ctx* ctx, ScratchBuf& b, size_t bytes, const char* what)
{
    if (bytes <= b.cap) return FS_OK;
    size_t want = b.cap ? b.cap : 4096;
    while (want < bytes) want *= 2;
    // nothing enqueued earlier may still use the old block when it is released
    hipError_t e = hipStreamSynchronize(ctx->stream);
    if (e != hipSuccess) return hip_fail(ctx, e, "hipStreamSynchronize");
    if (b.ptr) (void)hipFree(b.ptr);
    b.ptr = nullptr;
    b.cap = 0;
    e = hipMalloc(&b.ptr, want);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        b.ptr = nullptr;
        return fail(ctx, FS_ENOMEM, "scratch allocation failed (%s)", what);
    }
    b.cap = want;
    return FS_OK;
}

#define FS_TRY(expr)            \
    do {                        \
        int rc_ = (expr);       \
        if (rc_ != FS_OK) return rc_; \
    } while (0)

const char* const kGroupNames[FS_K_COUNT] = {"preprocess", "scan", "emit_pairs", "order_pairs", "tile_ranges",
                                             "render_fwd", "l1_grad", "photo_loss", "render_bwd", "preprocess_bwd",
                                             "error_mask", "score"};

hipEvent_t prof_event(fs_ctx* ctx)
{
    if (!ctx->prof_free.empty()) {
        hipEvent_t e = ctx->prof_free.back();
        ctx->prof_free.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
    return e;
}

// Records an event pair around the launches issued during its lifetime when the group is selected.
struct ProfScope {
    fs_ctx* ctx;
    int group;
    hipEvent_t a = nullptr, b = nullptr;
    ProfScope(fs_ctx* c, int g) : ctx(c), group(g)
    {
        if (!(ctx->prof_mask >> g & 1u)) return;
        a = prof_event(ctx);
        b = prof_event(ctx);
        if (a && b) (void)hipEventRecord(a, ctx->stream);
    }
    ~ProfScope()
    {
        if (!a || !b) return;
        (void)hipEventRecord(b, ctx->stream);
        ctx->prof_pending[group].emplace_back(a, b);
    }
};

bool make_cam(const fs_camera* cam, CamDev& d)
{
    if (!cam || cam->width <= 0 || cam->height <= 0 || !(cam->fx > 0.f) || !(cam->fy > 0.f)) return false;
    d.width = cam->width;
    d.height = cam->height;
    d.fx = cam->fx; d.fy = cam->fy; d.cx = cam->cx; d.cy = cam->cy;
    memcpy(d.R, cam->R, sizeof(d.R));
    memcpy(d.t, cam->t, sizeof(d.t));
    d.tiles_x = (cam->width + TILE - 1) / TILE;
    d.tiles_y = (cam->height + TILE - 1) / TILE;
    return d.tiles_x <= 65535 && d.tiles_y <= 65535;
}

CfgDev make_cfg(const fs_config& c)
{
    CfgDev d;
    d.z_near = c.z_near; d.lowpass = c.lowpass; d.alpha_min = c.alpha_min; d.alpha_max = c.alpha_max;
    d.T_min = c.T_min;
    d.bg[0] = c.bg[0]; d.bg[1] = c.bg[1]; d.bg[2] = c.bg[2];
    d.jclamp = c.jclamp;
    // conservative: for opacity <= 1, sigma*exp(power) < alpha_min whenever power < ln(alpha_min) - 0.01
    d.power_min = (float)(log((double)c.alpha_min) - 0.01);
    d.score_mode = c.score_mode;
    d.compact_box = c.compact_box != 0;
    d.cb_beta = c.cb_beta;
    return d;
}

int tile_bits(int tiles)
{
    int b = 0;
    while ((1 << b) < tiles) b++;
    return b;
}

bool proj_ok(const fs_projected* p)
{
    return p && p->mean2d && p->depth && p->conic_opacity && p->rgb && p->rect && p->tiles_touched && p->clamped;
}

// bins of an earlier fs_bin_sort (or of another ctx) point at memory that has been reused since
bool bins_stale(const fs_ctx* ctx, const fs_bins* bins) { return bins->generation != ctx->generation || ctx->generation == 0; }

// the record in ctx->pair_bits now describes the forward pass over these bins
void note_bits(fs_ctx* ctx, const fs_bins* bins, int tiles)
{
    ctx->bits_pairs = bins->num_pairs;
    ctx->bits_order = bins->gauss_sorted;
    ctx->bits_tiles = tiles;
}

}  // namespace

extern "C" {

void fs_default_config(fs_config* cfg)
{
    if (!cfg) return;
    cfg->tile = TILE;
    cfg->z_near = (float)0.2;
    cfg->lowpass = (float)0.3;
    cfg->alpha_min = 1.0f / 255.0f;
    cfg->alpha_max = (float)0.99;
    cfg->T_min = (float)1e-4;
    cfg->bg[0] = cfg->bg[1] = cfg->bg[2] = 0.0f;
    cfg->jclamp = (float)1.3;
    cfg->score_mode = FS_SCORE_WEIGHT;
    cfg->compact_box = 0;
    cfg->cb_beta = 1.0f;
    cfg->sort_mode = FS_SORT_AUTO;
}

int fs_create(fs_ctx** out, int device, void* hip_stream, const fs_config* cfg)
{
    if (!out) return FS_EINVAL;
    *out = nullptr;
    fs_config c;
    if (cfg) c = *cfg; else fs_default_config(&c);
    if (c.tile != TILE || !(c.alpha_min > 0.f) || !(c.alpha_min < c.alpha_max) || !(c.alpha_max < 1.f) ||
        !(c.T_min > 0.f) || !(c.T_min < 1.f) || !(c.lowpass >= 0.f) ||
        (c.score_mode != FS_SCORE_WEIGHT && c.score_mode != FS_SCORE_ALPHA) ||
        (c.compact_box != 0 && c.compact_box != 1) || (c.sort_mode != FS_SORT_AUTO && c.sort_mode != FS_SORT_RADIX) || (c.compact_box && !(c.cb_beta > 0.f && c.cb_beta <= 1.f)))
        return FS_EINVAL;
    if (hipSetDevice(device) != hipSuccess) { (void)hipGetLastError(); return FS_EHIP; }
    fs_ctx* ctx = new (std::nothrow) fs_ctx();
    if (!ctx) return FS_ENOMEM;
    ctx->device = device;
    ctx->stream = static_cast<hipStream_t>(hip_stream);
    ctx->cfg = c;
    ctx->err[0] = 0;
    if (hipEventCreateWithFlags(&ctx->totals_event, hipEventDisableTiming) != hipSuccess) {
        (void)hipGetLastError();
        ctx->totals_event = nullptr;
        fs_destroy(ctx);
        return FS_EHIP;
    }
    if (noalloc_setup(device) != hipSuccess) {
        (void)hipGetLastError();
        fs_destroy(ctx);
        return FS_EHIP;
    }
    if (hipMalloc(reinterpret_cast<void**>(&ctx->alloc_dev), 2 * sizeof(uint64_t)) != hipSuccess ||
        hipMemset(ctx->alloc_dev, 0, 2 * sizeof(uint64_t)) != hipSuccess ||
        hipMalloc(reinterpret_cast<void**>(&ctx->total_dev), 4 * sizeof(uint64_t)) != hipSuccess ||
        hipHostMalloc(reinterpret_cast<void**>(&ctx->total_host), 4 * sizeof(uint64_t), hipHostMallocDefault) != hipSuccess) {
        (void)hipGetLastError();
        fs_destroy(ctx);
        return FS_EHIP;
    }
    *out = ctx;
    return FS_OK;
}

void fs_destroy(fs_ctx* ctx)
{
    if (!ctx) return;
    (void)hipSetDevice(ctx->device);
    (void)hipStreamSynchronize(ctx->stream);
    ScratchBuf* all[] = {&ctx->offsets, &ctx->scan_tmp, &ctx->keys[0], &ctx->keys[1], &ctx->vals[0], &ctx->vals[1],
                         &ctx->hist, &ctx->ranges, &ctx->pair_grad, &ctx->splats, &ctx->rec_counts, &ctx->rec_offsets,
                         &ctx->err_map, &ctx->ssim_maps, &ctx->partial, &ctx->tile_partial, &ctx->pair_bits, &ctx->rec_valid,
                         &ctx->compact_pos, &ctx->compact_scan, &ctx->sel_keys[0], &ctx->sel_keys[1], &ctx->sel_vals[0],
                         &ctx->sel_vals[1], &ctx->sel_hist};
    for (ScratchBuf* b : all)
        if (b->ptr) (void)hipFree(b->ptr);
    if (ctx->total_dev) (void)hipFree(ctx->total_dev);
    if (ctx->alloc_dev) (void)hipFree(ctx->alloc_dev);
    if (ctx->total_host) (void)hipHostFree(ctx->total_host);
    if (ctx->totals_event) (void)hipEventDestroy(ctx->totals_event);
    for (auto& v : ctx->prof_pending)
        for (auto& pr : v) { (void)hipEventDestroy(pr.first); (void)hipEventDestroy(pr.second); }
    for (hipEvent_t e : ctx->prof_free) (void)hipEventDestroy(e);
    delete ctx;
}

const char* fs_last_error(const fs_ctx* ctx) { return ctx ? ctx->err : "null context"; }

int fs_preprocess(fs_ctx* ctx, const fs_gaussians* g, const fs_camera* cam, fs_projected* out)
{
    if (!ctx) return FS_EINVAL;
    CamDev cd;
    if (!g || g->n < 0 || g->sh_degree < 0 || g->sh_degree > 3 || !make_cam(cam, cd))
        return fail(ctx, FS_EINVAL, "fs_preprocess: bad scene or camera");
    if (g->n > 0 && (!g->means || !g->scales || !g->quats || !g->opacities || !g->sh || !proj_ok(out)))
        return fail(ctx, FS_EINVAL, "fs_preprocess: null array");
    if (g->n >= (int64_t)1 << 31) return fail(ctx, FS_ECAPACITY, "fs_preprocess: n does not fit 31 bits");
    FS_HIP(hipSetDevice(ctx->device), "hipSetDevice");
    ProfScope prof(ctx, FS_K_PREPROCESS);
    FS_HIP(launch_preprocess(ctx->stream, g->n, g->sh_degree, *g, cd, make_cfg(ctx->cfg), *out), "k_preprocess");
    return FS_OK;
}

int fs_bin_sort(fs_ctx* ctx, const fs_projected* proj, const fs_camera* cam, int64_t n, fs_bins* out)
{
    if (!ctx) return FS_EINVAL;
    CamDev cd;
    if (!out || n < 0 || !make_cam(cam, cd)) return fail(ctx, FS_EINVAL, "fs_bin_sort: bad arguments");
    if (n > 0 && !proj_ok(proj)) return fail(ctx, FS_EINVAL, "fs_bin_sort: null array");
    if (n >= (int64_t)1 << 31) return fail(ctx, FS_ECAPACITY, "fs_bin_sort: n does not fit 31 bits");
    ctx->bits_pairs = -1;
    ctx->generation++;      // whatever earlier fs_bins of this ctx point at is overwritten from here on
    out->generation = 0;    // (a call that fails leaves bins that every later call refuses)
    FS_HIP(hipSetDevice(ctx->device), "hipSetDevice");
    hipStream_t st = ctx->stream;
    const int tiles = cd.tiles_x * cd.tiles_y;

    // ranges [T,2] | tile_order [T] | tile totals [T] | per-tile counters [TILE_COPIES,T]
    FS_TRY(ensure(ctx, ctx->ranges, (size_t)tiles * (4 + TILE_COPIES) * sizeof(uint32_t), "tile ranges and order"));
    uint32_t* const ranges_p = static_cast<uint32_t*>(ctx->ranges.ptr);
    uint32_t* const order_p = ranges_p + 2 * (size_t)tiles;
    uint32_t* const ttotal_p = ranges_p + 3 * (size_t)tiles;
    uint32_t* const tcount_p = ranges_p + 4 * (size_t)tiles;
    const bool bucketed = ctx->cfg.sort_mode == FS_SORT_AUTO && tiles <= TILE_LDS_MAX_TILES;
    FS_TRY(ensure(ctx, ctx->offsets, (size_t)(n > 0 ? n : 1) * sizeof(uint32_t), "offsets"));
    FS_TRY(ensure(ctx, ctx->scan_tmp, scan_tmp_bytes(n), "scan"));
    FS_TRY(ensure(ctx, ctx->splats, (size_t)(n > 0 ? n : 1) * SPLAT_REC * sizeof(float), "splats"));

    // a2: where each Gaussian's pairs / backward records start, and the pair count P (the one host read-back of
    // the path).  With the Compact Box the records are indexed by candidate tile, so the boxes' areas get
    // offsets of their own.  The radix path emits its keys in index order from exclusive prefix sums; the
    // tile-bucketed path only needs disjoint places for the records and gets them from its counting kernel.
    const bool cb = ctx->cfg.compact_box != 0;
    const CfgDev cf = make_cfg(ctx->cfg);
    if (cb) {
        FS_TRY(ensure(ctx, ctx->rec_counts, (size_t)(n > 0 ? n : 1) * sizeof(uint32_t), "record counts"));
        FS_TRY(ensure(ctx, ctx->rec_offsets, (size_t)(n > 0 ? n : 1) * sizeof(uint32_t), "record offsets"));
    }
    auto prefix_sums = [&]() -> int {
        ProfScope prof(ctx, FS_K_SCAN);
        FS_HIP(launch_exclusive_scan(st, proj ? proj->tiles_touched : nullptr, static_cast<uint32_t*>(ctx->offsets.ptr),
                                     n, ctx->scan_tmp.ptr, ctx->total_dev),
               "scan");
        if (cb) {
            FS_HIP(launch_rect_area(st, n, proj ? proj->rect : nullptr, static_cast<uint32_t*>(ctx->rec_counts.ptr)),
                   "k_rect_area");
            FS_HIP(launch_exclusive_scan(st, static_cast<const uint32_t*>(ctx->rec_counts.ptr),
                                         static_cast<uint32_t*>(ctx->rec_offsets.ptr), n, ctx->scan_tmp.ptr,
                                         ctx->total_dev + 1),
                   "scan");
        }
        return FS_OK;
    };
    if (bucketed) {
        // first half: pairs per tile, ranges, longest list, record places (needs no P-sized memory, so it is
        // enqueued ahead of the read-back)
        ProfScope prof(ctx, FS_K_EMIT);
        fs_projected none = {};
        if (ctx->alloc_dirty) FS_HIP(launch_fill_u32(st, reinterpret_cast<uint32_t*>(ctx->alloc_dev), 0u, 4), "k_fill_u32");
        ctx->alloc_dirty = true;
        FS_HIP(launch_tile_count(st, n, proj ? *proj : none, cf, cd.tiles_x, tiles, tcount_p, ttotal_p,
                                 reinterpret_cast<uint2*>(ranges_p), order_p, ctx->total_host,
                                 static_cast<uint32_t*>(cb ? ctx->rec_offsets.ptr : ctx->offsets.ptr),
                                 cb ? static_cast<uint32_t*>(ctx->rec_counts.ptr) : nullptr, ctx->alloc_dev),
               "k_tile_pairs (count)");
        ctx->alloc_dirty = false;
    } else {
        FS_TRY(prefix_sums());
    }
    // (the per-tile ordering's scan kernel stores its four totals straight into the pinned host block, which the
    // device can address: a copy behind it would be one more small kernel in front of the placement)
    if (!bucketed)
        FS_HIP(hipMemcpyAsync(ctx->total_host, ctx->total_dev, 4 * sizeof(uint64_t), hipMemcpyDeviceToHost, st),
               "hipMemcpyAsync");
    FS_HIP(hipEventRecord(ctx->totals_event, st), "hipEventRecord");
    // Per-tile ordering, second half (placement into the tiles' segments -- keys[1] serves as the bucket array -- and
    // the per-tile LDS sorts; the ranges are already in place).  When this ctx has ordered pairs per tile before, the
    // second half is enqueued right here, ahead of the host's wait for the totals, sized by what the buffers hold, with
    // the sort launches the previous call's lists would have chosen: otherwise the GPU idles for the whole round trip (wait, wake-up, launch) once per
    // call.  The kernels write nothing beyond the capacities they are given; what the totals then say was not covered
    // (a longer list's sort variant, or buffers that have to grow first) is enqueued afterwards.
    const uint32_t* recs_p = cb ? static_cast<const uint32_t*>(ctx->rec_offsets.ptr) : static_cast<const uint32_t*>(ctx->offsets.ptr);
    fs_projected none = {};
    uint64_t cap_pairs = 0, cap_recs = 0;
    int spec_variants = 0;
    if (bucketed && ctx->spec_set != 0 && n > 0) {
        cap_pairs = ctx->keys[0].cap / sizeof(uint64_t);
        if (ctx->keys[1].cap / sizeof(uint64_t) < cap_pairs) cap_pairs = ctx->keys[1].cap / sizeof(uint64_t);
        if (ctx->vals[0].cap / sizeof(uint32_t) < cap_pairs) cap_pairs = ctx->vals[0].cap / sizeof(uint32_t);
        if (cap_pairs > 0x7fffffffull) cap_pairs = 0x7fffffffull;
        cap_recs = cb ? ctx->pair_grad.cap / (PAIR_REC * sizeof(float)) : 0;
        if (cap_recs > 0x7fffffffull) cap_recs = 0x7fffffffull;
        if (cap_pairs > 0 && (!cb || cap_recs > 0)) {
            ProfScope prof(ctx, FS_K_ORDER);
            spec_variants = ctx->spec_set;
            FS_HIP(launch_tile_scatter(st, n, proj ? *proj : none, cf, recs_p, cd.tiles_x, tiles, (uint32_t)cap_pairs,
                                       (uint32_t)cap_recs, reinterpret_cast<const uint2*>(ranges_p), tcount_p,
                                       static_cast<uint64_t*>(ctx->keys[1].ptr), static_cast<float*>(ctx->splats.ptr),
                                       static_cast<float*>(ctx->pair_grad.ptr)),
                   "k_tile_pairs (placement)");
            FS_HIP(launch_tile_sorts(st, tiles, spec_variants, (uint32_t)cap_pairs, reinterpret_cast<const uint2*>(ranges_p),
                                     order_p, static_cast<const uint64_t*>(ctx->keys[1].ptr),
                                     static_cast<uint64_t*>(ctx->keys[0].ptr), static_cast<uint32_t*>(ctx->vals[0].ptr)),
                   "k_tile_sort");
        }
    }
    FS_HIP(hipEventSynchronize(ctx->totals_event), "hipEventSynchronize");
    // bucketed: {sum of tiles_touched, records, pairs counted per tile, longest list}; else {pairs, records (CB)}
    const uint64_t P = bucketed ? ctx->total_host[2] : ctx->total_host[0];
    const uint64_t NR = cb || bucketed ? ctx->total_host[1] : P;
    ctx->spec_set = 0;
    if (bucketed && (ctx->total_host[0] != P || (!cb && NR != P)))
        return fail(ctx, FS_EINVAL, "fs_bin_sort: tiles_touched does not match rect (proj from another configuration?)");
    if (P >= (uint64_t)1 << 31) return fail(ctx, FS_ECAPACITY, "fs_bin_sort: pair count does not fit 31 bits");
    if (NR >= (uint64_t)1 << 31) return fail(ctx, FS_ECAPACITY, "fs_bin_sort: candidate tile count does not fit 31 bits");
    const uint64_t max_len = bucketed ? ctx->total_host[3] : 0;
    ctx->longest_list = (int64_t)max_len;
    const bool lds_sort = bucketed && max_len <= (uint64_t)TILE_SORT_HUGE;
    // did what was enqueued ahead cover this call?  (growing a buffer below waits for the stream first)
    const bool spec_fits = spec_variants != 0 && P <= cap_pairs && (!cb || NR <= cap_recs);
    if (cb) FS_TRY(ensure(ctx, ctx->pair_grad, (size_t)(NR ? NR : 1) * PAIR_REC * sizeof(float), "pair gradients"));

    const int64_t nb = radix_num_blocks((int64_t)P);
    for (int k = 0; k < 2; k++) {
        FS_TRY(ensure(ctx, ctx->keys[k], (size_t)(P ? P : 1) * sizeof(uint64_t), "keys"));
        FS_TRY(ensure(ctx, ctx->vals[k], (size_t)(P ? P : 1) * sizeof(uint32_t), "values"));
    }
    FS_TRY(ensure(ctx, ctx->hist, (size_t)(nb ? nb : 1) * RADIX_DIGITS * sizeof(uint32_t), "histograms"));
    FS_TRY(ensure(ctx, ctx->scan_tmp, scan_tmp_bytes(RADIX_DIGITS * nb), "scan"));

    uint64_t* keys[2] = {static_cast<uint64_t*>(ctx->keys[0].ptr), static_cast<uint64_t*>(ctx->keys[1].ptr)};
    uint32_t* vals[2] = {static_cast<uint32_t*>(ctx->vals[0].ptr), static_cast<uint32_t*>(ctx->vals[1].ptr)};
    int res = 0;
    if (lds_sort) {
        // (lists of more than 1024 entries on average: enough tiles beyond 2048 to give them a launch of their own)
        const bool long_lists = P > (uint64_t)1024 * (uint64_t)tiles;
        // placement and the sorts enqueued ahead have run (or are running) already: what do they leave to do?
        const int variants = P > 0 ? tile_sort_variants((int64_t)max_len, long_lists, spec_fits ? spec_variants : 0) : 0;
        if (!spec_fits || variants) {
            ProfScope prof(ctx, FS_K_ORDER);
            if (!spec_fits) {
                FS_HIP(launch_tile_scatter(st, n, proj ? *proj : none, cf, recs_p, cd.tiles_x, tiles, (uint32_t)P,
                                           (uint32_t)NR, reinterpret_cast<const uint2*>(ranges_p), tcount_p, keys[1],
                                           static_cast<float*>(ctx->splats.ptr), static_cast<float*>(ctx->pair_grad.ptr)),
                       "k_tile_pairs (placement)");
            }
            FS_HIP(launch_tile_sorts(st, tiles, variants, (uint32_t)P, reinterpret_cast<const uint2*>(ranges_p), order_p,
                                     keys[1], keys[0], vals[0]),
                   "k_tile_sort");
        }
        ctx->spec_set = tile_sort_variants((int64_t)max_len, long_lists, 0);
    } else {
        // (lists too long for the per-tile sort: the radix path's prefix sums have not been made yet)
        if (bucketed) FS_TRY(prefix_sums());
        if (P > 0) {
            // a3
            {
                ProfScope prof(ctx, FS_K_EMIT);
                if (cb)
                    FS_HIP(launch_emit_pairs_cb(st, n, *proj, cf, static_cast<const uint32_t*>(ctx->offsets.ptr),
                                                static_cast<const uint32_t*>(ctx->rec_offsets.ptr), cd.tiles_x, (int64_t)P,
                                                keys[0], vals[0], static_cast<float*>(ctx->splats.ptr),
                                                static_cast<float*>(ctx->pair_grad.ptr)),
                           "k_emit_pairs_cb");
                else
                    FS_HIP(launch_emit_pairs(st, n, *proj, static_cast<const uint32_t*>(ctx->offsets.ptr), cd.tiles_x,
                                             keys[0], vals[0], static_cast<float*>(ctx->splats.ptr)),
                           "k_emit_pairs");
            }
            // a4: 32 depth bits + the tile bits are live
            ProfScope prof(ctx, FS_K_ORDER);
            FS_HIP(launch_radix_sort(st, (int64_t)P, 32 + tile_bits(tiles), keys, vals, static_cast<uint32_t*>(ctx->hist.ptr),
                                     ctx->scan_tmp.ptr, ctx->total_dev, &res),
                   "radix sort");
        }
        // a5
        ProfScope prof(ctx, FS_K_RANGES);
        FS_HIP(launch_tile_ranges(st, (int64_t)P, keys[res], tiles, ranges_p, order_p), "k_tile_ranges");
    }
    out->num_pairs = (int64_t)P;
    out->keys_sorted = keys[res];
    out->gauss_sorted = vals[res];
    out->tile_ranges = static_cast<const uint32_t*>(ctx->ranges.ptr);
    out->pair_offsets = lds_sort ? nullptr : static_cast<const uint32_t*>(ctx->offsets.ptr);
    out->num_records = (int64_t)NR;
    out->record_offsets = static_cast<const uint32_t*>(cb ? ctx->rec_offsets.ptr : ctx->offsets.ptr);
    out->record_counts = cb ? static_cast<const uint32_t*>(ctx->rec_counts.ptr) : nullptr;
    out->splats = ctx->splats.ptr;
    out->tile_order = static_cast<const uint32_t*>(ctx->ranges.ptr) + 2 * (size_t)tiles;
    out->generation = ctx->generation;
    return FS_OK;
}

int fs_render_fwd(fs_ctx* ctx, const fs_projected* proj, const fs_bins* bins, const fs_camera* cam, float* image,
                  float* final_T, uint32_t* n_contrib)
{
    if (!ctx) return FS_EINVAL;
    CamDev cd;
    if (!make_cam(cam, cd) || !bins || !bins->tile_ranges || !bins->tile_order || !image || !final_T || !n_contrib)
        return fail(ctx, FS_EINVAL, "fs_render_fwd: bad arguments");
    if (bins->num_pairs > 0 && (!proj_ok(proj) || !bins->gauss_sorted || !bins->splats))
        return fail(ctx, FS_EINVAL, "fs_render_fwd: null array");
    if (bins_stale(ctx, bins)) return fail(ctx, FS_EINVAL, "fs_render_fwd: bins do not come from this context's latest fs_bin_sort");
    FS_HIP(hipSetDevice(ctx->device), "hipSetDevice");
    ctx->bits_pairs = -1;   // (what an earlier forward pass recorded for the count pass does not describe this one)
    const bool bits = ctx->record_bits && bins->num_pairs > 0;
    if (bits) FS_TRY(ensure(ctx, ctx->pair_bits, score_record_bytes(bins->num_pairs, cd.tiles_x * cd.tiles_y), "score record"));
    ProfScope prof(ctx, FS_K_RENDER_FWD);
    FS_HIP(launch_render_fwd(ctx->stream, cd, make_cfg(ctx->cfg), bins->tile_ranges, bins->tile_order, bins->gauss_sorted,
                             static_cast<const float*>(bins->splats), image, final_T, n_contrib,
                             bits ? score_record_at(ctx->pair_bits.ptr, bins->num_pairs) : ScoreRecord{nullptr, nullptr, nullptr}),
           "k_render_fwd");
    if (bits) note_bits(ctx, bins, cd.tiles_x * cd.tiles_y);
    return FS_OK;
}

int fs_render_fwd_loss(fs_ctx* ctx, const fs_projected* proj, const fs_bins* bins, const fs_camera* cam, const float* target,
                       float* image, float* final_T, uint32_t* n_contrib, float* dL_dimage, double* loss_out)
{
    if (!ctx) return FS_EINVAL;
    CamDev cd;
    if (!make_cam(cam, cd) || !bins || !bins->tile_ranges || !bins->tile_order || !image || !final_T || !n_contrib || !target)
        return fail(ctx, FS_EINVAL, "fs_render_fwd_loss: bad arguments");
    if (bins->num_pairs > 0 && (!proj_ok(proj) || !bins->gauss_sorted || !bins->splats))
        return fail(ctx, FS_EINVAL, "fs_render_fwd_loss: null array");
    if (bins_stale(ctx, bins)) return fail(ctx, FS_EINVAL, "fs_render_fwd_loss: bins do not come from this context's latest fs_bin_sort");
    FS_HIP(hipSetDevice(ctx->device), "hipSetDevice");
    const int tiles = cd.tiles_x * cd.tiles_y;
    const int64_t pixels = (int64_t)cd.width * cd.height;
    ctx->fused_pixels = 0;
    ctx->bits_pairs = -1;
    const bool bits = ctx->record_bits && bins->num_pairs > 0;
    FS_TRY(ensure(ctx, ctx->err_map, (size_t)(pixels + 1) * sizeof(float), "error map"));
    FS_TRY(ensure(ctx, ctx->partial, (size_t)fused_partials() * sizeof(double), "partials"));
    FS_TRY(ensure(ctx, ctx->tile_partial, (size_t)5 * tiles * sizeof(double), "tile partials"));
    if (bits) FS_TRY(ensure(ctx, ctx->pair_bits, score_record_bytes(bins->num_pairs, cd.tiles_x * cd.tiles_y), "score record"));
    {
        ProfScope prof(ctx, FS_K_RENDER_FWD);
        FS_HIP(launch_render_fwd_fused(ctx->stream, cd, make_cfg(ctx->cfg), bins->tile_ranges, bins->tile_order,
                                       bins->gauss_sorted, static_cast<const float*>(bins->splats), image, final_T, n_contrib,
                                       target, dL_dimage, static_cast<float*>(ctx->err_map.ptr),
                                       static_cast<double*>(ctx->tile_partial.ptr), bits ? score_record_at(ctx->pair_bits.ptr, bins->num_pairs) : ScoreRecord{nullptr, nullptr, nullptr}),
               "k_render_fwd");
    }
    if (bits) note_bits(ctx, bins, tiles);
    ProfScope prof(ctx, FS_K_L1);
    FS_HIP(launch_fold_tile_partials(ctx->stream, static_cast<const double*>(ctx->tile_partial.ptr), tiles, 3 * pixels,
                                     static_cast<double*>(ctx->partial.ptr), loss_out),
           "k_fold_tile_partials");
    ctx->fused_pixels = pixels;
    return FS_OK;
}

int fs_set_backward_mode(fs_ctx* ctx, int32_t mode)
{
    if (!ctx) return FS_EINVAL;
    if (mode != FS_BWD_PER_PIXEL && mode != FS_BWD_PER_SPLAT) return fail(ctx, FS_EINVAL, "fs_set_backward_mode: unknown mode");
    ctx->per_splat_bwd = mode == FS_BWD_PER_SPLAT;
    return FS_OK;
}

int fs_set_record_mode(fs_ctx* ctx, int32_t mode)
{
    if (!ctx) return FS_EINVAL;
    if (mode != FS_RECORDS_AUTO && mode != FS_RECORDS_DENSE && mode != FS_RECORDS_SPARSE)
        return fail(ctx, FS_EINVAL, "fs_set_record_mode: unknown mode");
    ctx->record_mode = mode;
    return FS_OK;
}

int fs_set_score_record(fs_ctx* ctx, int32_t on)
{
    if (!ctx) return FS_EINVAL;
    ctx->record_bits = on != 0;
    if (!ctx->record_bits) ctx->bits_pairs = -1;
    return FS_OK;
}

int fs_error_mask_fused(fs_ctx* ctx, int32_t height, int32_t width, int32_t rule, float k, uint8_t* mask, float* threshold_out)
{
    if (!ctx) return FS_EINVAL;
    if (!mask || height <= 0 || width <= 0 || (rule != FS_MASK_MEAN_STD && rule != FS_MASK_MINMAX_TAU))
        return fail(ctx, FS_EINVAL, "fs_error_mask_fused: bad arguments");
    const int64_t pixels = (int64_t)height * width;
    if (ctx->fused_pixels != pixels)
        return fail(ctx, FS_EINVAL, "fs_error_mask_fused: no error map of this size from fs_render_fwd_loss is pending");
    FS_HIP(hipSetDevice(ctx->device), "hipSetDevice");
    float* err = static_cast<float*>(ctx->err_map.ptr);
    float* thr = threshold_out ? threshold_out : err + pixels;
    ProfScope prof(ctx, FS_K_ERR_MASK);
    FS_HIP(launch_error_mask_from_map(ctx->stream, pixels, rule, k, err, static_cast<double*>(ctx->partial.ptr), mask, thr),
           "k_err_*");
    return FS_OK;
}

int fs_l1_grad(fs_ctx* ctx, const float* image, const float* target, int32_t height, int32_t width, float* dL_dimage,
               double* loss_out)
{
    if (!ctx) return FS_EINVAL;
    if (!image || !target || !dL_dimage || height <= 0 || width <= 0)
        return fail(ctx, FS_EINVAL, "fs_l1_grad: bad arguments");
    ctx->fused_pixels = 0;   // (the scratch that the fused forward pass leaves its error map in is reused here)
    FS_HIP(hipSetDevice(ctx->device), "hipSetDevice");
    FS_TRY(ensure(ctx, ctx->partial, (size_t)4 * mask_partials() * sizeof(double), "partials"));
    ProfScope prof(ctx, FS_K_L1);
    FS_HIP(launch_l1_grad(ctx->stream, image, target, (int64_t)3 * height * width, dL_dimage,
                          static_cast<double*>(ctx->partial.ptr), loss_out),
           "k_l1_grad");
    return FS_OK;
}

int fs_render_bwd(fs_ctx* ctx, const fs_gaussians* g, const fs_camera* cam, const fs_projected* proj,
                  const fs_bins* bins, const float* final_T, const uint32_t* n_contrib, const float* dL_dimage,
                  fs_grads* out)
{
    if (!ctx) return FS_EINVAL;
    CamDev cd;
    if (!g || g->n < 0 || g->sh_degree < 0 || g->sh_degree > 3 || !make_cam(cam, cd) || !bins || !bins->tile_ranges ||
        !bins->tile_order || !final_T || !n_contrib || !dL_dimage || !out)
        return fail(ctx, FS_EINVAL, "fs_render_bwd: bad arguments");
    const int64_t n = g->n;
    if (n == 0) return FS_OK;
    if (!g->means || !g->scales || !g->quats || !g->opacities || !g->sh || !proj_ok(proj) || !out->dmeans ||
        !out->dscales || !out->dquats || !out->dopacities || !out->dsh || !out->dmean2d ||
        (bins->num_pairs > 0 && !bins->gauss_sorted))
        return fail(ctx, FS_EINVAL, "fs_render_bwd: null array");
    FS_HIP(hipSetDevice(ctx->device), "hipSetDevice");
    hipStream_t st = ctx->stream;
    if (bins->num_pairs > 0 && (!bins->record_offsets || !bins->splats || bins->num_records < bins->num_pairs))
        return fail(ctx, FS_EINVAL, "fs_render_bwd: bins without record_offsets / splats");
    // (the records, their places and -- with the Compact Box -- the zeroed records of the candidate tiles that are
    // no pairs all live in this ctx and belong to its latest fs_bin_sort)
    if (bins_stale(ctx, bins)) return fail(ctx, FS_EINVAL, "fs_render_bwd: bins do not come from this context's latest fs_bin_sort");
    FS_TRY(ensure(ctx, ctx->pair_grad, (size_t)(bins->num_records ? bins->num_records : 1) * PAIR_REC * sizeof(float),
                  "pair gradients"));
    float* pair_grad = static_cast<float*>(ctx->pair_grad.ptr);
    // sparse records: one flag per record place, all zeros here (a fresh or left-over array is cleared first)
    const int tiles = cd.tiles_x * cd.tiles_y;
    const bool sparse = ctx->record_mode == FS_RECORDS_SPARSE ||
                        (ctx->record_mode == FS_RECORDS_AUTO && bins->num_pairs >= (int64_t)320 * tiles);
    uint8_t* rec_valid = nullptr;
    if (sparse) {
        FS_TRY(ensure(ctx, ctx->rec_valid, ((size_t)(bins->num_records ? bins->num_records : 1) + 3) / 4 * 4, "record flags"));
        if (ctx->rec_valid_zeroed != ctx->rec_valid.cap || ctx->rec_valid_dirty) {
            FS_HIP(launch_fill_u32(st, static_cast<uint32_t*>(ctx->rec_valid.ptr), 0u, (int64_t)(ctx->rec_valid.cap / 4)), "k_fill_u32");
            ctx->rec_valid_zeroed = ctx->rec_valid.cap;
        }
        rec_valid = static_cast<uint8_t*>(ctx->rec_valid.ptr);
        ctx->rec_valid_dirty = true;
    }
    const CfgDev cf = make_cfg(ctx->cfg);
    // a8: every pair's record is written exactly once (sparse: that of every pair that received something, and flagged)
    if (bins->num_pairs > 0) {
        ProfScope prof(ctx, FS_K_RENDER_BWD);
        FS_HIP(launch_render_bwd(st, cd, cf, bins->tile_ranges, bins->tile_order, bins->gauss_sorted,
                                 static_cast<const float*>(bins->splats), final_T, n_contrib, dL_dimage, pair_grad, rec_valid,
                                 out->dmean2d_abs != nullptr, ctx->per_splat_bwd),
               "k_render_bwd");
    }
    // a9: per-Gaussian sum of its records (sparse: the flagged ones; the flags go back to 0), then the chain through
    // the projection
    ProfScope prof(ctx, FS_K_PREPROCESS_BWD);
    FS_HIP(launch_preprocess_bwd(st, n, g->sh_degree, *g, cd, cf, proj->clamped, proj->tiles_touched,
                                 bins->record_counts ? bins->record_counts : proj->tiles_touched, bins->record_offsets,
                                 pair_grad, rec_valid, *out),
           "k_preprocess_bwd");
    if (sparse) ctx->rec_valid_dirty = false;
    return FS_OK;
}

int fs_error_mask(fs_ctx* ctx, const float* image, const float* target, int32_t height, int32_t width, int32_t rule,
                  float k, uint8_t* mask, float* threshold_out)
{
    if (!ctx) return FS_EINVAL;
    if (!image || !target || !mask || height <= 0 || width <= 0 ||
        (rule != FS_MASK_MEAN_STD && rule != FS_MASK_MINMAX_TAU))
        return fail(ctx, FS_EINVAL, "fs_error_mask: bad arguments");
    ctx->fused_pixels = 0;   // (the scratch that the fused forward pass leaves its error map in is reused here)
    FS_HIP(hipSetDevice(ctx->device), "hipSetDevice");
    const int64_t pixels = (int64_t)height * width;
    FS_TRY(ensure(ctx, ctx->err_map, (size_t)(pixels + 1) * sizeof(float), "error map"));
    FS_TRY(ensure(ctx, ctx->partial, (size_t)4 * mask_partials() * sizeof(double), "partials"));
    float* err = static_cast<float*>(ctx->err_map.ptr);
    float* thr = threshold_out ? threshold_out : err + pixels;
    ProfScope prof(ctx, FS_K_ERR_MASK);
    FS_HIP(launch_error_mask(ctx->stream, image, target, pixels, rule, k, err, static_cast<double*>(ctx->partial.ptr),
                             mask, thr),
           "k_err_*");
    return FS_OK;
}

int fs_error_mask_noalloc(fs_ctx* ctx, const float* image, const float* target, int32_t height, int32_t width,
                          int32_t rule, float k, uint8_t* mask, float* threshold_out)
{
    if (!ctx) return FS_EINVAL;
    if (!image || !target || !mask || height <= 0 || width <= 0 ||
        (rule != FS_MASK_MEAN_STD && rule != FS_MASK_MINMAX_TAU))
        return fail(ctx, FS_EINVAL, "fs_error_mask_noalloc: bad arguments");
    const int64_t pixels = (int64_t)height * width;
    if (pixels > (int64_t)FS_NOALLOC_MAX_PIXELS)
        return fail(ctx, FS_ECAPACITY, "fs_error_mask_noalloc: more than FS_NOALLOC_MAX_PIXELS pixels (use fs_error_mask)");
    unsigned char* base = ctx->device >= 0 && ctx->device < NOALLOC_MAX_DEVICES
                              ? static_cast<unsigned char*>(g_noalloc_ptr[ctx->device]) : nullptr;
    if (!base) return fail(ctx, FS_EHIP, "fs_error_mask_noalloc: no static scratch on this device");
    FS_HIP(hipSetDevice(ctx->device), "hipSetDevice");
    // every word the kernels read is written earlier in the same call (the error map and all 4 x RED_BLOCKS
    // partials by k_err_map's workgroups), so nothing of an earlier call's contents matters
    float* err = reinterpret_cast<float*>(base);
    double* partial = reinterpret_cast<double*>(base + NOALLOC_ERR_BYTES);
    float* thr = threshold_out ? threshold_out : err + pixels;
    FS_HIP(launch_error_mask(ctx->stream, image, target, pixels, rule, k, err, partial, mask, thr), "k_err_*");
    return FS_OK;
}

int fs_score_accumulate(fs_ctx* ctx, const fs_projected* proj, const fs_bins* bins, const fs_camera* cam,
                        const float* final_T, const uint32_t* n_contrib, const uint8_t* mask, int32_t* counts)
{
    if (!ctx) return FS_EINVAL;
    CamDev cd;
    (void)final_T;  // the walk recomputes T from the front, exactly as the forward pass did
    if (!make_cam(cam, cd) || !bins || !bins->tile_ranges || !bins->tile_order || !n_contrib || !mask)
        return fail(ctx, FS_EINVAL, "fs_score_accumulate: bad arguments");
    if (bins->num_pairs == 0) return FS_OK;
    if (!proj_ok(proj) || !bins->gauss_sorted || !bins->splats || !counts)
        return fail(ctx, FS_EINVAL, "fs_score_accumulate: null array");
    if (bins_stale(ctx, bins)) return fail(ctx, FS_EINVAL, "fs_score_accumulate: bins do not come from this context's latest fs_bin_sort");
    FS_HIP(hipSetDevice(ctx->device), "hipSetDevice");
    ProfScope prof(ctx, FS_K_SCORE);
    if (ctx->bits_pairs == bins->num_pairs && ctx->bits_order == bins->gauss_sorted &&
        ctx->bits_tiles == cd.tiles_x * cd.tiles_y) {
        // the latest forward pass over these bins recorded where each pair is counted: no second walk
        FS_HIP(launch_score_bits(ctx->stream, cd, bins->tile_ranges, score_record_at(ctx->pair_bits.ptr, bins->num_pairs),
                                 mask, counts, ctx->longest_list),
               "k_score_bits");
        return FS_OK;
    }
    FS_HIP(launch_score(ctx->stream, cd, make_cfg(ctx->cfg), bins->tile_ranges, bins->tile_order, bins->gauss_sorted,
                        static_cast<const float*>(bins->splats), n_contrib, mask, counts),
           "k_score");
    return FS_OK;
}

int fs_mask_score_fused(fs_ctx* ctx, const fs_projected* proj, const fs_bins* bins, const fs_camera* cam,
                        const uint32_t* n_contrib, int32_t rule, float k, uint8_t* mask, float* threshold_out, int32_t* counts)
{
    if (!ctx) return FS_EINVAL;
    CamDev cd;
    if (!make_cam(cam, cd) || !bins || !bins->tile_ranges || !bins->tile_order || !n_contrib || !mask ||
        (rule != FS_MASK_MEAN_STD && rule != FS_MASK_MINMAX_TAU))
        return fail(ctx, FS_EINVAL, "fs_mask_score_fused: bad arguments");
    const int64_t pixels = (int64_t)cd.width * cd.height;
    if (ctx->fused_pixels != pixels)
        return fail(ctx, FS_EINVAL, "fs_mask_score_fused: no error map of this size from fs_render_fwd_loss is pending");
    if (bins->num_pairs > 0 && (!proj_ok(proj) || !bins->gauss_sorted || !bins->splats || !counts))
        return fail(ctx, FS_EINVAL, "fs_mask_score_fused: null array");
    if (bins_stale(ctx, bins)) return fail(ctx, FS_EINVAL, "fs_mask_score_fused: bins do not come from this context's latest fs_bin_sort");
    FS_HIP(hipSetDevice(ctx->device), "hipSetDevice");
    float* err = static_cast<float*>(ctx->err_map.ptr);
    float* thr = threshold_out ? threshold_out : err + pixels;
    const int tiles = cd.tiles_x * cd.tiles_y;
    if (bins->num_pairs > 0 && ctx->bits_pairs == bins->num_pairs && ctx->bits_order == bins->gauss_sorted &&
        ctx->bits_tiles == tiles) {
        // one launch: every tile's first workgroup makes (and stores) the tile's part of the mask on its way
        ProfScope prof(ctx, FS_K_SCORE);
        FS_HIP(launch_mask_score_bits(ctx->stream, cd, bins->tile_ranges, score_record_at(ctx->pair_bits.ptr, bins->num_pairs),
                                      err, static_cast<const double*>(ctx->partial.ptr), rule, k, mask, thr, counts,
                                      ctx->longest_list),
               "k_score_bits");
        return FS_OK;
    }
    {
        ProfScope prof(ctx, FS_K_ERR_MASK);
        FS_HIP(launch_error_mask_from_map(ctx->stream, pixels, rule, k, err, static_cast<double*>(ctx->partial.ptr), mask, thr),
               "k_err_*");
    }
    if (bins->num_pairs == 0) return FS_OK;
    ProfScope prof(ctx, FS_K_SCORE);
    FS_HIP(launch_score(ctx->stream, cd, make_cfg(ctx->cfg), bins->tile_ranges, bins->tile_order, bins->gauss_sorted,
                        static_cast<const float*>(bins->splats), n_contrib, mask, counts),
           "k_score");
    return FS_OK;
}

int fs_score_record_rows(fs_ctx* ctx, const fs_bins* bins, const fs_camera* cam, int32_t* rows_per_tile)
{
    if (!ctx) return FS_EINVAL;
    CamDev cd;
    if (!make_cam(cam, cd) || !bins || !rows_per_tile) return fail(ctx, FS_EINVAL, "fs_score_record_rows: bad arguments");
    if (bins_stale(ctx, bins)) return fail(ctx, FS_EINVAL, "fs_score_record_rows: bins do not come from this context's latest fs_bin_sort");
    const int tiles = cd.tiles_x * cd.tiles_y;
    if (ctx->bits_pairs != bins->num_pairs || ctx->bits_order != bins->gauss_sorted || ctx->bits_tiles != tiles)
        return fail(ctx, FS_EINVAL, "fs_score_record_rows: the latest forward pass on this context left no record for these bins");
    if (!bins->tile_ranges) return fail(ctx, FS_EINVAL, "fs_score_record_rows: null array");
    FS_HIP(hipSetDevice(ctx->device), "hipSetDevice");
    FS_HIP(launch_record_rows(ctx->stream, tiles, score_record_at(ctx->pair_bits.ptr, bins->num_pairs), rows_per_tile),
           "k_record_rows");
    return FS_OK;
}

int fs_photo_loss(fs_ctx* ctx, const float* image, const float* target, int32_t height, int32_t width, float lambda,
                  float* dL_dimage, double* out3)
{
    if (!ctx) return FS_EINVAL;
    if (!image || !target || height <= 0 || width <= 0 || !(lambda >= 0.f && lambda <= 1.f) || (!dL_dimage && !out3))
        return fail(ctx, FS_EINVAL, "fs_photo_loss: bad arguments");
    ctx->fused_pixels = 0;   // (the scratch that the fused forward pass leaves its error map in is reused here)
    FS_HIP(hipSetDevice(ctx->device), "hipSetDevice");
    const size_t nb = (size_t)photo_blocks(height, width);
    FS_TRY(ensure(ctx, ctx->partial, (2 * nb > (size_t)4 * mask_partials() ? 2 * nb : (size_t)4 * mask_partials()) * sizeof(double),
                  "partials"));
    if (dL_dimage)
        FS_TRY(ensure(ctx, ctx->ssim_maps, (size_t)9 * height * width * sizeof(float), "SSIM derivative maps"));
    ProfScope prof(ctx, FS_K_PHOTO);
    FS_HIP(launch_photo_loss(ctx->stream, image, target, height, width, lambda, static_cast<float*>(ctx->ssim_maps.ptr),
                             static_cast<double*>(ctx->partial.ptr), dL_dimage, out3),
           "k_ssim_*");
    return FS_OK;
}

int fs_prune_score_accumulate(fs_ctx* ctx, const int32_t* counts_view, int64_t n, const double* E, double* acc)
{
    if (!ctx) return FS_EINVAL;
    if (n < 0 || (n > 0 && (!counts_view || !E || !acc))) return fail(ctx, FS_EINVAL, "fs_prune_score_accumulate: bad arguments");
    FS_HIP(hipSetDevice(ctx->device), "hipSetDevice");
    FS_HIP(launch_prune_accumulate(ctx->stream, counts_view, n, E, acc), "k_prune_accumulate");
    return FS_OK;
}

int fs_prune_score_normalize(fs_ctx* ctx, const double* acc, int64_t n, float* s_p)
{
    if (!ctx) return FS_EINVAL;
    if (n < 0 || (n > 0 && (!acc || !s_p))) return fail(ctx, FS_EINVAL, "fs_prune_score_normalize: bad arguments");
    ctx->fused_pixels = 0;   // (the scratch that the fused forward pass leaves its error map in is reused here)
    FS_HIP(hipSetDevice(ctx->device), "hipSetDevice");
    FS_TRY(ensure(ctx, ctx->partial, (size_t)4 * mask_partials() * sizeof(double), "partials"));
    FS_HIP(launch_prune_normalize(ctx->stream, acc, n, static_cast<double*>(ctx->partial.ptr), s_p), "k_prune_normalize");
    return FS_OK;
}

int fs_densify_accumulate(fs_ctx* ctx, const float* dmean2d, const float* dmean2d_abs, const uint32_t* tiles_touched,
                          int64_t n, float* grad_accum, float* abs_accum, uint32_t* denom)
{
    if (!ctx) return FS_EINVAL;
    if (n < 0 || (n > 0 && (!dmean2d || !tiles_touched || !grad_accum || !denom)) || ((dmean2d_abs != nullptr) != (abs_accum != nullptr)))
        return fail(ctx, FS_EINVAL, "fs_densify_accumulate: bad arguments");
    FS_HIP(hipSetDevice(ctx->device), "hipSetDevice");
    FS_HIP(launch_densify_accumulate(ctx->stream, n, dmean2d, dmean2d_abs, tiles_touched, grad_accum, abs_accum, denom),
           "k_densify_accumulate");
    return FS_OK;
}

int fs_select(fs_ctx* ctx, int64_t n, const float* grad_accum, const float* abs_accum, const uint32_t* denom,
              const int32_t* counts, const float* scales, const float* opacities, const float* s_p,
              const fs_select_params* params, uint8_t* clone, uint8_t* split, uint8_t* prune)
{
    if (!ctx) return FS_EINVAL;
    if (n < 0 || !params || params->K <= 0 ||
        (n > 0 && (!grad_accum || !denom || !counts || !scales || !opacities || !clone || !split || !prune)))
        return fail(ctx, FS_EINVAL, "fs_select: bad arguments");
    FS_HIP(hipSetDevice(ctx->device), "hipSetDevice");
    FS_HIP(launch_select(ctx->stream, n, grad_accum, abs_accum, denom, counts, scales, opacities, s_p, *params, clone,
                         split, prune),
           "k_select");
    return FS_OK;
}

int fs_compact(fs_ctx* ctx, const uint8_t* mask, int64_t n, uint32_t* indices, int64_t* count_host)
{
    if (!ctx) return FS_EINVAL;
    if (n < 0 || !count_host || (n > 0 && (!mask || !indices))) return fail(ctx, FS_EINVAL, "fs_compact: bad arguments");
    if (n >= (int64_t)1 << 31) return fail(ctx, FS_ECAPACITY, "fs_compact: n does not fit 31 bits");
    *count_host = 0;
    if (n == 0) return FS_OK;
    FS_HIP(hipSetDevice(ctx->device), "hipSetDevice");
    // (scratch of its own: what fs_bin_sort left for the backward pass must survive a compaction in between)
    FS_TRY(ensure(ctx, ctx->compact_pos, (size_t)n * sizeof(uint32_t), "compaction positions"));
    FS_TRY(ensure(ctx, ctx->compact_scan, scan_tmp_bytes(n), "scan"));
    FS_HIP(launch_compact(ctx->stream, n, mask, static_cast<uint32_t*>(ctx->compact_pos.ptr), ctx->compact_scan.ptr,
                          ctx->total_dev, indices),
           "compaction");
    FS_HIP(hipMemcpyAsync(ctx->total_host, ctx->total_dev, sizeof(uint64_t), hipMemcpyDeviceToHost, ctx->stream),
           "hipMemcpyAsync");
    FS_HIP(hipStreamSynchronize(ctx->stream), "hipStreamSynchronize");
    *count_host = (int64_t)ctx->total_host[0];
    return FS_OK;
}

int fs_gather_rows(fs_ctx* ctx, const float* src, int64_t row_floats, const uint32_t* indices, int64_t count, float* dst)
{
    if (!ctx) return FS_EINVAL;
    if (count < 0 || row_floats <= 0 || row_floats > 4096 || (count > 0 && (!src || !indices || !dst)))
        return fail(ctx, FS_EINVAL, "fs_gather_rows: bad arguments");
    FS_HIP(hipSetDevice(ctx->device), "hipSetDevice");
    FS_HIP(launch_gather_rows(ctx->stream, src, (int)row_floats, indices, count, dst), "k_gather_rows");
    return FS_OK;
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int fs_adam_step(fs_ctx* ctx, float* param, float* grad, float* m, float* v, int64_t count, float lr, float beta1,
                 float beta2, float eps, int32_t step, float grad_scale, int32_t zero_grad)
{
    if (!ctx) return FS_EINVAL;
    if (count < 0 || step < 1 || !(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f) || !(eps >= 0.f) ||
        (count > 0 && (!param || !grad || !m || !v)))
        return fail(ctx, FS_EINVAL, "fs_adam_step: bad arguments");
    if (!aligned16(param) || !aligned16(grad) || !aligned16(m) || !aligned16(v))
        return fail(ctx, FS_EINVAL, "fs_adam_step: arrays must be 16-byte aligned");
    FS_HIP(hipSetDevice(ctx->device), "hipSetDevice");
    FS_HIP(launch_adam(ctx->stream, param, grad, m, v, count, lr, beta1, beta2, eps, step, grad_scale, zero_grad != 0),
           "k_adam");
    return FS_OK;
}

int fs_grad_accumulate(fs_ctx* ctx, float* acc, const float* grad, int64_t count)
{
    if (!ctx) return FS_EINVAL;
    if (count < 0 || (count > 0 && (!acc || !grad)) || !aligned16(acc) || !aligned16(grad))
        return fail(ctx, FS_EINVAL, "fs_grad_accumulate: bad arguments");
    FS_HIP(hipSetDevice(ctx->device), "hipSetDevice");
    FS_HIP(launch_grad_accumulate(ctx->stream, acc, grad, count), "k_grad_accumulate");
    return FS_OK;
}

int32_t fs_adam_interval(int32_t iteration) { return iteration < 15000 ? 1 : (iteration < 20000 ? 32 : 64); }

int fs_activate(fs_ctx* ctx, int64_t n, const float* raw_scales, const float* raw_quats, const float* raw_opacities,
                float* scales, float* quats, float* opacities)
{
    if (!ctx) return FS_EINVAL;
    if (n < 0 || (n > 0 && (!raw_scales || !raw_quats || !raw_opacities || !scales || !quats || !opacities)) ||
        !aligned16(raw_quats) || !aligned16(quats))
        return fail(ctx, FS_EINVAL, "fs_activate: bad arguments");
    FS_HIP(hipSetDevice(ctx->device), "hipSetDevice");
    FS_HIP(launch_activate(ctx->stream, n, raw_scales, raw_quats, raw_opacities, scales, quats, opacities), "k_activate");
    return FS_OK;
}

int fs_activate_bwd(fs_ctx* ctx, int64_t n, const float* raw_scales, const float* raw_quats, const float* raw_opacities,
                    const float* d_scales, const float* d_quats, const float* d_opacities, float* d_raw_scales,
                    float* d_raw_quats, float* d_raw_opacities)
{
    if (!ctx) return FS_EINVAL;
    if (n < 0 ||
        (n > 0 && (!raw_scales || !raw_quats || !raw_opacities || !d_scales || !d_quats || !d_opacities ||
                   !d_raw_scales || !d_raw_quats || !d_raw_opacities)) ||
        !aligned16(raw_quats) || !aligned16(d_quats) || !aligned16(d_raw_quats))
        return fail(ctx, FS_EINVAL, "fs_activate_bwd: bad arguments");
    FS_HIP(hipSetDevice(ctx->device), "hipSetDevice");
    FS_HIP(launch_activate_bwd(ctx->stream, n, raw_scales, raw_quats, raw_opacities, d_scales, d_quats, d_opacities,
                               d_raw_scales, d_raw_quats, d_raw_opacities),
           "k_activate_bwd");
    return FS_OK;
}

int fs_combine_masks(fs_ctx* ctx, int64_t n, const uint8_t* clone, const uint8_t* split, const uint8_t* prune,
                     uint8_t* keep, uint8_t* clone_eff, uint8_t* split_eff)
{
    if (!ctx) return FS_EINVAL;
    if (n < 0 || (n > 0 && (!clone || !split || !prune || !keep || !clone_eff || !split_eff)))
        return fail(ctx, FS_EINVAL, "fs_combine_masks: bad arguments");
    FS_HIP(hipSetDevice(ctx->device), "hipSetDevice");
    FS_HIP(launch_combine_masks(ctx->stream, n, clone, split, prune, keep, clone_eff, split_eff), "k_combine_masks");
    return FS_OK;
}

int fs_counts_add(fs_ctx* ctx, int32_t* total, const int32_t* view, int64_t n)
{
    if (!ctx) return FS_EINVAL;
    if (n < 0 || (n > 0 && (!total || !view))) return fail(ctx, FS_EINVAL, "fs_counts_add: bad arguments");
    FS_HIP(hipSetDevice(ctx->device), "hipSetDevice");
    FS_HIP(launch_counts_add(ctx->stream, n, total, view), "k_counts_add");
    return FS_OK;
}

int fs_split_children(fs_ctx* ctx, const float* means, const float* scales, const float* quats, const uint32_t* parents,
                      int64_t m, const float* normals, float phi, float* child_means, float* child_scales)
{
    if (!ctx) return FS_EINVAL;
    if (m < 0 || !(phi > 0.f) || (m > 0 && (!means || !scales || !quats || !parents || !normals || !child_means || !child_scales)))
        return fail(ctx, FS_EINVAL, "fs_split_children: bad arguments");
    if (m >= (int64_t)1 << 30) return fail(ctx, FS_ECAPACITY, "fs_split_children: m does not fit 30 bits");
    if (m > 0 && !aligned16(quats)) return fail(ctx, FS_EINVAL, "fs_split_children: quats must be 16-byte aligned");
    FS_HIP(hipSetDevice(ctx->device), "hipSetDevice");
    FS_HIP(launch_split_children(ctx->stream, m, means, scales, quats, parents, normals, phi, child_means, child_scales),
           "k_split_children");
    return FS_OK;
}

int fs_sample_by_score(fs_ctx* ctx, const uint8_t* candidates, const float* scores, const float* exponentials, int64_t n,
                       uint8_t* sample, int64_t* sampled_host)
{
    if (!ctx) return FS_EINVAL;
    if (n < 0 || (n > 0 && (!candidates || !scores || !exponentials || !sample)))
        return fail(ctx, FS_EINVAL, "fs_sample_by_score: bad arguments");
    if (n >= (int64_t)1 << 31) return fail(ctx, FS_ECAPACITY, "fs_sample_by_score: n does not fit 31 bits");
    if (sampled_host) *sampled_host = 0;
    if (n == 0) return FS_OK;
    FS_HIP(hipSetDevice(ctx->device), "hipSetDevice");
    hipStream_t st = ctx->stream;
    // the candidates' indices, and their number m (one read-back: the sample size floor(m / 2) sizes what follows)
    FS_TRY(ensure(ctx, ctx->compact_pos, (size_t)n * sizeof(uint32_t), "compaction positions"));
    FS_TRY(ensure(ctx, ctx->compact_scan, scan_tmp_bytes(n), "scan"));
    for (int k = 0; k < 2; k++) {
        FS_TRY(ensure(ctx, ctx->sel_keys[k], (size_t)n * sizeof(uint64_t), "sampling keys"));
        FS_TRY(ensure(ctx, ctx->sel_vals[k], (size_t)n * sizeof(uint32_t), "sampling indices"));
    }
    uint64_t* keys[2] = {static_cast<uint64_t*>(ctx->sel_keys[0].ptr), static_cast<uint64_t*>(ctx->sel_keys[1].ptr)};
    uint32_t* vals[2] = {static_cast<uint32_t*>(ctx->sel_vals[0].ptr), static_cast<uint32_t*>(ctx->sel_vals[1].ptr)};
    FS_HIP(launch_compact(st, n, candidates, static_cast<uint32_t*>(ctx->compact_pos.ptr), ctx->compact_scan.ptr,
                          ctx->total_dev, vals[1]),
           "compaction");
    FS_HIP(hipMemcpyAsync(ctx->total_host, ctx->total_dev, sizeof(uint64_t), hipMemcpyDeviceToHost, st), "hipMemcpyAsync");
    FS_HIP(hipStreamSynchronize(st), "hipStreamSynchronize");
    const int64_t m = (int64_t)ctx->total_host[0];
    const int64_t k = m / 2;
    int res = 0;
    if (k > 0) {
        // arrival times e / score as sort keys (ties by index), a stable radix sort on all 64 bits, the first k
        const int64_t nb = radix_num_blocks(m);
        FS_TRY(ensure(ctx, ctx->sel_hist, (size_t)nb * RADIX_DIGITS * sizeof(uint32_t), "histograms"));
        FS_TRY(ensure(ctx, ctx->compact_scan, scan_tmp_bytes(RADIX_DIGITS * nb), "scan"));
        FS_HIP(launch_sample_keys(st, m, vals[1], scores, exponentials, keys[0], vals[0]), "k_sample_keys");
        FS_HIP(launch_radix_sort(st, m, 64, keys, vals, static_cast<uint32_t*>(ctx->sel_hist.ptr), ctx->compact_scan.ptr,
                                 ctx->total_dev, &res),
               "radix sort");
    }
    FS_HIP(launch_mark_indices(st, n, k, vals[res], sample), "k_mark_indices");
    if (sampled_host) *sampled_host = k;
    return FS_OK;
}

int fs_activate_inv(fs_ctx* ctx, int64_t n, const float* scales, const float* opacities, float lo, float hi,
                    float* raw_scales, float* raw_opacities)
{
    if (!ctx) return FS_EINVAL;
    if (n < 0 || !(lo > 0.f) || !(hi < 1.f) || !(lo <= hi) || (n > 0 && (!scales || !opacities || !raw_scales || !raw_opacities)))
        return fail(ctx, FS_EINVAL, "fs_activate_inv: bad arguments");
    FS_HIP(hipSetDevice(ctx->device), "hipSetDevice");
    FS_HIP(launch_activate_inv(ctx->stream, n, scales, opacities, lo, hi, raw_scales, raw_opacities), "k_activate_inv");
    return FS_OK;
}

int fs_measure_peaks(fs_ctx* ctx, int64_t copy_bytes, double* copy_gbs, double* fma_tflops)
{
    if (!ctx) return FS_EINVAL;
    if (copy_bytes < 0 || copy_bytes > ((int64_t)1 << 33)) return fail(ctx, FS_EINVAL, "fs_measure_peaks: bad size");
    ctx->fused_pixels = 0;   // (the scratch that the fused forward pass leaves its error map in is reused here)
    FS_HIP(hipSetDevice(ctx->device), "hipSetDevice");
    hipStream_t st = ctx->stream;
    hipEvent_t a = nullptr, b = nullptr;
    FS_HIP(hipEventCreate(&a), "hipEventCreate");
    if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return hip_fail(ctx, hipGetLastError(), "hipEventCreate"); }
    int rc = FS_OK;
    float ms = 0.f;
    if (copy_gbs && copy_bytes >= 16) {
        const int64_t bytes = copy_bytes / 16 * 16;
        void *src = nullptr, *dst = nullptr;
        if (hipMalloc(&src, (size_t)bytes) != hipSuccess || hipMalloc(&dst, (size_t)bytes) != hipSuccess) {
            (void)hipGetLastError();
            if (src) (void)hipFree(src);
            rc = fail(ctx, FS_ENOMEM, "fs_measure_peaks: allocation failed%s");
        } else {
            hipError_t e = launch_fill_u32(st, static_cast<uint32_t*>(src), 0x3f800000u, bytes / 4);
            for (int r = 0; r < 3 && e == hipSuccess; r++) {   // the third run is the timed one
                if (r == 2) e = hipEventRecord(a, st);
                if (e == hipSuccess) e = launch_copy(st, src, dst, bytes);
            }
            if (e == hipSuccess) e = hipEventRecord(b, st);
            if (e == hipSuccess) e = hipEventSynchronize(b);
            if (e == hipSuccess) e = hipEventElapsedTime(&ms, a, b);
            if (e != hipSuccess) rc = hip_fail(ctx, e, "fs_measure_peaks (copy)");
            else *copy_gbs = 2.0 * (double)bytes / ((double)ms * 1e-3) / 1e9;
            (void)hipStreamSynchronize(st);
            (void)hipFree(src);
            (void)hipFree(dst);
        }
    }
    if (rc == FS_OK && fma_tflops) {
        const int blocks = 256 * 32, iters = 4096;
        FS_TRY(ensure(ctx, ctx->err_map, (size_t)blocks * 256 * sizeof(float), "fma output"));
        hipError_t e = hipSuccess;
        for (int r = 0; r < 2 && e == hipSuccess; r++) {
            if (r == 1) e = hipEventRecord(a, st);
            if (e == hipSuccess) e = launch_fma_chain(st, static_cast<float*>(ctx->err_map.ptr), blocks, iters);
        }
        if (e == hipSuccess) e = hipEventRecord(b, st);
        if (e == hipSuccess) e = hipEventSynchronize(b);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, a, b);
        if (e != hipSuccess) rc = hip_fail(ctx, e, "fs_measure_peaks (fma)");
        else *fma_tflops = 2.0 * 8.0 * (double)iters * (double)blocks * 256.0 / ((double)ms * 1e-3) / 1e12;
    }
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(b);
    return rc;
}

static int prof_collect(fs_ctx* ctx)
{
    FS_HIP(hipStreamSynchronize(ctx->stream), "hipStreamSynchronize");
    for (int g = 0; g < FS_K_COUNT; g++) {
        for (auto& pr : ctx->prof_pending[g]) {
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, pr.first, pr.second) == hipSuccess) {
                ctx->prof_ms[g] += (double)ms;
                ctx->prof_launches[g] += 1;
            } else {
                (void)hipGetLastError();
            }
            ctx->prof_free.push_back(pr.first);
            ctx->prof_free.push_back(pr.second);
        }
        ctx->prof_pending[g].clear();
    }
    return FS_OK;
}

int fs_profile_enable(fs_ctx* ctx, uint32_t group_mask)
{
    if (!ctx) return FS_EINVAL;
    FS_HIP(hipSetDevice(ctx->device), "hipSetDevice");
    FS_TRY(prof_collect(ctx));
    for (int g = 0; g < FS_K_COUNT; g++) { ctx->prof_ms[g] = 0.0; ctx->prof_launches[g] = 0; }
    ctx->prof_mask = group_mask & ((1u << FS_K_COUNT) - 1u);
    return FS_OK;
}

int fs_profile_read(fs_ctx* ctx, int32_t group, const char** name, double* total_ms, int64_t* launches)
{
    if (!ctx) return FS_EINVAL;
    if (group < 0 || group >= FS_K_COUNT) return fail(ctx, FS_EINVAL, "fs_profile_read: bad group");
    FS_HIP(hipSetDevice(ctx->device), "hipSetDevice");
    FS_TRY(prof_collect(ctx));
    if (name) *name = kGroupNames[group];
    if (total_ms) *total_ms = ctx->prof_ms[group];
    if (launches) *launches = ctx->prof_launches[group];
    return FS_OK;
}

}  // extern "C"
