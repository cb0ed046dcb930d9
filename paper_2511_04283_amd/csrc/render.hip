// Per-tile alpha compositing (forward), its gradient (backward) and the high-error-pixel count
// (score) on gfx950.
//
// FastGS Sec. 3, Eq. (4): C(p) = sum_i c_i alpha_i prod_{j<i} (1 - alpha_j), alpha_i = sigma_i G'_i(p),
// Eq. (5): G'_i(p) = exp(-1/2 (p - mu_2D)^T Sigma_2D^-1 (p - mu_2D)).
// Sec. 4.2, Eq. for s_d: per Gaussian, the number of high-error pixels in its footprint.
//
// One workgroup (4 wavefronts) per 16x16 tile, one pixel per lane.  Wavefront w owns the 8x8
// quadrant (w&1, w>>1); each of its four rows of 16 lanes (the unit of the DPP row operations) owns
// one 4x4 sub-tile of that quadrant.  The tile's depth-ordered Gaussians are staged through LDS in
// batches of 256.  While staging, every Gaussian's support {alpha >= alpha_min} is bounded by an
// axis-aligned box (conservatively, see stage_batch) and each of the 16 sub-tiles gets its own
// order-preserving list of the staged Gaussians whose box meets it.  In the inner loops the four
// rows of a wavefront walk their own lists side by side, so one wavefront iteration evaluates
// four different Gaussians on 16 pixels each.  A wavefront stops as soon as all of its 64 pixels
// have terminated.
//
// alpha, T and the blend weights follow a fixed fp32 operation order (fused multiply-adds only
// where written as __builtin_fmaf; the file is compiled with -ffp-contract=off) so that the
// integer outputs they decide (n_contrib, counts) can be reproduced bit for bit on a CPU.  The
// box test only ever drops (Gaussian, pixel) pairs that this arithmetic would reject as well.
#include "common.hpp"

namespace fs {

namespace {

constexpr int BATCH = 256;

// exp(x) for pmin <= x <= 0: t = x*log2(e); n = rint(t); r = t - n; 2^r by a degree-5 polynomial
// (Horner, fused), scaled by 2^n.  The caller guarantees x >= about -5.6, so no range clamp.
__device__ __forceinline__ float exp_c(float x)
{
    const float t = x * 0x1.715476p+0f;
    const float n = __builtin_rintf(t);
    const float r = t - n;
    float p = 0x1.5bba14p-10f;
    p = __builtin_fmaf(p, r, 0x1.3cea88p-7f);
    p = __builtin_fmaf(p, r, 0x1.c6b752p-5f);
    p = __builtin_fmaf(p, r, 0x1.ebf9bcp-3f);
    p = __builtin_fmaf(p, r, 0x1.62e42ap-1f);
    p = __builtin_fmaf(p, r, 1.0f);
    return __builtin_ldexpf(p, (int)n);
}

// 16-byte streaming (non-temporal) store / load
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void nt_store(const uint4& v, uint4* dst)
{
    u32x4 t;
    t.x = v.x; t.y = v.y; t.z = v.z; t.w = v.w;
    __builtin_nontemporal_store(t, reinterpret_cast<u32x4*>(dst));
}
__device__ __forceinline__ uint4 nt_load(const uint4* src)
{
    const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src));
    return make_uint4(t.x, t.y, t.z, t.w);
}

struct Pixel {
    int x, y;
    bool inside;
    float px, py;
};

__device__ __forceinline__ Pixel pixel_of_thread(const CamDev& cam, int tile, int thread)
{
    const int wave = thread >> 6, lane = thread & 63;
    const int tx = tile % cam.tiles_x, ty = tile / cam.tiles_x;
    const int row = lane >> 4;  // 4x4 sub-tile (row & 1, row >> 1) of the quadrant
    Pixel p;
    p.x = tx * TILE + (wave & 1) * 8 + (row & 1) * 4 + (lane & 3);
    p.y = ty * TILE + (wave >> 1) * 8 + (row >> 1) * 4 + ((lane >> 2) & 3);
    p.inside = p.x < cam.width && p.y < cam.height;
    p.px = (float)p.x + 0.5f;
    p.py = (float)p.y + 0.5f;
    return p;
}

__device__ __forceinline__ Pixel pixel_of_thread(const CamDev& cam, int tile)
{
    return pixel_of_thread(cam, tile, (int)threadIdx.x);
}

// LDS image of one batch of a tile's list, shared by the kernels.  A staged Gaussian is one record of RS 16-byte
// words, so that the loops form one address per entry: (mu_x, mu_y, a, 2b), (c, sigma, r, g) and, with WITH_RGB,
// (r, g, b, -sigma/2).
template <bool WITH_RGB>
struct Stage {
    static constexpr int RS = WITH_RGB ? 3 : 2;
    float4 rec[BATCH * RS];
    uint64_t bits[16][4];      // per sub-tile, per staging wavefront: which of its 64 slots the sub-tile visits
    uint8_t list[16][BATCH];   // per sub-tile (index wave*4 + row): batch slots to visit, in list order
    int len[16];               // length of each sub-tile's list
    __device__ __forceinline__ const float4* at(int j) const { return rec + j * RS; }
    // unfilled slots must hold finite numbers: lanes past their list's end compute with a stale slot and
    // contribute exact zeros
    __device__ __forceinline__ void clear(int t)
    {
#pragma unroll
        for (int q = 0; q < RS; q++) rec[t * RS + q] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
};

// Sub-tile st = wave*4 + row of a tile sits at column kx = (wave&1)*2 + (row&1), line ky = (wave>>1)*2 + (row>>1).
// The 16-bit sets (bit st) of the sub-tiles in one column, one line, on one diagonal kx + ky = s or kx - ky = d.
struct SubTiles {
    static constexpr int kx(int st) { return ((st >> 2) & 1) * 2 + (st & 1); }
    static constexpr int ky(int st) { return (st >> 3) * 2 + ((st >> 1) & 1); }
    static constexpr uint32_t col(int k) { uint32_t m = 0; for (int st = 0; st < 16; st++) m |= kx(st) == k ? 1u << st : 0u; return m; }
    static constexpr uint32_t line(int k) { uint32_t m = 0; for (int st = 0; st < 16; st++) m |= ky(st) == k ? 1u << st : 0u; return m; }
    static constexpr uint32_t sum(int s) { uint32_t m = 0; for (int st = 0; st < 16; st++) m |= kx(st) + ky(st) == s ? 1u << st : 0u; return m; }
    static constexpr uint32_t dif(int d) { uint32_t m = 0; for (int st = 0; st < 16; st++) m |= kx(st) - ky(st) == d ? 1u << st : 0u; return m; }
};

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_shr_add(uint32_t v)
{
    return v + (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, false);
}

// Loads entries [first, first+m) of the tile's list into `s` (slot t <- entry first+t) and builds
// the 16 per-sub-tile slot lists.  Returns the length of the list of the calling lane's sub-tile.
// Contains two workgroup barriers; every thread of the workgroup must call it.
//
// Box of a Gaussian: it can only be blended where sigma*G >= alpha_min, i.e. where
// q <= qg = 2 ln(sigma/alpha_min), and the kernels also reject q > -2*power_min.  With
// Sigma_2D = conic^-1, the set {q <= Q} lies within |dx| <= sqrt(Q Sigma_xx), |dy| <= sqrt(Q Sigma_yy).
// Q is taken as min(qg, -2 power_min) + 0.1 + e, where e bounds the rounding error of the fp32 q
// for any pixel of a tile the Gaussian is paired with (|dx|,|dy| <= 3 sqrt(lambda_max) + 17), and the
// half-widths get a further 0.2 % + 0.01 px (the box itself is computed with the fast reciprocal,
// square root and logarithm): outside the box the pinned arithmetic yields alpha < 0.96 alpha_min
// (or power < power_min), so dropping the pair cannot change any result.  The same argument gives
// bounds on dx + dy and dx - dy (an octagon around the support).
//
// Lists: each staging wavefront ballots, per sub-tile, which of its 64 slots are kept (phase 1);
// then the 16 lanes that own a sub-tile in the render loops expand its 256-bit mask into slot
// numbers, 16 slots per lane, with a prefix sum over the row (phase 2).
// ID_MODE: 0 = s_id unused, 1 = s_id[t] <- Gaussian index, 2 = s_id[t] <- index of the pair's
// gradient record (where the pair was emitted before the sort: offset + place in the rectangle).
template <bool WITH_RGB, int ID_MODE>
__device__ __forceinline__ int stage_batch(Stage<WITH_RGB>& s, uint32_t* s_id, const CamDev& cam,
                                           const CfgDev& cfg, int tile, const uint32_t* __restrict__ gauss_sorted,
                                           const float4* __restrict__ splats, uint32_t first, int m)
{
    const int t = threadIdx.x;
    const int swave = t >> 6, lane = t & 63;
    uint32_t sub_mask = 0;  // bit (wave*4 + row) of every sub-tile the box meets
    if (t < m) {
        const uint32_t g = gauss_sorted[first + t];
        const float4* rec = splats + (size_t)g * (SPLAT_REC / 4);  // one 64-byte line
        const float4 r0 = rec[0], r1 = rec[1], r2 = rec[2];
        const float2 xy = make_float2(r0.x, r0.y);
        const float4 co = make_float4(r0.z, r0.w, r1.x, r1.y);
        s.rec[t * s.RS] = make_float4(xy.x, xy.y, co.x, co.y + co.y);
        s.rec[t * s.RS + 1] = make_float4(co.z, co.w, r1.z, r1.w);
        // (the backward pass takes the colour and -sigma / 2 with one aligned 16-byte read)
        if (WITH_RGB) s.rec[t * s.RS + 2] = make_float4(r1.z, r1.w, r2.x, -0.5f * co.w);
        if (ID_MODE == 1) s_id[t] = g;
        if (ID_MODE == 2) {
            const uint32_t r01 = __float_as_uint(r2.z), r23 = __float_as_uint(r2.w);
            const uint32_t x0 = r01 & 0xffffu, y0 = r01 >> 16, x1 = r23 & 0xffffu;
            s_id[t] = __float_as_uint(r2.y) + ((uint32_t)(tile / cam.tiles_x) - y0) * (x1 - x0) +
                      ((uint32_t)(tile % cam.tiles_x) - x0);
        }
        const float ratio = co.w * __builtin_amdgcn_rcpf(cfg.alpha_min);
        if (ratio >= 1.0f) {
            const float det = co.x * co.z - co.y * co.y;
            const float inv = __builtin_amdgcn_rcpf(det);
            const float sxx = co.z * inv, syy = co.x * inv;
            const float D = 3.0f * __builtin_amdgcn_sqrtf(sxx + syy) + 17.0f;
            const float e = 1e-6f * (fabsf(co.x) + 2.0f * fabsf(co.y) + fabsf(co.z)) * D * D;
            const float Q = fminf(2.0f * __logf(ratio), -2.0f * cfg.power_min) + 0.1f + e;
            const float hx = __builtin_amdgcn_sqrtf(Q * sxx) * 1.002f + 0.01f;
            const float hy = __builtin_amdgcn_sqrtf(Q * syy) * 1.002f + 0.01f;
            // sub-tile column k has its centre at +4k+2 from the tile origin; pixel centres reach 1.5 from it
            const float ox = xy.x - (float)((tile % cam.tiles_x) * TILE), oy = xy.y - (float)((tile / cam.tiles_x) * TILE);
            // Every test below concerns a whole family of sub-tiles at once (a column, a line, a diagonal), so each is
            // made once and switches on the family's 16-bit pattern (SubTiles::col ...): 22 tests and a few ANDs instead
            // of four tests per sub-tile.
            uint32_t colm = 0, rowm = 0;
#pragma unroll
            for (int k = 0; k < 4; k++) {
                colm |= (fabsf(ox - (float)(4 * k + 2)) <= hx + 1.5f) ? SubTiles::col(k) : 0u;
                rowm |= (fabsf(oy - (float)(4 * k + 2)) <= hy + 1.5f) ? SubTiles::line(k) : 0u;
            }
            // NaN half-widths (degenerate conic) keep the Gaussian everywhere: the exact test decides
            if (!(hx == hx) || !(hy == hy)) { colm = 0xffffu; rowm = 0xffffu; }
            // The same set also lies between the tangent lines at +-45 degrees: |dx + dy| <= sqrt(Q (Sxx + Syy + 2 Sxy)),
            // |dx - dy| <= sqrt(Q (Sxx + Syy - 2 Sxy)) with Sxy = -b/det; a sub-tile's pixel centres reach 3 from
            // its centre in these sums.  This trims the corners of the box for slanted, elongated Gaussians.
            const float sxy = -co.y * inv;
            const float hu = __builtin_amdgcn_sqrtf(fmaxf(Q * (sxx + syy + 2.0f * sxy), 0.f)) * 1.002f + 0.02f;
            const float hv = __builtin_amdgcn_sqrtf(fmaxf(Q * (sxx + syy - 2.0f * sxy), 0.f)) * 1.002f + 0.02f;
            const float su = ox + oy, sv = ox - oy;
            const bool nan8 = !(hu == hu) || !(hv == hv);
            // the sub-tile in column kx, line ky has its centre at sum 4 (kx + ky) + 4 and difference 4 (kx - ky)
            uint32_t summ = 0, difm = 0;
#pragma unroll
            for (int d = 0; d < 7; d++) {
                summ |= (fabsf(su - (float)(4 * d + 4)) <= hu + 3.0f) ? SubTiles::sum(d) : 0u;
                difm |= (fabsf(sv - (float)(4 * (d - 3))) <= hv + 3.0f) ? SubTiles::dif(d - 3) : 0u;
            }
            sub_mask = colm & rowm & (nan8 ? 0xffffu : (summ & difm));
        }
    }
    // phase 1: one 64-bit keep mask per (sub-tile, staging wavefront)
    uint64_t keep = 0;
#pragma unroll
    for (int st = 0; st < 16; st++) {
        const uint64_t bal = __ballot((sub_mask >> st) & 1u);
        keep = lane == st ? bal : keep;
    }
    if (lane < 16) s.bits[lane][swave] = keep;
    __syncthreads();
    // phase 2: lane i of the row that owns sub-tile st expands slots [16 i, 16 i + 16)
    const int st = swave * 4 + (lane >> 4);
    const int i = lane & 15;
    uint32_t b16 = (uint32_t)(s.bits[st][i >> 2] >> ((i & 3) * 16)) & 0xffffu;
    const uint32_t cnt = __popc(b16);
    uint32_t inc = cnt;
    inc = dpp_shr_add<0x111>(inc);  // row_shr:1
    inc = dpp_shr_add<0x112>(inc);  // row_shr:2
    inc = dpp_shr_add<0x114>(inc);  // row_shr:4
    inc = dpp_shr_add<0x118>(inc);  // row_shr:8
    uint32_t pos = inc - cnt;
    while (b16) {
        const uint32_t b = __builtin_ctz(b16);
        s.list[st][pos++] = (uint8_t)(16 * i + b);
        b16 &= b16 - 1u;
    }
    const int mine = __shfl((int)inc, (lane & 48) | 15, 64);
    if (i == 15) s.len[st] = (int)inc;
    __syncthreads();
    return mine;
}

// One step of a sum (three doubles) and a minimum / maximum (bit patterns of non-negative floats, which order like
// unsigned integers) over the lanes of a wavefront: every lane combines its values with those of the lane the DPP
// control names; a lane without such a source (the start of a row, a row the mask leaves out) adds zero and keeps
// its extrema.  SHIFT: a shift within the rows (all rows take part, a missing source reads as zero).
template <int CTRL, int ROW_MASK, bool SHIFT>
__device__ __forceinline__ void wave_step(double& a, double& b, double& c, uint32_t& lo, uint32_t& hi)
{
    auto moved = [](double v) {
        const long long bits = __double_as_longlong(v);
        const int l = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)bits, CTRL, ROW_MASK, 0xF, SHIFT);
        const int h = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)((unsigned long long)bits >> 32), CTRL, ROW_MASK, 0xF, SHIFT);
        return __longlong_as_double((long long)(((unsigned long long)(uint32_t)h << 32) | (uint32_t)l));
    };
    a += moved(a);
    b += moved(b);
    c += moved(c);
    // (the minimum must not meet the zero a missing source reads as: its own value stands in)
    lo = min(lo, (uint32_t)__builtin_amdgcn_update_dpp((int)lo, (int)lo, CTRL, ROW_MASK, 0xF, false));
    hi = max(hi, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)hi, CTRL, ROW_MASK, 0xF, SHIFT));
}

// Longest of the four sub-tile lists of the calling wavefront (`mine` is uniform within a row).
__device__ __forceinline__ int wave_max_of_rows(int mine)
{
    const int a = __builtin_amdgcn_readlane(mine, 0), b = __builtin_amdgcn_readlane(mine, 16);
    const int c = __builtin_amdgcn_readlane(mine, 32), d = __builtin_amdgcn_readlane(mine, 48);
    // (read back through a scalar register: a loop bound the compiler knows to be uniform is counted by the scalar unit)
    return __builtin_amdgcn_readfirstlane(max(max(a, b), max(c, d)));
}

// FUSED: the epilogue also does, per pixel, what the L1 term (FastGS Sec. 4.5) and the error map of the
// multi-view score (Sec. 4.2) need from the finished colour -- dL/dC = sign(C - target) * scale, the error
// e = ((|d0| + |d1|) + |d2|) / 3 -- and leaves this tile's partial sums (sum of |d|; sum, min, max and sum of squares
// of e) at tile_partial[q * num_tiles + tile], so that the image is not read again for them.
//
// BITS: the kernel also records, for every pair of the tile's list (by its position in the sorted order), at which
// of the tile's 256 pixels the Gaussian is counted by the multi-view score (Sec. 4.2): where it is blended and, in
// FS_SCORE_WEIGHT mode, alpha T > alpha_min.  32 bytes per pair: 16 sub-tiles (index wave*4 + row) x 16 bits (lane
// within the row); one more byte per pair says whether any of them is set, and only then is the row written.  With
// these the count pass is a population count per pair instead of a second walk over the lists (k_score_bits).
template <bool FUSED, bool BITS>
__global__ __launch_bounds__(256) void k_render_fwd(CamDev cam, CfgDev cfg, const uint2* __restrict__ ranges,
                                                    const uint32_t* __restrict__ tile_order,
                                                    const uint32_t* __restrict__ gauss_sorted,
                                                    const float4* __restrict__ splats, float* __restrict__ image,
                                                    float* __restrict__ final_T, uint32_t* __restrict__ n_contrib,
                                                    const float* __restrict__ target, float scale,
                                                    float* __restrict__ dL, float* __restrict__ err,
                                                    double* __restrict__ tile_partial, ScoreRecord record)
{
    __shared__ Stage<true> s;
    __shared__ __align__(16) uint16_t s_pb[BITS ? BATCH : 1][16];  // this batch's bits, [slot][sub-tile]
    __shared__ uint32_t s_rows;                                    // rows of the record this tile has written so far

    const int tile = (int)tile_order[blockIdx.x];  // longest lists first
    const int sub = (threadIdx.x >> 6) * 4 + ((threadIdx.x & 63) >> 4);  // this lane's sub-tile list
    const Pixel p = pixel_of_thread(cam, tile);
    const uint2 range = ranges[tile];
    const int total = (int)(range.y - range.x);

    bool done = !p.inside;
    float T = 1.0f, C0 = 0.f, C1 = 0.f, C2 = 0.f;
    uint32_t last = 0;

    // Slots a batch does not fill must still hold finite numbers: lanes past the end of their list
    // read a stale slot and multiply its colour by a zero weight.
    s.clear(threadIdx.x);

    // BITS: row t of s_pb is zeroed and written out by thread t alone; the other wavefronts set bits in it between
    // a batch's staging barriers and the barrier at the top of the next batch
    const float hit_above = cfg.score_mode == FS_SCORE_ALPHA ? 0.0f : cfg.alpha_min;
    int pending = -1, pending_m = 0;  // the batch whose bits are in s_pb and not yet in memory (uniform)
    if (BITS && threadIdx.x == 0) s_rows = 0;   // (the first use lies behind the barrier at the top of the second batch)
    auto write_bits = [&](int first, int count) {
        // A pair that is counted nowhere (at 500k Gaussians half of them: the rectangle's corners, entries behind the
        // last blended one) leaves nothing.  The others' rows are packed at the start of the tile's segment: a
        // wavefront reserves as many places as it has rows with one LDS atomic, so the order of the rows within the
        // tile depends on which wavefront comes first (the count pass adds integers: its result does not).
        uint4 lo = make_uint4(0u, 0u, 0u, 0u), hi = lo;
        if ((int)threadIdx.x < count) {
            const uint4* row = reinterpret_cast<const uint4*>(s_pb[threadIdx.x]);
            lo = row[0];
            hi = row[1];
        }
        const bool any = ((lo.x | lo.y) | (lo.z | lo.w) | (hi.x | hi.y) | (hi.z | hi.w)) != 0u;
        const uint64_t bal = __ballot(any);
        if (bal != 0) {   // (uniform over the wavefront)
            uint32_t base = 0;
            if ((threadIdx.x & 63) == 0) base = atomicAdd(&s_rows, (uint32_t)__popcll(bal));
            base = (uint32_t)__builtin_amdgcn_readfirstlane((int)base);
            if (any) {
                const uint32_t below = __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0u));
                const size_t at = (size_t)range.x + base + below;
                // (streaming stores: the record is read once, by the count pass, and should not displace the step's
                // other arrays from the caches)
                nt_store(lo, record.rows + at * 2);
                nt_store(hi, record.rows + at * 2 + 1);
                record.row_gauss[at] = gauss_sorted[(size_t)range.x + first + threadIdx.x];
            }
        }
    };
    for (int start = 0; start < total; start += BATCH) {
        const int alive = __syncthreads_count(!done);
        if (BITS && pending >= 0) {
            write_bits(pending, pending_m);
            pending = -1;
        }
        if (alive == 0) break;
        const int m = min(BATCH, total - start);
        if (BITS) {
            uint4* row = reinterpret_cast<uint4*>(s_pb[threadIdx.x]);
            row[0] = make_uint4(0u, 0u, 0u, 0u);
            row[1] = make_uint4(0u, 0u, 0u, 0u);
            pending = start;
            pending_m = m;
        }
        const int mine = stage_batch<true, 0>(s, nullptr, cam, cfg, tile, gauss_sorted, splats, range.x + start, m);
        // a row whose 16 pixels have all finished does not lengthen the wavefront's loop
        const bool row_alive = ((__ballot(!done) >> (threadIdx.x & 48)) & 0xffffull) != 0;
        const int longest = wave_max_of_rows(row_alive ? mine : 0);
        // Straight-line body with selects: lanes past their list's end (or finished) read a stale
        // slot and discard the result; one wave-uniform branch per iteration.  (Skipping the rest of an
        // iteration when no lane passes the range test does not pay: four rows look at four different
        // Gaussians, so all of them missing is rare, and the test costs more than it saves.)
        int lastj = -1;   // batch slot of the last Gaussian this pixel blended in this batch
        for (int k = 0; k < longest; k++) {
            // (every fourth trip: a wavefront whose pixels have all terminated leaves the loop)
            if ((k & 3) == 0 && __ballot(!done) == 0) break;
            const int j = s.list[sub][k];
            const float4* e = s.at(j);
            const float4 r0 = e[0], r1 = e[1];           // (mu_x, mu_y, a, 2b), (c, sigma, r, g)
            const float dx = p.px - r0.x, dy = p.py - r0.y;
            const float u = __builtin_fmaf(r0.w, dy, r0.z * dx);
            const float q = __builtin_fmaf(dx, u, (r1.x * dy) * dy);
            const float power = -0.5f * q;
            bool ok = (k < mine) & !done & !(power > 0.0f) & !(power < cfg.power_min);
            const float colb = e[2].z;
            const float G = exp_c(power);
            const float alpha = fminf(cfg.alpha_max, r1.y * G);
            ok = ok & (alpha >= cfg.alpha_min);
            const float Tn = T * (1.0f - alpha);
            const bool stop = ok & (Tn < cfg.T_min);
            const bool blend = ok & !stop;
            done = done | stop;
            const float w = blend ? alpha * T : 0.0f;  // a zero weight leaves C unchanged bit for bit
            C0 = __builtin_fmaf(r1.z, w, C0);
            C1 = __builtin_fmaf(r1.w, w, C1);
            C2 = __builtin_fmaf(colb, w, C2);
            if (BITS) {
                // (kept behind the colour update: scheduled ahead of it, the LDS store below would sit between the
                // colour's LDS read and the wait for it, and every iteration would wait for the store as well)
                asm volatile("" : "+v"(C0), "+v"(C1), "+v"(C2) : : "memory");
                // w is alpha T with the transmittance in front of this Gaussian where it is blended (> 0 then), else 0:
                // one comparison against alpha_min (FS_SCORE_WEIGHT) or 0 (FS_SCORE_ALPHA) decides
                const uint64_t hb = __builtin_amdgcn_ballot_w64(w > hit_above);
                // the row's first lane stores the row's 16 bits (past the end of the row's list j is stale)
                if ((threadIdx.x & 15) == 0 && k < mine) s_pb[j][sub] = (uint16_t)(hb >> (threadIdx.x & 48));
            }
            T = blend ? Tn : T;
            lastj = blend ? j : lastj;
        }
        last = lastj >= 0 ? (uint32_t)(start + lastj + 1) : last;
    }
    if (BITS) {
        if (pending >= 0) {
            __syncthreads();
            write_bits(pending, pending_m);
        }
        // (pairs the loop never reached -- every pixel had finished -- are blended nowhere and leave no row)
        __syncthreads();
        if (threadIdx.x == 0) record.tile_rows[tile] = (int32_t)s_rows;
    }
    double l1 = 0.0, esum = 0.0, esq = 0.0, emin = 1.0e300, emax = -1.0e300;
    if (p.inside) {
        const size_t hw = (size_t)cam.width * cam.height;
        const size_t pix = (size_t)p.y * cam.width + p.x;
        const float c0 = __builtin_fmaf(T, cfg.bg[0], C0), c1 = __builtin_fmaf(T, cfg.bg[1], C1);
        const float c2 = __builtin_fmaf(T, cfg.bg[2], C2);
        image[pix] = c0;
        image[hw + pix] = c1;
        image[2 * hw + pix] = c2;
        final_T[pix] = T;
        n_contrib[pix] = last;
        if (FUSED) {
            const float d0 = c0 - target[pix], d1 = c1 - target[hw + pix], d2 = c2 - target[2 * hw + pix];
            if (dL) {
                dL[pix] = d0 > 0.f ? scale : (d0 < 0.f ? -scale : 0.f);
                dL[hw + pix] = d1 > 0.f ? scale : (d1 < 0.f ? -scale : 0.f);
                dL[2 * hw + pix] = d2 > 0.f ? scale : (d2 < 0.f ? -scale : 0.f);
            }
            const float e = ((fabsf(d0) + fabsf(d1)) + fabsf(d2)) / 3.0f;
            err[pix] = e;
            l1 = ((double)fabsf(d0) + (double)fabsf(d1)) + (double)fabsf(d2);
            esum = emin = emax = (double)e;
            esq = (double)e * (double)e;
        }
    }
    if (FUSED) {
        // per-wavefront partials (sums in double, extrema of the fp32 errors in float: exact) by DPP moves -- four
        // shifts within the rows of 16 lanes, lane 15 of rows 0 and 2 into the row after it, lane 31 into rows 2 and
        // 3 -- which leave the totals in lane 63; combined across the four wavefronts through LDS with a single barrier
        // (errors are >= 0: threads outside the image carry +3e38 for the minimum and 0 for the maximum)
        uint32_t lo_e = __float_as_uint((float)emin == (float)emin && emin < 1.0e299 ? (float)emin : 3.0e38f);
        uint32_t hi_e = __float_as_uint(emax > -1.0e299 ? (float)emax : 0.0f);
        wave_step<0x111, 0xF, true>(l1, esum, esq, lo_e, hi_e);
        wave_step<0x112, 0xF, true>(l1, esum, esq, lo_e, hi_e);
        wave_step<0x114, 0xF, true>(l1, esum, esq, lo_e, hi_e);
        wave_step<0x118, 0xF, true>(l1, esum, esq, lo_e, hi_e);
        wave_step<0x142, 0xA, false>(l1, esum, esq, lo_e, hi_e);
        wave_step<0x143, 0xC, false>(l1, esum, esq, lo_e, hi_e);
        const float fmin_e = __uint_as_float(lo_e), fmax_e = __uint_as_float(hi_e);
        // (the staging masks serve as the 4 x 5 doubles of scratch: they are only live inside stage_batch, between
        // its two barriers, and every wavefront has left its last stage_batch before any of them gets here)
        static_assert(sizeof(s.bits) >= 4 * 5 * sizeof(double), "scratch for the per-wavefront partials");
        double (*s_part)[5] = reinterpret_cast<double (*)[5]>(&s.bits[0][0]);
        if ((threadIdx.x & 63) == 63) {
            double* w = s_part[threadIdx.x >> 6];
            w[0] = l1; w[1] = esum; w[2] = (double)fmin_e; w[3] = (double)fmax_e; w[4] = esq;
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            const size_t nt = (size_t)cam.tiles_x * cam.tiles_y;
            tile_partial[tile] = (s_part[0][0] + s_part[1][0]) + (s_part[2][0] + s_part[3][0]);
            tile_partial[nt + tile] = (s_part[0][1] + s_part[1][1]) + (s_part[2][1] + s_part[3][1]);
            tile_partial[2 * nt + tile] = fmin(fmin(s_part[0][2], s_part[1][2]), fmin(s_part[2][2], s_part[3][2]));
            tile_partial[3 * nt + tile] = fmax(fmax(s_part[0][3], s_part[1][3]), fmax(s_part[2][3], s_part[3][3]));
            tile_partial[4 * nt + tile] = (s_part[0][4] + s_part[1][4]) + (s_part[2][4] + s_part[3][4]);
        }
    }
}

// ---- row reduction of 9 values -------------------------------------------------------------
// A row of 16 lanes (one 4x4 sub-tile) sums 9 per-pixel values.  Instead of 9 separate butterflies
// the first three steps halve the number of live registers: at the step for lane bit b, a lane
// keeps the value whose index has that bit equal to its own and hands the other one to its partner.
// After the four steps lane i of the row holds the row total of value (i & 7); value 8 is summed
// the plain way and ends up in every lane.

template <int CTRL>
__device__ __forceinline__ float dpp_get(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}

// lanes with `bit` clear end up with sum(a) over the exchanged pair, lanes with it set with sum(b)
template <int CTRL>
__device__ __forceinline__ float fold(bool bit, float a, float b)
{
    const float keep = bit ? b : a, give = bit ? a : b;
    return keep + dpp_get<CTRL>(give);
}

__device__ __forceinline__ void row_reduce9(const float v[9], int lane, float& packed, float& ninth)
{
    constexpr int XOR1 = 0xB1, XOR2 = 0x4E, ROR4 = 0x124, ROR8 = 0x128;  // quad_perm swaps, row rotations
    const bool b0 = lane & 1, b1 = lane & 2, b2 = lane & 4;
    const float r01 = fold<XOR1>(b0, v[0], v[1]);
    const float r23 = fold<XOR1>(b0, v[2], v[3]);
    const float r45 = fold<XOR1>(b0, v[4], v[5]);
    const float r67 = fold<XOR1>(b0, v[6], v[7]);
    float r8 = v[8] + dpp_get<XOR1>(v[8]);
    const float s03 = fold<XOR2>(b1, r01, r23);
    const float s47 = fold<XOR2>(b1, r45, r67);
    r8 = r8 + dpp_get<XOR2>(r8);
    // lane i+4 has the opposite bit 2, so a rotation by 4 pairs the lanes like the earlier swaps did
    float u = fold<ROR4>(b2, s03, s47);
    r8 = r8 + dpp_get<ROR4>(r8);
    u = u + dpp_get<ROR8>(u);
    r8 = r8 + dpp_get<ROR8>(r8);
    packed = u;
    ninth = r8;
}

// Two more values: afterwards the even lanes of the row hold the total of a, the odd lanes that of b.
__device__ __forceinline__ float row_reduce2(float a, float b, int lane)
{
    constexpr int XOR1 = 0xB1, XOR2 = 0x4E, ROR4 = 0x124, ROR8 = 0x128;
    float r = fold<XOR1>(lane & 1, a, b);
    r = r + dpp_get<XOR2>(r);
    r = r + dpp_get<ROR4>(r);
    r = r + dpp_get<ROR8>(r);
    return r;
}

// Backward of the compositing.  Walks each sub-tile's list back to front from the furthest blended
// Gaussian; per Gaussian, 9 partial sums over the 16 pixels of a sub-tile are formed across the
// row's lanes and combined across the sub-tiles in LDS.  The 9 sums: dL/drgb (3), dL/dsigma, and with
// g = dL/dq the moments sum g dx^2, g dx dy, g dy^2, g dx, g dy, from which dL/dconic and dL/dmu_2D
// follow at the flush (dq/dmu is linear in d = p - mu).
//
// Every Gaussian-tile pair owns one record of PAIR_REC floats in `pair_grad`, at the position the
// pair had when it was emitted (pair_offsets[g] + its place in g's tile rectangle): the flush is a
// plain store (rgb 3, sigma, conic 3, mu_2D 2), every pair of the tile is written exactly once (zeros
// for the ones nothing blended), and the per-Gaussian sum over its contiguous records is left to the
// projection's backward kernel.  No global atomics.  The only sums whose order depends on scheduling are those of a
// Gaussian's (up to 16) sub-tile totals within a tile, taken in double precision in LDS: the record is the same from
// run to run unless the exponents of those terms span more than 29 bits.
//
// ABS adds the absolute positional gradient (used by FastGS for the split decision): per pixel the
// magnitudes |dL/dmu_x|, |dL/dmu_y| of its own contribution, summed like the other values and stored
// in the record's floats 9 and 10.
template <bool ABS, bool SPARSE>
__global__ __launch_bounds__(256) void k_render_bwd(
    CamDev cam, CfgDev cfg, const uint2* __restrict__ ranges, const uint32_t* __restrict__ tile_order,
    const uint32_t* __restrict__ gauss_sorted,
    const float4* __restrict__ splats, const float* __restrict__ final_T, const uint32_t* __restrict__ n_contrib,
    const float* __restrict__ dL_dimage, float4* __restrict__ pair_grad, uint8_t* __restrict__ rec_valid)
{
    __shared__ Stage<true> s;
    __shared__ uint32_t s_id[BATCH];
    constexpr int NV = ABS ? 11 : 9;
    // The sub-tiles' sums of a Gaussian meet in double precision: on this chip the LDS atomic add of a double is
    // markedly cheaper than that of a float (the kernel takes 0.19 ms instead of 0.23 at 500k Gaussians), and the
    // sum of up to 16 single-precision terms is then exact unless their exponents span more than 29 bits.
    typedef double acc_t;
    __shared__ acc_t s_acc[BATCH][NV];
    __shared__ int s_max;

    const int tile = (int)tile_order[blockIdx.x];  // longest lists first
    const Pixel p = pixel_of_thread(cam, tile);
    const uint2 range = ranges[tile];
    const size_t hw = (size_t)cam.width * cam.height;
    const size_t pix = (size_t)p.y * cam.width + p.x;
    const int lane = threadIdx.x & 63;
    const int sub = (threadIdx.x >> 6) * 4 + (lane >> 4);

    const int last = p.inside ? (int)n_contrib[pix] : 0;
    float T = p.inside ? final_T[pix] : 0.f;
    float dC0 = 0.f, dC1 = 0.f, dC2 = 0.f;
    if (p.inside) {
        dC0 = dL_dimage[pix];
        dC1 = dL_dimage[hw + pix];
        dC2 = dL_dimage[2 * hw + pix];
    }
    // dC . (colour composited behind the Gaussian at hand): all that dL/dalpha = T (dC . c - S) needs of it
    float S = __builtin_fmaf(dC2, cfg.bg[2], __builtin_fmaf(dC1, cfg.bg[1], dC0 * cfg.bg[0]));

    // unfilled slots must hold finite numbers (lanes past their list's end compute with them and
    // contribute exact zeros)
    s.clear(threadIdx.x);
    if (threadIdx.x == 0) s_max = 0;
    __syncthreads();
    atomicMax(&s_max, last);
    __syncthreads();
    const int total = s_max;  // entries at positions >= total are blended by no pixel of the tile

    // batches from the back: batch b covers positions [b*BATCH, min(total,(b+1)*BATCH))
    for (int start = ((total - 1) / BATCH) * BATCH; start >= 0 && total > 0; start -= BATCH) {
        const int m = min(BATCH, total - start);
        __syncthreads();  // the previous batch's flush has read s_acc / s_id
#pragma unroll
        for (int k = 0; k < NV; k++) s_acc[threadIdx.x][k] = (acc_t)0;
        const int mine = stage_batch<true, 2>(s, s_id, cam, cfg, tile, gauss_sorted, splats, range.x + start, m);
        // a row none of whose pixels reaches into this batch does not lengthen the wavefront's loop
        const bool row_walks = ((__ballot(start < last) >> (lane & 48)) & 0xffffull) != 0;
        const int longest = wave_max_of_rows(row_walks ? mine : 0);
        const int last_here = last - start;   // slots below this one hold entries this pixel blended (or examined)
        for (int it = 0; it < longest; it++) {
            const int k = mine - 1 - it;      // every row walks its own list from the back
            const int j = s.list[sub][k & (BATCH - 1)];
            const float4* e = s.at(j);
            const float4 r0 = e[0], r1 = e[1];           // (mu_x, mu_y, a, 2b), (c, sigma, r, g)
            const float dx = p.px - r0.x, dy = p.py - r0.y;
            const float u = __builtin_fmaf(r0.w, dy, r0.z * dx);
            const float q = __builtin_fmaf(dx, u, (r1.x * dy) * dy);
            const float power = -0.5f * q;
            bool act = (k >= 0) & (j < last_here) & !(power > 0.0f) & !(power < cfg.power_min);
            float G = exp_c(power);   // (whatever the exponent of a lane that fails the test: its result is dropped)
            const float sG = r1.y * G;
            float alpha = fminf(cfg.alpha_max, sG);
            act = act & (alpha >= cfg.alpha_min);
            const uint64_t act_mask = __ballot(act);
            if (act_mask == 0) continue;
            // lanes that do not blend this Gaussian run the same arithmetic with alpha = G = 0:
            // every one of their 9 contributions is then an exact zero (and T / (1 - 0) leaves T as it is)
            alpha = act ? alpha : 0.f;
            G = act ? G : 0.f;
            const float4 r2 = e[2];   // (r, g, b, -sigma / 2)
            T = T * __builtin_amdgcn_rcpf(1.0f - alpha);             // transmittance in front of this Gaussian
            const float w = alpha * T;
            float v[9];
            v[0] = w * dC0;
            v[1] = w * dC1;
            v[2] = w * dC2;
            const float cd = __builtin_fmaf(r2.z, dC2, __builtin_fmaf(r2.y, dC1, r2.x * dC0));   // dC . c
            const float diff = cd - S;
            float dL_dalpha = T * diff;
            S = __builtin_fmaf(alpha, diff, S);
            dL_dalpha = sG > cfg.alpha_max ? 0.f : dL_dalpha;  // capped alpha is a constant
            v[3] = G * dL_dalpha;                              // d/d sigma
            const float gq = r2.w * v[3];                      // d/d q = -1/2 sigma G dL/dalpha
            const float gx = gq * dx, gy = gq * dy;
            v[4] = gx * dx;
            v[5] = gx * dy;
            v[6] = gy * dy;
            v[7] = gx;
            v[8] = gy;
            float packed, ninth;
            row_reduce9(v, lane, packed, ninth);
            // lanes 0..7 of a row hold the totals of values 0..7, lane 8 adds the ninth
            const int li = lane & 15;
            if (ABS) {
                // |dq/dmu . g| per pixel: (2a dx + 2b dy, 2b dx + 2c dy) scaled by |g|  (r0.w holds 2b)
                const float ag = fabsf(gq);
                const float ax = ag * fabsf(__builtin_fmaf(r0.w, dy, 2.0f * r0.z * dx));
                const float ay = ag * fabsf(__builtin_fmaf(r0.w, dx, 2.0f * r1.x * dy));
                const float r2 = row_reduce2(ax, ay, lane);
                // lane 10 (even) holds the total of ax -> slot 9, lane 9 (odd) that of ay -> slot 10
                // (a row none of whose pixels blends the Gaussian has zero totals: nothing to add)
                const float tot = li < 8 ? packed : (li == 8 ? ninth : r2);
                if (li < 11 && tot != 0.f && k >= 0) atomicAdd(&s_acc[j][li < 9 ? li : 19 - li], (acc_t)tot);
            } else {
                const float tot = li < 8 ? packed : ninth;
                if (li < 9 && tot != 0.f && k >= 0) atomicAdd(&s_acc[j][li], (acc_t)tot);
            }
        }
        __syncthreads();
        if ((int)threadIdx.x < m) {
            float a[NV];
#pragma unroll
            for (int k = 0; k < NV; k++) a[k] = (float)s_acc[threadIdx.x][k];
            // SPARSE: a pair that received nothing (blended at no pixel of the tile) leaves no record; its flag stays 0
            // and k_preprocess_bwd does not read the record's place
            bool any = !SPARSE;
            if (SPARSE) {
#pragma unroll
                for (int k = 0; k < NV; k++) any = any | (a[k] != 0.f);
            }
            if (any) {
                const float4 f0 = s.at(threadIdx.x)[0], f1 = s.at(threadIdx.x)[1];
                const float4 co = make_float4(f0.z, f0.w, f1.x, f1.y);  // (a, 2b, c, sigma)
                const uint32_t idx = s_id[threadIdx.x];
                float4* rec = pair_grad + (size_t)idx * (PAIR_REC / 4);
                rec[0] = make_float4(a[0], a[1], a[2], a[3]);
                // d = p - mu  =>  dq/dmu = -(2 a dx + 2b dy, 2b dx + 2 c dy)
                rec[1] = make_float4(a[4], 2.0f * a[5], a[6], -(2.0f * co.x * a[7] + co.y * a[8]));
                rec[2] = make_float4(-(co.y * a[7] + 2.0f * co.z * a[8]), ABS ? a[NV - 2] : 0.f, ABS ? a[NV - 1] : 0.f, 0.f);
                if (SPARSE) rec_valid[idx] = 1;
            }
        }
    }
    // pairs behind the furthest blended Gaussian of the tile received nothing (SPARSE: their flags stay 0)
    if (!SPARSE) {
        for (uint32_t pos = range.x + total + threadIdx.x; pos < range.y; pos += 256) {
            const float4 r2 = splats[(size_t)gauss_sorted[pos] * (SPLAT_REC / 4) + 2];
            const uint32_t r01 = __float_as_uint(r2.z), r23 = __float_as_uint(r2.w);
            const uint32_t x0 = r01 & 0xffffu, y0 = r01 >> 16, x1 = r23 & 0xffffu;
            const uint32_t idx = __float_as_uint(r2.y) + ((uint32_t)(tile / cam.tiles_x) - y0) * (x1 - x0) +
                                 ((uint32_t)(tile % cam.tiles_x) - x0);
            float4* rec = pair_grad + (size_t)idx * (PAIR_REC / 4);
            rec[0] = make_float4(0.f, 0.f, 0.f, 0.f);
            rec[1] = make_float4(0.f, 0.f, 0.f, 0.f);
            rec[2] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
}

// ---- per-splat-parallel backward (the mapping of Taming-3DGS that the paper's baseline uses) -------------
// Alternative to k_render_bwd with the same inputs, outputs and record layout; kept for comparison.
// A wavefront owns one 8x8 quadrant of the tile.  Per batch it forms the quadrant's list (the staged entries
// whose box meets any of its four sub-tiles), takes it in chunks of 64 entries from the back, one entry per
// lane (lane 0 = the entry furthest back), and passes the quadrant's 64 pixels by one after the other.  For a
// pixel p every lane evaluates its own Gaussian; what the per-pixel kernel carries from entry to entry becomes
// two scans over the lanes:
//   T in front of entry l    = T_behind_chunk / prod_{k <= l} (1 - alpha_k)
//   S behind entry l         = the maps  S -> alpha_k (dC . c_k) + (1 - alpha_k) S  of the entries k < l applied,
//                              furthest first, to S_behind_chunk, where S = dC . (colour composited behind),
//                              which is all that dL/dalpha = T (dC . c - S) needs.
// The 9 (11) sums of a Gaussian over the pixels are then plain per-lane accumulators: no reduction across
// lanes.  Pixel p's state (T, S behind the part of the list already done) lives in lane p and is fetched with
// readlane.  The four quadrants' sums of a Gaussian meet in LDS as in k_render_bwd.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_from(float identity, float v)
{
    return __int_as_float(
        __builtin_amdgcn_update_dpp(__float_as_int(identity), __float_as_int(v), CTRL, ROW_MASK, 0xF, false));
}

// Inclusive scan over the lanes of the composition of the maps S -> b + m S, lane 0 applied first:
// afterwards (m, b) of lane l is the composition of the maps of lanes 0 .. l.
__device__ __forceinline__ void wave_scan_affine(float& m, float& b)
{
#define FS_AFFINE_STEP(CTRL, ROW_MASK)                                  \
    {                                                                   \
        const float mo = dpp_from<CTRL, ROW_MASK>(1.0f, m);             \
        const float bo = dpp_from<CTRL, ROW_MASK>(0.0f, b);             \
        b = __builtin_fmaf(m, bo, b);                                   \
        m = m * mo;                                                     \
    }
    FS_AFFINE_STEP(0x111, 0xF)   // row_shr:1
    FS_AFFINE_STEP(0x112, 0xF)   // row_shr:2
    FS_AFFINE_STEP(0x114, 0xF)   // row_shr:4
    FS_AFFINE_STEP(0x118, 0xF)   // row_shr:8
    FS_AFFINE_STEP(0x142, 0xA)   // row_bcast:15 into rows 1 and 3
    FS_AFFINE_STEP(0x143, 0xC)   // row_bcast:31 into rows 2 and 3
#undef FS_AFFINE_STEP
}

template <bool ABS, bool SPARSE>
__global__ __launch_bounds__(256) void k_render_bwd_splat(
    CamDev cam, CfgDev cfg, const uint2* __restrict__ ranges, const uint32_t* __restrict__ tile_order,
    const uint32_t* __restrict__ gauss_sorted,
    const float4* __restrict__ splats, const float* __restrict__ final_T, const uint32_t* __restrict__ n_contrib,
    const float* __restrict__ dL_dimage, float4* __restrict__ pair_grad, uint8_t* __restrict__ rec_valid)
{
    __shared__ Stage<true> s;
    __shared__ uint32_t s_id[BATCH];
    constexpr int NV = ABS ? 11 : 9;
    __shared__ double s_acc[BATCH][NV];   // (double: the cheaper LDS atomic add on this chip, see k_render_bwd)
    __shared__ uint8_t s_qlist[4][BATCH];   // per quadrant: the batch slots on its list, in list order
    __shared__ int s_max;

    const int tile = (int)tile_order[blockIdx.x];
    const Pixel p = pixel_of_thread(cam, tile);
    const uint2 range = ranges[tile];
    const size_t hw = (size_t)cam.width * cam.height;
    const size_t pix = (size_t)p.y * cam.width + p.x;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;

    // this lane's pixel: constants and the state behind the part of the list already done
    const int last = p.inside ? (int)n_contrib[pix] : 0;
    float T_st = p.inside ? final_T[pix] : 0.f;
    float dC0 = 0.f, dC1 = 0.f, dC2 = 0.f;
    if (p.inside) {
        dC0 = dL_dimage[pix];
        dC1 = dL_dimage[hw + pix];
        dC2 = dL_dimage[2 * hw + pix];
    }
    float S_st = __builtin_fmaf(dC2, cfg.bg[2], __builtin_fmaf(dC1, cfg.bg[1], dC0 * cfg.bg[0]));

    s.clear(threadIdx.x);
    if (threadIdx.x == 0) s_max = 0;
    __syncthreads();
    atomicMax(&s_max, last);
    __syncthreads();
    const int total = s_max;
    // the furthest position any pixel of this quadrant reaches (uniform in the wavefront)
    int wave_last = last;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) wave_last = max(wave_last, __shfl_xor(wave_last, d, 64));

    for (int start = ((total - 1) / BATCH) * BATCH; start >= 0 && total > 0; start -= BATCH) {
        const int m = min(BATCH, total - start);
        __syncthreads();  // the previous batch's flush has read s_acc / s_id, its walk s_qlist
#pragma unroll
        for (int k = 0; k < NV; k++) s_acc[threadIdx.x][k] = 0.0;
        stage_batch<true, 2>(s, s_id, cam, cfg, tile, gauss_sorted, splats, range.x + start, m);
        // the quadrant's list: lane l looks at slots 4 l .. 4 l + 3 of the union of its four sub-tiles' masks
        uint32_t b4 = 0;
        {
            const int word = lane >> 4, shift = (lane & 15) * 4;
            uint64_t u = 0;
#pragma unroll
            for (int r = 0; r < 4; r++) u |= s.bits[wave * 4 + r][word];
            b4 = (uint32_t)(u >> shift) & 0xFu;
        }
        const int cnt = __popc(b4);
        int inc = cnt;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int o = __shfl_up(inc, d, 64);
            if (lane >= d) inc += o;
        }
        const int qlen = __shfl(inc, 63, 64);
        {
            int pos = inc - cnt;
            uint32_t b = b4;
            while (b) {
                s_qlist[wave][pos++] = (uint8_t)(4 * lane + __builtin_ctz(b));
                b &= b - 1u;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();

        if (start < wave_last) {
            for (int c_end = qlen; c_end > 0; c_end -= 64) {
                // lane 0 takes the entry furthest back of the chunk
                const int idx = c_end - 1 - lane;
                const bool have = idx >= 0;
                const int j = have ? (int)s_qlist[wave][idx] : 0;
                const float4 f0 = s.at(j)[0], f1 = s.at(j)[1], f2 = s.at(j)[2];
                const float2 xy = make_float2(f0.x, f0.y);
                const float4 co = make_float4(f0.z, f0.w, f1.x, f1.y);    // (a, 2b, c, sigma)
                const float4 col = make_float4(f2.x, f2.y, f2.z, 0.f);
                const int pos_j = start + j;
                float acc[NV];
#pragma unroll
                for (int k = 0; k < NV; k++) acc[k] = 0.f;
                bool any = false;
                for (int q = 0; q < 64; q++) {
                    const int last_q = __builtin_amdgcn_readlane(last, q);
                    if (last_q <= start) continue;   // this pixel blends nothing of this batch
                    const float px = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(p.px), q));
                    const float py = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(p.py), q));
                    const float dx = px - xy.x, dy = py - xy.y;
                    const float u = __builtin_fmaf(co.y, dy, co.x * dx);
                    const float qq = __builtin_fmaf(dx, u, (co.z * dy) * dy);
                    const float power = -0.5f * qq;
                    bool act = have & (pos_j < last_q) & !(power > 0.0f) & !(power < cfg.power_min);
                    if (__ballot(act) == 0) continue;
                    float G = exp_c(act ? power : 0.0f);
                    const float sG = co.w * G;
                    float alpha = fminf(cfg.alpha_max, sG);
                    act = act & (alpha >= cfg.alpha_min);
                    if (__ballot(act) == 0) continue;
                    any = true;
                    alpha = act ? alpha : 0.f;
                    G = act ? G : 0.f;
                    const float d0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(dC0), q));
                    const float d1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(dC1), q));
                    const float d2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(dC2), q));
                    const float T_behind = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(T_st), q));
                    const float S_behind = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(S_st), q));
                    const float cd = __builtin_fmaf(col.z, d2, __builtin_fmaf(col.y, d1, col.x * d0));   // dC . c
                    float M = 1.0f - alpha, Bc = alpha * cd;
                    wave_scan_affine(M, Bc);
                    // maps of the lanes before this one (the entries behind it)
                    float Mx = __shfl_up(M, 1, 64), Bx = __shfl_up(Bc, 1, 64);
                    if (lane == 0) { Mx = 1.0f; Bx = 0.0f; }
                    const float T = T_behind * __builtin_amdgcn_rcpf(M);   // in front of this entry
                    const float S = __builtin_fmaf(Mx, S_behind, Bx);      // dC . (colour behind this entry)
                    const float w = alpha * T;
                    acc[0] = __builtin_fmaf(w, d0, acc[0]);
                    acc[1] = __builtin_fmaf(w, d1, acc[1]);
                    acc[2] = __builtin_fmaf(w, d2, acc[2]);
                    float dL_dalpha = T * (cd - S);
                    dL_dalpha = sG > cfg.alpha_max ? 0.f : dL_dalpha;   // capped alpha is a constant
                    acc[3] = __builtin_fmaf(G, dL_dalpha, acc[3]);
                    const float gq = -0.5f * (co.w * G) * dL_dalpha;
                    const float gx = gq * dx, gy = gq * dy;
                    acc[4] = __builtin_fmaf(gx, dx, acc[4]);
                    acc[5] = __builtin_fmaf(gx, dy, acc[5]);
                    acc[6] = __builtin_fmaf(gy, dy, acc[6]);
                    acc[7] += gx;
                    acc[8] += gy;
                    if (ABS) {
                        const float ag = fabsf(gq);
                        acc[NV - 2] = __builtin_fmaf(ag, fabsf(__builtin_fmaf(co.y, dy, 2.0f * co.x * dx)), acc[NV - 2]);
                        acc[NV - 1] = __builtin_fmaf(ag, fabsf(__builtin_fmaf(co.y, dx, 2.0f * co.z * dy)), acc[NV - 1]);
                    }
                    // pixel q moves in front of the chunk: the last lane holds the composition of all its maps
                    const float M_all = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(M), 63));
                    const float B_all = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(Bc), 63));
                    const float T_new = T_behind * __builtin_amdgcn_rcpf(M_all);
                    const float S_new = __builtin_fmaf(M_all, S_behind, B_all);
                    T_st = lane == q ? T_new : T_st;
                    S_st = lane == q ? S_new : S_st;
                }
                if (any && have) {
#pragma unroll
                    for (int k = 0; k < NV; k++)
                        if (acc[k] != 0.f) atomicAdd(&s_acc[j][k], (double)acc[k]);
                }
            }
        }
        __syncthreads();
        if ((int)threadIdx.x < m) {
            float a[NV];
#pragma unroll
            for (int k = 0; k < NV; k++) a[k] = (float)s_acc[threadIdx.x][k];
            // SPARSE: a pair that received nothing (blended at no pixel of the tile) leaves no record; its flag stays 0
            // and k_preprocess_bwd does not read the record's place
            bool any = !SPARSE;
            if (SPARSE) {
#pragma unroll
                for (int k = 0; k < NV; k++) any = any | (a[k] != 0.f);
            }
            if (any) {
                const float4 f0 = s.at(threadIdx.x)[0], f1 = s.at(threadIdx.x)[1];
                const float4 co = make_float4(f0.z, f0.w, f1.x, f1.y);  // (a, 2b, c, sigma)
                const uint32_t idx = s_id[threadIdx.x];
                float4* rec = pair_grad + (size_t)idx * (PAIR_REC / 4);
                rec[0] = make_float4(a[0], a[1], a[2], a[3]);
                // d = p - mu  =>  dq/dmu = -(2 a dx + 2b dy, 2b dx + 2 c dy)
                rec[1] = make_float4(a[4], 2.0f * a[5], a[6], -(2.0f * co.x * a[7] + co.y * a[8]));
                rec[2] = make_float4(-(co.y * a[7] + 2.0f * co.z * a[8]), ABS ? a[NV - 2] : 0.f, ABS ? a[NV - 1] : 0.f, 0.f);
                if (SPARSE) rec_valid[idx] = 1;
            }
        }
    }
    // pairs behind the furthest blended Gaussian of the tile received nothing (SPARSE: their flags stay 0)
    if (!SPARSE) {
        for (uint32_t pos = range.x + total + threadIdx.x; pos < range.y; pos += 256) {
            const float4 r2 = splats[(size_t)gauss_sorted[pos] * (SPLAT_REC / 4) + 2];
            const uint32_t r01 = __float_as_uint(r2.z), r23 = __float_as_uint(r2.w);
            const uint32_t x0 = r01 & 0xffffu, y0 = r01 >> 16, x1 = r23 & 0xffffu;
            const uint32_t idx = __float_as_uint(r2.y) + ((uint32_t)(tile / cam.tiles_x) - y0) * (x1 - x0) +
                                 ((uint32_t)(tile % cam.tiles_x) - x0);
            float4* rec = pair_grad + (size_t)idx * (PAIR_REC / 4);
            rec[0] = make_float4(0.f, 0.f, 0.f, 0.f);
            rec[1] = make_float4(0.f, 0.f, 0.f, 0.f);
            rec[2] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
}

// Count pass: re-walks the forward loop for the mask pixels only (other pixels cannot add to a
// count) up to each pixel's n_contrib, and counts per Gaussian the pixels where it is blended
// (and, in weight mode, alpha*T > alpha_min).  A ballot + population count gives each sub-tile's
// count without any cross-lane arithmetic.
__global__ __launch_bounds__(256) void k_score(CamDev cam, CfgDev cfg, const uint2* __restrict__ ranges,
                                               const uint32_t* __restrict__ tile_order,
                                               const uint32_t* __restrict__ gauss_sorted,
                                               const float4* __restrict__ splats,
                                               const uint32_t* __restrict__ n_contrib,
                                               const uint8_t* __restrict__ mask, int32_t* __restrict__ counts)
{
    __shared__ Stage<false> s;
    __shared__ uint32_t s_id[BATCH];
    __shared__ int s_cnt[BATCH];
    __shared__ int s_max;

    const int tile = (int)tile_order[blockIdx.x];  // longest lists first
    const Pixel p = pixel_of_thread(cam, tile);
    const uint2 range = ranges[tile];
    const size_t pix = (size_t)p.y * cam.width + p.x;
    const int lane = threadIdx.x & 63;
    const int sub = (threadIdx.x >> 6) * 4 + (lane >> 4);
    int last = 0;
    if (p.inside && mask[pix]) last = (int)n_contrib[pix];
    s.clear(threadIdx.x);
    if (threadIdx.x == 0) s_max = 0;
    __syncthreads();
    atomicMax(&s_max, last);
    __syncthreads();
    const int total = s_max;
    float T = 1.0f;

    // The walking pixels (mask pixels with at least one blended Gaussian) are usually a small part of the
    // tile.  When at most half of it walks, they are packed into the first lanes of the workgroup: lane c
    // takes over the c-th walking pixel, with that pixel's own sub-tile list, so that one or two wavefronts
    // run the loop instead of four mostly idle ones.  The per-pixel arithmetic is the same either way.
    __shared__ int s_wave_cnt[4];
    __shared__ uint8_t s_walker[256];
    const bool walks = last > 0;
    const uint64_t wb = __ballot(walks);
    if (lane == 0) s_wave_cnt[threadIdx.x >> 6] = __popcll(wb);
    __syncthreads();
    int before = 0, nwalk = 0;
#pragma unroll
    for (int w = 0; w < 4; w++) {
        before += w < (int)(threadIdx.x >> 6) ? s_wave_cnt[w] : 0;
        nwalk += s_wave_cnt[w];
    }
    if (walks) s_walker[before + __popcll(wb & ((1ull << lane) - 1ull))] = (uint8_t)threadIdx.x;
    __syncthreads();

    if (nwalk <= 128) {
        // Which wavefront takes the first 64 walkers rotates with the workgroup index: wavefront w of every
        // workgroup runs on the same SIMD of its CU, and the walk is the expensive part.
        const int c = (int)((((threadIdx.x >> 6) - blockIdx.x) & 3u) * 64u) + lane;
        const bool on = c < nwalk;
        const int me = on ? (int)s_walker[c] : 0;
        const Pixel pw = pixel_of_thread(cam, tile, me);
        const int my_sub = (me >> 6) * 4 + ((me & 63) >> 4);
        const int my_last = on ? (int)n_contrib[(size_t)pw.y * cam.width + pw.x] : 0;
        const bool wave_on = (c - lane) < nwalk;   // uniform per wavefront
        for (int start = 0; start < total; start += BATCH) {
            const int m = min(BATCH, total - start);
            __syncthreads();  // the previous batch's flush has read s_cnt / s_id
            s_cnt[threadIdx.x] = 0;
            stage_batch<false, 1>(s, s_id, cam, cfg, tile, gauss_sorted, splats, range.x + start, m);
            if (wave_on) {
                const int len = start < my_last ? s.len[my_sub] : 0;
                // two list entries per trip: their alphas are independent, only the transmittance chains
                for (int k = 0; __ballot(k < len) != 0; k += 2) {
                    const int j0 = s.list[my_sub][k & (BATCH - 1)], j1 = s.list[my_sub][(k + 1) & (BATCH - 1)];
                    const float4 a0 = s.at(j0)[0], b0 = s.at(j0)[1], a1 = s.at(j1)[0], b1 = s.at(j1)[1];
                    const float2 xy0 = make_float2(a0.x, a0.y), xy1 = make_float2(a1.x, a1.y);
                    const float4 co0 = make_float4(a0.z, a0.w, b0.x, b0.y), co1 = make_float4(a1.z, a1.w, b1.x, b1.y);
                    const float dx0 = pw.px - xy0.x, dy0 = pw.py - xy0.y;
                    const float dx1 = pw.px - xy1.x, dy1 = pw.py - xy1.y;
                    const float q0 = __builtin_fmaf(dx0, __builtin_fmaf(co0.y, dy0, co0.x * dx0), (co0.z * dy0) * dy0);
                    const float q1 = __builtin_fmaf(dx1, __builtin_fmaf(co1.y, dy1, co1.x * dx1), (co1.z * dy1) * dy1);
                    const float power0 = -0.5f * q0, power1 = -0.5f * q1;
                    bool act0 = (k < len) & (start + j0 < my_last) & !(power0 > 0.0f) & !(power0 < cfg.power_min);
                    bool act1 = (k + 1 < len) & (start + j1 < my_last) & !(power1 > 0.0f) & !(power1 < cfg.power_min);
                    if (__ballot(act0 | act1) == 0) continue;
                    // (an inactive entry's exponent may be anything: clamp it so that exp_c stays in range)
                    const float alpha0 = fminf(cfg.alpha_max, co0.w * exp_c(act0 ? power0 : 0.0f));
                    const float alpha1 = fminf(cfg.alpha_max, co1.w * exp_c(act1 ? power1 : 0.0f));
                    act0 = act0 & (alpha0 >= cfg.alpha_min);
                    act1 = act1 & (alpha1 >= cfg.alpha_min);
                    const bool hit0 = act0 & (cfg.score_mode == FS_SCORE_ALPHA || alpha0 * T > cfg.alpha_min);
                    T = act0 ? T * (1.0f - alpha0) : T;
                    const bool hit1 = act1 & (cfg.score_mode == FS_SCORE_ALPHA || alpha1 * T > cfg.alpha_min);
                    T = act1 ? T * (1.0f - alpha1) : T;
                    if (hit0) atomicAdd(&s_cnt[j0], 1);
                    if (hit1) atomicAdd(&s_cnt[j1], 1);
                }
            }
            __syncthreads();
            if ((int)threadIdx.x < m && s_cnt[threadIdx.x] != 0)
                atomicAdd(&counts[s_id[threadIdx.x]], s_cnt[threadIdx.x]);
        }
        return;
    }

    for (int start = 0; start < total; start += BATCH) {
        const int m = min(BATCH, total - start);
        __syncthreads();  // the previous batch's flush has read s_cnt / s_id
        s_cnt[threadIdx.x] = 0;
        const int mine = stage_batch<false, 1>(s, s_id, cam, cfg, tile, gauss_sorted, splats,
                                               range.x + start, m);
        // a row none of whose pixels is still walking (no mask pixel, or all past their last Gaussian)
        // has nothing to count in this batch
        const uint64_t walking = __ballot(start < last);
        if (walking != 0) {
            const bool row_walks = ((walking >> (lane & 48)) & 0xffffull) != 0;
            const int longest = wave_max_of_rows(row_walks ? mine : 0);
            for (int k = 0; k < longest; k++) {
                const int j = s.list[sub][k];
                const float4 a0 = s.at(j)[0], b0 = s.at(j)[1];
                const float2 xy = make_float2(a0.x, a0.y);
                const float4 co = make_float4(a0.z, a0.w, b0.x, b0.y);
                const float dx = p.px - xy.x, dy = p.py - xy.y;
                const float u = __builtin_fmaf(co.y, dy, co.x * dx);
                const float q = __builtin_fmaf(dx, u, (co.z * dy) * dy);
                const float power = -0.5f * q;
                bool act = (k < mine) & (start + j < last) & !(power > 0.0f) & !(power < cfg.power_min);
                if (__ballot(act) == 0) continue;
                const float alpha = fminf(cfg.alpha_max, co.w * exp_c(power));
                act = act & (alpha >= cfg.alpha_min);
                const float w = alpha * T;
                const bool hit = act & (cfg.score_mode == FS_SCORE_ALPHA || w > cfg.alpha_min);
                T = act ? T * (1.0f - alpha) : T;
                const uint32_t b = (uint32_t)(__ballot(hit) >> (lane & 48)) & 0xffffu;  // this row's pixels
                if (b != 0 && (lane & 15) == 0) atomicAdd(&s_cnt[j], (int)__popc(b));
            }
        }
        __syncthreads();
        if ((int)threadIdx.x < m && s_cnt[threadIdx.x] != 0) atomicAdd(&counts[s_id[threadIdx.x]], s_cnt[threadIdx.x]);
    }
}

// Count pass from the record a k_render_fwd<., true> launch left: per tile, the mask of its 256 pixels in the same
// layout as a row's bits, then one population count per row of the tile.  Tiles without rows or without mask pixels
// read nothing else.  Workgroup (x, y) takes rows [y * chunk, (y + 1) * chunk) of tile x (the last one whatever is
// left), so that thousands of rows are not one workgroup's chain of dependent rounds; a workgroup past the tile's last
// row leaves at once.  (Tiles in plain order: a tile's rows are few, and the detour over the order array would be one
// more dependent load.)
// FROM_ERR: the mask is not read but made here, mask[p] = err[p] > threshold (Sec. 4.2), by the first workgroup of
// every tile, which also stores it (mask_out) -- the mask kernel's launch saved.
template <bool FROM_ERR>
__global__ __launch_bounds__(256) void k_score_bits(CamDev cam, const uint2* __restrict__ ranges, ScoreRecord record,
                                                    const uint8_t* __restrict__ mask, int32_t* __restrict__ counts,
                                                    uint32_t chunk, const float* __restrict__ err,
                                                    const double* __restrict__ stats, int rule, float k,
                                                    uint8_t* __restrict__ mask_out, float* __restrict__ thr_out)
{
    __shared__ __align__(16) uint16_t s_m[16];
    const int tile = (int)blockIdx.x;
    const uint32_t rows = (uint32_t)record.tile_rows[tile];
    uint32_t first = blockIdx.y * chunk;
    if (rows <= first && !(FROM_ERR && blockIdx.y == 0)) return;   // (uniform over the workgroup)
    uint32_t end = blockIdx.y + 1 == gridDim.y ? rows : min(rows, first + chunk);
    const uint32_t seg = ranges[tile].x;
    first += seg;
    end += seg;
    const Pixel p = pixel_of_thread(cam, tile);
    const int lane = threadIdx.x & 63;
    const size_t pix = (size_t)p.y * cam.width + p.x;
    // the first 256 rows are requested before the tile's mask is known, so that the two latencies overlap
    uint32_t pos = first + threadIdx.x;
    uint4 a = make_uint4(0u, 0u, 0u, 0u), c = a;
    uint32_t g = 0;
    if (pos < end) {
        a = nt_load(record.rows + (size_t)pos * 2);
        c = nt_load(record.rows + (size_t)pos * 2 + 1);
        g = record.row_gauss[pos];
    }
    bool on;
    if (FROM_ERR) {
        const float thr = threshold_from_stats(stats[0], stats[1], stats[2], stats[3], (int64_t)cam.width * cam.height, rule, k);
        on = p.inside && err[pix] > thr;
        if (blockIdx.y == 0) {
            if (tile == 0 && threadIdx.x == 0) *thr_out = thr;
            if ((cam.width & 3) == 0 && (reinterpret_cast<uintptr_t>(mask_out) & 3) == 0) {
                // four neighbouring pixels of a line are four neighbouring lanes: one 4-byte store for them
                const uint32_t four = (uint32_t)(__ballot(on) >> (lane & 60)) & 0xfu;
                if ((lane & 3) == 0 && p.inside)
                    *reinterpret_cast<uint32_t*>(mask_out + pix) = (four & 1u) | (four & 2u) << 7 | (four & 4u) << 14 | (four & 8u) << 21;
            } else if (p.inside) {
                mask_out[pix] = on ? 1 : 0;
            }
        }
    } else {
        on = p.inside && mask[pix] != 0;
    }
    const uint64_t b = __ballot(on);
    if ((lane & 15) == 0) s_m[(threadIdx.x >> 6) * 4 + (lane >> 4)] = (uint16_t)((b >> (lane & 48)) & 0xffffull);
    if (__syncthreads_or(on) == 0 || first >= end) return;
    const uint4 m0 = reinterpret_cast<const uint4*>(s_m)[0], m1 = reinterpret_cast<const uint4*>(s_m)[1];
    for (;;) {
        // (the next round's rows are requested before this round's are counted)
        const uint32_t next = pos + 256;
        uint4 a2 = make_uint4(0u, 0u, 0u, 0u), c2 = a2;
        uint32_t g2 = 0;
        if (next < end) {
            a2 = nt_load(record.rows + (size_t)next * 2);
            c2 = nt_load(record.rows + (size_t)next * 2 + 1);
            g2 = record.row_gauss[next];
        }
        const int n = __popc(a.x & m0.x) + __popc(a.y & m0.y) + __popc(a.z & m0.z) + __popc(a.w & m0.w) +
                      __popc(c.x & m1.x) + __popc(c.y & m1.y) + __popc(c.z & m1.z) + __popc(c.w & m1.w);
        if (n != 0) atomicAdd(&counts[g], n);   // (all zeros for a thread past the last row)
        if (next >= end) break;
        pos = next; a = a2; c = c2; g = g2;
    }
}

__global__ __launch_bounds__(256) void k_record_rows(int tiles, const int32_t* __restrict__ tile_rows, int32_t* __restrict__ rows)
{
    const int tile = (int)(blockIdx.x * 256 + threadIdx.x);
    if (tile < tiles) rows[tile] = tile_rows[tile];
}

}  // namespace

hipError_t launch_render_fwd(hipStream_t st, const CamDev& cam, const CfgDev& cfg, const uint32_t* ranges,
                             const uint32_t* tile_order, const uint32_t* gauss_sorted, const float* splats, float* image, float* final_T,
                             uint32_t* n_contrib, const ScoreRecord& record)
{
    const int tiles = cam.tiles_x * cam.tiles_y;
    if (tiles == 0) return hipSuccess;
    const ScoreRecord none = {nullptr, nullptr, nullptr};
    if (record.rows)
        hipLaunchKernelGGL((k_render_fwd<false, true>), dim3(tiles), dim3(256), 0, st, cam, cfg,
                           reinterpret_cast<const uint2*>(ranges), tile_order, gauss_sorted,
                           reinterpret_cast<const float4*>(splats), image, final_T, n_contrib, nullptr, 0.f, nullptr,
                           nullptr, nullptr, record);
    else
        hipLaunchKernelGGL((k_render_fwd<false, false>), dim3(tiles), dim3(256), 0, st, cam, cfg,
                           reinterpret_cast<const uint2*>(ranges), tile_order, gauss_sorted,
                           reinterpret_cast<const float4*>(splats), image, final_T, n_contrib, nullptr, 0.f, nullptr,
                           nullptr, nullptr, none);
    return hipGetLastError();
}

hipError_t launch_render_fwd_fused(hipStream_t st, const CamDev& cam, const CfgDev& cfg, const uint32_t* ranges,
                                   const uint32_t* tile_order, const uint32_t* gauss_sorted, const float* splats,
                                   float* image, float* final_T, uint32_t* n_contrib, const float* target, float* dL,
                                   float* err, double* tile_partial, const ScoreRecord& record)
{
    const int tiles = cam.tiles_x * cam.tiles_y;
    if (tiles == 0) return hipSuccess;
    const float scale = 1.0f / (float)((int64_t)3 * cam.width * cam.height);
    const ScoreRecord none = {nullptr, nullptr, nullptr};
    if (record.rows)
        hipLaunchKernelGGL((k_render_fwd<true, true>), dim3(tiles), dim3(256), 0, st, cam, cfg,
                           reinterpret_cast<const uint2*>(ranges), tile_order, gauss_sorted,
                           reinterpret_cast<const float4*>(splats), image, final_T, n_contrib, target, scale, dL, err,
                           tile_partial, record);
    else
        hipLaunchKernelGGL((k_render_fwd<true, false>), dim3(tiles), dim3(256), 0, st, cam, cfg,
                           reinterpret_cast<const uint2*>(ranges), tile_order, gauss_sorted,
                           reinterpret_cast<const float4*>(splats), image, final_T, n_contrib, target, scale, dL, err,
                           tile_partial, none);
    return hipGetLastError();
}

namespace {
// a workgroup of k_score_bits takes SCORE_CHUNK rows (the last one of a tile whatever is left); the longest list bounds
// the rows of any tile (0: not known)
constexpr uint32_t SCORE_CHUNK = 4096;
unsigned score_chunks(int64_t longest_list)
{
    int64_t chunks = longest_list > 0 ? (longest_list + SCORE_CHUNK - 1) / SCORE_CHUNK : 4;
    return (unsigned)(chunks > 64 ? 64 : chunks);
}
}  // namespace

hipError_t launch_score_bits(hipStream_t st, const CamDev& cam, const uint32_t* ranges, const ScoreRecord& record,
                             const uint8_t* mask, int32_t* counts, int64_t longest_list)
{
    const int tiles = cam.tiles_x * cam.tiles_y;
    if (tiles == 0) return hipSuccess;
    hipLaunchKernelGGL(k_score_bits<false>, dim3(tiles, score_chunks(longest_list)), dim3(256), 0, st, cam,
                       reinterpret_cast<const uint2*>(ranges), record, mask, counts, SCORE_CHUNK, nullptr, nullptr, 0, 0.f,
                       nullptr, nullptr);
    return hipGetLastError();
}

hipError_t launch_mask_score_bits(hipStream_t st, const CamDev& cam, const uint32_t* ranges, const ScoreRecord& record,
                                  const float* err, const double* stats, int rule, float k, uint8_t* mask, float* thr_out,
                                  int32_t* counts, int64_t longest_list)
{
    const int tiles = cam.tiles_x * cam.tiles_y;
    if (tiles == 0) return hipSuccess;
    hipLaunchKernelGGL(k_score_bits<true>, dim3(tiles, score_chunks(longest_list)), dim3(256), 0, st, cam,
                       reinterpret_cast<const uint2*>(ranges), record, nullptr, counts, SCORE_CHUNK, err, stats, rule, k, mask,
                       thr_out);
    return hipGetLastError();
}

hipError_t launch_record_rows(hipStream_t st, int tiles, const ScoreRecord& record, int32_t* rows)
{
    if (tiles == 0) return hipSuccess;
    hipLaunchKernelGGL(k_record_rows, dim3((tiles + 255) / 256), dim3(256), 0, st, tiles, record.tile_rows, rows);
    return hipGetLastError();
}

hipError_t launch_render_bwd(hipStream_t st, const CamDev& cam, const CfgDev& cfg, const uint32_t* ranges,
                             const uint32_t* tile_order, const uint32_t* gauss_sorted, const float* splats, const float* final_T,
                             const uint32_t* n_contrib, const float* dL_dimage, float* pair_grad, uint8_t* rec_valid,
                             bool abs_grad, bool per_splat)
{
    const int tiles = cam.tiles_x * cam.tiles_y;
    if (tiles == 0) return hipSuccess;
    const uint2* r2 = reinterpret_cast<const uint2*>(ranges);
    const float4* sp = reinterpret_cast<const float4*>(splats);
    float4* pg = reinterpret_cast<float4*>(pair_grad);
    const dim3 grid(tiles), block(256);
    // rec_valid: null = dense records, else the flags of the sparse records
#define FS_BWD(KERNEL, ABS, SPARSE)                                                                                  \
    hipLaunchKernelGGL((KERNEL<ABS, SPARSE>), grid, block, 0, st, cam, cfg, r2, tile_order, gauss_sorted, sp, final_T, \
                       n_contrib, dL_dimage, pg, rec_valid)
#define FS_BWD_MODE(KERNEL)                         \
    do {                                            \
        if (abs_grad) {                             \
            if (rec_valid) FS_BWD(KERNEL, true, true);   \
            else FS_BWD(KERNEL, true, false);       \
        } else {                                    \
            if (rec_valid) FS_BWD(KERNEL, false, true);  \
            else FS_BWD(KERNEL, false, false);      \
        }                                           \
    } while (0)
    if (per_splat) FS_BWD_MODE(k_render_bwd_splat);
    else FS_BWD_MODE(k_render_bwd);
#undef FS_BWD_MODE
#undef FS_BWD
    return hipGetLastError();
}

hipError_t launch_score(hipStream_t st, const CamDev& cam, const CfgDev& cfg, const uint32_t* ranges,
                        const uint32_t* tile_order, const uint32_t* gauss_sorted, const float* splats, const uint32_t* n_contrib,
                        const uint8_t* mask, int32_t* counts)
{
    const int tiles = cam.tiles_x * cam.tiles_y;
    if (tiles == 0) return hipSuccess;
    hipLaunchKernelGGL(k_score, dim3(tiles), dim3(256), 0, st, cam, cfg, reinterpret_cast<const uint2*>(ranges),
                       tile_order, gauss_sorted, reinterpret_cast<const float4*>(splats), n_contrib, mask, counts);
    return hipGetLastError();
}

}  // namespace fs
