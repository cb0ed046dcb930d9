// Gaussian-tile pair binning on gfx950: exclusive scans, the pairs of every Gaussian, their order
// (tile, depth, index) and the per-tile ranges.  All integer work; results are unique and reproducible
// bit for bit.
//
// FastGS Sec. 3 blends "Gaussians sorted by depth" per pixel; Sec. 4.4 names the Gaussian-tile pairs that
// the 3-sigma rule (or the Compact Box) produces.  A pair's key is tile_id << 32 | bits(depth).  Two ways
// to the same order live here: the tile-bucketed one (count per tile, place, sort each tile's segment in
// LDS), used whenever the lists are short enough, and a global stable LSD radix sort of index-ordered keys.
#include "common.hpp"

namespace fs {

namespace {

constexpr int SCAN_THREADS = 256;
constexpr int SCAN_ITEMS = 8;
constexpr int SCAN_BLOCK = SCAN_THREADS * SCAN_ITEMS;  // 2048 values per workgroup

__device__ __forceinline__ uint32_t lane_id() { return threadIdx.x & 63u; }

// Inclusive scan across the 64 lanes of a wavefront with data-parallel-primitive moves instead of shuffles through
// LDS: four shifts within the rows of 16 lanes (zeros move in at a row's start), then lane 15 of rows 0 and 2 is
// added to every lane of the row after it, then lane 31 to every lane of rows 2 and 3.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_or_zero(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xF, false);
}
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v)
{
    v += dpp_or_zero<0x111, 0xF>(v);   // row_shr:1
    v += dpp_or_zero<0x112, 0xF>(v);   // row_shr:2
    v += dpp_or_zero<0x114, 0xF>(v);   // row_shr:4
    v += dpp_or_zero<0x118, 0xF>(v);   // row_shr:8
    v += dpp_or_zero<0x142, 0xA>(v);   // row_bcast:15 into rows 1 and 3
    v += dpp_or_zero<0x143, 0xC>(v);   // row_bcast:31 into rows 2 and 3
    return v;
}
// The same with max (on unsigned values, for which zero is the neutral element).
__device__ __forceinline__ uint32_t wave_inclusive_max(uint32_t v)
{
    v = max(v, dpp_or_zero<0x111, 0xF>(v));
    v = max(v, dpp_or_zero<0x112, 0xF>(v));
    v = max(v, dpp_or_zero<0x114, 0xF>(v));
    v = max(v, dpp_or_zero<0x118, 0xF>(v));
    v = max(v, dpp_or_zero<0x142, 0xA>(v));
    v = max(v, dpp_or_zero<0x143, 0xC>(v));
    return v;
}

// Exclusive scan over the 256 threads of a workgroup; returns the thread's exclusive prefix and
// the workgroup total.
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* total, uint32_t* smem /*[4]*/)
{
    const uint32_t inc = wave_inclusive_scan(v);
    const int wave = threadIdx.x >> 6;
    __syncthreads();
    if (lane_id() == 63) smem[wave] = inc;
    __syncthreads();
    uint32_t base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < 4; w++) {
        const uint32_t s = smem[w];
        if (w < wave) base += s;
        tot += s;
    }
    *total = tot;
    return base + inc - v;
}

// Pass 1: per-workgroup sums (64-bit, so that a total beyond 2^32 is detected by the caller).
__global__ __launch_bounds__(SCAN_THREADS) void k_scan_block_sums(const uint32_t* __restrict__ in, int64_t n,
                                                                 uint64_t* __restrict__ block_sums)
{
    __shared__ uint32_t smem[4];
    const int64_t base = (int64_t)blockIdx.x * SCAN_BLOCK + threadIdx.x * SCAN_ITEMS;
    uint32_t s = 0;
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; k++)
        if (base + k < n) s += in[base + k];
    uint32_t tot;
    block_exclusive_scan(s, &tot, smem);
    if (threadIdx.x == 0) block_sums[blockIdx.x] = tot;
}

// Pass 2: one workgroup turns the block sums into exclusive block offsets (sequential chunks).
__global__ __launch_bounds__(SCAN_THREADS) void k_scan_block_offsets(uint64_t* __restrict__ block_sums,
                                                                    int64_t num_blocks,
                                                                    uint64_t* __restrict__ total_out)
{
    __shared__ uint64_t wave_tot[4];
    __shared__ uint64_t carry_s;
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    for (int64_t c = 0; c < num_blocks; c += SCAN_THREADS) {
        const int64_t i = c + threadIdx.x;
        const uint64_t v = i < num_blocks ? block_sums[i] : 0;
        // 64-bit inclusive scan within the wave
        uint64_t inc = v;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const uint32_t lo = __shfl_up((uint32_t)inc, d, 64);
            const uint32_t hi = __shfl_up((uint32_t)(inc >> 32), d, 64);
            if ((int)lane_id() >= d) inc += ((uint64_t)hi << 32) | lo;
        }
        const int wave = threadIdx.x >> 6;
        if (lane_id() == 63) wave_tot[wave] = inc;
        __syncthreads();
        uint64_t base = carry_s;
        for (int w = 0; w < wave; w++) base += wave_tot[w];
        if (i < num_blocks) block_sums[i] = base + inc - v;
        __syncthreads();
        if (threadIdx.x == SCAN_THREADS - 1) carry_s = base + inc;
        __syncthreads();
    }
    if (threadIdx.x == 0) *total_out = carry_s;
}

// Pass 3: exclusive scan inside each workgroup plus its block offset.
// `in` and `out` may be the same array (each thread reads its values before writing them).
__global__ __launch_bounds__(SCAN_THREADS) void k_scan_apply(const uint32_t* in, uint32_t* out, int64_t n,
                                                            const uint64_t* __restrict__ block_offsets)
{
    __shared__ uint32_t smem[4];
    const int64_t base = (int64_t)blockIdx.x * SCAN_BLOCK + threadIdx.x * SCAN_ITEMS;
    uint32_t v[SCAN_ITEMS];
    uint32_t s = 0;
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; k++) {
        v[k] = base + k < n ? in[base + k] : 0u;
        s += v[k];
    }
    uint32_t tot;
    uint32_t run = block_exclusive_scan(s, &tot, smem) + (uint32_t)block_offsets[blockIdx.x];
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; k++) {
        if (base + k < n) out[base + k] = run;
        run += v[k];
    }
}

// One key per tile of each Gaussian's rectangle, rows then columns, starting at offsets[i].  A
// wavefront takes 64 consecutive Gaussians; their pairs occupy one contiguous run of the output, and
// the wavefront writes that run 64 pairs at a time (lane j of a round finds the Gaussian that owns
// output slot j by a binary search over the lanes' running counts), so a Gaussian that touches
// hundreds of tiles does not stall its 63 neighbours and every store is coalesced.  Each lane also
// packs its own Gaussian's projected splat, rectangle and pair offset into one 64-byte record, so
// that the render kernels gather one cache line per (Gaussian, tile) pair instead of five.
__global__ __launch_bounds__(256) void k_emit_pairs(int64_t n, const ushort4* __restrict__ rect,
                                                    const float* __restrict__ depth,
                                                    const float2* __restrict__ mean2d,
                                                    const float4* __restrict__ conic_opacity,
                                                    const float* __restrict__ rgb,
                                                    const uint32_t* __restrict__ offsets, int tiles_x,
                                                    uint64_t* __restrict__ keys, uint32_t* __restrict__ vals,
                                                    float4* __restrict__ splats)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const bool valid = i < n;
    const uint32_t lane = lane_id();
    const ushort4 r = valid ? rect[i] : make_ushort4(0, 0, 0, 0);
    const uint32_t w = r.z > r.x ? (uint32_t)(r.z - r.x) : 0u, h = r.w > r.y ? (uint32_t)(r.w - r.y) : 0u;
    const uint32_t cnt = w * h;
    const uint32_t off = valid ? offsets[i] : 0u;
    const uint32_t dbits = cnt ? __float_as_uint(depth[i]) : 0u;
    if (cnt) {
        const float2 m = mean2d[i];
        const float4 co = conic_opacity[i];
        float4* rec = splats + (size_t)i * (SPLAT_REC / 4);
        rec[0] = make_float4(m.x, m.y, co.x, co.y);
        rec[1] = make_float4(co.z, co.w, rgb[3 * i], rgb[3 * i + 1]);
        rec[2] = make_float4(rgb[3 * i + 2], __uint_as_float(off), __uint_as_float((uint32_t)r.x | (uint32_t)r.y << 16),
                             __uint_as_float((uint32_t)r.z | (uint32_t)r.w << 16));
    }
    const uint32_t inc = wave_inclusive_scan(cnt);
    const uint32_t excl = inc - cnt;                       // this lane's first slot within the wave's run
    const uint32_t total = (uint32_t)__shfl((int)inc, 63, 64);
    const uint32_t run_start = (uint32_t)__shfl((int)off, 0, 64);  // offsets[] of the wave's first Gaussian
    const uint32_t rect_xy = (uint32_t)r.x | (uint32_t)r.y << 16;
    for (uint32_t j0 = 0; j0 < total; j0 += 64) {
        const uint32_t j = min(j0 + lane, total - 1);     // clamped: every lane takes part in the shuffles
        // owner = last lane whose first slot is <= j (lanes without pairs share their successor's first slot)
        uint32_t s = 0;
#pragma unroll
        for (uint32_t step = 32; step >= 1; step >>= 1) {
            const uint32_t t = s + step;
            const uint32_t e = (uint32_t)__shfl((int)excl, (int)t, 64);
            s = e <= j ? t : s;
        }
        const uint32_t k = j - (uint32_t)__shfl((int)excl, (int)s, 64);  // place in the owner's rectangle, row-major
        const uint32_t ow = (uint32_t)__shfl((int)w, (int)s, 64);
        const uint32_t oxy = (uint32_t)__shfl((int)rect_xy, (int)s, 64);
        const uint32_t od = (uint32_t)__shfl((int)dbits, (int)s, 64);
        // estimate with the fast reciprocal, off by at most one (k < 2^32 and ow < 2^16 make the quotient's error < 0.02):
        // corrected by one step either way, never by a loop that bad operands could keep a wavefront in
        uint32_t row = (uint32_t)((float)k * __builtin_amdgcn_rcpf((float)ow));
        row -= row * ow > k ? 1u : 0u;
        row += (row + 1) * ow <= k ? 1u : 0u;
        const uint32_t col = k - row * ow;
        const uint32_t tx = (oxy & 0xffffu) + col, ty = (oxy >> 16) + row;
        if (j0 + lane < total) {
            const size_t o = (size_t)run_start + j0 + lane;
            keys[o] = ((uint64_t)(ty * (uint32_t)tiles_x + tx) << 32) | od;
            vals[o] = (uint32_t)(i - lane + s);
        }
    }
}

// Compact Box: tiles in each Gaussian's box (the candidates of the ellipse test).
__global__ __launch_bounds__(256) void k_rect_area(int64_t n, const ushort4* __restrict__ rect,
                                                   uint32_t* __restrict__ area)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const ushort4 r = rect[i];
    area[i] = r.z > r.x && r.w > r.y ? (uint32_t)(r.z - r.x) * (uint32_t)(r.w - r.y) : 0u;
}

// Compact Box emission.  Same wave-cooperative walk as k_emit_pairs, but over the candidates (all tiles
// of each box): the lane that takes a candidate runs the ellipse-tile test; a hit becomes a key at
// offsets[owner] + (hits of the same Gaussian before it, in row-major order), a miss gets its gradient
// record zeroed.  Hits of one Gaussian before a candidate = those of earlier rounds (kept by the owner
// lane in `emitted`) + those on lower lanes of this round (one ballot, masked to the owner's lanes).
__global__ __launch_bounds__(256) void k_emit_pairs_cb(int64_t n, const ushort4* __restrict__ rect,
                                                       const float* __restrict__ depth,
                                                       const float2* __restrict__ mean2d,
                                                       const float4* __restrict__ conic_opacity,
                                                       const float* __restrict__ rgb, CfgDev cfg,
                                                       const uint32_t* __restrict__ offsets,
                                                       const uint32_t* __restrict__ rec_offsets, int tiles_x,
                                                       uint32_t P, uint64_t* __restrict__ keys,
                                                       uint32_t* __restrict__ vals,
                                                       float4* __restrict__ splats, float4* __restrict__ pair_grad)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const bool valid = i < n;
    const uint32_t lane = lane_id();
    const ushort4 r = valid ? rect[i] : make_ushort4(0, 0, 0, 0);
    const uint32_t w = r.z > r.x ? (uint32_t)(r.z - r.x) : 0u, h = r.w > r.y ? (uint32_t)(r.w - r.y) : 0u;
    const uint32_t cnt = w * h;                              // candidates
    const uint32_t off = valid ? offsets[i] : 0u;           // first pair
    const uint32_t roff = valid ? rec_offsets[i] : 0u;      // first gradient record
    const uint32_t dbits = cnt ? __float_as_uint(depth[i]) : 0u;
    float mx = 0.f, my = 0.f, A = 1.f, B = 0.f, C = 1.f, Q = 0.f;
    if (cnt) {
        const float2 m = mean2d[i];
        const float4 co = conic_opacity[i];
        mx = m.x; my = m.y; A = co.x; B = co.y; C = co.z;
        Q = cb_threshold(co.w, cfg);
        float4* rec = splats + (size_t)i * (SPLAT_REC / 4);
        rec[0] = make_float4(m.x, m.y, co.x, co.y);
        rec[1] = make_float4(co.z, co.w, rgb[3 * i], rgb[3 * i + 1]);
        rec[2] = make_float4(rgb[3 * i + 2], __uint_as_float(roff), __uint_as_float((uint32_t)r.x | (uint32_t)r.y << 16),
                             __uint_as_float((uint32_t)r.z | (uint32_t)r.w << 16));
    }
    const uint32_t inc = wave_inclusive_scan(cnt);
    const uint32_t excl = inc - cnt;
    const uint32_t total = (uint32_t)__shfl((int)inc, 63, 64);
    const uint32_t rect_xy = (uint32_t)r.x | (uint32_t)r.y << 16;
    uint32_t emitted = 0;                                    // hits of this lane's own Gaussian so far
    for (uint32_t j0 = 0; j0 < total; j0 += 64) {
        const bool live = j0 + lane < total;
        const uint32_t j = min(j0 + lane, total - 1);
        uint32_t s = 0;
#pragma unroll
        for (uint32_t step = 32; step >= 1; step >>= 1) {
            const uint32_t t = s + step;
            const uint32_t e = (uint32_t)__shfl((int)excl, (int)t, 64);
            s = e <= j ? t : s;
        }
        const uint32_t oexcl = (uint32_t)__shfl((int)excl, (int)s, 64);
        const uint32_t k = j - oexcl;
        const uint32_t ow = (uint32_t)__shfl((int)w, (int)s, 64);
        const uint32_t oxy = (uint32_t)__shfl((int)rect_xy, (int)s, 64);
        const uint32_t od = (uint32_t)__shfl((int)dbits, (int)s, 64);
        const uint32_t ooff = (uint32_t)__shfl((int)off, (int)s, 64);
        const uint32_t oroff = (uint32_t)__shfl((int)roff, (int)s, 64);
        const uint32_t oem = (uint32_t)__shfl((int)emitted, (int)s, 64);
        const float omx = __shfl(mx, (int)s, 64), omy = __shfl(my, (int)s, 64);
        const float oA = __shfl(A, (int)s, 64), oB = __shfl(B, (int)s, 64), oC = __shfl(C, (int)s, 64);
        const float oQ = __shfl(Q, (int)s, 64);
        // estimate with the fast reciprocal, off by at most one (k < 2^32 and ow < 2^16 make the quotient's error < 0.02):
        // corrected by one step either way, never by a loop that bad operands could keep a wavefront in
        uint32_t row = (uint32_t)((float)k * __builtin_amdgcn_rcpf((float)ow));
        row -= row * ow > k ? 1u : 0u;
        row += (row + 1) * ow <= k ? 1u : 0u;
        const uint32_t col = k - row * ow;
        const uint32_t tx = (oxy & 0xffffu) + col, ty = (oxy >> 16) + row;
        const bool hit = live && cb_tile_hit(omx, omy, oA, oB, oC, oQ, (int)tx, (int)ty);
        const uint64_t hb = __ballot(hit);
        // lanes of this round that belong to the same Gaussian and come before this one
        const uint32_t seg0 = oexcl > j0 ? oexcl - j0 : 0u;                 // first lane of the owner's run
        const uint64_t below = (lane ? (~0ull >> (64 - lane)) : 0ull) & (~0ull << seg0);
        if (hit) {
            const size_t o = (size_t)ooff + oem + (uint32_t)__popcll(hb & below);
            if (o < P) {   // always true when tiles_touched came from k_preprocess with the same configuration
                keys[o] = ((uint64_t)(ty * (uint32_t)tiles_x + tx) << 32) | od;
                vals[o] = (uint32_t)(i - lane + s);
            }
        } else if (live) {
            float4* g = pair_grad + ((size_t)oroff + k) * (PAIR_REC / 4);
            const float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
            g[0] = z; g[1] = z; g[2] = z;
        }
        // each owner adds the hits of its own run in this round
        const uint32_t a0 = excl > j0 ? excl - j0 : 0u;                      // run of this lane's Gaussian: [a0, a1)
        const uint32_t a1 = inc > j0 ? min(inc - j0, 64u) : 0u;
        if (a1 > a0) {
            const uint64_t mine = (a1 >= 64 ? ~0ull : ((1ull << a1) - 1ull)) & (~0ull << a0);
            emitted += (uint32_t)__popcll(hb & mine);
        }
    }
}

// ---- tile-bucketed ordering ----------------------------------------------------------------
// The order wanted is (tile, depth, Gaussian index): instead of one global sort on 45 live key bits, the
// pairs are (1) counted per tile, (2) placed into their tile's segment in arrival order, and (3) every
// tile's segment is sorted in LDS on the 64-bit word depth_bits << 32 | Gaussian index.  Those words are
// unique within a tile, so the result does not depend on the arrival order and equals what a stable global
// sort of index-ordered keys gives.  The per-tile ranges fall out of step (1).

// Steps (1) and (2) are launched as TILE_COPIES workgroups, each keeping its own counter per tile in LDS
// (so num_tiles * 4 bytes must fit there) and walking the same Gaussians in both steps; step (1) ends by
// writing its counters as one row of a [TILE_COPIES, num_tiles] table, which k_tile_sum turns into each
// workgroup's start within every tile's segment, and step (2) starts from that row.  Global atomics reach
// about 45 G/s on this chip whatever the contention; LDS atomics are an order of magnitude cheaper.
//
// Steps (1) and (2) walk the candidate tiles of 64 consecutive Gaussians per wavefront the way k_emit_pairs
// does.  SCATTER = false: count[tile] += 1 per pair.  SCATTER = true: slot = first[tile] + counter[tile]++
// (k_tile_sum has turned each copy's counter into that copy's start within the tile's segment),
// bucket[slot] = depth_bits << 32 | index; also packs the splat records and, with
// the Compact Box, zeroes the gradient records of the candidates that are no pairs.  In this mode `P` and `rec_limit`
// are the numbers of words / records the buffers hold: nothing is written at or beyond them (the kernel may be
// enqueued before the host has seen the real totals).
//
// Step (1) also hands every Gaussian the place of its backward records (one per tile of its rectangle): a
// workgroup first adds up the records of all its Gaussians and reserves them with one add on a global counter
// (adds on one address take about 10 ns each, so one per wavefront and round would cost more than the prefix sum
// it replaces); inside the reservation the wavefronts, their rounds and the 64 Gaussians of a round follow each
// other.  The places are disjoint, each Gaussian's are contiguous and so are those of 64 consecutive Gaussians,
// which is all their users need -- no prefix sum over the Gaussians.  A second counter receives the sum of
// tiles_touched, which the host compares with the number of pairs counted per tile.
struct RecAlloc {
    const uint32_t* tiles_touched;   // [n]
    uint32_t* rec_offsets;           // [n] out: first record of each Gaussian
    uint32_t* rec_counts;            // [n] out (may be null): records of each Gaussian = area of its rectangle
    unsigned long long* counters;    // [2]: records handed out, sum of tiles_touched
};

template <bool CB, bool SCATTER>
__global__ __launch_bounds__(TILE_PAIR_THREADS) void k_tile_pairs(int64_t n, const ushort4* __restrict__ rect,
                                                    const float* __restrict__ depth,
                                                    const float2* __restrict__ mean2d,
                                                    const float4* __restrict__ conic_opacity,
                                                    const float* __restrict__ rgb, CfgDev cfg,
                                                    const uint32_t* __restrict__ rec_offsets, int tiles_x,
                                                    int num_tiles, uint32_t* __restrict__ tile_counter,
                                                    const uint2* __restrict__ ranges, uint32_t P, uint32_t rec_limit,
                                                    uint64_t* __restrict__ bucket, float4* __restrict__ splats,
                                                    float4* __restrict__ pair_grad, RecAlloc ra)
{
    extern __shared__ uint32_t s_tile[];   // this workgroup's counter per tile
    uint32_t* const my_row = tile_counter + (size_t)blockIdx.x * num_tiles;
    // placement: the counter starts at the absolute position of this workgroup's first pair of the tile
    for (int t = threadIdx.x; t < num_tiles; t += TILE_PAIR_THREADS) s_tile[t] = SCATTER ? ranges[t].x + my_row[t] : 0u;
    __syncthreads();
    const uint32_t lane = lane_id();
    __shared__ uint32_t s_mark[TILE_PAIR_THREADS / 64][64];
    uint32_t* const mark = s_mark[threadIdx.x >> 6];   // this wavefront's own
    uint32_t rec_next = 0;   // (counting) where the records of this wavefront's next round start
    if (!SCATTER) {
        __shared__ uint32_t s_wave_recs[TILE_PAIR_THREADS / 64];
        __shared__ uint32_t s_tt[TILE_PAIR_THREADS / 64];
        __shared__ uint32_t s_base[2];
        uint32_t recs = 0, tt = 0;
        // (four rounds' loads are requested together: with one wavefront's worth of loads in flight per round the
        // loop would take one memory latency per round)
        const int64_t stride = (int64_t)gridDim.x * TILE_PAIR_THREADS;
        for (int64_t i = (int64_t)blockIdx.x * TILE_PAIR_THREADS + threadIdx.x; i < n; i += 4 * stride) {
            ushort4 r[4];
            uint32_t t4[4];
#pragma unroll
            for (int q = 0; q < 4; q++) {
                const bool in = i + q * stride < n;
                r[q] = in ? rect[i + q * stride] : make_ushort4(0, 0, 0, 0);
                t4[q] = in ? ra.tiles_touched[i + q * stride] : 0u;
            }
#pragma unroll
            for (int q = 0; q < 4; q++) {
                recs += (r[q].z > r[q].x ? (uint32_t)(r[q].z - r[q].x) : 0u) * (r[q].w > r[q].y ? (uint32_t)(r[q].w - r[q].y) : 0u);
                tt += t4[q];
            }
        }
        recs = wave_inclusive_scan(recs);
        tt = wave_inclusive_scan(tt);
        if (lane == 63) { s_wave_recs[threadIdx.x >> 6] = recs; s_tt[threadIdx.x >> 6] = tt; }
        __syncthreads();
        if (threadIdx.x == 0) {
            unsigned long long all = 0, all_tt = 0;
            for (int w = 0; w < TILE_PAIR_THREADS / 64; w++) { all += s_wave_recs[w]; all_tt += s_tt[w]; }
            unsigned long long b = 0;
            if (all | all_tt) {
                b = atomicAdd(&ra.counters[0], all);
                atomicAdd(&ra.counters[1], all_tt);
            }
            // (a reservation that reaches beyond 32 bits is never used: the host rejects the call on the total)
            s_base[0] = (uint32_t)b;
            s_base[1] = (b + all) >> 32 ? 1u : 0u;
        }
        __syncthreads();
        rec_next = s_base[1] ? 0u : s_base[0];
        for (int w = 0; w < (int)(threadIdx.x >> 6); w++) rec_next += s_base[1] ? 0u : s_wave_recs[w];
    }
    // (every wavefront of the workgroup walks its own 64 Gaussians per round; no barrier inside the rounds)
    // (the next round's rectangle, record place and depth are requested before this round's candidates are walked)
    const int64_t i_first = (int64_t)blockIdx.x * TILE_PAIR_THREADS + threadIdx.x;
    const int64_t round_stride = (int64_t)gridDim.x * TILE_PAIR_THREADS;
    ushort4 r_next = i_first < n ? rect[i_first] : make_ushort4(0, 0, 0, 0);
    uint32_t roff_next = (SCATTER && i_first < n) ? rec_offsets[i_first] : 0u;
    uint32_t dbits_next = (SCATTER && i_first < n) ? __float_as_uint(depth[i_first]) : 0u;
    for (int64_t i = i_first; i - lane < n; i += round_stride) {
        const bool valid = i < n;
        const ushort4 r = r_next;
        const uint32_t roff = roff_next;
        const uint32_t w = r.z > r.x ? (uint32_t)(r.z - r.x) : 0u, h = r.w > r.y ? (uint32_t)(r.w - r.y) : 0u;
        const uint32_t cnt = w * h;
        const uint32_t dbits = cnt ? dbits_next : 0u;
        {
            const int64_t i2 = i + round_stride;
            const bool in = i2 < n;
            r_next = in ? rect[i2] : make_ushort4(0, 0, 0, 0);
            if (SCATTER) {
                roff_next = in ? rec_offsets[i2] : 0u;
                dbits_next = in ? __float_as_uint(depth[i2]) : 0u;
            }
        }
        float mx = 0.f, my = 0.f, A = 1.f, B = 0.f, C = 1.f, Q = 0.f;
        if (cnt && (CB || SCATTER)) {
            const float2 m = mean2d[i];
            const float4 co = conic_opacity[i];
            if (CB) { mx = m.x; my = m.y; A = co.x; B = co.y; C = co.z; Q = cb_threshold(co.w, cfg); }
            if (SCATTER) {
                float4* rec = splats + (size_t)i * (SPLAT_REC / 4);
                rec[0] = make_float4(m.x, m.y, co.x, co.y);
                rec[1] = make_float4(co.z, co.w, rgb[3 * i], rgb[3 * i + 1]);
                rec[2] = make_float4(rgb[3 * i + 2], __uint_as_float(roff), __uint_as_float((uint32_t)r.x | (uint32_t)r.y << 16),
                                     __uint_as_float((uint32_t)r.z | (uint32_t)r.w << 16));
            }
        }
        const uint32_t inc = wave_inclusive_scan(cnt);
        const uint32_t excl = inc - cnt;
        const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)inc, 63);
        const uint32_t rect_xy = (uint32_t)r.x | (uint32_t)r.y << 16;
        if (!SCATTER) {
            if (valid) {
                ra.rec_offsets[i] = rec_next + excl;
                if (ra.rec_counts) ra.rec_counts[i] = cnt;
            }
            rec_next += total;
        }
        uint32_t carry = 0;   // 1 + the lane whose rectangle holds candidate j0 - 1 (uniform)
        for (uint32_t j0 = 0; j0 < total; j0 += 64) {
            const bool live = j0 + lane < total;
            const uint32_t j = min(j0 + lane, total - 1);
            // Whose candidate is number j?  Every Gaussian with candidates leaves 1 + its lane at the slot of its first
            // one (if that falls into this window of 64; the slots are distinct), and a running maximum over the slots
            // spreads it over the rest of its run; the window's first slots belong to `carry`.  One trip through LDS
            // (a wavefront's LDS operations complete in the order they were issued) instead of the six dependent
            // shuffles of a binary search over the prefix sums.
            mark[lane] = 0u;
            const uint32_t rel = excl - j0;
            if (cnt != 0u && rel < 64u) mark[rel] = lane + 1u;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            uint32_t own = mark[lane];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            own = wave_inclusive_max(lane == 0u ? max(own, carry) : own);
            carry = (uint32_t)__builtin_amdgcn_readlane((int)own, 63);
            const uint32_t s = (own - 1u) & 63u;   // (own >= 1 wherever live: candidate 0 is some lane's first)
            const uint32_t k = j - (uint32_t)__shfl((int)excl, (int)s, 64);
            const uint32_t ow = (uint32_t)__shfl((int)w, (int)s, 64);
            const uint32_t oxy = (uint32_t)__shfl((int)rect_xy, (int)s, 64);
            // estimate with the fast reciprocal, off by at most one (k < 2^32 and ow < 2^16 make the quotient's error < 0.02):
            // corrected by one step either way, never by a loop that bad operands could keep a wavefront in
            uint32_t row = (uint32_t)((float)k * __builtin_amdgcn_rcpf((float)ow));
            row -= row * ow > k ? 1u : 0u;
            row += (row + 1) * ow <= k ? 1u : 0u;
            const uint32_t col = k - row * ow;
            const uint32_t tx = (oxy & 0xffffu) + col, ty = (oxy >> 16) + row;
            bool hit = live;
            if (CB) {
                const float omx = __shfl(mx, (int)s, 64), omy = __shfl(my, (int)s, 64);
                const float oA = __shfl(A, (int)s, 64), oB = __shfl(B, (int)s, 64), oC = __shfl(C, (int)s, 64);
                const float oQ = __shfl(Q, (int)s, 64);
                hit = live && cb_tile_hit(omx, omy, oA, oB, oC, oQ, (int)tx, (int)ty);
            }
            const uint32_t tile = ty * (uint32_t)tiles_x + tx;
            hit = hit && tile < (uint32_t)num_tiles;   // (always true for a rect made for this camera)
            if (!SCATTER) {
                if (hit) atomicAdd(&s_tile[tile], 1u);
            } else {
                const uint32_t od = (uint32_t)__shfl((int)dbits, (int)s, 64);
                const uint32_t oroff = (uint32_t)__shfl((int)roff, (int)s, 64);
                if (hit) {
                    const uint32_t slot = atomicAdd(&s_tile[tile], 1u);
                    if (slot < P) bucket[slot] = ((uint64_t)od << 32) | (uint32_t)(i - lane + s);
                } else if (CB && live && (uint64_t)oroff + k < rec_limit) {
                    float4* g = pair_grad + ((size_t)oroff + k) * (PAIR_REC / 4);
                    const float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
                    g[0] = z; g[1] = z; g[2] = z;
                }
            }
        }
    }
    if (!SCATTER) {
        __syncthreads();
        for (int t = threadIdx.x; t < num_tiles; t += TILE_PAIR_THREADS) my_row[t] = s_tile[t];
    }
}

// Per tile: its count summed over the workgroups' rows -> tile_total; each row's counter is replaced by the
// number of the tile's pairs in the rows before it (where that workgroup's pairs start within the tile's
// segment).  A workgroup takes 64 tiles; its wavefront g takes rows [64 g, 64 g + 64) of each.
__global__ __launch_bounds__(64 * (TILE_COPIES / 64)) void k_tile_sum(uint32_t* __restrict__ count, int num_tiles,
                                                                     uint32_t* __restrict__ tile_total)
{
    constexpr int GROUPS = TILE_COPIES / 64;
    // Order of the workgroups' shares within a tile's segment: workgroups are handed to the 8 XCDs in turn, so
    // those with the same index mod 8 share an L2; putting their shares next to each other lets the 8-byte words
    // they scatter into a segment fill whole lines in one L2 before they are written back.
    auto row_at = [](int pos) { return (pos % (TILE_COPIES / 8)) * 8 + pos / (TILE_COPIES / 8); };
    __shared__ uint32_t gsum[GROUPS][64];
    const int g = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int t = blockIdx.x * 64 + lane;
    uint32_t part[64];
    uint32_t sum = 0;
#pragma unroll
    for (int k = 0; k < 64; k++) {
        part[k] = t < num_tiles ? count[(size_t)row_at(g * 64 + k) * num_tiles + t] : 0u;
        sum += part[k];
    }
    gsum[g][lane] = sum;
    __syncthreads();
    uint32_t run = 0, all = 0;
#pragma unroll
    for (int q = 0; q < GROUPS; q++) {
        run += q < g ? gsum[q][lane] : 0u;
        all += gsum[q][lane];
    }
    if (t >= num_tiles) return;
#pragma unroll
    for (int k = 0; k < 64; k++) {
        count[(size_t)row_at(g * 64 + k) * num_tiles + t] = run;
        run += part[k];
    }
    if (g == 0) tile_total[t] = all;
}

// One workgroup: exclusive scan of the tile totals -> ranges [first, last); totals[2] = sum,
// totals[3] = longest list (totals[0..1] come from the counting kernel's two counters); and the order in which
// the render kernels take the tiles (longest list first, bucketed by length / 8, as k_tile_order).  Thread t owns the consecutive tiles [t*per, t*per + per).
__global__ __launch_bounds__(1024) void k_tile_scan(const uint32_t* __restrict__ tile_total, int num_tiles,
                                                    uint2* __restrict__ ranges, uint32_t* __restrict__ order,
                                                    uint64_t* __restrict__ totals,
                                                    unsigned long long* __restrict__ counters)
{
    constexpr int NB = 512;
    __shared__ uint32_t wsum[16];
    __shared__ uint32_t max_s;
    __shared__ uint32_t cnt[NB];
    for (int b = threadIdx.x; b < NB; b += 1024) cnt[b] = 0;
    if (threadIdx.x == 0) max_s = 0;
    __syncthreads();
    constexpr int PER_MAX = (TILE_LDS_MAX_TILES + 1023) / 1024;   // this path is only taken up to that many tiles
    const int per = (num_tiles + 1023) / 1024;
    const int t0 = threadIdx.x * per;
    auto bucket = [](uint32_t len) { return (int)(NB - 1 - min(len >> 3, (uint32_t)NB - 1)); };
    uint32_t c[PER_MAX];   // this thread's tile totals, read once
    uint32_t v = 0, mymax = 0;
#pragma unroll
    for (int q = 0; q < PER_MAX; q++) {
        const bool in = q < per && t0 + q < num_tiles;
        c[q] = in ? tile_total[t0 + q] : 0u;
        v += c[q];
        mymax = max(mymax, c[q]);
        if (in) atomicAdd(&cnt[bucket(c[q])], 1u);
    }
    const uint32_t inc = wave_inclusive_scan(v);
    if (lane_id() == 63) wsum[threadIdx.x >> 6] = inc;
    if (mymax) atomicMax(&max_s, mymax);
    __syncthreads();
    uint32_t run = inc - v;
    for (int w = 0; w < (int)(threadIdx.x >> 6); w++) run += wsum[w];
#pragma unroll
    for (int q = 0; q < PER_MAX; q++) {
        if (q < per && t0 + q < num_tiles) ranges[t0 + q] = c[q] ? make_uint2(run, run + c[q]) : make_uint2(0u, 0u);
        run += c[q];
    }
    if (threadIdx.x == 1023) {
        // totals: sum of tiles_touched, backward records, pairs counted per tile, longest list; the two counters of
        // the counting kernel start the next call at zero
        totals[0] = counters[1];
        totals[1] = counters[0];
        totals[2] = run;
        totals[3] = max_s;
        counters[0] = 0ull;
        counters[1] = 0ull;
    }
    // tile order: exclusive prefix over the 512 length buckets by one wavefront, then a counting placement
    if (threadIdx.x < 64) {
        uint32_t b8[8], sum = 0;
#pragma unroll
        for (int q = 0; q < 8; q++) { b8[q] = cnt[threadIdx.x * 8 + q]; sum += b8[q]; }
        uint32_t pre = wave_inclusive_scan(sum) - sum;
#pragma unroll
        for (int q = 0; q < 8; q++) { cnt[threadIdx.x * 8 + q] = pre; pre += b8[q]; }
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < PER_MAX; q++)
        if (q < per && t0 + q < num_tiles) order[atomicAdd(&cnt[bucket(c[q])], 1u)] = (uint32_t)(t0 + q);
}

// Step (3): one workgroup sorts one tile's segment in LDS (bitonic network on the 64-bit words, padded to
// a power of two with all-ones words) and writes the final keys tile << 32 | depth_bits and the Gaussian
// indices.  The network is bound by LDS traffic (every step reads and writes every word), so the steps at
// distances 4, 2, 1 of a stage -- which stay inside aligned groups of 8 words -- are done in registers: a thread
// loads a group, runs the three steps (all of the stages 2, 4, 8 at the start) and stores it back; the steps at
// larger distances are taken three at a time as well, on groups of 8 words the right distance apart, which makes
// 13 passes over LDS of the 36 steps of a 256-word sort.  Long lists use groups of 16 words (four steps a pass).
// Groups are 16 bytes further apart in LDS than their size so that the 16-byte accesses of neighbouring lanes fall
// into different banks.  (Replacing the workgroup barrier by a wavefront-level one for the steps at
// distance <= 64, a register/shuffle variant of those steps, and giving short lists to single wavefronts were
// all measured slower.)
// Handles the tiles whose length is in (len_lo, CAP]; the others are left to another launch.
__device__ __forceinline__ void cmpx(uint64_t& a, uint64_t& b, bool up)
{
    const bool sw = (a > b) == up;
    const uint64_t x = sw ? b : a, y = sw ? a : b;
    a = x;
    b = y;
}

// GG words at distance 2^a from each other through registers: the GG/2 .. 1 steps of stage k2 at distances
// 2^a GG/2 .. 2^a.  The words of a group agree in every index bit outside [a, a + log2 GG), the stage's bit
// among them, so one direction serves the group.  Ends with a workgroup barrier.
template <int GG, int LG, int THREADS>
__device__ __forceinline__ void tile_sort_strided(uint64_t* k, int N, int a, int k2)
{
    constexpr int LGG = GG == 2 ? 1 : GG == 4 ? 2 : GG == 8 ? 3 : 4;
    auto at = [](int e) { return e + ((e >> LG) << 1); };
    for (int g = threadIdx.x; g < N / GG; g += THREADS) {
        const int e0 = ((g >> a) << (a + LGG)) | (g & ((1 << a) - 1));
        const bool up = (e0 & k2) == 0;
        uint64_t v[GG];
#pragma unroll
        for (int q = 0; q < GG; q++) v[q] = k[at(e0 + (q << a))];
#pragma unroll
        for (int jj = GG / 2; jj > 0; jj >>= 1)
#pragma unroll
            for (int q = 0; q < GG; q++)
                if ((q & jj) == 0) cmpx(v[q], v[q | jj], up);
#pragma unroll
        for (int q = 0; q < GG; q++) k[at(e0 + (q << a))] = v[q];
    }
    __syncthreads();
}

// The sort proper, with G (8 or 16) words per register group; k holds N + 2 N / G words.  A stage's steps are
// taken log2 G at a time, from the largest distance down: first the odd ones out (a smaller group), then groups
// of G words ever closer together, last the contiguous groups with 16-byte LDS accesses.
template <int G, int THREADS, int CAP>
__device__ __forceinline__ void tile_sort_lds(uint64_t* k, int N, int n, uint32_t tile, uint32_t first,
                                              const uint64_t* __restrict__ bucket, uint64_t* __restrict__ keys_out,
                                              uint32_t* __restrict__ vals_out)
{
    constexpr int LG = G == 8 ? 3 : 4;
    static_assert(G == 8 || G == 16, "group of 8 or 16 words");
    auto at = [](int e) { return e + ((e >> LG) << 1); };   // word e of the sequence -> its place in k
    {
        // (all of a thread's loads are issued before the first LDS write: written as one loop, each load would be
        // waited for in turn)
        constexpr int PER = (CAP + THREADS - 1) / THREADS;
        uint64_t w[PER];
#pragma unroll
        for (int u = 0; u < PER; u++) {
            const int i = threadIdx.x + u * THREADS;
            w[u] = i < n ? bucket[first + i] : ~0ull;
        }
#pragma unroll
        for (int u = 0; u < PER; u++) {
            const int i = threadIdx.x + u * THREADS;
            if (i < N) k[at(i)] = w[u];
        }
    }
    __syncthreads();
    // one contiguous group through registers: FIRST = the complete stages 2 .. G, otherwise the steps at
    // distances G/2 .. 1 of a later stage, whose direction `up` is the same for the whole group
    auto local = [&](int g, bool first_stages, bool up) {
        uint4* q = reinterpret_cast<uint4*>(&k[(G + 2) * g]);
        uint64_t v[G];
#pragma unroll
        for (int h = 0; h < G / 2; h++) {
            const uint4 w = q[h];
            v[2 * h] = ((uint64_t)w.y << 32) | w.x;
            v[2 * h + 1] = ((uint64_t)w.w << 32) | w.z;
        }
        if (first_stages) {
#pragma unroll
            for (int k2 = 2; k2 < G; k2 <<= 1)
#pragma unroll
                for (int j = k2 >> 1; j > 0; j >>= 1)
#pragma unroll
                    for (int e = 0; e < G; e++)
                        if ((e & j) == 0) cmpx(v[e], v[e | j], (e & k2) == 0);
        }
#pragma unroll
        for (int j = G / 2; j > 0; j >>= 1)
#pragma unroll
            for (int e = 0; e < G; e++)
                if ((e & j) == 0) cmpx(v[e], v[e | j], up);
#pragma unroll
        for (int h = 0; h < G / 2; h++)
            q[h] = make_uint4((uint32_t)v[2 * h], (uint32_t)(v[2 * h] >> 32), (uint32_t)v[2 * h + 1],
                              (uint32_t)(v[2 * h + 1] >> 32));
    };
    for (int g = threadIdx.x; g < (N >> LG); g += THREADS) local(g, true, ((G * g) & G) == 0);
    __syncthreads();
    for (int k2 = 2 * G, m = LG + 1; k2 <= N; k2 <<= 1, m++) {   // m = log2 k2: the stage has steps 2^(m-1) .. 1
        int top = m;
        const int odd = (m - LG) % LG;
        if (odd == 1) tile_sort_strided<2, LG, THREADS>(k, N, top - 1, k2);
        if (odd == 2) tile_sort_strided<4, LG, THREADS>(k, N, top - 2, k2);
        if (odd == 3) tile_sort_strided<8, LG, THREADS>(k, N, top - 3, k2);
        top -= odd;
        for (; top > LG; top -= LG) tile_sort_strided<G, LG, THREADS>(k, N, top - LG, k2);
        for (int g = threadIdx.x; g < (N >> LG); g += THREADS) local(g, false, ((G * g) & k2) == 0);
        __syncthreads();
    }
    for (int i = threadIdx.x; i < n; i += THREADS) {
        const uint64_t v = k[at(i)];
        keys_out[first + i] = ((uint64_t)tile << 32) | (v >> 32);
        vals_out[first + i] = (uint32_t)v;
    }
}

template <int CAP, int THREADS>
__global__ __launch_bounds__(THREADS) void k_tile_sort(const uint2* __restrict__ ranges,
                                                   const uint32_t* __restrict__ tile_order,
                                                   const uint64_t* __restrict__ bucket, int len_lo, uint32_t limit,
                                                   uint64_t* __restrict__ keys_out, uint32_t* __restrict__ vals_out)
{
    // (groups of 8 words are padded by a quarter, groups of 16, which every list beyond 512 words uses, by an eighth)
    __shared__ __align__(16) uint64_t k[CAP + CAP / (CAP > 8192 ? 8 : 4)];
    const uint32_t tile = tile_order[blockIdx.x];
    const uint2 r = ranges[tile];
    const int n = (int)(r.y - r.x);
    // (uniform over the workgroup; `limit` = the words the buffers hold: a segment that reaches beyond it is left alone)
    if (n <= len_lo || n > CAP || r.y > limit) return;
    int N = 16;
    while (N < n) N <<= 1;
    // groups of 16 words make fewer passes over LDS but leave N / 16 threads busy in the register phases:
    // measured better from 1024 words on
    if (N <= TILE_SORT_GROUP16_FROM / 2)
        tile_sort_lds<8, THREADS, CAP>(k, N, n, tile, r.x, bucket, keys_out, vals_out);
    else
        tile_sort_lds<16, THREADS, CAP>(k, N, n, tile, r.x, bucket, keys_out, vals_out);
}

// ---- radix sort -------------------------------------------------------------------------
// One pass ranks RADIX_BLOCK_KEYS keys per workgroup on a digit of up to RADIX_BITS bits (the live key
// bits are split into the fewest such digits, of equal width).  Wave w of the workgroup owns the
// contiguous chunk [w*512, w*512+512) of the block's keys and walks it in 8 rounds of 64 consecutive
// keys, so (wave, round, lane) order is the input order and the ranking is stable.

constexpr int RADIX_ROUNDS = RADIX_BLOCK_KEYS / 256;  // rounds per wave

// Per-workgroup digit histogram, stored digit-major: hist[digit * num_blocks + block].
__global__ __launch_bounds__(256) void k_radix_hist(const uint64_t* __restrict__ keys, uint32_t P, int shift,
                                                    uint32_t mask, uint32_t num_blocks,
                                                    uint32_t* __restrict__ hist)
{
    __shared__ uint32_t cnt[RADIX_DIGITS];
    for (int d = threadIdx.x; d < RADIX_DIGITS; d += 256) cnt[d] = 0;
    __syncthreads();
    const uint32_t base = blockIdx.x * RADIX_BLOCK_KEYS;
#pragma unroll
    for (int r = 0; r < RADIX_ROUNDS; r++) {
        const uint32_t i = base + r * 256 + threadIdx.x;
        if (i < P) atomicAdd(&cnt[(uint32_t)(keys[i] >> shift) & mask], 1u);
    }
    __syncthreads();
    for (uint32_t d = threadIdx.x; d <= mask; d += 256) hist[d * num_blocks + blockIdx.x] = cnt[d];
}

__global__ __launch_bounds__(256) void k_radix_scatter(const uint64_t* __restrict__ kin,
                                                       const uint32_t* __restrict__ vin,
                                                       uint64_t* __restrict__ kout, uint32_t* __restrict__ vout,
                                                       const uint32_t* __restrict__ hist_scanned, uint32_t P,
                                                       int shift, int bits, uint32_t num_blocks)
{
    __shared__ uint32_t cnt[4][RADIX_DIGITS];
    const int wave = threadIdx.x >> 6;
    const uint32_t lane = lane_id();
    const uint32_t mask = (1u << bits) - 1u;
#pragma unroll
    for (int w = 0; w < 4; w++)
        for (int d = threadIdx.x; d < RADIX_DIGITS; d += 256) cnt[w][d] = 0;
    __syncthreads();

    const uint32_t wave_start = blockIdx.x * RADIX_BLOCK_KEYS + wave * (RADIX_ROUNDS * 64);
    uint64_t key[RADIX_ROUNDS];
    uint32_t val[RADIX_ROUNDS], rank[RADIX_ROUNDS];
#pragma unroll
    for (int r = 0; r < RADIX_ROUNDS; r++) {
        const uint32_t i = wave_start + r * 64 + lane;
        const bool valid = i < P;
        key[r] = valid ? kin[i] : 0ull;
        val[r] = valid ? vin[i] : 0u;
    }
#pragma unroll
    for (int r = 0; r < RADIX_ROUNDS; r++) {
        const uint32_t i = wave_start + r * 64 + lane;
        const bool valid = i < P;
        const uint32_t d = (uint32_t)(key[r] >> shift) & mask;
        // lanes of this wave holding the same digit
        uint64_t peers = __ballot(valid);
        for (int b = 0; b < bits; b++) {
            const bool bit = (d >> b) & 1u;
            const uint64_t bal = __ballot(valid && bit);
            peers &= bit ? bal : ~bal;
        }
        const uint32_t below = __popcll(peers & ((1ull << lane) - 1ull));
        const uint32_t count = __popcll(peers);
        uint32_t prev = 0;
        if (valid) prev = cnt[wave][d];
        __builtin_amdgcn_wave_barrier();
        if (valid && below == 0) cnt[wave][d] = prev + count;
        __builtin_amdgcn_wave_barrier();
        rank[r] = prev + below;
    }
    __syncthreads();
    // per digit: global start of this block's run of that digit, then per-wave starts
    for (uint32_t d = threadIdx.x; d <= mask; d += 256) {
        uint32_t run = hist_scanned[d * num_blocks + blockIdx.x];
#pragma unroll
        for (int w = 0; w < 4; w++) {
            const uint32_t c = cnt[w][d];
            cnt[w][d] = run;
            run += c;
        }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < RADIX_ROUNDS; r++) {
        const uint32_t i = wave_start + r * 64 + lane;
        if (i < P) {
            const uint32_t d = (uint32_t)(key[r] >> shift) & mask;
            const uint32_t pos = cnt[wave][d] + rank[r];
            kout[pos] = key[r];
            vout[pos] = val[r];
        }
    }
}

// ranges[t] = [first,last) for every tile present in the sorted keys (ranges pre-filled with 0).
__global__ __launch_bounds__(256) void k_tile_ranges(const uint64_t* __restrict__ keys, uint32_t P,
                                                     uint32_t* __restrict__ ranges)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= P) return;
    const uint32_t t = (uint32_t)(keys[i] >> 32);
    if (i == 0 || (uint32_t)(keys[i - 1] >> 32) != t) ranges[2 * t] = i;
    if (i + 1 == P || (uint32_t)(keys[i + 1] >> 32) != t) ranges[2 * t + 1] = i + 1;
}

// Order in which the render kernels take the tiles: longest list first (bucketed by length / 8), so
// that the last workgroups of a launch are the cheapest ones.  One workgroup; any order is valid.
__global__ __launch_bounds__(1024) void k_tile_order(const uint2* __restrict__ ranges, int num_tiles,
                                                     uint32_t* __restrict__ order)
{
    constexpr int NB = 512;
    __shared__ uint32_t cnt[NB];
    for (int b = threadIdx.x; b < NB; b += 1024) cnt[b] = 0;
    __syncthreads();
    auto bucket = [](uint2 r) { const uint32_t len = r.y - r.x; return (int)(NB - 1 - min(len >> 3, (uint32_t)NB - 1)); };
    for (int t = threadIdx.x; t < num_tiles; t += 1024) atomicAdd(&cnt[bucket(ranges[t])], 1u);
    __syncthreads();
    if (threadIdx.x < 64) {  // exclusive prefix over the 512 buckets by one wavefront, 8 buckets per lane
        uint32_t c[8], sum = 0;
#pragma unroll
        for (int k = 0; k < 8; k++) { c[k] = cnt[threadIdx.x * 8 + k]; sum += c[k]; }
        uint32_t run = wave_inclusive_scan(sum) - sum;
#pragma unroll
        for (int k = 0; k < 8; k++) { cnt[threadIdx.x * 8 + k] = run; run += c[k]; }
    }
    __syncthreads();
    for (int t = threadIdx.x; t < num_tiles; t += 1024) order[atomicAdd(&cnt[bucket(ranges[t])], 1u)] = (uint32_t)t;
}

__global__ __launch_bounds__(256) void k_fill_u32(uint32_t* __restrict__ p, uint32_t v, int64_t count)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = v;
}

}  // namespace

size_t scan_tmp_bytes(int64_t n)
{
    const int64_t nb = (n + SCAN_BLOCK - 1) / SCAN_BLOCK;
    return (size_t)(nb > 0 ? nb : 1) * sizeof(uint64_t);
}

hipError_t launch_exclusive_scan(hipStream_t st, const uint32_t* in, uint32_t* out, int64_t n, void* tmp,
                                 uint64_t* total_dev)
{
    const int64_t nb = (n + SCAN_BLOCK - 1) / SCAN_BLOCK;
    uint64_t* bs = static_cast<uint64_t*>(tmp);
    if (nb > 0) hipLaunchKernelGGL(k_scan_block_sums, dim3((unsigned)nb), dim3(SCAN_THREADS), 0, st, in, n, bs);
    hipLaunchKernelGGL(k_scan_block_offsets, dim3(1), dim3(SCAN_THREADS), 0, st, bs, nb, total_dev);
    if (nb > 0) hipLaunchKernelGGL(k_scan_apply, dim3((unsigned)nb), dim3(SCAN_THREADS), 0, st, in, out, n, bs);
    return hipGetLastError();
}

hipError_t launch_emit_pairs(hipStream_t st, int64_t n, const fs_projected& proj, const uint32_t* offsets,
                             int tiles_x, uint64_t* keys, uint32_t* vals, float* splats)
{
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(k_emit_pairs, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, n,
                       reinterpret_cast<const ushort4*>(proj.rect), proj.depth,
                       reinterpret_cast<const float2*>(proj.mean2d), reinterpret_cast<const float4*>(proj.conic_opacity),
                       proj.rgb, offsets, tiles_x, keys, vals, reinterpret_cast<float4*>(splats));
    return hipGetLastError();
}

hipError_t launch_rect_area(hipStream_t st, int64_t n, const uint16_t* rect, uint32_t* rec_counts)
{
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(k_rect_area, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, n,
                       reinterpret_cast<const ushort4*>(rect), rec_counts);
    return hipGetLastError();
}

hipError_t launch_emit_pairs_cb(hipStream_t st, int64_t n, const fs_projected& proj, const CfgDev& cfg,
                                const uint32_t* offsets, const uint32_t* rec_offsets, int tiles_x, int64_t P,
                                uint64_t* keys, uint32_t* vals, float* splats, float* pair_grad)
{
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(k_emit_pairs_cb, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, n,
                       reinterpret_cast<const ushort4*>(proj.rect), proj.depth,
                       reinterpret_cast<const float2*>(proj.mean2d), reinterpret_cast<const float4*>(proj.conic_opacity),
                       proj.rgb, cfg, offsets, rec_offsets, tiles_x, (uint32_t)P, keys, vals,
                       reinterpret_cast<float4*>(splats),
                       reinterpret_cast<float4*>(pair_grad));
    return hipGetLastError();
}

hipError_t launch_tile_count(hipStream_t st, int64_t n, const fs_projected& proj, const CfgDev& cfg, int tiles_x,
                             int num_tiles, uint32_t* tile_count, uint32_t* tile_total, uint2* ranges,
                             uint32_t* tile_order, uint64_t* totals, uint32_t* rec_offsets, uint32_t* rec_counts,
                             uint64_t* counters)
{
    const RecAlloc ra = {proj.tiles_touched, rec_offsets, rec_counts, reinterpret_cast<unsigned long long*>(counters)};
    {
        const dim3 grid(TILE_COPIES), block(TILE_PAIR_THREADS);
        const size_t lds = (size_t)num_tiles * sizeof(uint32_t);
        const ushort4* rect = reinterpret_cast<const ushort4*>(proj.rect);
        const float2* m2 = reinterpret_cast<const float2*>(proj.mean2d);
        const float4* co = reinterpret_cast<const float4*>(proj.conic_opacity);
        if (cfg.compact_box)
            hipLaunchKernelGGL((k_tile_pairs<true, false>), grid, block, lds, st, n, rect, proj.depth, m2, co, proj.rgb, cfg,
                               nullptr, tiles_x, num_tiles, tile_count, nullptr, 0u, 0u, nullptr, nullptr, nullptr, ra);
        else
            hipLaunchKernelGGL((k_tile_pairs<false, false>), grid, block, lds, st, n, rect, proj.depth, m2, co, proj.rgb,
                               cfg, nullptr, tiles_x, num_tiles, tile_count, nullptr, 0u, 0u, nullptr, nullptr, nullptr, ra);
    }
    hipLaunchKernelGGL(k_tile_sum, dim3((unsigned)((num_tiles + 63) / 64)), dim3(64 * (TILE_COPIES / 64)), 0, st, tile_count,
                       num_tiles, tile_total);
    hipLaunchKernelGGL(k_tile_scan, dim3(1), dim3(1024), 0, st, tile_total, num_tiles, ranges, tile_order, totals,
                       reinterpret_cast<unsigned long long*>(counters));
    return hipGetLastError();
}

hipError_t launch_tile_scatter(hipStream_t st, int64_t n, const fs_projected& proj, const CfgDev& cfg,
                               const uint32_t* rec_offsets, int tiles_x, int num_tiles, uint32_t pair_limit,
                               uint32_t rec_limit, const uint2* ranges, uint32_t* cursor, uint64_t* bucket, float* splats,
                               float* pair_grad)
{
    if (n <= 0) return hipSuccess;
    const dim3 grid(TILE_COPIES), block(TILE_PAIR_THREADS);
    const size_t lds = (size_t)num_tiles * sizeof(uint32_t);
    const ushort4* rect = reinterpret_cast<const ushort4*>(proj.rect);
    const float2* m2 = reinterpret_cast<const float2*>(proj.mean2d);
    const float4* co = reinterpret_cast<const float4*>(proj.conic_opacity);
    if (cfg.compact_box)
        hipLaunchKernelGGL((k_tile_pairs<true, true>), grid, block, lds, st, n, rect, proj.depth, m2, co, proj.rgb, cfg,
                           rec_offsets, tiles_x, num_tiles, cursor, ranges, pair_limit, rec_limit, bucket,
                           reinterpret_cast<float4*>(splats), reinterpret_cast<float4*>(pair_grad), RecAlloc{});
    else
        hipLaunchKernelGGL((k_tile_pairs<false, true>), grid, block, lds, st, n, rect, proj.depth, m2, co, proj.rgb, cfg,
                           rec_offsets, tiles_x, num_tiles, cursor, ranges, pair_limit, rec_limit, bucket,
                           reinterpret_cast<float4*>(splats), reinterpret_cast<float4*>(pair_grad), RecAlloc{});
    return hipGetLastError();
}

int tile_sort_variants(int64_t max_len, bool long_lists, int have)
{
    // which length classes still need a launch: (0, SMALL], (SMALL, MID], (MID, MAX], (MAX, HUGE]
    int v = 0;
    if (!(have & TS_SMALL)) v |= TS_SMALL;
    const bool need_mid = max_len > TILE_SORT_SMALL && !(have & (TS_MID | TS_MIDMAX));
    const bool need_max = max_len > TILE_SORT_MID && !(have & (TS_MAX | TS_MIDMAX));
    if (need_mid && need_max) v |= long_lists ? (TS_MID | TS_MAX) : TS_MIDMAX;
    else if (need_mid) v |= long_lists || (have & TS_MAX) ? TS_MID : TS_MIDMAX;
    else if (need_max) v |= TS_MAX;
    if (max_len > TILE_SORT_MAX && !(have & TS_HUGE)) v |= TS_HUGE;
    return v;
}

hipError_t launch_tile_sorts(hipStream_t st, int num_tiles, int variants, uint32_t pair_limit, const uint2* ranges,
                             const uint32_t* tile_order, const uint64_t* bucket, uint64_t* keys_out, uint32_t* vals_out)
{
    if (num_tiles <= 0) return hipSuccess;
    // the long lists first: few workgroups, each a long chain of steps, which more threads shorten
    if (variants & TS_HUGE)
        hipLaunchKernelGGL((k_tile_sort<TILE_SORT_HUGE, 1024>), dim3(num_tiles), dim3(1024), 0, st, ranges, tile_order,
                           bucket, TILE_SORT_MAX, pair_limit, keys_out, vals_out);
    if (variants & (TS_MAX | TS_MIDMAX))
        hipLaunchKernelGGL((k_tile_sort<TILE_SORT_MAX, 1024>), dim3(num_tiles), dim3(1024), 0, st, ranges, tile_order,
                           bucket, (variants & TS_MIDMAX) ? TILE_SORT_SMALL : TILE_SORT_MID, pair_limit, keys_out, vals_out);
    if (variants & TS_MID)
        hipLaunchKernelGGL((k_tile_sort<TILE_SORT_MID, 512>), dim3(num_tiles), dim3(512), 0, st, ranges, tile_order,
                           bucket, TILE_SORT_SMALL, pair_limit, keys_out, vals_out);
    if (variants & TS_SMALL)
        hipLaunchKernelGGL((k_tile_sort<TILE_SORT_SMALL, 256>), dim3(num_tiles), dim3(256), 0, st, ranges, tile_order, bucket,
                           0, pair_limit, keys_out, vals_out);
    return hipGetLastError();
}

hipError_t launch_radix_sort(hipStream_t st, int64_t P, int total_bits, uint64_t* keys[2], uint32_t* vals[2],
                             uint32_t* hist, void* scan_tmp, uint64_t* scan_total_dev, int* result_index)
{
    int cur = 0;
    if (P > 0) {
        const uint32_t nb = (uint32_t)radix_num_blocks(P);
        const int passes = (total_bits + RADIX_BITS - 1) / RADIX_BITS;
        const int bits = (total_bits + passes - 1) / passes;  // equal-width digits, at most RADIX_BITS
        for (int p = 0; p < passes; p++) {
            const int shift = bits * p;
            const uint32_t mask = (1u << bits) - 1u;
            hipLaunchKernelGGL(k_radix_hist, dim3(nb), dim3(256), 0, st, keys[cur], (uint32_t)P, shift, mask, nb,
                               hist);
            hipError_t e = launch_exclusive_scan(st, hist, hist, (int64_t)(mask + 1) * nb, scan_tmp, scan_total_dev);
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL(k_radix_scatter, dim3(nb), dim3(256), 0, st, keys[cur], vals[cur], keys[cur ^ 1],
                               vals[cur ^ 1], hist, (uint32_t)P, shift, bits, nb);
            cur ^= 1;
        }
    }
    *result_index = cur;
    return hipGetLastError();
}

hipError_t launch_tile_ranges(hipStream_t st, int64_t P, const uint64_t* keys_sorted, int num_tiles,
                              uint32_t* ranges, uint32_t* tile_order)
{
    hipError_t e = launch_fill_u32(st, ranges, 0u, (int64_t)2 * num_tiles);
    if (e != hipSuccess) return e;
    if (P > 0)
        hipLaunchKernelGGL(k_tile_ranges, dim3((unsigned)((P + 255) / 256)), dim3(256), 0, st, keys_sorted,
                           (uint32_t)P, ranges);
    if (num_tiles > 0)
        hipLaunchKernelGGL(k_tile_order, dim3(1), dim3(1024), 0, st, reinterpret_cast<const uint2*>(ranges), num_tiles,
                           tile_order);
    return hipGetLastError();
}

hipError_t launch_fill_u32(hipStream_t st, uint32_t* p, uint32_t v, int64_t count)
{
    if (count <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_fill_u32, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st, p, v, count);
    return hipGetLastError();
}

}  // namespace fs
