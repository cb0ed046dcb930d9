// Per-tile alpha compositing (forward), its gradient (backward) and the high-error-pixel count
// (score) on gfx950.
//
// FastGS Sec. 3, Eq. (4): C(p) = sum_i c_i alpha_i prod_{j<i} (1 - alpha_j), alpha_i = sigma_i G'_i(p),
// Eq. (5): G'_i(p) = exp(-1/2 (p - mu_2D)^T Sigma_2D^-1 (p - mu_2D)).
// Sec. 4.2, Eq. for s_d: per Gaussian, the number of high-error pixels in its footprint.
//
// One workgroup (4 wavefronts) per 16x16 tile; wavefront w owns the 8x8 quadrant (w&1, w>>1), one
// pixel per lane.  The tile's depth-ordered Gaussians are staged through LDS in batches of 256;
// a wavefront stops evaluating as soon as all of its 64 pixels have terminated.
//
// alpha, T and the blend weights follow a fixed fp32 operation order (fused multiply-adds only
// where written as __builtin_fmaf; the file is compiled with -ffp-contract=off) so that the
// integer outputs they decide (n_contrib, counts) can be reproduced bit for bit on a CPU.
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

struct Pixel {
    int x, y;
    bool inside;
    float px, py;
};

__device__ __forceinline__ Pixel pixel_of_thread(const CamDev& cam, int tile)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int tx = tile % cam.tiles_x, ty = tile / cam.tiles_x;
    Pixel p;
    p.x = tx * TILE + (wave & 1) * 8 + (lane & 7);
    p.y = ty * TILE + (wave >> 1) * 8 + (lane >> 3);
    p.inside = p.x < cam.width && p.y < cam.height;
    p.px = (float)p.x + 0.5f;
    p.py = (float)p.y + 0.5f;
    return p;
}

// alpha of one Gaussian at one pixel; false if it takes no part (exponent > 0, alpha < alpha_min).
// xy = mu_2D, co = (a, 2b, c, sigma).
__device__ __forceinline__ bool alpha_at(const Pixel& p, float2 xy, float4 co, const CfgDev& cfg, float& alpha,
                                         float& dx, float& dy, float& G)
{
    dx = p.px - xy.x;
    dy = p.py - xy.y;
    const float u = __builtin_fmaf(co.y, dy, co.x * dx);
    const float q = __builtin_fmaf(dx, u, (co.z * dy) * dy);
    const float power = -0.5f * q;
    if (power > 0.0f || power < cfg.power_min) return false;
    G = exp_c(power);
    alpha = fminf(cfg.alpha_max, co.w * G);
    return alpha >= cfg.alpha_min;
}

__global__ __launch_bounds__(256) void k_render_fwd(CamDev cam, CfgDev cfg, const uint2* __restrict__ ranges,
                                                    const uint32_t* __restrict__ gauss_sorted,
                                                    const float2* __restrict__ mean2d,
                                                    const float4* __restrict__ conic_opacity,
                                                    const float* __restrict__ rgb, float* __restrict__ image,
                                                    float* __restrict__ final_T, uint32_t* __restrict__ n_contrib)
{
    __shared__ float2 s_xy[BATCH];
    __shared__ float4 s_co[BATCH];
    __shared__ float s_rgb[BATCH * 3];

    const int tile = blockIdx.x;
    const Pixel p = pixel_of_thread(cam, tile);
    const uint2 range = ranges[tile];
    const int total = (int)(range.y - range.x);

    bool done = !p.inside;
    float T = 1.0f, C0 = 0.f, C1 = 0.f, C2 = 0.f;
    uint32_t last = 0;

    for (int start = 0; start < total; start += BATCH) {
        if (__syncthreads_count(!done) == 0) break;
        const int m = min(BATCH, total - start);
        if ((int)threadIdx.x < m) {
            const uint32_t g = gauss_sorted[range.x + start + threadIdx.x];
            float4 co = conic_opacity[g];
            co.y = co.y + co.y;
            s_xy[threadIdx.x] = mean2d[g];
            s_co[threadIdx.x] = co;
            s_rgb[3 * threadIdx.x + 0] = rgb[3 * g + 0];
            s_rgb[3 * threadIdx.x + 1] = rgb[3 * g + 1];
            s_rgb[3 * threadIdx.x + 2] = rgb[3 * g + 2];
        }
        __syncthreads();
        for (int j = 0; j < m; j++) {
            if (__ballot(!done) == 0) break;
            if (done) continue;
            float alpha, dx, dy, G;
            if (!alpha_at(p, s_xy[j], s_co[j], cfg, alpha, dx, dy, G)) continue;
            const float Tn = T * (1.0f - alpha);
            if (Tn < cfg.T_min) { done = true; continue; }
            const float w = alpha * T;
            C0 = __builtin_fmaf(s_rgb[3 * j + 0], w, C0);
            C1 = __builtin_fmaf(s_rgb[3 * j + 1], w, C1);
            C2 = __builtin_fmaf(s_rgb[3 * j + 2], w, C2);
            T = Tn;
            last = (uint32_t)(start + j + 1);
        }
    }
    if (p.inside) {
        const size_t hw = (size_t)cam.width * cam.height;
        const size_t pix = (size_t)p.y * cam.width + p.x;
        image[pix] = __builtin_fmaf(T, cfg.bg[0], C0);
        image[hw + pix] = __builtin_fmaf(T, cfg.bg[1], C1);
        image[2 * hw + pix] = __builtin_fmaf(T, cfg.bg[2], C2);
        final_T[pix] = T;
        n_contrib[pix] = last;
    }
}

// Sum over the 64 lanes of a wavefront; the total is returned in every lane of the last row
// (callers read lane 63).  Cross-lane moves use DPP: quad swaps, half-row and row mirrors, then
// the row broadcasts of the gfx9 family.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_step(float v)
{
    const int moved = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xF, false);
    return v + __int_as_float(moved);
}

__device__ __forceinline__ float wave_sum_to_lane63(float v)
{
    v = dpp_step<0xB1, 0xF>(v);   // quad_perm [1,0,3,2]
    v = dpp_step<0x4E, 0xF>(v);   // quad_perm [2,3,0,1]
    v = dpp_step<0x141, 0xF>(v);  // row_half_mirror
    v = dpp_step<0x140, 0xF>(v);  // row_mirror: every lane of a row of 16 holds the row sum
    v = dpp_step<0x142, 0xA>(v);  // row_bcast:15 into rows 1 and 3
    v = dpp_step<0x143, 0xC>(v);  // row_bcast:31 into rows 2 and 3
    return v;
}

// Backward of the compositing.  Walks each tile's list back to front from the furthest blended
// Gaussian; per Gaussian, the 9 partial gradients of the 64 pixels of a wavefront are summed
// across lanes, combined across the 4 wavefronts in LDS, and flushed with one atomic per value.
__global__ __launch_bounds__(256) void k_render_bwd(
    CamDev cam, CfgDev cfg, const uint2* __restrict__ ranges, const uint32_t* __restrict__ gauss_sorted,
    const float2* __restrict__ mean2d, const float4* __restrict__ conic_opacity, const float* __restrict__ rgb,
    const float* __restrict__ final_T, const uint32_t* __restrict__ n_contrib, const float* __restrict__ dL_dimage,
    float* __restrict__ d_mean2d, float* __restrict__ d_conic, float* __restrict__ d_opac, float* __restrict__ d_rgb)
{
    __shared__ float2 s_xy[BATCH];
    __shared__ float4 s_co[BATCH];
    __shared__ float s_rgb[BATCH * 3];
    __shared__ uint32_t s_id[BATCH];
    __shared__ float s_acc[BATCH][9];
    __shared__ uint32_t s_touched[BATCH];
    __shared__ int s_max;

    const int tile = blockIdx.x;
    const Pixel p = pixel_of_thread(cam, tile);
    const uint2 range = ranges[tile];
    const size_t hw = (size_t)cam.width * cam.height;
    const size_t pix = (size_t)p.y * cam.width + p.x;
    const int lane = threadIdx.x & 63;

    const int last = p.inside ? (int)n_contrib[pix] : 0;
    float T = p.inside ? final_T[pix] : 0.f;
    float dC0 = 0.f, dC1 = 0.f, dC2 = 0.f;
    if (p.inside) {
        dC0 = dL_dimage[pix];
        dC1 = dL_dimage[hw + pix];
        dC2 = dL_dimage[2 * hw + pix];
    }
    float B0 = cfg.bg[0], B1 = cfg.bg[1], B2 = cfg.bg[2];

    if (threadIdx.x == 0) s_max = 0;
    __syncthreads();
    atomicMax(&s_max, last);
    __syncthreads();
    const int total = s_max;  // entries at positions >= total are blended by no pixel of the tile

    // batches from the back: batch b covers positions [b*BATCH, min(total,(b+1)*BATCH))
    for (int start = ((total - 1) / BATCH) * BATCH; start >= 0 && total > 0; start -= BATCH) {
        const int m = min(BATCH, total - start);
        __syncthreads();
        if ((int)threadIdx.x < m) {
            const uint32_t g = gauss_sorted[range.x + start + threadIdx.x];
            float4 co = conic_opacity[g];
            co.y = co.y + co.y;
            s_id[threadIdx.x] = g;
            s_xy[threadIdx.x] = mean2d[g];
            s_co[threadIdx.x] = co;
            s_rgb[3 * threadIdx.x + 0] = rgb[3 * g + 0];
            s_rgb[3 * threadIdx.x + 1] = rgb[3 * g + 1];
            s_rgb[3 * threadIdx.x + 2] = rgb[3 * g + 2];
        }
#pragma unroll
        for (int k = 0; k < 9; k++) s_acc[threadIdx.x][k] = 0.f;
        s_touched[threadIdx.x] = 0;
        __syncthreads();

        for (int j = m - 1; j >= 0; j--) {
            const float2 xy = s_xy[j];
            const float4 co = s_co[j];
            float alpha = 0.f, dx = 0.f, dy = 0.f, G = 0.f;
            const bool act = (start + j < last) && alpha_at(p, xy, co, cfg, alpha, dx, dy, G);
            if (__ballot(act) == 0) continue;
            float v[9];
#pragma unroll
            for (int k = 0; k < 9; k++) v[k] = 0.f;
            if (act) {
                const float c0 = s_rgb[3 * j + 0], c1 = s_rgb[3 * j + 1], c2 = s_rgb[3 * j + 2];
                const float om = 1.0f - alpha;
                T = T * __builtin_amdgcn_rcpf(om);  // transmittance in front of this Gaussian
                const float w = alpha * T;
                v[0] = w * dC0;
                v[1] = w * dC1;
                v[2] = w * dC2;
                const float e0 = c0 - B0, e1 = c1 - B1, e2 = c2 - B2;
                float dL_dalpha = T * (e0 * dC0 + e1 * dC1 + e2 * dC2);
                B0 = B0 + alpha * e0;
                B1 = B1 + alpha * e1;
                B2 = B2 + alpha * e2;
                const float sG = co.w * G;
                if (sG > cfg.alpha_max) dL_dalpha = 0.f;  // capped alpha is a constant
                v[3] = G * dL_dalpha;                      // d/d sigma
                const float gq = -0.5f * sG * dL_dalpha;   // d/d q,  q = a dx^2 + 2 b dx dy + c dy^2
                v[4] = gq * dx * dx;
                v[5] = gq * 2.0f * dx * dy;
                v[6] = gq * dy * dy;
                // d = p - mu  =>  dq/dmu = -(2 a dx + 2b dy, 2b dx + 2 c dy);  co.y already holds 2b
                v[7] = -gq * (2.0f * co.x * dx + co.y * dy);
                v[8] = -gq * (co.y * dx + 2.0f * co.z * dy);
            }
#pragma unroll
            for (int k = 0; k < 9; k++) v[k] = wave_sum_to_lane63(v[k]);
            if (lane == 63) {
#pragma unroll
                for (int k = 0; k < 9; k++) atomicAdd(&s_acc[j][k], v[k]);
                s_touched[j] = 1;
            }
        }
        __syncthreads();
        if ((int)threadIdx.x < m && s_touched[threadIdx.x]) {
            const uint32_t g = s_id[threadIdx.x];
            const float* a = s_acc[threadIdx.x];
            atomicAdd(&d_rgb[3 * g + 0], a[0]);
            atomicAdd(&d_rgb[3 * g + 1], a[1]);
            atomicAdd(&d_rgb[3 * g + 2], a[2]);
            atomicAdd(&d_opac[g], a[3]);
            atomicAdd(&d_conic[3 * g + 0], a[4]);
            atomicAdd(&d_conic[3 * g + 1], a[5]);
            atomicAdd(&d_conic[3 * g + 2], a[6]);
            atomicAdd(&d_mean2d[2 * g + 0], a[7]);
            atomicAdd(&d_mean2d[2 * g + 1], a[8]);
        }
    }
}

// Count pass: re-walks the forward loop for the mask pixels only (other pixels cannot add to a
// count) up to each pixel's n_contrib, and counts per Gaussian the pixels where it is blended
// (and, in weight mode, alpha*T > alpha_min).  A ballot + population count gives the wavefront's
// count without any cross-lane arithmetic.
__global__ __launch_bounds__(256) void k_score(CamDev cam, CfgDev cfg, const uint2* __restrict__ ranges,
                                               const uint32_t* __restrict__ gauss_sorted,
                                               const float2* __restrict__ mean2d,
                                               const float4* __restrict__ conic_opacity,
                                               const uint32_t* __restrict__ n_contrib,
                                               const uint8_t* __restrict__ mask, int32_t* __restrict__ counts)
{
    __shared__ float2 s_xy[BATCH];
    __shared__ float4 s_co[BATCH];
    __shared__ uint32_t s_id[BATCH];
    __shared__ int s_cnt[BATCH];
    __shared__ int s_max;

    const int tile = blockIdx.x;
    const Pixel p = pixel_of_thread(cam, tile);
    const uint2 range = ranges[tile];
    const size_t pix = (size_t)p.y * cam.width + p.x;
    const int lane = threadIdx.x & 63;
    int last = 0;
    if (p.inside && mask[pix]) last = (int)n_contrib[pix];
    if (threadIdx.x == 0) s_max = 0;
    __syncthreads();
    atomicMax(&s_max, last);
    __syncthreads();
    const int total = s_max;
    float T = 1.0f;

    for (int start = 0; start < total; start += BATCH) {
        const int m = min(BATCH, total - start);
        __syncthreads();
        if ((int)threadIdx.x < m) {
            const uint32_t g = gauss_sorted[range.x + start + threadIdx.x];
            float4 co = conic_opacity[g];
            co.y = co.y + co.y;
            s_id[threadIdx.x] = g;
            s_xy[threadIdx.x] = mean2d[g];
            s_co[threadIdx.x] = co;
        }
        s_cnt[threadIdx.x] = 0;
        __syncthreads();
        for (int j = 0; j < m; j++) {
            float alpha = 0.f, dx, dy, G;
            const bool act = (start + j < last) && alpha_at(p, s_xy[j], s_co[j], cfg, alpha, dx, dy, G);
            bool hit = false;
            if (act) {
                const float w = alpha * T;
                hit = cfg.score_mode == FS_SCORE_ALPHA || w > cfg.alpha_min;
                T = T * (1.0f - alpha);
            }
            const uint64_t b = __ballot(hit);
            if (b != 0 && lane == 0) atomicAdd(&s_cnt[j], (int)__popcll(b));
        }
        __syncthreads();
        if ((int)threadIdx.x < m && s_cnt[threadIdx.x] != 0) atomicAdd(&counts[s_id[threadIdx.x]], s_cnt[threadIdx.x]);
    }
}

}  // namespace

hipError_t launch_render_fwd(hipStream_t st, const CamDev& cam, const CfgDev& cfg, const uint32_t* ranges,
                             const uint32_t* gauss_sorted, const float* mean2d, const float* conic_opacity,
                             const float* rgb, float* image, float* final_T, uint32_t* n_contrib)
{
    const int tiles = cam.tiles_x * cam.tiles_y;
    if (tiles == 0) return hipSuccess;
    hipLaunchKernelGGL(k_render_fwd, dim3(tiles), dim3(256), 0, st, cam, cfg, reinterpret_cast<const uint2*>(ranges),
                       gauss_sorted, reinterpret_cast<const float2*>(mean2d),
                       reinterpret_cast<const float4*>(conic_opacity), rgb, image, final_T, n_contrib);
    return hipGetLastError();
}

hipError_t launch_render_bwd(hipStream_t st, const CamDev& cam, const CfgDev& cfg, const uint32_t* ranges,
                             const uint32_t* gauss_sorted, const float* mean2d, const float* conic_opacity,
                             const float* rgb, const float* final_T, const uint32_t* n_contrib,
                             const float* dL_dimage, float* dmean2d, float* dconic, float* dopac, float* drgb)
{
    const int tiles = cam.tiles_x * cam.tiles_y;
    if (tiles == 0) return hipSuccess;
    hipLaunchKernelGGL(k_render_bwd, dim3(tiles), dim3(256), 0, st, cam, cfg, reinterpret_cast<const uint2*>(ranges),
                       gauss_sorted, reinterpret_cast<const float2*>(mean2d),
                       reinterpret_cast<const float4*>(conic_opacity), rgb, final_T, n_contrib, dL_dimage, dmean2d,
                       dconic, dopac, drgb);
    return hipGetLastError();
}

hipError_t launch_score(hipStream_t st, const CamDev& cam, const CfgDev& cfg, const uint32_t* ranges,
                        const uint32_t* gauss_sorted, const float* mean2d, const float* conic_opacity,
                        const uint32_t* n_contrib, const uint8_t* mask, int32_t* counts)
{
    const int tiles = cam.tiles_x * cam.tiles_y;
    if (tiles == 0) return hipSuccess;
    hipLaunchKernelGGL(k_score, dim3(tiles), dim3(256), 0, st, cam, cfg, reinterpret_cast<const uint2*>(ranges),
                       gauss_sorted, reinterpret_cast<const float2*>(mean2d),
                       reinterpret_cast<const float4*>(conic_opacity), n_contrib, mask, counts);
    return hipGetLastError();
}

}  // namespace fs
