// Image-space helpers of the hot path (gfx950): L1 term with its gradient, the per-pixel
// error map / threshold / high-error mask of FastGS Sec. 4.2 (first three equations), the
// photometric loss E = (1 - lambda) L1 + lambda (1 - SSIM) of Sec. 4.3 / Sec. 4.5 with its
// gradient, and the pruning score of Sec. 4.3.
//
// Reductions over the image run in double precision in a fixed tree (per-thread strided sums,
// wavefront shuffle tree, per-workgroup partials, one final workgroup), so results do not depend
// on scheduling.
#include "common.hpp"

namespace fs {

namespace {

// final reduction of RED_BLOCKS partials by one workgroup (thread i takes partials i, i+256, ... in order)
template <RedOp OP>
__device__ __forceinline__ double final_reduce(const double* partial, double* smem)
{
    double v = partial[threadIdx.x];
#pragma unroll
    for (int k = 1; k < RED_BLOCKS / RED_THREADS; k++) v = red_combine<OP>(v, partial[k * RED_THREADS + threadIdx.x]);
    return block_reduce<OP>(v, smem);
}

// VEC = 4: 16-byte accesses (count a multiple of 4, arrays 16-byte aligned); VEC = 1 otherwise.  The sum is
// accumulated per thread in element order either way.
template <int VEC>
__global__ __launch_bounds__(RED_THREADS) void k_l1_grad(const float* __restrict__ image,
                                                        const float* __restrict__ target, int64_t count,
                                                        float scale, float* __restrict__ dL,
                                                        double* __restrict__ partial)
{
    __shared__ double smem[4];
    double s = 0.0;
    const int64_t stride = (int64_t)RED_BLOCKS * RED_THREADS;
    if (VEC == 4) {
        const float4* a4 = reinterpret_cast<const float4*>(image);
        const float4* b4 = reinterpret_cast<const float4*>(target);
        float4* d4 = reinterpret_cast<float4*>(dL);
        for (int64_t i = (int64_t)blockIdx.x * RED_THREADS + threadIdx.x; i < (count >> 2); i += stride) {
            const float4 a = a4[i], b = b4[i];
            const float d0 = a.x - b.x, d1 = a.y - b.y, d2 = a.z - b.z, d3 = a.w - b.w;
            s += (double)fabsf(d0); s += (double)fabsf(d1); s += (double)fabsf(d2); s += (double)fabsf(d3);
            d4[i] = make_float4(d0 > 0.f ? scale : (d0 < 0.f ? -scale : 0.f), d1 > 0.f ? scale : (d1 < 0.f ? -scale : 0.f),
                                d2 > 0.f ? scale : (d2 < 0.f ? -scale : 0.f), d3 > 0.f ? scale : (d3 < 0.f ? -scale : 0.f));
        }
    } else {
        for (int64_t i = (int64_t)blockIdx.x * RED_THREADS + threadIdx.x; i < count; i += stride) {
            const float d = image[i] - target[i];
            s += (double)fabsf(d);
            dL[i] = d > 0.f ? scale : (d < 0.f ? -scale : 0.f);
        }
    }
    s = block_reduce<RED_SUM>(s, smem);
    if (threadIdx.x == 0) partial[blockIdx.x] = s;
}

__global__ __launch_bounds__(RED_THREADS) void k_l1_final(const double* __restrict__ partial, int64_t count,
                                                         double* __restrict__ loss_out)
{
    __shared__ double smem[4];
    const double s = final_reduce<RED_SUM>(partial, smem);
    if (threadIdx.x == 0) *loss_out = s / (double)count;
}

// e = ((|d0| + |d1|) + |d2|) / 3 per pixel; partial sums / minima / maxima / sums of squares per workgroup.
// VEC = 4: four neighbouring pixels per thread with 16-byte accesses (pixels a multiple of 4, arrays aligned).
template <int VEC>
__global__ __launch_bounds__(RED_THREADS) void k_err_map(const float* __restrict__ image,
                                                        const float* __restrict__ target, int64_t pixels,
                                                        float* __restrict__ err, double* __restrict__ partial)
{
    __shared__ double smem[4];
    double s = 0.0, sq = 0.0, lo = 1.0e300, hi = -1.0e300;
    const int64_t stride = (int64_t)RED_BLOCKS * RED_THREADS;
    auto one = [&](float i0, float i1, float i2, float t0, float t1, float t2) {
        const float e = ((fabsf(i0 - t0) + fabsf(i1 - t1)) + fabsf(i2 - t2)) / 3.0f;
        s += (double)e;
        sq += (double)e * (double)e;
        lo = (double)e < lo ? (double)e : lo;
        hi = (double)e > hi ? (double)e : hi;
        return e;
    };
    if (VEC == 4) {
        const int64_t q = pixels >> 2;
        const float4* a4 = reinterpret_cast<const float4*>(image);
        const float4* b4 = reinterpret_cast<const float4*>(target);
        float4* e4 = reinterpret_cast<float4*>(err);
        for (int64_t i = (int64_t)blockIdx.x * RED_THREADS + threadIdx.x; i < q; i += stride) {
            const float4 a0 = a4[i], a1 = a4[q + i], a2 = a4[2 * q + i];
            const float4 b0 = b4[i], b1 = b4[q + i], b2 = b4[2 * q + i];
            float4 e;
            e.x = one(a0.x, a1.x, a2.x, b0.x, b1.x, b2.x);
            e.y = one(a0.y, a1.y, a2.y, b0.y, b1.y, b2.y);
            e.z = one(a0.z, a1.z, a2.z, b0.z, b1.z, b2.z);
            e.w = one(a0.w, a1.w, a2.w, b0.w, b1.w, b2.w);
            e4[i] = e;
        }
    } else {
        for (int64_t i = (int64_t)blockIdx.x * RED_THREADS + threadIdx.x; i < pixels; i += stride)
            err[i] = one(image[i], image[pixels + i], image[2 * pixels + i], target[i], target[pixels + i],
                         target[2 * pixels + i]);
    }
    s = block_reduce<RED_SUM>(s, smem);
    lo = block_reduce<RED_MIN>(lo, smem);
    hi = block_reduce<RED_MAX>(hi, smem);
    sq = block_reduce<RED_SUM>(sq, smem);
    if (threadIdx.x == 0) {
        partial[blockIdx.x] = s;
        partial[RED_BLOCKS + blockIdx.x] = lo;
        partial[2 * RED_BLOCKS + blockIdx.x] = hi;
        partial[3 * RED_BLOCKS + blockIdx.x] = sq;
    }
}

// After the fused forward kernel: one workgroup adds up its per-tile partials ([5][tiles]: sum |d|; sum, min,
// max, sum of squares of e) in a fixed order (thread b takes tiles b, b + 1024, ...; then a shuffle tree) and leaves
// stats[0..3] = {sum e, min e, max e, sum e^2} and the L1 loss.
constexpr int FOLD_THREADS = 1024;
__global__ __launch_bounds__(FOLD_THREADS) void k_fold_tile_stats(const double* __restrict__ tile_partial, int tiles,
                                                                  int64_t count, double* __restrict__ stats,
                                                                  double* __restrict__ loss_out)
{
    __shared__ double sm[5][FOLD_THREADS / 64];
    double l1 = 0.0, s = 0.0, sq = 0.0, lo = 1.0e300, hi = -1.0e300;
    for (int t0 = threadIdx.x; t0 < tiles; t0 += 4 * FOLD_THREADS) {   // 20 loads in flight per round
        double v[4][5];
#pragma unroll
        for (int u = 0; u < 4; u++) {
            const int t = t0 + u * FOLD_THREADS;
            const bool in = t < tiles;
            v[u][0] = in ? tile_partial[t] : 0.0;
            v[u][1] = in ? tile_partial[(size_t)tiles + t] : 0.0;
            v[u][2] = in ? tile_partial[2 * (size_t)tiles + t] : 1.0e300;
            v[u][3] = in ? tile_partial[3 * (size_t)tiles + t] : -1.0e300;
            v[u][4] = in ? tile_partial[4 * (size_t)tiles + t] : 0.0;
        }
#pragma unroll
        for (int u = 0; u < 4; u++) {
            l1 += v[u][0];
            s += v[u][1];
            lo = v[u][2] < lo ? v[u][2] : lo;
            hi = v[u][3] > hi ? v[u][3] : hi;
            sq += v[u][4];
        }
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        l1 += shfl_down_f64(l1, d);
        s += shfl_down_f64(s, d);
        sq += shfl_down_f64(sq, d);
        const double a = shfl_down_f64(lo, d), b = shfl_down_f64(hi, d);
        lo = a < lo ? a : lo;
        hi = b > hi ? b : hi;
    }
    if ((threadIdx.x & 63) == 0) {
        const int w = threadIdx.x >> 6;
        sm[0][w] = l1; sm[1][w] = s; sm[2][w] = lo; sm[3][w] = hi; sm[4][w] = sq;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        l1 = 0.0; s = 0.0; sq = 0.0; lo = 1.0e300; hi = -1.0e300;
        for (int w = 0; w < FOLD_THREADS / 64; w++) {
            l1 += sm[0][w];
            s += sm[1][w];
            lo = sm[2][w] < lo ? sm[2][w] : lo;
            hi = sm[3][w] > hi ? sm[3][w] : hi;
            sq += sm[4][w];
        }
        stats[0] = s; stats[1] = lo; stats[2] = hi; stats[3] = sq;
        if (loss_out) *loss_out = l1 / (double)count;
    }
}

// threshold from the RED_BLOCKS-wide partials of k_err_map (one workgroup), written as one float
__global__ __launch_bounds__(RED_THREADS) void k_err_threshold(const double* __restrict__ partial, int64_t pixels,
                                                              int rule, float k, float* __restrict__ thr)
{
    __shared__ double smem[4];
    const double tot = final_reduce<RED_SUM>(partial, smem);
    const double lo = final_reduce<RED_MIN>(partial + RED_BLOCKS, smem);
    const double hi = final_reduce<RED_MAX>(partial + 2 * RED_BLOCKS, smem);
    const double sq = final_reduce<RED_SUM>(partial + 3 * RED_BLOCKS, smem);
    if (threadIdx.x == 0) *thr = threshold_from_stats(tot, lo, hi, sq, pixels, rule, k);
}

__global__ __launch_bounds__(256) void k_err_mask(const float* __restrict__ err, int64_t pixels,
                                                  const float* __restrict__ thr, uint8_t* __restrict__ mask)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < pixels) mask[i] = err[i] > *thr;
}

// the mask straight from the four statistics that k_fold_tile_stats left (every thread forms the threshold itself;
// the first one also stores it)
__global__ __launch_bounds__(256) void k_err_mask_stats(const float* __restrict__ err, int64_t pixels,
                                                        const double* __restrict__ stats, int rule, float k,
                                                        uint8_t* __restrict__ mask, float* __restrict__ thr_out)
{
    const float thr = threshold_from_stats(stats[0], stats[1], stats[2], stats[3], pixels, rule, k);
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0) *thr_out = thr;
    if (i < pixels) mask[i] = err[i] > thr;
}

// ---- photometric loss: (1 - lambda) L1 + lambda (1 - SSIM) ---------------------------------------
// SSIM per channel under an 11x11 Gaussian window (sigma 1.5, sum 1, separable), image continued by
// zeros, C1 = 0.01^2, C2 = 0.03^2; its mean over channels and pixels.  With the window sums
// mu1 = <x>, mu2 = <y>, e11 = <x^2>, e22 = <y^2>, e12 = <x y>:
//   ssim = (2 mu1 mu2 + C1)(2 (e12 - mu1 mu2) + C2) / ((mu1^2 + mu2^2 + C1)(e11 - mu1^2 + e22 - mu2^2 + C2)).
// Gradient with respect to x: the three maps d ssim/d mu1, d ssim/d e11, d ssim/d e12 are window-summed
// again (the window is symmetric) and combined as  g = <d_mu1> + 2 x <d_e11> + y <d_e12>.
//
// One workgroup produces a 32x32 block of one channel: the (32+10)x(32+10) input region goes to LDS,
// a horizontal 11-tap pass (one lane: 4 neighbouring columns of one row, sliding over 14 inputs) leaves
// NQ row-filtered planes in LDS, and a vertical pass (one lane: 4 neighbouring rows of one column) finishes.
constexpr int SS_R = 5, SS_TAPS = 2 * SS_R + 1;
constexpr int SS_TW = 32, SS_TH = 32;   // (32x16: 9 % slower, 64x16: the same, 64x32: 5 % slower, 16x32: 27 % slower)
constexpr int SS_VO = SS_TW * SS_TH / 256;                         // outputs (neighbouring rows of one column) per lane
constexpr int SS_IW = SS_TW + 2 * SS_R, SS_IH = SS_TH + 2 * SS_R;   // 42 x 42
constexpr int SS_IP = SS_IW + 2;                                     // padded LDS row

struct SsimWin { float w[SS_TAPS]; };

// zero-continued load of the block's input region of NP planes: every global load is issued before the
// first LDS write, so that their latencies overlap
template <int NP>
__device__ __forceinline__ void ss_load(const float* const (&base)[NP], int H, int W, int x0, int y0,
                                        float (*dst)[SS_IH][SS_IP])
{
    constexpr int IT = (SS_IH * SS_IW + 255) / 256;
    float v[NP][IT];
#pragma unroll
    for (int it = 0; it < IT; it++) {
        const int e = threadIdx.x + 256 * it;
        const int r = e / SS_IW, c = e - r * SS_IW;
        const int gy = y0 + r - SS_R, gx = x0 + c - SS_R;
        const bool in = e < SS_IH * SS_IW && gy >= 0 && gy < H && gx >= 0 && gx < W;
        const size_t off = in ? (size_t)gy * W + gx : 0;
#pragma unroll
        for (int p = 0; p < NP; p++) {
            const float t = base[p][off];   // (off = 0 is always a valid address)
            v[p][it] = in ? t : 0.0f;
        }
    }
#pragma unroll
    for (int it = 0; it < IT; it++) {
        const int e = threadIdx.x + 256 * it;
        const int r = e / SS_IW, c = e - r * SS_IW;
        if (e < SS_IH * SS_IW) {
#pragma unroll
            for (int p = 0; p < NP; p++) dst[p][r][c] = v[p][it];
        }
    }
}

// vertical pass for the SS_VO outputs of this lane: rows r0 .. r0+SS_VO-1 of column c of one row-filtered plane
__device__ __forceinline__ void ss_vertical(const float (*h)[SS_TW], int r0, int c, const SsimWin& win,
                                            float out[SS_VO])
{
    float col[SS_TAPS + SS_VO - 1];
#pragma unroll
    for (int i = 0; i < SS_TAPS + SS_VO - 1; i++) col[i] = h[r0 + i][c];
#pragma unroll
    for (int o = 0; o < SS_VO; o++) {
        float a = 0.f;
#pragma unroll
        for (int k = 0; k < SS_TAPS; k++) a = __builtin_fmaf(win.w[k], col[k + o], a);
        out[o] = a;
    }
}

__global__ __launch_bounds__(256) void k_ssim_fwd(const float* __restrict__ image, const float* __restrict__ target,
                                                  int H, int W, SsimWin win, float* __restrict__ dmaps,
                                                  double* __restrict__ partial, int nblocks)
{
    __shared__ __attribute__((aligned(16))) float s_in[2][SS_IH][SS_IP];
    __shared__ __attribute__((aligned(16))) float s_h[4][SS_IH][SS_TW];
    __shared__ double smem[4];
    const int x0 = blockIdx.x * SS_TW, y0 = blockIdx.y * SS_TH;
    const size_t plane = (size_t)blockIdx.z * H * W;
    const float* const src[2] = {image + plane, target + plane};
    ss_load<2>(src, H, W, x0, y0, s_in);
    __syncthreads();
    for (int u = threadIdx.x; u < SS_IH * (SS_TW / 4); u += 256) {
        const int r = u / (SS_TW / 4), c0 = (u % (SS_TW / 4)) * 4;
        // 16-byte LDS accesses: a lane's 16 inputs are four aligned float4s, and 8 neighbouring lanes cover
        // all banks (a 4-byte access pattern with stride 4 would hit every fourth bank only)
        // (only the sum e11 + e22 enters the index, so x^2 + y^2 is filtered as one plane)
        float xv[16], yv[16], sq[SS_TAPS + 3], xy[SS_TAPS + 3];
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const float4 a = *reinterpret_cast<const float4*>(&s_in[0][r][c0 + 4 * i]);
            const float4 b = *reinterpret_cast<const float4*>(&s_in[1][r][c0 + 4 * i]);
            xv[4 * i] = a.x; xv[4 * i + 1] = a.y; xv[4 * i + 2] = a.z; xv[4 * i + 3] = a.w;
            yv[4 * i] = b.x; yv[4 * i + 1] = b.y; yv[4 * i + 2] = b.z; yv[4 * i + 3] = b.w;
        }
#pragma unroll
        for (int i = 0; i < SS_TAPS + 3; i++) {
            sq[i] = __builtin_fmaf(xv[i], xv[i], yv[i] * yv[i]);
            xy[i] = xv[i] * yv[i];
        }
        float o[4][4];
#pragma unroll
        for (int j = 0; j < 4; j++) {
            float m1 = 0.f, m2 = 0.f, esq = 0.f, e12 = 0.f;
#pragma unroll
            for (int k = 0; k < SS_TAPS; k++) {
                const float wk = win.w[k];
                m1 = __builtin_fmaf(wk, xv[j + k], m1);
                m2 = __builtin_fmaf(wk, yv[j + k], m2);
                esq = __builtin_fmaf(wk, sq[j + k], esq);
                e12 = __builtin_fmaf(wk, xy[j + k], e12);
            }
            o[0][j] = m1; o[1][j] = m2; o[2][j] = esq; o[3][j] = e12;
        }
#pragma unroll
        for (int k = 0; k < 4; k++)
            *reinterpret_cast<float4*>(&s_h[k][r][c0]) = make_float4(o[k][0], o[k][1], o[k][2], o[k][3]);
    }
    __syncthreads();
    const int c = threadIdx.x % SS_TW, r0 = (threadIdx.x / SS_TW) * SS_VO;
    float q[4][SS_VO];
#pragma unroll
    for (int k = 0; k < 4; k++) ss_vertical(s_h[k], r0, c, win, q[k]);
    const float C1 = 0.01f * 0.01f, C2 = 0.03f * 0.03f;
    double ssum = 0.0, lsum = 0.0;
#pragma unroll
    for (int o = 0; o < SS_VO; o++) {
        const int gy = y0 + r0 + o, gx = x0 + c;
        if (gy < H && gx < W) {
            const float m1 = q[0][o], m2 = q[1][o];
            const float mm = m1 * m1 + m2 * m2, s12 = q[3][o] - m1 * m2;
            const float A = 2.f * m1 * m2 + C1, B = 2.f * s12 + C2, Cq = mm + C1, D = (q[2][o] - mm) + C2;
            const float inv = 1.0f / (Cq * D);
            const float sv = A * B * inv;
            ssum += (double)sv;
            lsum += (double)fabsf(s_in[0][r0 + o + SS_R][c + SS_R] - s_in[1][r0 + o + SS_R][c + SS_R]);
            if (dmaps) {
                const size_t n3 = (size_t)3 * H * W, p = plane + (size_t)gy * W + gx;
                dmaps[p] = (2.f * m2 * (B - A) - sv * 2.f * m1 * (D - Cq)) * inv;
                dmaps[n3 + p] = -sv / D;
                dmaps[2 * n3 + p] = 2.f * A * inv;
            }
        }
    }
    ssum = block_reduce<RED_SUM>(ssum, smem);
    lsum = block_reduce<RED_SUM>(lsum, smem);
    if (threadIdx.x == 0) {
        const int b = (blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x;
        partial[b] = ssum;
        partial[nblocks + b] = lsum;
    }
}

// out3 = {L1, SSIM, (1 - lambda) L1 + lambda (1 - SSIM)}: one workgroup adds the partials in a fixed order
__global__ __launch_bounds__(RED_THREADS) void k_photo_final(const double* __restrict__ partial, int nblocks,
                                                            double count, double lambda, double* __restrict__ out3)
{
    __shared__ double smem[4];
    // 2 x 8 loads in flight per lane and round; the order of the additions is fixed
    double s = 0.0, l = 0.0;
    for (int i0 = threadIdx.x; i0 < nblocks; i0 += 8 * RED_THREADS) {
        double a[8], b[8];
#pragma unroll
        for (int k = 0; k < 8; k++) {
            const int i = i0 + k * RED_THREADS;
            a[k] = i < nblocks ? partial[i] : 0.0;
            b[k] = i < nblocks ? partial[nblocks + i] : 0.0;
        }
#pragma unroll
        for (int k = 0; k < 8; k++) { s += a[k]; l += b[k]; }
    }
    s = block_reduce<RED_SUM>(s, smem);
    l = block_reduce<RED_SUM>(l, smem);
    if (threadIdx.x == 0) {
        const double ssim = s / count, l1 = l / count;
        out3[0] = l1;
        out3[1] = ssim;
        out3[2] = (1.0 - lambda) * l1 + lambda * (1.0 - ssim);
    }
}

// dE/dx = c_l1 sign(x - y) - c_ss (<d_mu1> + 2 x <d_e11> + y <d_e12>),  c_l1 = (1-lambda)/N, c_ss = lambda/N
__global__ __launch_bounds__(256) void k_ssim_bwd(const float* __restrict__ image, const float* __restrict__ target,
                                                  int H, int W, SsimWin win, const float* __restrict__ dmaps,
                                                  float c_l1, float c_ss, float* __restrict__ dL)
{
    __shared__ __attribute__((aligned(16))) float s_in[3][SS_IH][SS_IP];
    __shared__ __attribute__((aligned(16))) float s_h[3][SS_IH][SS_TW];
    const int x0 = blockIdx.x * SS_TW, y0 = blockIdx.y * SS_TH;
    const size_t plane = (size_t)blockIdx.z * H * W, n3 = (size_t)3 * H * W;
    const float* const src[3] = {dmaps + plane, dmaps + n3 + plane, dmaps + 2 * n3 + plane};
    ss_load<3>(src, H, W, x0, y0, s_in);
    __syncthreads();
    for (int u = threadIdx.x; u < SS_IH * (SS_TW / 4); u += 256) {
        const int r = u / (SS_TW / 4), c0 = (u % (SS_TW / 4)) * 4;
#pragma unroll
        for (int k = 0; k < 3; k++) {
            float v[16], o[4];
#pragma unroll
            for (int i = 0; i < 4; i++) {
                const float4 a = *reinterpret_cast<const float4*>(&s_in[k][r][c0 + 4 * i]);
                v[4 * i] = a.x; v[4 * i + 1] = a.y; v[4 * i + 2] = a.z; v[4 * i + 3] = a.w;
            }
#pragma unroll
            for (int j = 0; j < 4; j++) {
                float a = 0.f;
#pragma unroll
                for (int t = 0; t < SS_TAPS; t++) a = __builtin_fmaf(win.w[t], v[j + t], a);
                o[j] = a;
            }
            *reinterpret_cast<float4*>(&s_h[k][r][c0]) = make_float4(o[0], o[1], o[2], o[3]);
        }
    }
    __syncthreads();
    const int c = threadIdx.x % SS_TW, r0 = (threadIdx.x / SS_TW) * SS_VO;
    float q[3][SS_VO];
#pragma unroll
    for (int k = 0; k < 3; k++) ss_vertical(s_h[k], r0, c, win, q[k]);
#pragma unroll
    for (int o = 0; o < SS_VO; o++) {
        const int gy = y0 + r0 + o, gx = x0 + c;
        if (gy < H && gx < W) {
            const size_t p = plane + (size_t)gy * W + gx;
            const float x = image[p], y = target[p];
            const float g = q[0][o] + 2.f * x * q[1][o] + y * q[2][o];
            const float d = x - y;
            const float sg = d > 0.f ? c_l1 : (d < 0.f ? -c_l1 : 0.f);
            dL[p] = sg - c_ss * g;
        }
    }
}

// ---- pruning score (Sec. 4.3): s_p = N(sum_j count_i^j E^j) -------------------------------------
__global__ __launch_bounds__(256) void k_prune_accumulate(const int32_t* __restrict__ counts, int64_t n,
                                                          const double* __restrict__ E, double* __restrict__ acc)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) acc[i] = acc[i] + (double)counts[i] * *E;
}

__global__ __launch_bounds__(RED_THREADS) void k_minmax_f64(const double* __restrict__ v, int64_t n,
                                                           double* __restrict__ partial)
{
    __shared__ double smem[4];
    double lo = 1.0e300, hi = -1.0e300;
    for (int64_t i = (int64_t)blockIdx.x * RED_THREADS + threadIdx.x; i < n; i += (int64_t)RED_BLOCKS * RED_THREADS) {
        lo = v[i] < lo ? v[i] : lo;
        hi = v[i] > hi ? v[i] : hi;
    }
    lo = block_reduce<RED_MIN>(lo, smem);
    hi = block_reduce<RED_MAX>(hi, smem);
    if (threadIdx.x == 0) { partial[blockIdx.x] = lo; partial[RED_BLOCKS + blockIdx.x] = hi; }
}

__global__ __launch_bounds__(RED_THREADS) void k_minmax_final(double* __restrict__ partial)
{
    __shared__ double smem[4];
    const double lo = final_reduce<RED_MIN>(partial, smem);
    const double hi = final_reduce<RED_MAX>(partial + RED_BLOCKS, smem);
    if (threadIdx.x == 0) { partial[2 * RED_BLOCKS] = lo; partial[2 * RED_BLOCKS + 1] = hi; }
}

__global__ __launch_bounds__(256) void k_prune_normalize(const double* __restrict__ acc, int64_t n,
                                                         const double* __restrict__ lohi, float* __restrict__ out)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const double lo = lohi[0], hi = lohi[1];
    out[i] = hi > lo ? (float)((acc[i] - lo) / (hi - lo)) : 0.0f;
}

}  // namespace

int l1_partials() { return RED_BLOCKS; }
int mask_partials() { return RED_BLOCKS; }
int fused_partials() { return 4; }

hipError_t launch_l1_grad(hipStream_t st, const float* image, const float* target, int64_t count, float* dL,
                          double* partial, double* loss_out)
{
    if (count <= 0) return hipSuccess;
    const float scale = 1.0f / (float)count;
    const bool vec = count % 4 == 0 && ((reinterpret_cast<uintptr_t>(image) | reinterpret_cast<uintptr_t>(target) |
                                         reinterpret_cast<uintptr_t>(dL)) & 15u) == 0;
    if (vec)
        hipLaunchKernelGGL(k_l1_grad<4>, dim3(RED_BLOCKS), dim3(RED_THREADS), 0, st, image, target, count, scale, dL, partial);
    else
        hipLaunchKernelGGL(k_l1_grad<1>, dim3(RED_BLOCKS), dim3(RED_THREADS), 0, st, image, target, count, scale, dL, partial);
    if (loss_out) hipLaunchKernelGGL(k_l1_final, dim3(1), dim3(RED_THREADS), 0, st, partial, count, loss_out);
    return hipGetLastError();
}

hipError_t launch_error_mask(hipStream_t st, const float* image, const float* target, int64_t pixels, int rule,
                             float k, float* err, double* partial, uint8_t* mask, float* thr)
{
    if (pixels <= 0) return hipSuccess;
    const bool vec = pixels % 4 == 0 && ((reinterpret_cast<uintptr_t>(image) | reinterpret_cast<uintptr_t>(target) |
                                          reinterpret_cast<uintptr_t>(err)) & 15u) == 0;
    if (vec)
        hipLaunchKernelGGL(k_err_map<4>, dim3(RED_BLOCKS), dim3(RED_THREADS), 0, st, image, target, pixels, err, partial);
    else
        hipLaunchKernelGGL(k_err_map<1>, dim3(RED_BLOCKS), dim3(RED_THREADS), 0, st, image, target, pixels, err, partial);
    hipLaunchKernelGGL(k_err_threshold, dim3(1), dim3(RED_THREADS), 0, st, partial, pixels, rule, k, thr);
    hipLaunchKernelGGL(k_err_mask, dim3((unsigned)((pixels + 255) / 256)), dim3(256), 0, st, err, pixels, thr, mask);
    return hipGetLastError();
}

int photo_blocks(int H, int W) { return ((W + SS_TW - 1) / SS_TW) * ((H + SS_TH - 1) / SS_TH) * 3; }

hipError_t launch_photo_loss(hipStream_t st, const float* image, const float* target, int H, int W, float lambda,
                             float* dmaps, double* partial, float* dL, double* out3)
{
    SsimWin win;
    double w[SS_TAPS], sum = 0.0;
    for (int k = 0; k < SS_TAPS; k++) { w[k] = exp(-(double)((k - SS_R) * (k - SS_R)) / (2.0 * 1.5 * 1.5)); sum += w[k]; }
    for (int k = 0; k < SS_TAPS; k++) win.w[k] = (float)(w[k] / sum);
    const dim3 grid((unsigned)((W + SS_TW - 1) / SS_TW), (unsigned)((H + SS_TH - 1) / SS_TH), 3);
    const int nb = photo_blocks(H, W);
    const double count = 3.0 * (double)H * (double)W;
    hipLaunchKernelGGL(k_ssim_fwd, grid, dim3(256), 0, st, image, target, H, W, win, dL ? dmaps : nullptr, partial, nb);
    if (out3) hipLaunchKernelGGL(k_photo_final, dim3(1), dim3(RED_THREADS), 0, st, partial, nb, count, (double)lambda, out3);
    if (dL)
        hipLaunchKernelGGL(k_ssim_bwd, grid, dim3(256), 0, st, image, target, H, W, win, dmaps,
                           (float)((1.0 - (double)lambda) / count), (float)((double)lambda / count), dL);
    return hipGetLastError();
}

hipError_t launch_prune_accumulate(hipStream_t st, const int32_t* counts, int64_t n, const double* E, double* acc)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_prune_accumulate, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, counts, n, E, acc);
    return hipGetLastError();
}

hipError_t launch_prune_normalize(hipStream_t st, const double* acc, int64_t n, double* partial, float* out)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_minmax_f64, dim3(RED_BLOCKS), dim3(RED_THREADS), 0, st, acc, n, partial);
    hipLaunchKernelGGL(k_minmax_final, dim3(1), dim3(RED_THREADS), 0, st, partial);
    hipLaunchKernelGGL(k_prune_normalize, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, acc, n,
                       partial + 2 * RED_BLOCKS, out);
    return hipGetLastError();
}

// After the fused forward kernel: its per-tile partials -> stats[0..3] and, optionally, the L1 loss.
hipError_t launch_fold_tile_partials(hipStream_t st, const double* tile_partial, int tiles, int64_t count,
                                     double* stats, double* loss_out)
{
    hipLaunchKernelGGL(k_fold_tile_stats, dim3(1), dim3(FOLD_THREADS), 0, st, tile_partial, tiles, count, stats, loss_out);
    return hipGetLastError();
}

// fs_error_mask without its first pass: the error map and its statistics are already in place
hipError_t launch_error_mask_from_map(hipStream_t st, int64_t pixels, int rule, float k, const float* err,
                                      const double* stats, uint8_t* mask, float* thr)
{
    if (pixels <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_err_mask_stats, dim3((unsigned)((pixels + 255) / 256)), dim3(256), 0, st, err, pixels, stats, rule, k,
                       mask, thr);
    return hipGetLastError();
}

}  // namespace fs
