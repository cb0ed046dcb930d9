// Image-space helpers of the hot path (gfx950): L1 term with its gradient, and the per-pixel
// error map / threshold / high-error mask of FastGS Sec. 4.2 (first three equations).
//
// Reductions over the image run in double precision in a fixed tree (per-thread strided sums,
// wavefront shuffle tree, per-workgroup partials, one final workgroup), so results do not depend
// on scheduling.
#include "common.hpp"

namespace fs {

namespace {

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

// final reduction of RED_BLOCKS partials by one workgroup (thread i takes partials i, i+256, ... in order)
template <RedOp OP>
__device__ __forceinline__ double final_reduce(const double* partial, double* smem)
{
    double v = partial[threadIdx.x];
#pragma unroll
    for (int k = 1; k < RED_BLOCKS / RED_THREADS; k++) v = red_combine<OP>(v, partial[k * RED_THREADS + threadIdx.x]);
    return block_reduce<OP>(v, smem);
}

__global__ __launch_bounds__(RED_THREADS) void k_l1_grad(const float* __restrict__ image,
                                                        const float* __restrict__ target, int64_t count,
                                                        float scale, float* __restrict__ dL,
                                                        double* __restrict__ partial)
{
    __shared__ double smem[4];
    double s = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * RED_THREADS + threadIdx.x; i < count; i += (int64_t)RED_BLOCKS * RED_THREADS) {
        const float d = image[i] - target[i];
        s += (double)fabsf(d);
        dL[i] = d > 0.f ? scale : (d < 0.f ? -scale : 0.f);
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

// e = ((|d0| + |d1|) + |d2|) / 3 per pixel; partial sums / minima / maxima per workgroup.
__global__ __launch_bounds__(RED_THREADS) void k_err_map(const float* __restrict__ image,
                                                        const float* __restrict__ target, int64_t pixels,
                                                        float* __restrict__ err, double* __restrict__ partial)
{
    __shared__ double smem[4];
    double s = 0.0, lo = 1.0e300, hi = -1.0e300;
    for (int64_t i = (int64_t)blockIdx.x * RED_THREADS + threadIdx.x; i < pixels; i += (int64_t)RED_BLOCKS * RED_THREADS) {
        const float d0 = fabsf(image[i] - target[i]);
        const float d1 = fabsf(image[pixels + i] - target[pixels + i]);
        const float d2 = fabsf(image[2 * pixels + i] - target[2 * pixels + i]);
        const float e = ((d0 + d1) + d2) / 3.0f;
        err[i] = e;
        s += (double)e;
        lo = (double)e < lo ? (double)e : lo;
        hi = (double)e > hi ? (double)e : hi;
    }
    s = block_reduce<RED_SUM>(s, smem);
    lo = block_reduce<RED_MIN>(lo, smem);
    hi = block_reduce<RED_MAX>(hi, smem);
    if (threadIdx.x == 0) {
        partial[blockIdx.x] = s;
        partial[RED_BLOCKS + blockIdx.x] = lo;
        partial[2 * RED_BLOCKS + blockIdx.x] = hi;
    }
}

// second pass of the two-pass variance: partial sums of (e - mean)^2
__global__ __launch_bounds__(RED_THREADS) void k_err_var(const float* __restrict__ err, int64_t pixels,
                                                        double* __restrict__ partial)
{
    __shared__ double smem[4];
    __shared__ double mean_s;
    const double tot = final_reduce<RED_SUM>(partial, smem);
    if (threadIdx.x == 0) mean_s = tot / (double)pixels;
    __syncthreads();
    const double mean = mean_s;
    double s = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * RED_THREADS + threadIdx.x; i < pixels; i += (int64_t)RED_BLOCKS * RED_THREADS) {
        const double d = (double)err[i] - mean;
        s += d * d;
    }
    s = block_reduce<RED_SUM>(s, smem);
    if (threadIdx.x == 0) partial[3 * RED_BLOCKS + blockIdx.x] = s;
}

// threshold from the partials (one workgroup), written as one float
__global__ __launch_bounds__(RED_THREADS) void k_err_threshold(const double* __restrict__ partial, int64_t pixels,
                                                              int rule, float k, float* __restrict__ thr)
{
    __shared__ double smem[4];
    if (rule == FS_MASK_MEAN_STD) {
        const double tot = final_reduce<RED_SUM>(partial, smem);
        const double var = final_reduce<RED_SUM>(partial + 3 * RED_BLOCKS, smem);
        if (threadIdx.x == 0) {
            const double mean = tot / (double)pixels;
            *thr = (float)(mean + (double)k * sqrt(var / (double)pixels));
        }
    } else {
        const double lo = final_reduce<RED_MIN>(partial + RED_BLOCKS, smem);
        const double hi = final_reduce<RED_MAX>(partial + 2 * RED_BLOCKS, smem);
        if (threadIdx.x == 0) {
            const float l = (float)lo, h = (float)hi;
            *thr = l + k * (h - l);
        }
    }
}

__global__ __launch_bounds__(256) void k_err_mask(const float* __restrict__ err, int64_t pixels,
                                                  const float* __restrict__ thr, uint8_t* __restrict__ mask)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < pixels) mask[i] = err[i] > *thr;
}

}  // namespace

int l1_partials() { return RED_BLOCKS; }
int mask_partials() { return RED_BLOCKS; }

hipError_t launch_l1_grad(hipStream_t st, const float* image, const float* target, int64_t count, float* dL,
                          double* partial, double* loss_out)
{
    if (count <= 0) return hipSuccess;
    const float scale = 1.0f / (float)count;
    hipLaunchKernelGGL(k_l1_grad, dim3(RED_BLOCKS), dim3(RED_THREADS), 0, st, image, target, count, scale, dL, partial);
    if (loss_out) hipLaunchKernelGGL(k_l1_final, dim3(1), dim3(RED_THREADS), 0, st, partial, count, loss_out);
    return hipGetLastError();
}

hipError_t launch_error_mask(hipStream_t st, const float* image, const float* target, int64_t pixels, int rule,
                             float k, float* err, double* partial, uint8_t* mask, float* thr)
{
    if (pixels <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_err_map, dim3(RED_BLOCKS), dim3(RED_THREADS), 0, st, image, target, pixels, err, partial);
    if (rule == FS_MASK_MEAN_STD)
        hipLaunchKernelGGL(k_err_var, dim3(RED_BLOCKS), dim3(RED_THREADS), 0, st, err, pixels, partial);
    hipLaunchKernelGGL(k_err_threshold, dim3(1), dim3(RED_THREADS), 0, st, partial, pixels, rule, k, thr);
    hipLaunchKernelGGL(k_err_mask, dim3((unsigned)((pixels + 255) / 256)), dim3(256), 0, st, err, pixels, thr, mask);
    return hipGetLastError();
}

}  // namespace fs
