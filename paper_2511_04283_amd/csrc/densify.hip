// Densification / pruning decisions of FastGS (Sec. 4.2 VCD, Sec. 4.3 VCP, supplement "Implementation
// Details") and the index plumbing that turns a decision mask into tensor surgery (gfx950).
//
// All element-wise and HBM-bound: a few bytes per Gaussian per call.  The comparisons are made in fp32
// with correctly rounded divisions, so that a CPU implementation following the same order decides
// identically.
#include "common.hpp"

namespace fs {

namespace {

// Per training iteration: add the norm of this view's positional gradient (and of the absolute one) to
// the running sums of every Gaussian that was visible in the view, and count the view.
__global__ __launch_bounds__(256) void k_densify_accumulate(int64_t n, const float2* __restrict__ dmean2d,
                                                            const float2* __restrict__ dabs,
                                                            const uint32_t* __restrict__ touched,
                                                            float* __restrict__ grad_accum,
                                                            float* __restrict__ abs_accum,
                                                            uint32_t* __restrict__ denom)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n || touched[i] == 0) return;
    const float2 g = dmean2d[i];
    grad_accum[i] = grad_accum[i] + sqrtf(g.x * g.x + g.y * g.y);
    if (dabs) {
        const float2 a = dabs[i];
        abs_accum[i] = abs_accum[i] + sqrtf(a.x * a.x + a.y * a.y);
    }
    denom[i] = denom[i] + 1u;
}

// clone: mean gradient norm >= tau_grad, largest scale <= size_limit, s_d > tau_d
// split: mean absolute-gradient norm >= tau_abs, largest scale > size_limit, s_d > tau_d
// prune: opacity < min_opacity, or s_p > tau_p
__global__ __launch_bounds__(256) void k_select(int64_t n, const float* __restrict__ grad_accum,
                                                const float* __restrict__ abs_accum,
                                                const uint32_t* __restrict__ denom, const int32_t* __restrict__ counts,
                                                const float* __restrict__ scales, const float* __restrict__ opac,
                                                const float* __restrict__ s_p, fs_select_params prm,
                                                uint8_t* __restrict__ clone, uint8_t* __restrict__ split,
                                                uint8_t* __restrict__ prune)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const float d = fmaxf((float)denom[i], 1.0f);
    const float g = grad_accum[i] / d;
    const float ga = abs_accum ? abs_accum[i] / d : 0.0f;
    const float sd = (float)counts[i] / (float)prm.K;
    const bool important = sd > prm.tau_d;
    const float smax = fmaxf(fmaxf(scales[3 * i], scales[3 * i + 1]), scales[3 * i + 2]);
    const bool big = smax > prm.size_limit;
    clone[i] = (g >= prm.tau_grad) && !big && important;
    split[i] = abs_accum && (ga >= prm.tau_abs) && big && important;
    prune[i] = (opac[i] < prm.min_opacity) || (s_p && s_p[i] > prm.tau_p);
}

__global__ __launch_bounds__(256) void k_mask_flags(int64_t n, const uint8_t* __restrict__ mask,
                                                    uint32_t* __restrict__ flags)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) flags[i] = mask[i] ? 1u : 0u;
}

// positions[i] = number of selected elements before i: element i goes to slot positions[i]
__global__ __launch_bounds__(256) void k_compact_scatter(int64_t n, const uint8_t* __restrict__ mask,
                                                         const uint32_t* __restrict__ positions,
                                                         uint32_t* __restrict__ indices)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n && mask[i]) indices[positions[i]] = (uint32_t)i;
}

// dst[r, :] = src[indices[r], :], one lane per float (rows are short: 1..48 floats)
__global__ __launch_bounds__(256) void k_gather_rows(const float* __restrict__ src, int row_floats,
                                                     const uint32_t* __restrict__ indices, int64_t count,
                                                     float* __restrict__ dst)
{
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= count * row_floats) return;
    const int64_t r = e / row_floats;
    const int c = (int)(e - r * row_floats);
    dst[e] = src[(size_t)indices[r] * row_floats + c];
}

}  // namespace

hipError_t launch_densify_accumulate(hipStream_t st, int64_t n, const float* dmean2d, const float* dabs,
                                     const uint32_t* touched, float* grad_accum, float* abs_accum, uint32_t* denom)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_densify_accumulate, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, n,
                       reinterpret_cast<const float2*>(dmean2d), reinterpret_cast<const float2*>(dabs), touched,
                       grad_accum, abs_accum, denom);
    return hipGetLastError();
}

hipError_t launch_select(hipStream_t st, int64_t n, const float* grad_accum, const float* abs_accum,
                         const uint32_t* denom, const int32_t* counts, const float* scales, const float* opac,
                         const float* s_p, const fs_select_params& prm, uint8_t* clone, uint8_t* split, uint8_t* prune)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_select, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, n, grad_accum, abs_accum, denom,
                       counts, scales, opac, s_p, prm, clone, split, prune);
    return hipGetLastError();
}

hipError_t launch_compact(hipStream_t st, int64_t n, const uint8_t* mask, uint32_t* positions, void* scan_tmp,
                          uint64_t* total_dev, uint32_t* indices)
{
    if (n <= 0) return hipSuccess;
    const dim3 grid((unsigned)((n + 255) / 256)), block(256);
    hipLaunchKernelGGL(k_mask_flags, grid, block, 0, st, n, mask, positions);
    hipError_t e = launch_exclusive_scan(st, positions, positions, n, scan_tmp, total_dev);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_compact_scatter, grid, block, 0, st, n, mask, positions, indices);
    return hipGetLastError();
}

hipError_t launch_gather_rows(hipStream_t st, const float* src, int row_floats, const uint32_t* indices,
                              int64_t count, float* dst)
{
    if (count <= 0 || row_floats <= 0) return hipSuccess;
    const int64_t total = count * row_floats;
    hipLaunchKernelGGL(k_gather_rows, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, src, row_floats, indices,
                       count, dst);
    return hipGetLastError();
}

}  // namespace fs
