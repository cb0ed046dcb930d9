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


// What the three decisions do to the array when applied together: a pruned Gaussian is neither cloned nor
// split; a split parent is replaced by its children; everything else stays.
__global__ __launch_bounds__(256) void k_combine_masks(int64_t n, const uint8_t* __restrict__ clone,
                                                       const uint8_t* __restrict__ split,
                                                       const uint8_t* __restrict__ prune, uint8_t* __restrict__ keep,
                                                       uint8_t* __restrict__ clone_eff, uint8_t* __restrict__ split_eff)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const bool c = clone[i] != 0, s = split[i] != 0, p = prune[i] != 0;
    keep[i] = !p && !s;
    clone_eff[i] = c && !p;
    split_eff[i] = s && !p;
}

__global__ __launch_bounds__(256) void k_counts_add(int64_t n, int32_t* __restrict__ total,
                                                    const int32_t* __restrict__ view)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) total[i] = total[i] + view[i];
}

// Children of the split parents (vanilla 3DGS's split, which the paper keeps): child c of the r-th parent p sits
// at mu_p + R(q_p) (s_p * xi[r, c]) with xi the caller's standard normal draws, and has scales s_p / phi.
// One lane per (parent, child); row c*m + r.
__global__ __launch_bounds__(256) void k_split_children(int64_t m, const float* __restrict__ means,
                                                        const float* __restrict__ scales,
                                                        const float4* __restrict__ quats,
                                                        const uint32_t* __restrict__ parents,
                                                        const float* __restrict__ normals, float phi,
                                                        float* __restrict__ child_means,
                                                        float* __restrict__ child_scales)
{
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= 2 * m) return;
    const int64_t r = e % m;
    const int c = (int)(e / m);
    const size_t p = parents[r];
    const float4 q = quats[p];
    const float w = q.x, x = q.y, y = q.z, z = q.w;
    const float s0 = scales[3 * p], s1 = scales[3 * p + 1], s2 = scales[3 * p + 2];
    const float* xi = normals + (size_t)(2 * r + c) * 3;
    const float l0 = s0 * xi[0], l1 = s1 * xi[1], l2 = s2 * xi[2];
    const float r00 = 1.0f - 2.0f * (y * y + z * z), r01 = 2.0f * (x * y - w * z), r02 = 2.0f * (x * z + w * y);
    const float r10 = 2.0f * (x * y + w * z), r11 = 1.0f - 2.0f * (x * x + z * z), r12 = 2.0f * (y * z - w * x);
    const float r20 = 2.0f * (x * z - w * y), r21 = 2.0f * (y * z + w * x), r22 = 1.0f - 2.0f * (x * x + y * y);
    child_means[3 * e + 0] = means[3 * p + 0] + ((r00 * l0 + r01 * l1) + r02 * l2);
    child_means[3 * e + 1] = means[3 * p + 1] + ((r10 * l0 + r11 * l1) + r12 * l2);
    child_means[3 * e + 2] = means[3 * p + 2] + ((r20 * l0 + r21 * l1) + r22 * l2);
    child_scales[3 * e + 0] = s0 / phi;
    child_scales[3 * e + 1] = s1 / phi;
    child_scales[3 * e + 2] = s2 / phi;
}

// Arrival time of each listed candidate under an exponential clock of rate score: e / score (one correctly
// rounded division), +inf for a score <= 0 (or a NaN); the sort key is bits(time) << 32 | index, so that equal
// times are ordered by index.  Times are >= 0, for which the bit pattern orders like the value.
__global__ __launch_bounds__(256) void k_sample_keys(int64_t m, const uint32_t* __restrict__ cand_idx,
                                                     const float* __restrict__ scores,
                                                     const float* __restrict__ exponentials,
                                                     uint64_t* __restrict__ keys, uint32_t* __restrict__ vals)
{
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= m) return;
    const uint32_t i = cand_idx[j];
    const float w = scores[i];
    float t = w > 0.0f ? exponentials[i] / w : __builtin_inff();
    if (!(t >= 0.0f)) t = __builtin_inff();
    keys[j] = ((uint64_t)__float_as_uint(t) << 32) | i;
    vals[j] = i;
}

__global__ __launch_bounds__(256) void k_mark_indices(int64_t k, const uint32_t* __restrict__ idx,
                                                      uint8_t* __restrict__ mask)
{
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j < k) mask[idx[j]] = 1;
}

__global__ __launch_bounds__(256) void k_fill_u8(int64_t n, uint8_t* __restrict__ p, uint8_t v)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
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

hipError_t launch_combine_masks(hipStream_t st, int64_t n, const uint8_t* clone, const uint8_t* split,
                                const uint8_t* prune, uint8_t* keep, uint8_t* clone_eff, uint8_t* split_eff)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_combine_masks, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, n, clone, split, prune, keep,
                       clone_eff, split_eff);
    return hipGetLastError();
}

hipError_t launch_counts_add(hipStream_t st, int64_t n, int32_t* total, const int32_t* view)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_counts_add, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, n, total, view);
    return hipGetLastError();
}

hipError_t launch_split_children(hipStream_t st, int64_t m, const float* means, const float* scales, const float* quats,
                                 const uint32_t* parents, const float* normals, float phi, float* child_means,
                                 float* child_scales)
{
    if (m <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_split_children, dim3((unsigned)((2 * m + 255) / 256)), dim3(256), 0, st, m, means, scales,
                       reinterpret_cast<const float4*>(quats), parents, normals, phi, child_means, child_scales);
    return hipGetLastError();
}

hipError_t launch_sample_keys(hipStream_t st, int64_t m, const uint32_t* cand_idx, const float* scores,
                              const float* exponentials, uint64_t* keys, uint32_t* vals)
{
    if (m <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_sample_keys, dim3((unsigned)((m + 255) / 256)), dim3(256), 0, st, m, cand_idx, scores,
                       exponentials, keys, vals);
    return hipGetLastError();
}

hipError_t launch_mark_indices(hipStream_t st, int64_t n, int64_t k, const uint32_t* idx, uint8_t* mask)
{
    if (n > 0) hipLaunchKernelGGL(k_fill_u8, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, n, mask, (uint8_t)0);
    if (k > 0) hipLaunchKernelGGL(k_mark_indices, dim3((unsigned)((k + 255) / 256)), dim3(256), 0, st, k, idx, mask);
    return hipGetLastError();
}

}  // namespace fs
