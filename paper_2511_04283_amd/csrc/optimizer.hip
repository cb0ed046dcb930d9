// Optimiser side of the training iteration (gfx950): fused Adam update (FastGS Sec. 5.1 trains with Adam;
// supplement "Implementation Details": updates every 32 / 64 iterations late in training, the gradients
// of the iterations in between being summed), and the stored -> used parameter activations of vanilla 3DGS
// with their chain rule.  All HBM-bound streaming kernels.
#include "common.hpp"

namespace fs {

namespace {

struct AdamArgs {
    float lr, beta1, beta2, omb1, omb2, eps, grad_scale;
    float inv_bc1, inv_bc2;   // 1 / (1 - beta1^t), 1 / (1 - beta2^t), computed on the host in double
};

__device__ __forceinline__ void adam_one(float& p, float g, float& m, float& v, const AdamArgs& a)
{
    g = g * a.grad_scale;
    m = a.beta1 * m + a.omb1 * g;
    v = a.beta2 * v + a.omb2 * (g * g);
    const float mhat = m * a.inv_bc1;
    const float vhat = v * a.inv_bc2;
    p = p - a.lr * mhat / (sqrtf(vhat) + a.eps);
}

// 28 bytes of traffic per parameter (p, g, m, v read; p, m, v written); 16-byte accesses on the aligned body.
// When zero_grad is set the gradient is cleared in the same pass (+4 bytes), which saves the separate fill
// that an accumulate-then-step schedule needs.
__global__ __launch_bounds__(256) void k_adam(float* __restrict__ p, float* __restrict__ g, float* __restrict__ m,
                                              float* __restrict__ v, int64_t count, AdamArgs a, int zero_grad)
{
    const int64_t nvec = count >> 2;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    float4* p4 = reinterpret_cast<float4*>(p);
    float4* g4 = reinterpret_cast<float4*>(g);
    float4* m4 = reinterpret_cast<float4*>(m);
    float4* v4 = reinterpret_cast<float4*>(v);
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nvec; i += stride) {
        float4 pp = p4[i], mm = m4[i], vv = v4[i];
        const float4 gg = g4[i];
        adam_one(pp.x, gg.x, mm.x, vv.x, a);
        adam_one(pp.y, gg.y, mm.y, vv.y, a);
        adam_one(pp.z, gg.z, mm.z, vv.z, a);
        adam_one(pp.w, gg.w, mm.w, vv.w, a);
        p4[i] = pp; m4[i] = mm; v4[i] = vv;
        if (zero_grad) g4[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    // tail (count not a multiple of 4)
    const int64_t t = (nvec << 2) + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < count) {
        float pp = p[t], mm = m[t], vv = v[t];
        adam_one(pp, g[t], mm, vv, a);
        p[t] = pp; m[t] = mm; v[t] = vv;
        if (zero_grad) g[t] = 0.f;
    }
}

__global__ __launch_bounds__(256) void k_grad_accumulate(float* __restrict__ acc, const float* __restrict__ g,
                                                         int64_t count)
{
    const int64_t nvec = count >> 2;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    float4* a4 = reinterpret_cast<float4*>(acc);
    const float4* g4 = reinterpret_cast<const float4*>(g);
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nvec; i += stride) {
        float4 a = a4[i];
        const float4 b = g4[i];
        a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
        a4[i] = a;
    }
    const int64_t t = (nvec << 2) + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < count) acc[t] = acc[t] + g[t];
}

// s = exp(raw), q = raw / |raw|, sigma = 1 / (1 + exp(-raw))
__global__ __launch_bounds__(256) void k_activate(int64_t n, const float* __restrict__ raw_s,
                                                  const float4* __restrict__ raw_q, const float* __restrict__ raw_o,
                                                  float* __restrict__ s, float4* __restrict__ q, float* __restrict__ o)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
#pragma unroll
    for (int k = 0; k < 3; k++) s[3 * i + k] = expf(raw_s[3 * i + k]);
    const float4 r = raw_q[i];
    const float inv = 1.0f / sqrtf(r.x * r.x + r.y * r.y + r.z * r.z + r.w * r.w);
    q[i] = make_float4(r.x * inv, r.y * inv, r.z * inv, r.w * inv);
    o[i] = 1.0f / (1.0f + expf(-raw_o[i]));
}

// chain rule through k_activate; gradients may be written over the incoming ones
__global__ __launch_bounds__(256) void k_activate_bwd(int64_t n, const float* __restrict__ raw_s,
                                                      const float4* __restrict__ raw_q,
                                                      const float* __restrict__ raw_o, const float* d_s,
                                                      const float4* d_q, const float* d_o, float* d_raw_s,
                                                      float4* d_raw_q, float* d_raw_o)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
#pragma unroll
    for (int k = 0; k < 3; k++) d_raw_s[3 * i + k] = d_s[3 * i + k] * expf(raw_s[3 * i + k]);
    const float4 r = raw_q[i];
    const float inv = 1.0f / sqrtf(r.x * r.x + r.y * r.y + r.z * r.z + r.w * r.w);
    const float4 u = make_float4(r.x * inv, r.y * inv, r.z * inv, r.w * inv);
    const float4 g = d_q[i];
    const float dot = u.x * g.x + u.y * g.y + u.z * g.z + u.w * g.w;
    d_raw_q[i] = make_float4((g.x - u.x * dot) * inv, (g.y - u.y * dot) * inv, (g.z - u.z * dot) * inv,
                             (g.w - u.w * dot) * inv);
    const float sg = 1.0f / (1.0f + expf(-raw_o[i]));
    d_raw_o[i] = d_o[i] * sg * (1.0f - sg);
}

// the inverse of k_activate for scale and opacity: raw scale = ln s, raw opacity = ln(o' / (1 - o')) with the
// opacity limited to [lo, hi]
__global__ __launch_bounds__(256) void k_activate_inv(int64_t n, const float* __restrict__ s,
                                                      const float* __restrict__ o, float lo, float hi,
                                                      float* __restrict__ raw_s, float* __restrict__ raw_o)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
#pragma unroll
    for (int k = 0; k < 3; k++) raw_s[3 * i + k] = logf(s[3 * i + k]);
    const float v = fminf(fmaxf(o[i], lo), hi);
    raw_o[i] = logf(v / (1.0f - v));
}

// ---- reference measurements ------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_copy(const float4* __restrict__ src, float4* __restrict__ dst, int64_t nvec)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nvec; i += stride) dst[i] = src[i];
}

// 8 independent chains of fused multiply-adds per lane; the result is stored so that nothing is optimised away
__global__ __launch_bounds__(256) void k_fma_chain(float* __restrict__ out, int iters, float a, float b)
{
    float x0 = (float)threadIdx.x, x1 = x0 + 1.f, x2 = x0 + 2.f, x3 = x0 + 3.f, x4 = x0 + 4.f, x5 = x0 + 5.f,
          x6 = x0 + 6.f, x7 = x0 + 7.f;
    for (int i = 0; i < iters; i++) {
        x0 = __builtin_fmaf(x0, a, b); x1 = __builtin_fmaf(x1, a, b); x2 = __builtin_fmaf(x2, a, b);
        x3 = __builtin_fmaf(x3, a, b); x4 = __builtin_fmaf(x4, a, b); x5 = __builtin_fmaf(x5, a, b);
        x6 = __builtin_fmaf(x6, a, b); x7 = __builtin_fmaf(x7, a, b);
    }
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = ((x0 + x1) + (x2 + x3)) + ((x4 + x5) + (x6 + x7));
}

int stream_blocks(int64_t work_items)
{
    const int64_t b = (work_items + 255) / 256;
    return (int)(b < 1 ? 1 : (b > 8192 ? 8192 : b));   // grid-stride beyond 32 waves per CU
}

}  // namespace

hipError_t launch_adam(hipStream_t st, float* p, float* g, float* m, float* v, int64_t count, float lr, float beta1,
                       float beta2, float eps, int step, float grad_scale, bool zero_grad)
{
    if (count <= 0) return hipSuccess;
    AdamArgs a;
    a.lr = lr; a.beta1 = beta1; a.beta2 = beta2; a.omb1 = (float)(1.0 - (double)beta1);
    a.omb2 = (float)(1.0 - (double)beta2); a.eps = eps; a.grad_scale = grad_scale;
    a.inv_bc1 = (float)(1.0 / (1.0 - pow((double)beta1, (double)step)));
    a.inv_bc2 = (float)(1.0 / (1.0 - pow((double)beta2, (double)step)));
    hipLaunchKernelGGL(k_adam, dim3(stream_blocks(count >> 2)), dim3(256), 0, st, p, g, m, v, count, a, zero_grad ? 1 : 0);
    return hipGetLastError();
}

hipError_t launch_grad_accumulate(hipStream_t st, float* acc, const float* g, int64_t count)
{
    if (count <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_grad_accumulate, dim3(stream_blocks(count >> 2)), dim3(256), 0, st, acc, g, count);
    return hipGetLastError();
}

hipError_t launch_activate(hipStream_t st, int64_t n, const float* raw_s, const float* raw_q, const float* raw_o,
                           float* s, float* q, float* o)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_activate, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, n, raw_s,
                       reinterpret_cast<const float4*>(raw_q), raw_o, s, reinterpret_cast<float4*>(q), o);
    return hipGetLastError();
}

hipError_t launch_activate_bwd(hipStream_t st, int64_t n, const float* raw_s, const float* raw_q, const float* raw_o,
                               const float* d_s, const float* d_q, const float* d_o, float* d_raw_s, float* d_raw_q,
                               float* d_raw_o)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_activate_bwd, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, n, raw_s,
                       reinterpret_cast<const float4*>(raw_q), raw_o, d_s, reinterpret_cast<const float4*>(d_q), d_o,
                       d_raw_s, reinterpret_cast<float4*>(d_raw_q), d_raw_o);
    return hipGetLastError();
}

hipError_t launch_activate_inv(hipStream_t st, int64_t n, const float* s, const float* o, float lo, float hi,
                               float* raw_s, float* raw_o)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_activate_inv, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, n, s, o, lo, hi, raw_s, raw_o);
    return hipGetLastError();
}

hipError_t launch_copy(hipStream_t st, const void* src, void* dst, int64_t bytes)
{
    const int64_t nvec = bytes / 16;
    if (nvec <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_copy, dim3(stream_blocks(nvec)), dim3(256), 0, st, static_cast<const float4*>(src),
                       static_cast<float4*>(dst), nvec);
    return hipGetLastError();
}

hipError_t launch_fma_chain(hipStream_t st, float* out, int blocks, int iters)
{
    hipLaunchKernelGGL(k_fma_chain, dim3(blocks), dim3(256), 0, st, out, iters, 0.999f, 0.001f);
    return hipGetLastError();
}

}  // namespace fs
