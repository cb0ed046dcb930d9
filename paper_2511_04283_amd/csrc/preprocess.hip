// Projection of Gaussians to screen-space splats and its reverse-mode derivative (gfx950).
//
// FastGS Sec. 3: Sigma_3D = R S S^T R^T (Eq. (2)); Sigma' = J W Sigma_3D W^T J^T (Eq. (3)), of
// which the upper-left 2x2 block is Sigma_2D; Sec. 4.4: the 3-sigma rule gives the tiles a
// Gaussian is paired with.  One Gaussian per lane.
//
// Everything that decides an integer output (culling, tile rectangle, depth key, colour clamp)
// is computed in a fixed IEEE fp32 operation order, left to right as written, with no fused
// multiply-adds (this file is compiled with -ffp-contract=off), so that a CPU implementation
// following the same order reproduces it bit for bit.
#include "common.hpp"

namespace fs {

namespace {

// Real spherical-harmonics constants (orthonormal, no Condon-Shortley sign); double literals
// rounded once to float.
__device__ constexpr float K0 = (float)0.28209479177387814;
__device__ constexpr float K1 = (float)0.4886025119029199;
__device__ constexpr float K2A = (float)1.0925484305920792;
__device__ constexpr float K2B = (float)0.31539156525252005;
__device__ constexpr float K2C = (float)0.5462742152960396;
__device__ constexpr float K3A = (float)0.5900435899266435;
__device__ constexpr float K3B = (float)2.890611442640554;
__device__ constexpr float K3C = (float)0.4570457994644658;
__device__ constexpr float K3D = (float)0.3731763325901154;
__device__ constexpr float K3E = (float)1.445305721320277;

__device__ __forceinline__ void sh_basis(int deg, float x, float y, float z, float* Y)
{
    Y[0] = K0;
    if (deg < 1) return;
    Y[1] = K1 * y;
    Y[2] = K1 * z;
    Y[3] = K1 * x;
    if (deg < 2) return;
    float xx = x * x, yy = y * y, zz = z * z;
    Y[4] = K2A * (x * y);
    Y[5] = K2A * (y * z);
    Y[6] = K2B * (2.0f * zz - xx - yy);
    Y[7] = K2A * (x * z);
    Y[8] = K2C * (xx - yy);
    if (deg < 3) return;
    Y[9] = K3A * (y * (3.0f * xx - yy));
    Y[10] = K3B * ((x * y) * z);
    Y[11] = K3C * (y * (4.0f * zz - xx - yy));
    Y[12] = K3D * (z * (2.0f * zz - 3.0f * xx - 3.0f * yy));
    Y[13] = K3C * (x * (4.0f * zz - xx - yy));
    Y[14] = K3E * (z * (xx - yy));
    Y[15] = K3A * (x * (xx - 3.0f * yy));
}

// Intermediate quantities of one projection, shared by the forward and the backward kernels.
struct Splat {
    bool visible;
    float tx, ty, tz;    // camera-space mean
    float txz, tyz;      // t_x/t_z, t_y/t_z
    float cxz, cyz;      // limited copies used inside J
    bool xin, yin;
    float T00, T01, T02, T10, T11, T12;  // J * R_cam (2x3)
    float r00, r01, r02, r10, r11, r12, r20, r21, r22;  // R(q)
    float s00, s01, s02, s11, s12, s22;  // Sigma_3D (symmetric)
    float a, b, c, det;
    float mx, my, radius;
    float Q;             // Compact Box threshold
    int x0, y0, x1, y1;
};

// `sigma` (the opacity) only matters with the Compact Box, whose box depends on it.  With the Compact
// Box, s.visible still has to be and-ed with "some tile of the box meets the ellipse" by the caller.
__device__ __forceinline__ void project(const float* __restrict__ means, const float* __restrict__ scales,
                                        const float* __restrict__ quats, float sigma, int64_t i, const CamDev& cam,
                                        const CfgDev& cfg, Splat& s)
{
    s.visible = false;
    const float m0 = means[3 * i], m1 = means[3 * i + 1], m2 = means[3 * i + 2];
    s.tx = cam.R[0] * m0 + cam.R[1] * m1 + cam.R[2] * m2 + cam.t[0];
    s.ty = cam.R[3] * m0 + cam.R[4] * m1 + cam.R[5] * m2 + cam.t[1];
    s.tz = cam.R[6] * m0 + cam.R[7] * m1 + cam.R[8] * m2 + cam.t[2];
    if (!(s.tz > cfg.z_near)) return;

    const float4 q = *reinterpret_cast<const float4*>(quats + 4 * i);
    const float w = q.x, x = q.y, y = q.z, z = q.w;
    s.r00 = 1.0f - 2.0f * (y * y + z * z);
    s.r01 = 2.0f * (x * y - w * z);
    s.r02 = 2.0f * (x * z + w * y);
    s.r10 = 2.0f * (x * y + w * z);
    s.r11 = 1.0f - 2.0f * (x * x + z * z);
    s.r12 = 2.0f * (y * z - w * x);
    s.r20 = 2.0f * (x * z - w * y);
    s.r21 = 2.0f * (y * z + w * x);
    s.r22 = 1.0f - 2.0f * (x * x + y * y);
    const float sx = scales[3 * i], sy = scales[3 * i + 1], sz = scales[3 * i + 2];
    const float M00 = s.r00 * sx, M01 = s.r01 * sy, M02 = s.r02 * sz;
    const float M10 = s.r10 * sx, M11 = s.r11 * sy, M12 = s.r12 * sz;
    const float M20 = s.r20 * sx, M21 = s.r21 * sy, M22 = s.r22 * sz;
    s.s00 = M00 * M00 + M01 * M01 + M02 * M02;
    s.s01 = M00 * M10 + M01 * M11 + M02 * M12;
    s.s02 = M00 * M20 + M01 * M21 + M02 * M22;
    s.s11 = M10 * M10 + M11 * M11 + M12 * M12;
    s.s12 = M10 * M20 + M11 * M21 + M12 * M22;
    s.s22 = M20 * M20 + M21 * M21 + M22 * M22;

    s.txz = s.tx / s.tz;
    s.tyz = s.ty / s.tz;
    s.cxz = s.txz; s.cyz = s.tyz; s.xin = true; s.yin = true;
    if (cfg.jclamp > 0.0f) {
        const float limx = cfg.jclamp * (0.5f * (float)cam.width / cam.fx);
        const float limy = cfg.jclamp * (0.5f * (float)cam.height / cam.fy);
        if (s.txz > limx) { s.cxz = limx; s.xin = false; }
        if (s.txz < -limx) { s.cxz = -limx; s.xin = false; }
        if (s.tyz > limy) { s.cyz = limy; s.yin = false; }
        if (s.tyz < -limy) { s.cyz = -limy; s.yin = false; }
    }
    const float X = s.cxz * s.tz, Y = s.cyz * s.tz;
    const float iz = 1.0f / s.tz;
    const float iz2 = iz * iz;
    const float J00 = cam.fx * iz;
    const float J02 = -(cam.fx * X) * iz2;
    const float J11 = cam.fy * iz;
    const float J12 = -(cam.fy * Y) * iz2;
    s.T00 = J00 * cam.R[0] + J02 * cam.R[6];
    s.T01 = J00 * cam.R[1] + J02 * cam.R[7];
    s.T02 = J00 * cam.R[2] + J02 * cam.R[8];
    s.T10 = J11 * cam.R[3] + J12 * cam.R[6];
    s.T11 = J11 * cam.R[4] + J12 * cam.R[7];
    s.T12 = J11 * cam.R[5] + J12 * cam.R[8];
    const float U00 = s.T00 * s.s00 + s.T01 * s.s01 + s.T02 * s.s02;
    const float U01 = s.T00 * s.s01 + s.T01 * s.s11 + s.T02 * s.s12;
    const float U02 = s.T00 * s.s02 + s.T01 * s.s12 + s.T02 * s.s22;
    const float U10 = s.T10 * s.s00 + s.T11 * s.s01 + s.T12 * s.s02;
    const float U11 = s.T10 * s.s01 + s.T11 * s.s11 + s.T12 * s.s12;
    const float U12 = s.T10 * s.s02 + s.T11 * s.s12 + s.T12 * s.s22;
    const float c00 = U00 * s.T00 + U01 * s.T01 + U02 * s.T02;
    const float c01 = U00 * s.T10 + U01 * s.T11 + U02 * s.T12;
    const float c11 = U10 * s.T10 + U11 * s.T11 + U12 * s.T12;
    s.a = c00 + cfg.lowpass;
    s.b = c01;
    s.c = c11 + cfg.lowpass;
    s.det = s.a * s.c - s.b * s.b;
    if (!(s.det > 0.0f)) return;

    s.mx = cam.fx * s.txz + cam.cx;
    s.my = cam.fy * s.tyz + cam.cy;
    float hx, hy;   // half-widths of the box round mu_2D
    if (!cfg.compact_box) {
        const float mid = 0.5f * (s.a + s.c);
        const float hd = 0.5f * (s.a - s.c);
        const float lam = mid + sqrtf(hd * hd + s.b * s.b);
        s.radius = ceilf(3.0f * sqrtf(lam));
        hx = hy = s.radius;
    } else {
        // the ellipse q <= Q spans sqrt(Q Sigma_xx) horizontally and sqrt(Q Sigma_yy) vertically
        s.Q = cb_threshold(sigma, cfg);
        if (!(s.Q > 0.0f)) return;
        hx = sqrtf(s.Q * s.a);
        hy = sqrtf(s.Q * s.c);
        s.radius = ceilf(hx > hy ? hx : hy);
    }
    if (!(hx < 1e6f) || !(hy < 1e6f) || !(fabsf(s.mx) < 1e7f) || !(fabsf(s.my) < 1e7f)) return;

    const float it = 1.0f / (float)TILE;
    const float fx0 = floorf((s.mx - hx) * it);
    const float fy0 = floorf((s.my - hy) * it);
    const float fx1 = floorf((s.mx + hx) * it) + 1.0f;
    const float fy1 = floorf((s.my + hy) * it) + 1.0f;
    const float TXf = (float)cam.tiles_x, TYf = (float)cam.tiles_y;
    s.x0 = (int)fminf(fmaxf(fx0, 0.0f), TXf);
    s.y0 = (int)fminf(fmaxf(fy0, 0.0f), TYf);
    s.x1 = (int)fminf(fmaxf(fx1, 0.0f), TXf);
    s.y1 = (int)fminf(fmaxf(fy1, 0.0f), TYf);
    if ((s.x1 - s.x0) * (s.y1 - s.y0) <= 0) return;
    s.visible = true;
}

// Unit direction from the camera centre (-R^T t) to the mean, and its length.
__device__ __forceinline__ void view_dir(const float* __restrict__ means, int64_t i, const CamDev& cam,
                                         float d[3], float& len)
{
    float dir[3];
    for (int k = 0; k < 3; k++) {
        const float campos = -(cam.R[0 + k] * cam.t[0] + cam.R[3 + k] * cam.t[1] + cam.R[6 + k] * cam.t[2]);
        dir[k] = means[3 * i + k] - campos;
    }
    len = sqrtf(dir[0] * dir[0] + dir[1] * dir[1] + dir[2] * dir[2]);
    d[0] = dir[0] / len;
    d[1] = dir[1] / len;
    d[2] = dir[2] / len;
}

template <int DEG>
__global__ __launch_bounds__(256) void k_preprocess(int64_t n, const float* __restrict__ means,
                                                    const float* __restrict__ scales,
                                                    const float* __restrict__ quats,
                                                    const float* __restrict__ opac, const float* __restrict__ sh,
                                                    CamDev cam, CfgDev cfg, float* __restrict__ mean2d,
                                                    float* __restrict__ depth, float* __restrict__ conic_opacity,
                                                    float* __restrict__ rgb, uint16_t* __restrict__ rect,
                                                    uint32_t* __restrict__ touched, uint8_t* __restrict__ clamped)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    Splat s;
    project(means, scales, quats, opac[i], i, cam, cfg, s);
    uint32_t hits = 0;
    if (s.visible) {
        if (!cfg.compact_box) {
            hits = (uint32_t)((s.x1 - s.x0) * (s.y1 - s.y0));
        } else {
            const float idet = 1.0f / s.det;
            const float A = s.c * idet, B = -s.b * idet, C = s.a * idet;
            for (int ty = s.y0; ty < s.y1; ty++)
                for (int tx = s.x0; tx < s.x1; tx++) hits += cb_tile_hit(s.mx, s.my, A, B, C, s.Q, tx, ty) ? 1u : 0u;
            s.visible = hits > 0;
        }
    }
    float2 m2 = make_float2(0.f, 0.f);
    float4 co = make_float4(0.f, 0.f, 0.f, 0.f);
    float col[3] = {0.f, 0.f, 0.f};
    uint8_t cl[3] = {0, 0, 0};
    float dep = 0.f;
    ushort4 rc = make_ushort4(0, 0, 0, 0);
    uint32_t tt = 0;
    if (s.visible) {
        const float idet = 1.0f / s.det;
        co = make_float4(s.c * idet, -s.b * idet, s.a * idet, opac[i]);
        m2 = make_float2(s.mx, s.my);
        dep = s.tz;
        rc = make_ushort4((unsigned short)s.x0, (unsigned short)s.y0, (unsigned short)s.x1, (unsigned short)s.y1);
        tt = hits;
        float d[3], len;
        view_dir(means, i, cam, d, len);
        constexpr int K = (DEG + 1) * (DEG + 1);
        float Y[K];
        sh_basis(DEG, d[0], d[1], d[2], Y);
        const float* c = sh + (int64_t)3 * K * i;
        float v0 = Y[0] * c[0], v1 = Y[0] * c[1], v2 = Y[0] * c[2];
#pragma unroll
        for (int k = 1; k < K; k++) {
            v0 = v0 + Y[k] * c[3 * k + 0];
            v1 = v1 + Y[k] * c[3 * k + 1];
            v2 = v2 + Y[k] * c[3 * k + 2];
        }
        v0 = v0 + 0.5f; v1 = v1 + 0.5f; v2 = v2 + 0.5f;
        cl[0] = v0 < 0.0f; cl[1] = v1 < 0.0f; cl[2] = v2 < 0.0f;
        col[0] = cl[0] ? 0.0f : v0;
        col[1] = cl[1] ? 0.0f : v1;
        col[2] = cl[2] ? 0.0f : v2;
    }
    *reinterpret_cast<float2*>(mean2d + 2 * i) = m2;
    depth[i] = dep;
    *reinterpret_cast<float4*>(conic_opacity + 4 * i) = co;
    rgb[3 * i + 0] = col[0]; rgb[3 * i + 1] = col[1]; rgb[3 * i + 2] = col[2];
    *reinterpret_cast<ushort4*>(rect + 4 * i) = rc;
    touched[i] = tt;
    clamped[3 * i + 0] = cl[0]; clamped[3 * i + 1] = cl[1]; clamped[3 * i + 2] = cl[2];
}

// d(Y_k)/d(x,y,z) dotted with per-channel weights: accumulates g_d += sum_k w_k * grad Y_k.
template <int DEG>
__device__ __forceinline__ void sh_dir_grad(float x, float y, float z, const float* wk /*[K]*/, float g[3])
{
    float gx = 0.f, gy = 0.f, gz = 0.f;
    if (DEG >= 1) {
        gy += K1 * wk[1];
        gz += K1 * wk[2];
        gx += K1 * wk[3];
    }
    if (DEG >= 2) {
        gx += K2A * y * wk[4];  gy += K2A * x * wk[4];
        gy += K2A * z * wk[5];  gz += K2A * y * wk[5];
        gx += K2B * -2.f * x * wk[6];  gy += K2B * -2.f * y * wk[6];  gz += K2B * 4.f * z * wk[6];
        gx += K2A * z * wk[7];  gz += K2A * x * wk[7];
        gx += K2C * 2.f * x * wk[8];  gy += K2C * -2.f * y * wk[8];
    }
    if (DEG >= 3) {
        const float xx = x * x, yy = y * y, zz = z * z;
        gx += K3A * 6.f * x * y * wk[9];   gy += K3A * (3.f * xx - 3.f * yy) * wk[9];
        gx += K3B * y * z * wk[10];  gy += K3B * x * z * wk[10];  gz += K3B * x * y * wk[10];
        gx += K3C * -2.f * x * y * wk[11];  gy += K3C * (4.f * zz - xx - 3.f * yy) * wk[11];  gz += K3C * 8.f * y * z * wk[11];
        gx += K3D * -6.f * x * z * wk[12];  gy += K3D * -6.f * y * z * wk[12];  gz += K3D * (6.f * zz - 3.f * xx - 3.f * yy) * wk[12];
        gx += K3C * (4.f * zz - 3.f * xx - yy) * wk[13];  gy += K3C * -2.f * x * y * wk[13];  gz += K3C * 8.f * x * z * wk[13];
        gx += K3E * 2.f * x * z * wk[14];  gy += K3E * -2.f * y * z * wk[14];  gz += K3E * (xx - yy) * wk[14];
        gx += K3A * (3.f * xx - 3.f * yy) * wk[15];  gy += K3A * -6.f * x * y * wk[15];
    }
    g[0] = gx; g[1] = gy; g[2] = gz;
}

// Sum over the 64 lanes of a wavefront, left in lane 63: four shifts within the rows of 16 lanes (zeros move in at a
// row's start), then lane 15 of rows 0 and 2 is added to the row after it, then lane 31 to rows 2 and 3.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_or_zero_f(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xF, false));
}
__device__ __forceinline__ float wave_sum_to_last(float v)
{
    v += dpp_or_zero_f<0x111, 0xF>(v);   // row_shr:1
    v += dpp_or_zero_f<0x112, 0xF>(v);   // row_shr:2
    v += dpp_or_zero_f<0x114, 0xF>(v);   // row_shr:4
    v += dpp_or_zero_f<0x118, 0xF>(v);   // row_shr:8
    v += dpp_or_zero_f<0x142, 0xA>(v);   // row_bcast:15 into rows 1 and 3
    v += dpp_or_zero_f<0x143, 0xC>(v);   // row_bcast:31 into rows 2 and 3
    return v;
}

// Reverse of project().  First the screen-space gradients of Gaussian i are formed by adding up
// its pairs' records (contiguous: pair_offsets[i] .. + tiles_touched[i], each record = dL/drgb 3,
// dL/dsigma, dL/dconic 3, dL/dmu_2D 2, padded to PAIR_REC floats), in a fixed order; then they are
// chained to the gradients of mean, scale, quaternion and SH coefficients (dL/d opacity needs no
// chaining).  Outputs are overwritten; culled Gaussians get zeros.  Plain fp32 (not bit-pinned).
template <int DEG, bool SPARSE>
__global__ __launch_bounds__(256) void k_preprocess_bwd(
    int64_t n, const float* __restrict__ means, const float* __restrict__ scales, const float* __restrict__ quats,
    const float* __restrict__ opac, const float* __restrict__ sh, CamDev cam, CfgDev cfg,
    const uint8_t* __restrict__ clamped, const uint32_t* __restrict__ touched,
    const uint32_t* __restrict__ rec_counts, const uint32_t* __restrict__ offsets,
    const float4* __restrict__ pair_grad, uint8_t* __restrict__ rec_valid, float* __restrict__ d_means,
    float* __restrict__ d_scales,
    float* __restrict__ d_quats, float* __restrict__ d_sh, float* __restrict__ d_opac,
    float* __restrict__ d_mean2d, float* __restrict__ d_conic /* may be null */,
    float* __restrict__ d_rgb /* may be null */, float* __restrict__ d_abs /* may be null */)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    constexpr int K = (DEG + 1) * (DEG + 1);
    constexpr int F = 3 * K;                      // SH floats per Gaussian
    constexpr int ROW = F + 1;                    // padded row: lane-strided LDS access without bank conflicts
    constexpr int CH = 128;                       // pair records per chunk and wavefront
    constexpr int HALF = 32;                      // Gaussians whose SH rows are in LDS at a time
    constexpr int WAVE_FLOATS = HALF * ROW > CH * PAIR_REC ? HALF * ROW : CH * PAIR_REC;
    // one buffer per wavefront, used in turn for the pair records and, half a wavefront at a time, for the SH
    // coefficients and their gradients (kept this small so that more wavefronts fit a compute unit: the kernel
    // is bound by memory and needs them to keep enough loads in flight)
    __shared__ __attribute__((aligned(16))) float s_buf[4][(WAVE_FLOATS + 3) / 4 * 4];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const bool in_range = i < n;
    // (a Gaussian with tiles_touched > 0 passed the forward pass's culling: the count stands in for visibility)
    const bool vis0 = in_range && touched[i] > 0;
    const int64_t wave_first = (int64_t)blockIdx.x * blockDim.x + wave * 64;
    const int valid_rows = (int)min((int64_t)64, max((int64_t)0, n - wave_first));
    constexpr int NV = (HALF / 4 * F + 63) / 64;  // float4 per lane for the SH rows of a full half
    // The SH rows of the first half are requested before the pair records are streamed, so that the two latencies
    // overlap (they wait in registers: the LDS buffer serves the records first).
    float4 vh[NV];
    int pre = -1;   // the half whose rows are on their way into vh (uniform over the wavefront)
    auto request_half = [&](int h) {
        if (valid_rows < (h + 1) * HALF || __ballot(vis0 && (lane / HALF) == h) == 0) return;
        const float4* src4 = reinterpret_cast<const float4*>(sh + (wave_first + h * HALF) * F);
#pragma unroll
        for (int it = 0; it < NV; it++) {
            const int q = lane + 64 * it;
            vh[it] = q < HALF / 4 * F ? src4[q] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
        pre = h;
    };
    request_half(0);

    // ---- screen-space gradients: sum of this Gaussian's pair records, in tile order ----------
    // The 64 Gaussians of a wavefront own one contiguous run of records.  The wavefront streams that
    // run through LDS in chunks with coalesced 16-byte loads; each lane then adds up its own records.
    float4 ra = make_float4(0.f, 0.f, 0.f, 0.f), rb = ra;
    float rc = 0.f, rabs_x = 0.f, rabs_y = 0.f;
    {
        const uint32_t off = in_range ? offsets[i] : 0u;
        const uint32_t cnt = in_range && touched[i] ? rec_counts[i] : 0u;
        uint32_t lo_all = cnt ? off : 0xffffffffu, hi_all = cnt ? off + cnt : 0u;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            lo_all = min(lo_all, (uint32_t)__shfl_xor((int)lo_all, d, 64));
            hi_all = max(hi_all, (uint32_t)__shfl_xor((int)hi_all, d, 64));
        }
        float4* buf = reinterpret_cast<float4*>(s_buf[wave]);
        // Chunk k+1 is requested as soon as chunk k has gone from registers to LDS, so that its latency passes
        // while chunk k is added up.  (All loads of a chunk are issued before the first LDS write: written as one
        // loop, each load would be waited for in turn.)
        constexpr int LPL = CH * (PAIR_REC / 4) / 64;
        static_assert(CH == 128 && PAIR_REC == 12 && LPL == 6, "two records (flag bytes) per lane and chunk, three 16-byte words per record");
        float4 v[LPL];
        // !SPARSE (dense records, rec_valid unused): every place holds a record; the chunk is read as one run of 16-byte words.
        // Otherwise (sparse records) only the places whose flag the backward kernel set hold anything: the others are
        // not read and count as zeros.  Lane l then takes the three words of records l and l + 64 of the chunk (its own
        // two flags decide, no exchange between the lanes); a chunk's flags are requested one chunk ahead of its
        // records, and the wavefront puts them back to zero, so that the array is all zeros again when the kernel ends
        // (the places between lo_all and hi_all are this wavefront's own: no other one looks at their flags).
        constexpr bool sparse = SPARSE;
        uint8_t f0 = 0, f1 = 0;
        auto request_flags = [&](uint32_t cs) {
            const uint32_t p0 = cs + lane, p1 = cs + 64 + lane;
            f0 = p0 < hi_all ? rec_valid[p0] : (uint8_t)0;
            f1 = p1 < hi_all ? rec_valid[p1] : (uint8_t)0;
        };
        auto request = [&](uint32_t cs) {
            if (sparse) {
                const bool s0 = f0 != 0, s1 = f1 != 0;   // (the flags of chunk cs have arrived; zero beyond hi_all)
                if (s0) rec_valid[cs + lane] = 0;
                if (s1) rec_valid[cs + 64 + lane] = 0;
                const float4* src = pair_grad + ((size_t)cs + lane) * (PAIR_REC / 4);
#pragma unroll
                for (int k = 0; k < 3; k++) {
                    v[k] = s0 ? src[k] : make_float4(0.f, 0.f, 0.f, 0.f);
                    v[3 + k] = s1 ? src[64 * 3 + k] : make_float4(0.f, 0.f, 0.f, 0.f);
                }
            } else {
                const uint32_t nq = min((uint32_t)CH, hi_all - cs) * (PAIR_REC / 4);
                const float4* src = pair_grad + (size_t)cs * (PAIR_REC / 4);
#pragma unroll
                for (int u = 0; u < LPL; u++) {
                    const uint32_t q = lane + 64 * u;
                    v[u] = q < nq ? src[q] : make_float4(0.f, 0.f, 0.f, 0.f);
                }
            }
        };
        if (lo_all < hi_all) {
            if (sparse) request_flags(lo_all);
            request(lo_all);
            if (sparse && lo_all + CH < hi_all) request_flags(lo_all + CH);
        }
        for (uint32_t cs = lo_all; cs < hi_all; cs += CH) {
            const uint32_t nrec = min((uint32_t)CH, hi_all - cs);
            if (sparse) {
#pragma unroll
                for (int k = 0; k < 3; k++) {
                    if ((uint32_t)lane < nrec) buf[lane * 3 + k] = v[k];
                    if ((uint32_t)lane + 64 < nrec) buf[(lane + 64) * 3 + k] = v[3 + k];
                }
            } else {
#pragma unroll
                for (int u = 0; u < LPL; u++) {
                    const uint32_t q = lane + 64 * u;
                    if (q < nrec * (PAIR_REC / 4)) buf[q] = v[u];
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            if (cs + CH < hi_all) {
                request(cs + CH);
                if (sparse && cs + 2 * CH < hi_all) request_flags(cs + 2 * CH);
            }
            const uint32_t r0 = max(off, cs), r1 = min(off + cnt, cs + nrec);
            // A Gaussian with many records in the chunk (a large splat: one per tile of its rectangle) would keep its
            // lane busy for as many trips while the other 63 wait.  Such runs are added up by the whole wavefront
            // instead, one after the other: lane l takes records l and l + 64 of the run, a sum over the lanes follows,
            // and the owner adds the total.  (The order of the additions is fixed either way.)
            constexpr uint32_t BIG = 32;   // (8: slower everywhere; 16 .. 64: within 2 % of each other, 32 best)
            const bool big = r1 > r0 && r1 - r0 >= BIG;
            for (uint64_t todo = __ballot(big); todo != 0; todo &= todo - 1) {
                const int o = __builtin_ctzll(todo);
                const uint32_t q0 = (uint32_t)__builtin_amdgcn_readlane((int)r0, o) - cs;   // the run within the chunk:
                const uint32_t q1 = (uint32_t)__builtin_amdgcn_readlane((int)r1, o) - cs;   // [q0, q1), q1 <= nrec <= CH
                float t[11];
#pragma unroll
                for (int k = 0; k < 11; k++) t[k] = 0.f;
#pragma unroll
                for (uint32_t h = 0; h < CH / 64; h++) {
                    const uint32_t q = q0 + lane + 64 * h;
                    if (q < q1) {
                        const float4 a = buf[q * 3], b = buf[q * 3 + 1], c4 = buf[q * 3 + 2];
                        t[0] += a.x; t[1] += a.y; t[2] += a.z; t[3] += a.w;
                        t[4] += b.x; t[5] += b.y; t[6] += b.z; t[7] += b.w;
                        t[8] += c4.x; t[9] += c4.y; t[10] += c4.z;
                    }
                }
#pragma unroll
                for (int k = 0; k < 11; k++) t[k] = wave_sum_to_last(t[k]);
                float tot[11];
#pragma unroll
                for (int k = 0; k < 11; k++) tot[k] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(t[k]), 63));
                if (lane == o) {
                    ra.x += tot[0]; ra.y += tot[1]; ra.z += tot[2]; ra.w += tot[3];
                    rb.x += tot[4]; rb.y += tot[5]; rb.z += tot[6]; rb.w += tot[7];
                    rc += tot[8]; rabs_x += tot[9]; rabs_y += tot[10];
                }
            }
            const uint32_t r1s = big ? r0 : r1;   // the short runs: every lane its own
            uint32_t r = r0;
            for (; r + 2 <= r1s; r += 2) {   // two records per trip: their LDS reads overlap
                const float4 a = buf[(r - cs) * 3], b = buf[(r - cs) * 3 + 1], c4 = buf[(r - cs) * 3 + 2];
                const float4 a2 = buf[(r - cs) * 3 + 3], b2 = buf[(r - cs) * 3 + 4], c5 = buf[(r - cs) * 3 + 5];
                ra.x += a.x; ra.y += a.y; ra.z += a.z; ra.w += a.w;
                rb.x += b.x; rb.y += b.y; rb.z += b.z; rb.w += b.w;
                rc += c4.x; rabs_x += c4.y; rabs_y += c4.z;
                ra.x += a2.x; ra.y += a2.y; ra.z += a2.z; ra.w += a2.w;
                rb.x += b2.x; rb.y += b2.y; rb.z += b2.z; rb.w += b2.w;
                rc += c5.x; rabs_x += c5.y; rabs_y += c5.z;
            }
            if (r < r1s) {
                const float4 a = buf[(r - cs) * 3], b = buf[(r - cs) * 3 + 1], c4 = buf[(r - cs) * 3 + 2];
                ra.x += a.x; ra.y += a.y; ra.z += a.z; ra.w += a.w;
                rb.x += b.x; rb.y += b.y; rb.z += b.z; rb.w += b.w;
                rc += c4.x;
                rabs_x += c4.y; rabs_y += c4.z;   // (only meaningful when the records carry them)
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
    }

    // ---- SH coefficients of HALF consecutive Gaussians of the wavefront: one contiguous block of HALF*F floats,
    //      copied to LDS with coalesced loads (a lane reading its own F floats straight from memory would touch
    //      64 different cache lines per instruction); the gradients go back the same way ----
    float* rows = s_buf[wave];
    float* c = rows + (lane & (HALF - 1)) * ROW;  // this lane's coefficients, later its gradients
    // float4 number q of a half's block -> its four floats into the padded rows
    auto commit = [&](const float4 (&v)[NV]) {
#pragma unroll
        for (int it = 0; it < NV; it++) {
            const int q = lane + 64 * it;
            if (q < HALF / 4 * F) {
                const float comp[4] = {v[it].x, v[it].y, v[it].z, v[it].w};
                int row = (4 * q) / F, col = 4 * q - row * F;
#pragma unroll
                for (int jj = 0; jj < 4; jj++) {
                    rows[row * ROW + col] = comp[jj];
                    if (++col == F) { col = 0; row++; }
                }
            }
        }
    };
    auto load_half = [&](int h) {
        const int vr = min(HALF, max(0, valid_rows - h * HALF));
        const float* src = sh + (wave_first + h * HALF) * F;
        if (pre == h) {
            commit(vh);
        } else if (vr == HALF) {
            // all loads issued before the first LDS write
            const float4* src4 = reinterpret_cast<const float4*>(src);
            float4 v[NV];
#pragma unroll
            for (int it = 0; it < NV; it++) {
                const int q = lane + 64 * it;
                v[it] = q < HALF / 4 * F ? src4[q] : make_float4(0.f, 0.f, 0.f, 0.f);
            }
            commit(v);
        } else {
            for (int e = lane; e < HALF * F; e += 64) {
                const int row = e / F;
                if (row < vr) rows[row * ROW + (e - row * F)] = src[e];
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    };
    auto store_half = [&](int h) {
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        const int vr = min(HALF, max(0, valid_rows - h * HALF));
        float* dst = d_sh + (wave_first + h * HALF) * F;
        if (vr == HALF) {
            float4* dst4 = reinterpret_cast<float4*>(dst);
#pragma unroll
            for (int it = 0; it < NV; it++) {
                const int q = lane + 64 * it;
                if (q < HALF / 4 * F) {
                    float comp[4];
                    int row = (4 * q) / F, col = 4 * q - row * F;
#pragma unroll
                    for (int jj = 0; jj < 4; jj++) {
                        comp[jj] = rows[row * ROW + col];
                        if (++col == F) { col = 0; row++; }
                    }
                    dst4[q] = make_float4(comp[0], comp[1], comp[2], comp[3]);
                }
            }
        } else {
            for (int e = lane; e < HALF * F; e += 64) {
                const int row = e / F;
                if (row < vr) dst[e] = rows[row * ROW + (e - row * F)];
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    };

    // ---- colour -> SH coefficients (and the weights the view direction's gradient needs), half a wavefront at a
    //      time; done before the projection is recomputed so that few registers are live across it.
    float d[3] = {0.f, 0.f, 1.f}, len = 1.f;
    float wk[K];
#pragma unroll
    for (int k = 0; k < K; k++) wk[k] = 0.f;
    for (int h = 0; h < 64 / HALF; h++) {
        // (culled Gaussians come in runs -- whole clusters outside the frustum -- so a half often needs no
        // coefficients at all: its gradients are zeros whatever the buffer holds)
        if (__ballot(vis0 && (lane / HALF) == h) != 0) load_half(h);
        // (requesting the second half's rows here, while the first is worked on, was measured slower: the registers
        // they wait in take a wavefront per SIMD away)
        if ((lane / HALF) == h && in_range) {
            float Y[K], gcol[3] = {0.f, 0.f, 0.f};
#pragma unroll
            for (int k = 0; k < K; k++) Y[k] = 0.f;
            if (vis0) {
                view_dir(means, i, cam, d, len);
                sh_basis(DEG, d[0], d[1], d[2], Y);
                gcol[0] = clamped[3 * i] ? 0.f : ra.x;
                gcol[1] = clamped[3 * i + 1] ? 0.f : ra.y;
                gcol[2] = clamped[3 * i + 2] ? 0.f : ra.z;
            }
            // (culled Gaussians: gcol = 0, so their gradients come out as zeros)
#pragma unroll
            for (int k = 0; k < K; k++) {
                wk[k] = gcol[0] * c[3 * k] + gcol[1] * c[3 * k + 1] + gcol[2] * c[3 * k + 2];
                c[3 * k + 0] = gcol[0] * Y[k];   // the coefficient has been read: its slot now holds its gradient
                c[3 * k + 1] = gcol[1] * Y[k];
                c[3 * k + 2] = gcol[2] * Y[k];
            }
        }
        store_half(h);
    }
    Splat s;
    s.visible = false;
    if (vis0) {   // (tiles_touched = 0: culled in the forward pass, or a Compact Box none of whose tiles meets the ellipse)
        project(means, scales, quats, opac[i], i, cam, cfg, s);
    }
    if (in_range && !s.visible) {
        for (int k = 0; k < 3; k++) { d_means[3 * i + k] = 0.f; d_scales[3 * i + k] = 0.f; }
        *reinterpret_cast<float4*>(d_quats + 4 * i) = make_float4(0.f, 0.f, 0.f, 0.f);
        d_opac[i] = 0.f;
        d_mean2d[2 * i] = 0.f; d_mean2d[2 * i + 1] = 0.f;
        if (d_conic) for (int k = 0; k < 3; k++) d_conic[3 * i + k] = 0.f;
        if (d_rgb) for (int k = 0; k < 3; k++) d_rgb[3 * i + k] = 0.f;
        if (d_abs) { d_abs[2 * i] = 0.f; d_abs[2 * i + 1] = 0.f; }
    }
    const bool vis = in_range && s.visible;
    const float g_rgb3[3] = {ra.x, ra.y, ra.z};
    if (vis) {
        const float g_conic3[3] = {rb.x, rb.y, rb.z};
        const float g_m2[2] = {rb.w, rc};
        d_opac[i] = ra.w;
        d_mean2d[2 * i] = g_m2[0]; d_mean2d[2 * i + 1] = g_m2[1];
        if (d_conic) { d_conic[3 * i] = g_conic3[0]; d_conic[3 * i + 1] = g_conic3[1]; d_conic[3 * i + 2] = g_conic3[2]; }
        if (d_rgb) { d_rgb[3 * i] = g_rgb3[0]; d_rgb[3 * i + 1] = g_rgb3[1]; d_rgb[3 * i + 2] = g_rgb3[2]; }
        if (d_abs) { d_abs[2 * i] = rabs_x; d_abs[2 * i + 1] = rabs_y; }
        float gd[3];
        sh_dir_grad<DEG>(d[0], d[1], d[2], wk, gd);
        const float dot = gd[0] * d[0] + gd[1] * d[1] + gd[2] * d[2];
        const float ilen = 1.0f / len;
        float gm0 = (gd[0] - d[0] * dot) * ilen;
        float gm1 = (gd[1] - d[1] * dot) * ilen;
        float gm2 = (gd[2] - d[2] * dot) * ilen;

        // ---- conic = Sigma_2D^-1 -> (a,b,c) ----
        const float idet = 1.0f / s.det;
        const float g0 = g_conic3[0], g1 = g_conic3[1], g2 = g_conic3[2];
        const float g_det = -(g0 * s.c - g1 * s.b + g2 * s.a) * idet * idet;
        const float ga = g2 * idet + g_det * s.c;
        const float gb = -g1 * idet - 2.f * g_det * s.b;
        const float gc = g0 * idet + g_det * s.a;
        const float hb = 0.5f * gb;
        // Sigma_2D = T Sigma_3D T^T:  dSigma_3D = T^T G T ;  dT = 2 G T Sigma_3D   (G = [[ga,hb],[hb,gc]])
        const float T0[3] = {s.T00, s.T01, s.T02}, T1[3] = {s.T10, s.T11, s.T12};
        const float S3[3][3] = {{s.s00, s.s01, s.s02}, {s.s01, s.s11, s.s12}, {s.s02, s.s12, s.s22}};
        float GT0[3], GT1[3];  // rows of G*T
        for (int k = 0; k < 3; k++) { GT0[k] = ga * T0[k] + hb * T1[k]; GT1[k] = hb * T0[k] + gc * T1[k]; }
        float gS[3][3];
        for (int r = 0; r < 3; r++)
            for (int q = 0; q < 3; q++) gS[r][q] = T0[r] * GT0[q] + T1[r] * GT1[q];
        float gT0[3], gT1[3];
        for (int r = 0; r < 3; r++) {
            gT0[r] = 2.f * (GT0[0] * S3[0][r] + GT0[1] * S3[1][r] + GT0[2] * S3[2][r]);
            gT1[r] = 2.f * (GT1[0] * S3[0][r] + GT1[1] * S3[1][r] + GT1[2] * S3[2][r]);
        }
        // T = J R_cam
        const float gJ00 = gT0[0] * cam.R[0] + gT0[1] * cam.R[1] + gT0[2] * cam.R[2];
        const float gJ02 = gT0[0] * cam.R[6] + gT0[1] * cam.R[7] + gT0[2] * cam.R[8];
        const float gJ11 = gT1[0] * cam.R[3] + gT1[1] * cam.R[4] + gT1[2] * cam.R[5];
        const float gJ12 = gT1[0] * cam.R[6] + gT1[1] * cam.R[7] + gT1[2] * cam.R[8];
        // J00 = fx/tz, J02 = -fx X/tz^2, J11 = fy/tz, J12 = -fy Y/tz^2, X = cxz*tz, Y = cyz*tz
        const float iz = 1.0f / s.tz, iz2 = iz * iz;
        const float X = s.cxz * s.tz, Yc = s.cyz * s.tz;
        const float g_iz = cam.fx * gJ00 + cam.fy * gJ11 - 2.f * cam.fx * X * iz * gJ02 - 2.f * cam.fy * Yc * iz * gJ12;
        const float gX = -cam.fx * iz2 * gJ02, gY = -cam.fy * iz2 * gJ12;
        float gtz = gX * s.cxz + gY * s.cyz - g_iz * iz2;
        float gtxz = s.xin ? gX * s.tz : 0.f;
        float gtyz = s.yin ? gY * s.tz : 0.f;
        gtxz += cam.fx * g_m2[0];
        gtyz += cam.fy * g_m2[1];
        const float gtx = gtxz * iz, gty = gtyz * iz;
        gtz -= (gtxz * s.tx + gtyz * s.ty) * iz2;
        gm0 += cam.R[0] * gtx + cam.R[3] * gty + cam.R[6] * gtz;
        gm1 += cam.R[1] * gtx + cam.R[4] * gty + cam.R[7] * gtz;
        gm2 += cam.R[2] * gtx + cam.R[5] * gty + cam.R[8] * gtz;
        d_means[3 * i] = gm0; d_means[3 * i + 1] = gm1; d_means[3 * i + 2] = gm2;

        // ---- Sigma_3D = M M^T, M = R(q) diag(s) ----
        const float Rq[3][3] = {{s.r00, s.r01, s.r02}, {s.r10, s.r11, s.r12}, {s.r20, s.r21, s.r22}};
        const float sc[3] = {scales[3 * i], scales[3 * i + 1], scales[3 * i + 2]};
        float gR[3][3];
        float gs[3] = {0.f, 0.f, 0.f};
        for (int r = 0; r < 3; r++)
            for (int q = 0; q < 3; q++) {
                float gM = 0.f;
                for (int k = 0; k < 3; k++) gM += (gS[r][k] + gS[k][r]) * (Rq[k][q] * sc[q]);
                gs[q] += gM * Rq[r][q];
                gR[r][q] = gM * sc[q];
            }
        d_scales[3 * i] = gs[0]; d_scales[3 * i + 1] = gs[1]; d_scales[3 * i + 2] = gs[2];
        const float4 qq = *reinterpret_cast<const float4*>(quats + 4 * i);
        const float w = qq.x, x = qq.y, y = qq.z, z = qq.w;
        float4 gq;
        gq.x = 2.f * (-z * gR[0][1] + y * gR[0][2] + z * gR[1][0] - x * gR[1][2] - y * gR[2][0] + x * gR[2][1]);
        gq.y = 2.f * (y * gR[0][1] + z * gR[0][2] + y * gR[1][0] - 2.f * x * gR[1][1] - w * gR[1][2] + z * gR[2][0] +
                      w * gR[2][1] - 2.f * x * gR[2][2]);
        gq.z = 2.f * (-2.f * y * gR[0][0] + x * gR[0][1] + w * gR[0][2] + x * gR[1][0] + z * gR[1][2] - w * gR[2][0] +
                      z * gR[2][1] - 2.f * y * gR[2][2]);
        gq.w = 2.f * (-2.f * z * gR[0][0] - w * gR[0][1] + x * gR[0][2] + w * gR[1][0] - 2.f * z * gR[1][1] +
                      y * gR[1][2] + x * gR[2][0] + y * gR[2][1]);
        *reinterpret_cast<float4*>(d_quats + 4 * i) = gq;
    }
}

}  // namespace

hipError_t launch_preprocess(hipStream_t st, int64_t n, int deg, const fs_gaussians& g, const CamDev& cam,
                             const CfgDev& cfg, const fs_projected& o)
{
    if (n == 0) return hipSuccess;
    const dim3 grid((unsigned)((n + 255) / 256)), block(256);
#define FS_LAUNCH(D)                                                                                         \
    hipLaunchKernelGGL(k_preprocess<D>, grid, block, 0, st, n, g.means, g.scales, g.quats, g.opacities, g.sh, \
                       cam, cfg, o.mean2d, o.depth, o.conic_opacity, o.rgb, o.rect, o.tiles_touched, o.clamped)
    switch (deg) {
        case 0: FS_LAUNCH(0); break;
        case 1: FS_LAUNCH(1); break;
        case 2: FS_LAUNCH(2); break;
        default: FS_LAUNCH(3); break;
    }
#undef FS_LAUNCH
    return hipGetLastError();
}

// rec_valid: null = dense records (every place of pair_grad holds one), else the flags of the sparse records
hipError_t launch_preprocess_bwd(hipStream_t st, int64_t n, int deg, const fs_gaussians& g, const CamDev& cam,
                                 const CfgDev& cfg, const uint8_t* clamped, const uint32_t* touched,
                                 const uint32_t* rec_counts, const uint32_t* rec_offsets, const float* pair_grad,
                                 uint8_t* rec_valid, const fs_grads& o)
{
    if (n == 0) return hipSuccess;
    const dim3 grid((unsigned)((n + 255) / 256)), block(256);
#define FS_LAUNCH_S(D, S)                                                                                          \
    hipLaunchKernelGGL((k_preprocess_bwd<D, S>), grid, block, 0, st, n, g.means, g.scales, g.quats, g.opacities,    \
                       g.sh, cam, cfg, clamped, touched, rec_counts, rec_offsets,                                   \
                       reinterpret_cast<const float4*>(pair_grad), rec_valid, o.dmeans, o.dscales, o.dquats, o.dsh, \
                       o.dopacities, o.dmean2d, o.dconic, o.drgb, o.dmean2d_abs)
#define FS_LAUNCH(D)                         \
    do {                                     \
        if (rec_valid) FS_LAUNCH_S(D, true); \
        else FS_LAUNCH_S(D, false);          \
    } while (0)
    switch (deg) {
        case 0: FS_LAUNCH(0); break;
        case 1: FS_LAUNCH(1); break;
        case 2: FS_LAUNCH(2); break;
        default: FS_LAUNCH(3); break;
    }
#undef FS_LAUNCH
#undef FS_LAUNCH_S
    return hipGetLastError();
}

}  // namespace fs
