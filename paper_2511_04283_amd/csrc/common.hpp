// Internal declarations shared by the HIP translation units of libfastgs_hip (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fastgs.h"

namespace fs {

constexpr int TILE = 16;           // pixels per tile edge (the binning unit of the ABI)
constexpr int TILE_PIX = TILE * TILE;

// Camera and conventions as passed by value to kernels.
struct CamDev {
    int width, height;
    float fx, fy, cx, cy;
    float R[9];
    float t[3];
    int tiles_x, tiles_y;
};

struct CfgDev {
    float z_near, lowpass, alpha_min, alpha_max, T_min;
    float bg[3];
    float jclamp;
    float power_min;  // exponents below this cannot reach alpha_min for opacity <= 1 (conservative)
    int score_mode;
};

// ---- launchers (each enqueues on `st` and returns hipGetLastError()) ------------------------
hipError_t launch_preprocess(hipStream_t st, int64_t n, int deg, const fs_gaussians& g, const CamDev& cam,
                             const CfgDev& cfg, const fs_projected& out);
// pair_grad: [P] records of PAIR_REC floats (see render.hip); offsets/touched as in fs_bins/fs_projected
constexpr int PAIR_REC = 12;
hipError_t launch_preprocess_bwd(hipStream_t st, int64_t n, int deg, const fs_gaussians& g, const CamDev& cam,
                                 const CfgDev& cfg, const uint8_t* clamped, const uint32_t* touched,
                                 const uint32_t* offsets, const float* pair_grad, const fs_grads& out);

// exclusive scan of n uint32 values; total (uint64) written to *total_dev. tmp: >= scan_tmp_bytes(n).
size_t scan_tmp_bytes(int64_t n);
hipError_t launch_exclusive_scan(hipStream_t st, const uint32_t* in, uint32_t* out, int64_t n, void* tmp,
                                 uint64_t* total_dev);

// Splat record (SPLAT_REC floats = 64 bytes, one per Gaussian): mx my a b | c sigma r g | b offset rect01 rect23 | unused
constexpr int SPLAT_REC = 16;
hipError_t launch_emit_pairs(hipStream_t st, int64_t n, const fs_projected& proj, const uint32_t* offsets,
                             int tiles_x, uint64_t* keys, uint32_t* vals, float* splats);

constexpr int RADIX_BLOCK_KEYS = 2048;  // keys ranked by one workgroup per pass
constexpr int RADIX_BITS = 9;            // widest digit
constexpr int RADIX_DIGITS = 1 << RADIX_BITS;
inline int64_t radix_num_blocks(int64_t P) { return (P + RADIX_BLOCK_KEYS - 1) / RADIX_BLOCK_KEYS; }
// Stable LSD sort of P (key,val) pairs on key bits [0,total_bits). Result ends in *keys_out/*vals_out,
// which point into one of the two ping-pong buffers. hist: RADIX_DIGITS*radix_num_blocks(P) uint32.
hipError_t launch_radix_sort(hipStream_t st, int64_t P, int total_bits, uint64_t* keys[2], uint32_t* vals[2],
                             uint32_t* hist, void* scan_tmp, uint64_t* scan_total_dev, int* result_index);

// ranges [num_tiles,2] and tile_order [num_tiles] (tiles by decreasing list length)
hipError_t launch_tile_ranges(hipStream_t st, int64_t P, const uint64_t* keys_sorted, int num_tiles,
                              uint32_t* ranges, uint32_t* tile_order);

hipError_t launch_render_fwd(hipStream_t st, const CamDev& cam, const CfgDev& cfg, const uint32_t* ranges,
                             const uint32_t* tile_order, const uint32_t* gauss_sorted, const float* splats, float* image, float* final_T,
                             uint32_t* n_contrib);

hipError_t launch_render_bwd(hipStream_t st, const CamDev& cam, const CfgDev& cfg, const uint32_t* ranges,
                             const uint32_t* tile_order, const uint32_t* gauss_sorted, const float* splats, const float* final_T,
                             const uint32_t* n_contrib, const float* dL_dimage, float* pair_grad);

hipError_t launch_score(hipStream_t st, const CamDev& cam, const CfgDev& cfg, const uint32_t* ranges,
                        const uint32_t* tile_order, const uint32_t* gauss_sorted, const float* splats, const uint32_t* n_contrib,
                        const uint8_t* mask, int32_t* counts);

hipError_t launch_l1_grad(hipStream_t st, const float* image, const float* target, int64_t count,
                          float* dL, double* partial /* >= l1_partials() doubles */, double* loss_out);
int l1_partials();

// err: [H*W] floats, partial: >= 4*mask_partials() doubles
hipError_t launch_error_mask(hipStream_t st, const float* image, const float* target, int64_t pixels, int rule,
                             float k, float* err, double* partial, uint8_t* mask, float* thr_out);
int mask_partials();

hipError_t launch_fill_u32(hipStream_t st, uint32_t* p, uint32_t v, int64_t count);

}  // namespace fs
