"""Seeded synthetic scenes shaped like the five benchmark workloads.

This module only DRAWS inputs (Gaussian parameters, cameras, target images).
It holds none of the rasterizer's arithmetic: both the CPU oracle's tests and
the HIP path's tests/bench consume the arrays it returns, so neither side has to
reproduce a random-number stream.  Everything is numpy, float32 on output.

Draw order inside every recipe is fixed (documented per function) so a seed
names one scene forever.  Seeds: BASE_SEED + cfg for the scene, BASE_SEED + cfg
+ 500 + view for the target image of a view.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List

import numpy as np

BASE_SEED = 251104000
_Y00 = 0.28209479177387814  # value of the constant (degree-0) real SH basis function


@dataclass
class Camera:
    """Pinhole camera.  x_cam = R @ x_world + t ; pixel = (fx*x/z + cx, fy*y/z + cy)."""
    width: int
    height: int
    fx: float
    fy: float
    cx: float
    cy: float
    R: np.ndarray = field(default_factory=lambda: np.eye(3, dtype=np.float32))
    t: np.ndarray = field(default_factory=lambda: np.zeros(3, dtype=np.float32))


@dataclass
class Scene:
    name: str
    sh_degree: int
    means: np.ndarray      # [n,3] world space
    scales: np.ndarray     # [n,3] activated (>0)
    quats: np.ndarray      # [n,4] unit (w,x,y,z)
    opacities: np.ndarray  # [n]   activated, in (0,1)
    sh: np.ndarray         # [n,(deg+1)^2,3]
    cameras: List[Camera]
    seed: int

    @property
    def n(self) -> int:
        return int(self.means.shape[0])


def _sigmoid(x):
    return 1.0 / (1.0 + np.exp(-x))


def _unit_quats(rng, n):
    q = rng.standard_normal((n, 4))
    q /= np.linalg.norm(q, axis=1, keepdims=True)
    return q


def _rand_rot(rng):
    q = _unit_quats(rng, 1)[0]
    w, x, y, z = q
    return np.array([
        [1 - 2 * (y * y + z * z), 2 * (x * y - w * z), 2 * (x * z + w * y)],
        [2 * (x * y + w * z), 1 - 2 * (x * x + z * z), 2 * (y * z - w * x)],
        [2 * (x * z - w * y), 2 * (y * z + w * x), 1 - 2 * (x * x + y * y)]])


def _sh_deg3(rng, n, dc_std=0.5, band_std=0.05):
    sh = np.empty((n, 16, 3))
    sh[:, 0, :] = rng.normal(0.0, dc_std, (n, 3))
    sh[:, 1:, :] = rng.normal(0.0, band_std, (n, 15, 3))
    return sh


def _cluster_mixture(rng, n, centres, depth_scale, std_lo, std_hi):
    """Draw n points from an equal-weight mixture of anisotropic 3D Gaussian clusters.

    Cluster k has principal standard deviations depth_scale[k] * U[std_lo,std_hi]
    (one draw per axis) in a random orientation.  Draw order: per cluster
    (axis stds, rotation); then assignment; then standard normals."""
    k = centres.shape[0]
    stds = np.empty((k, 3))
    rots = np.empty((k, 3, 3))
    for c in range(k):
        stds[c] = depth_scale[c] * rng.uniform(std_lo, std_hi, 3)
        rots[c] = _rand_rot(rng)
    assign = rng.integers(0, k, n)
    z = rng.standard_normal((n, 3)) * stds[assign]
    pts = np.einsum('nij,nj->ni', rots[assign], z) + centres[assign]
    return pts


def _frustum_dirs(rng, k, width, height, fx, fy, widen):
    """Unit directions whose pinhole projection falls in the image widened by `widen`."""
    u = rng.uniform(-1.0, 1.0, k) * widen * 0.5 * width / fx
    v = rng.uniform(-1.0, 1.0, k) * widen * 0.5 * height / fy
    d = np.stack([u, v, np.ones(k)], axis=1)
    return d / np.linalg.norm(d, axis=1, keepdims=True)


def _finish(name, cfg, deg, means, log_scales, quats, opac, sh, cams):
    f32 = np.float32
    return Scene(name=name, sh_degree=deg,
                 means=np.ascontiguousarray(means, f32),
                 scales=np.ascontiguousarray(np.exp(log_scales), f32),
                 quats=np.ascontiguousarray(quats, f32),
                 opacities=np.ascontiguousarray(opac, f32),
                 sh=np.ascontiguousarray(sh, f32),
                 cameras=cams, seed=BASE_SEED + cfg)


def config1(n: int = 4096) -> Scene:
    """4,096 Gaussians, SH degree 0, one 128x128 camera (fx=fy=128, centred).
    Draw order: x,y ; z ; log-scales ; quats ; opacity logits ; rgb."""
    rng = np.random.default_rng(BASE_SEED + 1)
    xy = rng.uniform(-1.0, 1.0, (n, 2))
    z = rng.uniform(2.0, 6.0, (n, 1))
    ls = rng.normal(-3.5, 0.3, (n, 3))
    q = _unit_quats(rng, n)
    op = _sigmoid(rng.normal(0.0, 1.0, n))
    rgb = rng.uniform(0.0, 1.0, (n, 3))
    sh = ((rgb - 0.5) / _Y00)[:, None, :]
    cam = Camera(128, 128, 128.0, 128.0, 64.0, 64.0)
    return _finish("cfg1_4k_sh0_128x128", 1, 0, np.concatenate([xy, z], 1), ls, q, op, sh, [cam])


def config2(n: int = 100_000) -> Scene:
    """100k Gaussians, SH degree 3, one 980x545 camera (fx=fy=0.8*width).
    32 clusters inside the frustum at depth U[2,20]; cluster std proportional to depth.
    Draw order: cluster dirs ; depths ; clusters ; log-scales ; quats ; opacity ; SH."""
    W, H = 980, 545
    fx = 0.8 * W
    rng = np.random.default_rng(BASE_SEED + 2)
    k = 32
    dirs = _frustum_dirs(rng, k, W, H, fx, fx, 0.9)
    depth = rng.uniform(2.0, 20.0, k)
    centres = dirs * (depth / dirs[:, 2])[:, None]
    means = _cluster_mixture(rng, n, centres, depth, 0.02, 0.12)
    ls = rng.normal(-4.0, 0.5, (n, 3))
    q = _unit_quats(rng, n)
    op = _sigmoid(rng.normal(0.0, 1.5, n))
    sh = _sh_deg3(rng, n)
    cam = Camera(W, H, fx, fx, W / 2.0, H / 2.0)
    return _finish("cfg2_100k_sh3_980x545", 2, 3, means, ls, q, op, sh, [cam])


def config3(n: int = 500_000) -> Scene:
    """500k Gaussians, SH degree 3, one 1600x1064 camera (fx=fy=1280).
    64 clusters on a shell of radius U[5,30] around the camera, directions inside the
    frustum widened x1.2 (so culling is exercised); log-scales N(-4.5,0.7)."""
    W, H = 1600, 1064
    fx = 0.8 * W
    rng = np.random.default_rng(BASE_SEED + 3)
    k = 64
    dirs = _frustum_dirs(rng, k, W, H, fx, fx, 1.2)
    radius = rng.uniform(5.0, 30.0, k)
    centres = dirs * radius[:, None]
    means = _cluster_mixture(rng, n, centres, radius, 0.02, 0.12)
    ls = rng.normal(-4.5, 0.7, (n, 3))
    q = _unit_quats(rng, n)
    op = _sigmoid(rng.normal(0.0, 1.5, n))
    sh = _sh_deg3(rng, n)
    cam = Camera(W, H, fx, fx, W / 2.0, H / 2.0)
    return _finish("cfg3_500k_sh3_1600x1064", 3, 3, means, ls, q, op, sh, [cam])


def _look_at(eye, target, up):
    """World->camera rotation/translation with +z forward, +x right, +y down-image."""
    fwd = target - eye
    fwd = fwd / np.linalg.norm(fwd)
    right = np.cross(fwd, up)
    right = right / np.linalg.norm(right)
    down = np.cross(fwd, right)
    R = np.stack([right, down, fwd], axis=0)
    t = -R @ eye
    return R.astype(np.float32), t.astype(np.float32)


def config4(n: int = 300_000, views: int = 10) -> Scene:
    """300k Gaussians, SH degree 3, `views` cameras 1332x876 (fx=fy=0.8*width) on a
    horizontal 30-degree arc (-15..+15 deg inclusive) at distance 8 from the scene
    centroid, looking at it.  48 clusters of extent ~3 around the origin."""
    W, H = 1332, 876
    fx = 0.8 * W
    rng = np.random.default_rng(BASE_SEED + 4)
    k = 48
    centres = rng.normal(0.0, 1.0, (k, 3)) * np.array([1.5, 1.0, 1.5])
    means = _cluster_mixture(rng, n, centres, np.full(k, 3.0), 0.03, 0.15)
    ls = rng.normal(-4.0, 0.5, (n, 3))
    q = _unit_quats(rng, n)
    op = _sigmoid(rng.normal(0.0, 1.5, n))
    sh = _sh_deg3(rng, n)
    centroid = means.mean(axis=0)
    cams = []
    for ang in np.linspace(-15.0, 15.0, views):
        a = np.deg2rad(ang)
        eye = centroid + 8.0 * np.array([np.sin(a), 0.0, -np.cos(a)])
        R, t = _look_at(eye, centroid, np.array([0.0, -1.0, 0.0]))
        cams.append(Camera(W, H, fx, fx, W / 2.0, H / 2.0, R, t))
    return _finish("cfg4_300k_sh3_10x1332x876", 4, 3, means, ls, q, op, sh, cams)


def config5(n: int = 3_000_000, scale_sigma: float = 0.8) -> Scene:
    """3M Gaussians, SH degree 3, one 1920x1080 camera (fx=fy=1536).  256 clusters at
    depth U[1,50] inside the frustum widened x1.2; log-scales N(-5,0.8) (10.0 M pairs).
    `scale_sigma` = 1.2 is the wide-tail variant whose pair count reaches 27 M (same draws,
    the standard normal of the log-scale multiplied by 1.2 instead of 0.8)."""
    W, H = 1920, 1080
    fx = 0.8 * W
    rng = np.random.default_rng(BASE_SEED + 5)
    k = 256
    dirs = _frustum_dirs(rng, k, W, H, fx, fx, 1.2)
    depth = rng.uniform(1.0, 50.0, k)
    centres = dirs * (depth / dirs[:, 2])[:, None]
    means = _cluster_mixture(rng, n, centres, depth, 0.02, 0.12)
    ls = -5.0 + scale_sigma * ((rng.normal(-5.0, 0.8, (n, 3)) + 5.0) / 0.8)
    q = _unit_quats(rng, n)
    op = _sigmoid(rng.normal(0.0, 1.5, n))
    sh = _sh_deg3(rng, n)
    cam = Camera(W, H, fx, fx, W / 2.0, H / 2.0)
    return _finish("cfg5_3m_sh3_1920x1080", 5, 3, means, ls, q, op, sh, [cam])


CONFIGS = {1: config1, 2: config2, 3: config3, 4: config4, 5: config5}


def make_scene(cfg: int, n: int | None = None, **kw) -> Scene:
    """Scene for benchmark config `cfg` (1..5); `n` overrides the Gaussian count
    (same recipe and seed, fewer or more draws) for scaled-down parity cases."""
    fn = CONFIGS[cfg]
    return fn(**kw) if n is None else fn(n, **kw)


def target_image(cfg: int, view: int, cam: Camera) -> np.ndarray:
    """Seeded U[0,1] target image, planar [3,H,W] float32."""
    rng = np.random.default_rng(BASE_SEED + cfg + 500 + view)
    return rng.uniform(0.0, 1.0, (3, cam.height, cam.width)).astype(np.float32)


def tiny_scene(seed: int, n: int, width: int, height: int, sh_degree: int = 3,
               depth=(2.0, 6.0), log_scale=(-2.5, 0.3), spread: float = 0.6) -> Scene:
    """Small free-form scene for unit tests and finite differences (float64 kept by
    the caller if needed: arrays are returned as float32 like the rest)."""
    rng = np.random.default_rng(seed)
    fx = 0.8 * max(width, height)
    z = rng.uniform(depth[0], depth[1], (n, 1))
    xy = rng.uniform(-spread, spread, (n, 2)) * z * np.array([0.5 * width / fx, 0.5 * height / fx])
    ls = rng.normal(log_scale[0], log_scale[1], (n, 3))
    q = _unit_quats(rng, n)
    op = _sigmoid(rng.normal(0.0, 1.0, n))
    k = (sh_degree + 1) ** 2
    sh = np.empty((n, k, 3))
    sh[:, 0, :] = rng.normal(0.5, 0.5, (n, 3))
    if k > 1:
        sh[:, 1:, :] = rng.normal(0.0, 0.2, (n, k - 1, 3))
    R = _rand_rot(np.random.default_rng(seed + 7))
    # small rotation about a random axis so R is not the identity but the scene stays in view
    A = 0.15 * (R - R.T) / 2
    Rm = np.eye(3) + A + A @ A / 2
    U, _, Vt = np.linalg.svd(Rm)
    Rc = (U @ Vt)
    t0 = np.array([0.05, -0.03, 0.1])
    means_cam = np.concatenate([xy, z], 1)
    means = (means_cam - t0) @ Rc  # world = Rc^T (cam - t)
    cam = Camera(width, height, fx, fx, width / 2.0, height / 2.0,
                 Rc.astype(np.float32), t0.astype(np.float32))
    sc = _finish(f"tiny_{seed}", 0, sh_degree, means, ls, q, op, sh, [cam])
    sc.seed = seed
    return sc
