"""TEST INFRASTRUCTURE -- not part of the product.

numpy front end of the plain-C CPU oracle (fastgs_oracle.c).  Only tests, the smoke check
and the benchmark's CPU-baseline leg may import this package; the HIP path never does.

`Oracle(np.float32)` is the pinned-operation-order build used for parity with the GPU;
`Oracle(np.float64)` is the build used for finite differences and closed forms.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fastgs_oracle.c")
_LIB = os.path.join(_HERE, "libfastgs_oracle.so")


def _cpu_has_fma() -> bool:
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("flags"):
                    return " fma" in line
    except OSError:
        pass
    return False


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no contraction).  Returns the .so path."""
    deps = [_SRC, os.path.join(_HERE, "fastgs_oracle_impl.h")]
    if (not force and os.path.exists(_LIB)
            and all(os.path.getmtime(_LIB) >= os.path.getmtime(d) for d in deps)):
        return _LIB
    cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
           "-Wall", "-Wno-unused-function", "-o", _LIB, _SRC, "-lm"]
    if _cpu_has_fma():
        cmd.insert(1, "-mfma")
    subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.orc_exclusive_scan.restype = ctypes.c_uint64
        _lib.orc_emit_pairs.restype = ctypes.c_uint64
        _lib.orc_pairs_bruteforce.restype = ctypes.c_uint64
        _lib.orc_exp_neg_f32.restype = ctypes.c_float
        _lib.orc_exp_neg_f32.argtypes = [ctypes.c_float]
        _lib.orc_log_c_f32.restype = ctypes.c_float
        _lib.orc_log_c_f32.argtypes = [ctypes.c_float]
        for sfx, ct in (("_f32", ctypes.c_float), ("_f64", ctypes.c_double)):
            getattr(_lib, "orc_l1" + sfx).restype = ctypes.c_double
            getattr(_lib, "orc_error_mask" + sfx).restype = ct
            getattr(_lib, "orc_count_evals" + sfx).restype = ctypes.c_int64
            getattr(_lib, "orc_emit_pairs_cb" + sfx).restype = ctypes.c_uint64
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


@dataclass
class Config:
    """Blending / projection conventions the paper leaves open (see the design notes)."""
    tile: int = 16
    z_near: float = 0.2
    lowpass: float = 0.3
    alpha_min: float = 1.0 / 255.0
    alpha_max: float = 0.99
    T_min: float = 1e-4
    bg: tuple = (0.0, 0.0, 0.0)
    jclamp: float = 1.3
    score_mode: int = 0  # 0 = WEIGHT (alpha*T > alpha_min), 1 = ALPHA
    compact_box: bool = False  # pairs from the exact ellipse-tile test of the Compact Box instead of the 3-sigma square
    cb_beta: float = 1.0

    def array(self, dtype):
        # fp32 build: constants are the fp32 roundings (1/255 computed in fp32 division)
        if dtype == np.float32:
            amin = np.float32(self.alpha_min)
            if self.alpha_min == 1.0 / 255.0:
                amin = np.float32(1.0) / np.float32(255.0)
        else:
            amin = self.alpha_min
        return np.array([self.z_near, self.lowpass, amin, self.alpha_max, self.T_min,
                         self.bg[0], self.bg[1], self.bg[2], self.jclamp, 1.0 if self.compact_box else 0.0,
                         self.cb_beta], dtype=dtype)


def cam_array(cam, dtype):
    return np.concatenate([[cam.fx, cam.fy, cam.cx, cam.cy],
                           np.asarray(cam.R, dtype=np.float64).reshape(9),
                           np.asarray(cam.t, dtype=np.float64).reshape(3)]).astype(dtype)


@dataclass
class Projected:
    mean2d: np.ndarray
    depth: np.ndarray
    conic_opacity: np.ndarray
    rgb: np.ndarray
    rect: np.ndarray          # int32 [n,4] x0,y0,x1,y1 (tiles, half-open)
    tiles_touched: np.ndarray  # uint32 [n]
    clamped: np.ndarray       # uint8 [n,3]
    radius: np.ndarray        # int32 [n]


@dataclass
class Bins:
    num_pairs: int
    keys_sorted: np.ndarray   # uint64 [P]
    gauss_sorted: np.ndarray  # uint32 [P]
    tile_ranges: np.ndarray   # uint32 [T,2]
    keys_unsorted: np.ndarray
    gauss_unsorted: np.ndarray
    offsets: np.ndarray


class Oracle:
    def __init__(self, dtype=np.float32, config: Config | None = None):
        self.dtype = np.dtype(dtype).type
        assert self.dtype in (np.float32, np.float64)
        self.sfx = "_f32" if self.dtype == np.float32 else "_f64"
        self.cfg = config or Config()
        self.L = lib()

    # -- helpers ---------------------------------------------------------------------
    def _f(self, name):
        return getattr(self.L, name + self.sfx)

    def _a(self, x):
        return np.ascontiguousarray(x, dtype=self.dtype)

    def _tiles(self, cam):
        t = self.cfg.tile
        return (cam.width + t - 1) // t, (cam.height + t - 1) // t

    @staticmethod
    def _tl(tile_list):
        if tile_list is None:
            return None, 0
        tl = np.ascontiguousarray(tile_list, dtype=np.int32)
        return tl, int(tl.size)

    # -- a1 --------------------------------------------------------------------------
    def preprocess(self, sc, cam) -> Projected:
        n, dt = sc.n, self.dtype
        out = Projected(np.zeros((n, 2), dt), np.zeros(n, dt), np.zeros((n, 4), dt), np.zeros((n, 3), dt),
                        np.zeros((n, 4), np.int32), np.zeros(n, np.uint32), np.zeros((n, 3), np.uint8),
                        np.zeros(n, np.int32))
        self._f("orc_preprocess")(
            ctypes.c_int64(n), ctypes.c_int(sc.sh_degree), _p(self._a(sc.means)), _p(self._a(sc.scales)),
            _p(self._a(sc.quats)), _p(self._a(sc.opacities)), _p(self._a(sc.sh)),
            ctypes.c_int(cam.width), ctypes.c_int(cam.height), _p(cam_array(cam, dt)),
            _p(self.cfg.array(dt)), ctypes.c_int(self.cfg.tile),
            _p(out.mean2d), _p(out.depth), _p(out.conic_opacity), _p(out.rgb), _p(out.rect),
            _p(out.tiles_touched), _p(out.clamped), _p(out.radius))
        return out

    # -- a2..a5 ----------------------------------------------------------------------
    def bin_sort(self, proj: Projected, cam) -> Bins:
        n = proj.depth.shape[0]
        TX, TY = self._tiles(cam)
        offsets = np.zeros(n, np.uint64)
        P = int(self.L.orc_exclusive_scan(ctypes.c_int64(n), _p(proj.tiles_touched), _p(offsets)))
        depth32 = np.ascontiguousarray(proj.depth, dtype=np.float32)
        keys = np.zeros(max(P, 1), np.uint64)
        vals = np.zeros(max(P, 1), np.uint32)
        if self.cfg.compact_box:
            P2 = int(self._f("orc_emit_pairs_cb")(
                ctypes.c_int64(n), _p(proj.rect), _p(depth32.view(np.uint32)), _p(self._a(proj.mean2d)),
                _p(self._a(proj.conic_opacity)), _p(self.cfg.array(self.dtype)), ctypes.c_int(TX),
                ctypes.c_int(self.cfg.tile), _p(keys), _p(vals)))
        else:
            P2 = int(self.L.orc_emit_pairs(ctypes.c_int64(n), _p(proj.rect), _p(depth32), ctypes.c_int(TX),
                                           _p(keys), _p(vals)))
        assert P2 == P
        keys, vals = keys[:P], vals[:P]
        ks, vs = keys.copy(), vals.copy()
        self.L.orc_sort_pairs(ctypes.c_uint64(P), _p(ks), _p(vs))
        ranges = np.zeros((TX * TY, 2), np.uint32)
        self.L.orc_tile_ranges(ctypes.c_uint64(P), _p(ks), ctypes.c_int(TX * TY), _p(ranges))
        return Bins(P, ks, vs, ranges, keys, vals, offsets)

    def pairs_bruteforce(self, proj: Projected, cam):
        n = proj.depth.shape[0]
        TX, TY = self._tiles(cam)
        hit = np.zeros((n, TY * TX), np.uint8)
        m2 = np.ascontiguousarray(proj.mean2d, dtype=np.float32)
        tot = int(self.L.orc_pairs_bruteforce(ctypes.c_int64(n), _p(m2), _p(proj.radius), ctypes.c_int(cam.width),
                                              ctypes.c_int(cam.height), ctypes.c_int(self.cfg.tile), _p(hit)))
        return tot, hit

    # -- a6 --------------------------------------------------------------------------
    def render_fwd(self, proj: Projected, bins: Bins, cam, tile_list=None, out=None):
        H, W, dt = cam.height, cam.width, self.dtype
        if out is None:
            out = (np.zeros((3, H, W), dt), np.ones((H, W), dt), np.zeros((H, W), np.uint32))
        image, final_T, n_contrib = out
        tl, ntl = self._tl(tile_list)
        self._f("orc_render_fwd")(
            _p(proj.mean2d), _p(proj.conic_opacity), _p(proj.rgb), _p(bins.gauss_sorted), _p(bins.tile_ranges),
            ctypes.c_int(W), ctypes.c_int(H), _p(self.cfg.array(dt)), ctypes.c_int(self.cfg.tile),
            _p(tl), ctypes.c_int(ntl), _p(image), _p(final_T), _p(n_contrib))
        return image, final_T, n_contrib

    def count_evals(self, proj, bins, cam, tile_list=None) -> int:
        tl, ntl = self._tl(tile_list)
        return int(self._f("orc_count_evals")(
            _p(proj.mean2d), _p(proj.conic_opacity), _p(bins.gauss_sorted), _p(bins.tile_ranges),
            ctypes.c_int(cam.width), ctypes.c_int(cam.height), _p(self.cfg.array(self.dtype)),
            ctypes.c_int(self.cfg.tile), _p(tl), ctypes.c_int(ntl)))

    # -- a7 --------------------------------------------------------------------------
    def l1(self, image, target):
        H, W = image.shape[1:]
        g = np.zeros_like(image)
        loss = float(self._f("orc_l1")(_p(self._a(image)), _p(self._a(target)), ctypes.c_int(W),
                                       ctypes.c_int(H), _p(g)))
        return loss, g

    # -- a8 --------------------------------------------------------------------------
    def render_bwd(self, proj: Projected, bins: Bins, cam, dL_dimage, tile_list=None):
        n, dt = proj.depth.shape[0], self.dtype
        d_mean2d = np.zeros((n, 2)); d_conic = np.zeros((n, 3)); d_op = np.zeros(n); d_rgb = np.zeros((n, 3))
        d_abs = np.zeros((n, 2))
        tl, ntl = self._tl(tile_list)
        self._f("orc_render_bwd")(
            _p(proj.mean2d), _p(proj.conic_opacity), _p(proj.rgb), _p(bins.gauss_sorted), _p(bins.tile_ranges),
            ctypes.c_int(cam.width), ctypes.c_int(cam.height), _p(self.cfg.array(dt)),
            ctypes.c_int(self.cfg.tile), _p(tl), ctypes.c_int(ntl), _p(self._a(dL_dimage)),
            _p(d_mean2d), _p(d_conic), _p(d_op), _p(d_rgb), _p(d_abs))
        return d_mean2d, d_conic, d_op, d_rgb, d_abs

    # -- a9 --------------------------------------------------------------------------
    def preprocess_bwd(self, sc, cam, d_mean2d, d_conic, d_opacity, d_rgb):
        n, dt = sc.n, self.dtype
        K = (sc.sh_degree + 1) ** 2
        g = dict(means=np.zeros((n, 3)), scales=np.zeros((n, 3)), quats=np.zeros((n, 4)),
                 opacities=np.zeros(n), sh=np.zeros((n, K, 3)))
        c = lambda a: np.ascontiguousarray(a, dtype=np.float64)
        self._f("orc_preprocess_bwd")(
            ctypes.c_int64(n), ctypes.c_int(sc.sh_degree), _p(self._a(sc.means)), _p(self._a(sc.scales)),
            _p(self._a(sc.quats)), _p(self._a(sc.opacities)), _p(self._a(sc.sh)), ctypes.c_int(cam.width),
            ctypes.c_int(cam.height), _p(cam_array(cam, dt)), _p(self.cfg.array(dt)), ctypes.c_int(self.cfg.tile),
            _p(c(d_mean2d)), _p(c(d_conic)), _p(c(d_opacity)), _p(c(d_rgb)),
            _p(g["means"]), _p(g["scales"]), _p(g["quats"]), _p(g["opacities"]), _p(g["sh"]))
        return g

    # -- a10 -------------------------------------------------------------------------
    def error_mask(self, image, target, rule=0, k=1.0):
        H, W = image.shape[1:]
        mask = np.zeros((H, W), np.uint8)
        err = np.zeros((H, W), self.dtype)
        thr = self._f("orc_error_mask")(_p(self._a(image)), _p(self._a(target)), ctypes.c_int(W), ctypes.c_int(H),
                                        ctypes.c_int(rule), self._ct(k), _p(mask), _p(err))
        return mask, self.dtype(thr), err

    def _ct(self, v):
        return ctypes.c_float(v) if self.dtype == np.float32 else ctypes.c_double(v)

    # -- a11 -------------------------------------------------------------------------
    def score(self, proj, bins, cam, mask, counts, tile_list=None):
        tl, ntl = self._tl(tile_list)
        assert counts.dtype == np.int32 and mask.dtype == np.uint8
        self._f("orc_score")(
            _p(proj.mean2d), _p(proj.conic_opacity), _p(bins.gauss_sorted), _p(bins.tile_ranges),
            ctypes.c_int(cam.width), ctypes.c_int(cam.height), _p(self.cfg.array(self.dtype)),
            ctypes.c_int(self.cfg.tile), ctypes.c_int(self.cfg.score_mode), _p(np.ascontiguousarray(mask)),
            _p(tl), ctypes.c_int(ntl), _p(counts))
        return counts

    # -- test-harness convenience: the same single-threaded routines called from several Python
    #    threads on disjoint tile subsets (ctypes releases the GIL).  Forward outputs are disjoint
    #    per tile; accumulated outputs get one private array per thread, added up in thread order.
    def _split(self, cam, tile_list, threads):
        TX, TY = self._tiles(cam)
        tl = np.arange(TX * TY, dtype=np.int32) if tile_list is None else np.asarray(tile_list, np.int32)
        return [tl[k::threads] for k in range(threads) if tl[k::threads].size]

    def render_fwd_mt(self, proj, bins, cam, tile_list=None, threads=8):
        from concurrent.futures import ThreadPoolExecutor
        H, W, dt = cam.height, cam.width, self.dtype
        out = (np.zeros((3, H, W), dt), np.ones((H, W), dt), np.zeros((H, W), np.uint32))
        parts = self._split(cam, tile_list, threads)
        with ThreadPoolExecutor(len(parts) or 1) as ex:
            list(ex.map(lambda tl: self.render_fwd(proj, bins, cam, tl, out), parts))
        return out

    def render_bwd_mt(self, proj, bins, cam, dL_dimage, tile_list=None, threads=8):
        from concurrent.futures import ThreadPoolExecutor
        parts = self._split(cam, tile_list, threads)
        with ThreadPoolExecutor(len(parts) or 1) as ex:
            res = list(ex.map(lambda tl: self.render_bwd(proj, bins, cam, dL_dimage, tl), parts))
        if not res:
            return self.render_bwd(proj, bins, cam, dL_dimage, np.zeros(0, np.int32))
        acc = [a.copy() for a in res[0]]
        for r in res[1:]:
            for a, b in zip(acc, r):
                a += b
        return tuple(acc)

    def score_mt(self, proj, bins, cam, mask, counts, tile_list=None, threads=8):
        from concurrent.futures import ThreadPoolExecutor
        parts = self._split(cam, tile_list, threads)
        with ThreadPoolExecutor(len(parts) or 1) as ex:
            res = list(ex.map(lambda tl: self.score(proj, bins, cam, mask, np.zeros_like(counts), tl), parts))
        for r in res:
            counts += r
        return counts

    def backward_mt(self, sc, cam, proj, bins, dL_dimage, tile_list=None, threads=8):
        d2 = self.render_bwd_mt(proj, bins, cam, dL_dimage, tile_list, threads)
        g = self.preprocess_bwd(sc, cam, *d2[:4])
        g["mean2d"], g["conic"], g["rgb"], g["mean2d_abs"] = d2[0], d2[1], d2[3], d2[4]
        return g

    # -- whole path (used by finite differences and by the timed CPU baseline) ---------
    def forward(self, sc, cam):
        proj = self.preprocess(sc, cam)
        bins = self.bin_sort(proj, cam)
        image, final_T, n_contrib = self.render_fwd(proj, bins, cam)
        return proj, bins, image, final_T, n_contrib

    def backward(self, sc, cam, proj, bins, dL_dimage, tile_list=None):
        d2 = self.render_bwd(proj, bins, cam, dL_dimage, tile_list)
        g = self.preprocess_bwd(sc, cam, *d2[:4])
        g["mean2d"] = d2[0]
        g["conic"] = d2[1]
        g["rgb"] = d2[3]
        g["mean2d_abs"] = d2[4]
        return g


# ---- photometric loss (Sec. 4.3, Sec. 4.5) and pruning score (Sec. 4.3) --------------------------
def ssim(image, target, want_grad=False, threads=1):
    """Mean SSIM of `image` against `target` ([C,H,W]), the SSIM map, and d mean / d image (or None).
    Double precision whatever the inputs' type.  threads > 1 runs the channels side by side (test
    harness convenience; each channel is the same single-threaded routine)."""
    L = lib()
    L.orc_ssim.restype = ctypes.c_double
    x = np.ascontiguousarray(image, dtype=np.float64)
    y = np.ascontiguousarray(target, dtype=np.float64)
    C, H, W = x.shape
    smap = np.zeros((C, H, W))
    grad = np.zeros((C, H, W)) if want_grad else None
    if threads <= 1 or C == 1:
        mean = float(L.orc_ssim(ctypes.c_int(C), ctypes.c_int(H), ctypes.c_int(W), _p(x), _p(y), _p(smap), _p(grad)))
        return mean, smap, grad
    import threading
    means = [0.0] * C

    def work(c):
        g = grad[c:c + 1] if want_grad else None
        means[c] = float(L.orc_ssim(ctypes.c_int(1), ctypes.c_int(H), ctypes.c_int(W), _p(x[c:c + 1]), _p(y[c:c + 1]),
                                    _p(smap[c:c + 1]), _p(g)))
    ts = [threading.Thread(target=work, args=(c,)) for c in range(C)]
    [t.start() for t in ts]
    [t.join() for t in ts]
    if want_grad:
        grad /= C
    return float(sum(means) / C), smap, grad


def photometric(image, target, lam=0.2, want_grad=True, threads=1):
    """E = (1 - lam) * L1 + lam * (1 - SSIM) over the whole image, and dE / d image."""
    x = np.ascontiguousarray(image, dtype=np.float64)
    y = np.ascontiguousarray(target, dtype=np.float64)
    l1 = float(np.abs(x - y).mean())
    s, _, g = ssim(x, y, want_grad=want_grad, threads=threads)
    out = dict(L1=l1, ssim=s, E=(1.0 - lam) * l1 + lam * (1.0 - s))
    if want_grad:
        out["grad"] = (1.0 - lam) * np.sign(x - y) / x.size - lam * g
    return out


def prune_score(counts, E):
    """s_p = N(sum_j counts[j, i] * E[j]) with N the min-max normalisation over the Gaussians;
    returns (raw sums, s_p)."""
    L = lib()
    c = np.ascontiguousarray(counts, dtype=np.int32)
    K, n = c.shape
    e = np.ascontiguousarray(E, dtype=np.float64)
    raw = np.zeros(n)
    sp = np.zeros(n)
    L.orc_prune_score(ctypes.c_int(K), ctypes.c_int64(n), _p(c), _p(e), _p(raw), _p(sp))
    return raw, sp


# ---- densification / pruning decisions (Sec. 4.2, Sec. 4.3, supplement "Implementation Details") ---
def densify_accumulate(dmean2d, dmean2d_abs, tiles_touched, grad_accum, abs_accum, denom):
    """Per training view: add the Euclidean norms of the positional gradient (and of the absolute one) of
    every Gaussian visible in the view to the running sums; count the view.  In place, in the arrays' type."""
    vis = np.asarray(tiles_touched) > 0
    dt = grad_accum.dtype
    g = np.asarray(dmean2d, dt)
    grad_accum[vis] = grad_accum[vis] + np.sqrt(g[vis, 0] * g[vis, 0] + g[vis, 1] * g[vis, 1])
    if dmean2d_abs is not None:
        a = np.asarray(dmean2d_abs, dt)
        abs_accum[vis] = abs_accum[vis] + np.sqrt(a[vis, 0] * a[vis, 0] + a[vis, 1] * a[vis, 1])
    denom[vis] += 1


def densify_prune_masks(grad_norm, grad_abs_norm, denom, counts, K, max_scale, opacity, s_p, *, tau_grad, tau_abs,
                        tau_d=5.0, size_limit, min_opacity=0.1, tau_p=0.9, dtype=np.float64):
    """The selection rules as the paper states them, per Gaussian:
      clone  : mean positional-gradient norm >= tau_grad, largest scale <= size_limit, and s_d > tau_d
      split  : mean ABSOLUTE positional-gradient norm >= tau_abs, largest scale > size_limit, and s_d > tau_d
      prune  : opacity < min_opacity, or s_p > tau_p
    grad_norm / grad_abs_norm are sums over `denom` iterations of the per-iteration norms; s_d = counts / K.
    The gradient thresholds and the size limit follow vanilla 3DGS ("we follow 3DGS ... gradient for
    cloning, ... absolute gradient ... for splitting"); their values are the caller's.  All divisions and
    comparisons are made in `dtype` (IEEE, correctly rounded).  Returns uint8 masks."""
    f = lambda v: np.asarray(v, dtype=dtype)
    d = np.maximum(f(denom), dtype(1))
    g = f(grad_norm) / d
    ga = f(grad_abs_norm) / d
    s_d = f(counts) / dtype(K)
    important = s_d > dtype(tau_d)
    big = f(max_scale) > dtype(size_limit)
    clone = (g >= dtype(tau_grad)) & ~big & important
    split = (ga >= dtype(tau_abs)) & big & important
    prune = (f(opacity) < dtype(min_opacity)) | (f(s_p) > dtype(tau_p))
    return clone.astype(np.uint8), split.astype(np.uint8), prune.astype(np.uint8)


# ---- optimiser (Sec. 5.1: Adam; supplement "Implementation Details": the 32/64 schedule) -------------
def adam_step(param, grad, m, v, step, lr, beta1=0.9, beta2=0.999, eps=1e-15, grad_scale=1.0):
    """One Adam update (Kingma & Ba, Algorithm 1, with bias correction), in place, in the arrays' type:
         g = grad_scale * grad;  m = b1 m + (1-b1) g;  v = b2 v + (1-b2) g^2;
         param -= lr * (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps),   t = step >= 1."""
    dt = param.dtype.type
    g = np.asarray(grad, param.dtype) * dt(grad_scale)
    m[...] = dt(beta1) * m + dt(1 - beta1) * g
    v[...] = dt(beta2) * v + dt(1 - beta2) * (g * g)
    mhat = m / dt(1 - beta1 ** step)
    vhat = v / dt(1 - beta2 ** step)
    param[...] = param - dt(lr) * mhat / (np.sqrt(vhat) + dt(eps))


def adam_interval(iteration):
    """Iterations between optimiser updates: every iteration before 15 000, every 32 iterations from 15 000 to
    20 000, every 64 afterwards; gradients of the iterations in between are summed."""
    return 1 if iteration < 15000 else (32 if iteration < 20000 else 64)


def activate(raw_scales, raw_quats, raw_opac):
    """Stored -> used parameters, as in vanilla 3DGS (which the paper keeps): s = exp(raw), q = raw / |raw|,
    sigma = 1 / (1 + exp(-raw))."""
    q = raw_quats / np.sqrt((raw_quats * raw_quats).sum(1, keepdims=True))
    return np.exp(raw_scales), q, 1.0 / (1.0 + np.exp(-raw_opac))


def activate_bwd(raw_scales, raw_quats, raw_opac, d_scales, d_quats, d_opac):
    """Chain rule through `activate`."""
    s, q, o = activate(raw_scales, raw_quats, raw_opac)
    nrm = np.sqrt((raw_quats * raw_quats).sum(1, keepdims=True))
    d_raw_q = (d_quats - q * (q * d_quats).sum(1, keepdims=True)) / nrm
    return d_scales * s, d_raw_q, d_opac * o * (1.0 - o)


def activate_inv(scales, opacities, lo=1e-4, hi=1.0 - 1e-4):
    """Used -> stored parameters (the inverse of `activate` for the scale and the opacity): raw scale = ln s,
    raw opacity = ln(o' / (1 - o')) with o' = the opacity limited to [lo, hi] (a stored opacity of exactly 0 or 1
    has no finite logit).  In the arrays' type."""
    o = np.minimum(np.maximum(opacities, opacities.dtype.type(lo)), opacities.dtype.type(hi))
    return np.log(scales), np.log(o / (1 - o))


def _quat_rotation(q):
    """R(q) of unit quaternions q = (w, x, y, z), [m, 3, 3]: the R_i of Sec. 3 Eq. (2)."""
    w, x, y, z = (q[:, k] for k in range(4))
    R = np.empty((q.shape[0], 3, 3), q.dtype)
    R[:, 0, 0] = 1 - 2 * (y * y + z * z); R[:, 0, 1] = 2 * (x * y - w * z); R[:, 0, 2] = 2 * (x * z + w * y)
    R[:, 1, 0] = 2 * (x * y + w * z); R[:, 1, 1] = 1 - 2 * (x * x + z * z); R[:, 1, 2] = 2 * (y * z - w * x)
    R[:, 2, 0] = 2 * (x * z - w * y); R[:, 2, 1] = 2 * (y * z + w * x); R[:, 2, 2] = 1 - 2 * (x * x + y * y)
    return R


def split_children(means, scales, quats, parents, normals, phi=1.6):
    """Splitting (supplement, "Implementation Details": the paper keeps vanilla 3DGS's densification and
    selects the Gaussians to split with the absolute gradient).  Every selected parent p is replaced by two
    children: child c is placed at a sample of the parent's own density,
        mu_c = mu_p + R(q_p) (s_p * xi_c),    xi_c ~ N(0, I_3) supplied by the caller (normals[r, c, :]),
    with scales s_p / phi (phi = 1.6 = 0.8 x the number of children in vanilla 3DGS) and the parent's rotation,
    opacity and colour.  means [n,3], scales [n,3] (activated), quats [n,4] (unit), parents [m] indices,
    normals [m,2,3].  Returns (child_means [2m,3], child_scales [2m,3]); child c of the r-th parent is row
    c*m + r.  The copies of the other attributes and the removal of the parents are row gathers."""
    p = np.asarray(parents, dtype=np.int64)
    dt = means.dtype
    xi = np.asarray(normals, dt)
    R = _quat_rotation(np.asarray(quats, dt)[p])
    s = np.asarray(scales, dt)[p]
    mu = np.asarray(means, dt)[p]
    out_m, out_s = [], []
    for c in range(2):
        local = s * xi[:, c, :]
        off = np.stack([(R[:, r, 0] * local[:, 0] + R[:, r, 1] * local[:, 1]) + R[:, r, 2] * local[:, 2] for r in range(3)], 1)
        out_m.append(mu + off)
        out_s.append(s / dt.type(phi))
    return np.concatenate(out_m), np.concatenate(out_s)


def sample_by_score(candidates, scores, exponentials, k=None):
    """"Sampling half of the candidate Gaussians according to their pruning scores" (supplement,
    "Implementation Details": pruning before iteration 15 000).  Read as weighted sampling without
    replacement: of the m candidates, k = floor(m / 2) are drawn one after the other, each time with
    probability proportional to the score s_p among those still left.  That process is realised with one
    independent Exp(1) variate e_i per Gaussian, supplied by the caller: the k candidates with the smallest
    arrival times e_i / s_p_i are the sample (an exponential clock of rate s_p_i per candidate; the order of
    the first arrivals is exactly successive sampling proportional to the rates).  A candidate with a score
    <= 0 never arrives (time +inf) and is only taken when nothing else is left; equal times go to the lower
    index.  The division is made in the type of `scores`.  Returns the uint8 mask of the sample."""
    c = np.asarray(candidates) != 0
    w = np.asarray(scores)
    e = np.asarray(exponentials, w.dtype)
    idx = np.nonzero(c)[0]
    m = idx.size
    if k is None:
        k = m // 2
    with np.errstate(divide="ignore", invalid="ignore"):
        t = np.where(w[idx] > 0, e[idx] / w[idx], np.inf).astype(w.dtype)
    order = np.lexsort((idx, t))          # by time, ties by index
    out = np.zeros(c.shape[0], np.uint8)
    out[idx[order[:k]]] = 1
    return out


def combine_masks(clone, split, prune):
    """What the three decisions do to the array of Gaussians when they are applied together: a pruned
    Gaussian is neither cloned nor split; a split parent is replaced by its children (removed); everything
    else stays.  Returns (keep, clone_eff, split_eff) as uint8."""
    c, s, p = (np.asarray(a) != 0 for a in (clone, split, prune))
    return (~p & ~s).astype(np.uint8), (c & ~p).astype(np.uint8), (s & ~p).astype(np.uint8)
