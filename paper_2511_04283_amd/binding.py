"""ctypes binding of libfastgs_hip.so (the C ABI of include/fastgs.h).

Argument marshalling only: tensors are allocated with torch (device memory, stream), their
`data_ptr()`s are handed to the library, and every step of the path runs in the HIP kernels.
There is no fallback: if the library is missing or fails to load this module raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
# FASTGS_HIP_LIB names another build of the same library (e.g. an experimental variant); load_library says so on
# stderr when it is used, so that no run takes a substituted library unnoticed
LIB_PATH = os.environ.get("FASTGS_HIP_LIB") or os.path.join(_PKG, "libfastgs_hip.so")

FS_OK = 0
FS_SCORE_WEIGHT, FS_SCORE_ALPHA = 0, 1
FS_SORT_AUTO, FS_SORT_RADIX = 0, 1
FS_BWD_PER_PIXEL, FS_BWD_PER_SPLAT = 0, 1
FS_RECORDS_AUTO, FS_RECORDS_DENSE, FS_RECORDS_SPARSE = 0, 1, 2
FS_MASK_MEAN_STD, FS_MASK_MINMAX_TAU = 0, 1
_STATUS = {0: "FS_OK", -1: "FS_EINVAL", -2: "FS_ENOMEM", -3: "FS_EHIP", -4: "FS_ECAPACITY"}

EXPORTS = ("fs_default_config", "fs_create", "fs_destroy", "fs_last_error", "fs_preprocess", "fs_bin_sort",
           "fs_render_fwd", "fs_render_fwd_loss", "fs_set_score_record", "fs_set_backward_mode", "fs_set_record_mode", "fs_error_mask_fused", "fs_l1_grad", "fs_render_bwd", "fs_error_mask", "fs_error_mask_noalloc", "fs_score_accumulate", "fs_score_record_rows", "fs_mask_score_fused",
           "fs_photo_loss", "fs_prune_score_accumulate", "fs_prune_score_normalize",
           "fs_densify_accumulate", "fs_select", "fs_compact", "fs_gather_rows",
           "fs_combine_masks", "fs_counts_add", "fs_split_children", "fs_sample_by_score", "fs_activate_inv",
           "fs_adam_step", "fs_grad_accumulate", "fs_adam_interval", "fs_activate", "fs_activate_bwd",
           "fs_profile_enable", "fs_profile_read", "fs_measure_peaks")
KERNEL_GROUPS = ("preprocess", "scan", "emit_pairs", "order_pairs", "tile_ranges", "render_fwd", "l1_grad", "photo_loss",
                 "render_bwd", "preprocess_bwd", "error_mask", "score")


class fs_config(ctypes.Structure):
    _fields_ = [("tile", ctypes.c_int32), ("z_near", ctypes.c_float), ("lowpass", ctypes.c_float),
                ("alpha_min", ctypes.c_float), ("alpha_max", ctypes.c_float), ("T_min", ctypes.c_float),
                ("bg", ctypes.c_float * 3), ("jclamp", ctypes.c_float), ("score_mode", ctypes.c_int32),
                ("compact_box", ctypes.c_int32), ("cb_beta", ctypes.c_float), ("sort_mode", ctypes.c_int32)]


class fs_camera(ctypes.Structure):
    _fields_ = [("width", ctypes.c_int32), ("height", ctypes.c_int32), ("fx", ctypes.c_float), ("fy", ctypes.c_float),
                ("cx", ctypes.c_float), ("cy", ctypes.c_float), ("R", ctypes.c_float * 9), ("t", ctypes.c_float * 3)]


class fs_gaussians(ctypes.Structure):
    _fields_ = [("n", ctypes.c_int64), ("sh_degree", ctypes.c_int32), ("means", ctypes.c_void_p),
                ("scales", ctypes.c_void_p), ("quats", ctypes.c_void_p), ("opacities", ctypes.c_void_p),
                ("sh", ctypes.c_void_p)]


class fs_projected(ctypes.Structure):
    _fields_ = [("mean2d", ctypes.c_void_p), ("depth", ctypes.c_void_p), ("conic_opacity", ctypes.c_void_p),
                ("rgb", ctypes.c_void_p), ("rect", ctypes.c_void_p), ("tiles_touched", ctypes.c_void_p),
                ("clamped", ctypes.c_void_p)]


class fs_bins(ctypes.Structure):
    _fields_ = [("num_pairs", ctypes.c_int64), ("keys_sorted", ctypes.c_void_p), ("gauss_sorted", ctypes.c_void_p),
                ("tile_ranges", ctypes.c_void_p), ("pair_offsets", ctypes.c_void_p),
                ("num_records", ctypes.c_int64), ("record_offsets", ctypes.c_void_p),
                ("record_counts", ctypes.c_void_p),
                ("tile_order", ctypes.c_void_p), ("splats", ctypes.c_void_p), ("generation", ctypes.c_uint64)]


class fs_select_params(ctypes.Structure):
    _fields_ = [("tau_grad", ctypes.c_float), ("tau_abs", ctypes.c_float), ("tau_d", ctypes.c_float),
                ("size_limit", ctypes.c_float), ("min_opacity", ctypes.c_float), ("tau_p", ctypes.c_float),
                ("K", ctypes.c_int32)]


class fs_grads(ctypes.Structure):
    _fields_ = [("dmeans", ctypes.c_void_p), ("dscales", ctypes.c_void_p), ("dquats", ctypes.c_void_p),
                ("dopacities", ctypes.c_void_p), ("dsh", ctypes.c_void_p), ("dmean2d", ctypes.c_void_p),
                ("dconic", ctypes.c_void_p), ("drgb", ctypes.c_void_p), ("dmean2d_abs", ctypes.c_void_p)]


_lib = None


def load_library() -> ctypes.CDLL:
    """Loads libfastgs_hip.so (building is a separate, explicit step: paper_2511_04283_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2511_04283_amd.build` "
                           "(there is no CPU fallback)")
    if os.environ.get("FASTGS_HIP_LIB"):
        import sys
        print(f"paper_2511_04283_amd: loading the library named by FASTGS_HIP_LIB: {LIB_PATH}", file=sys.stderr, flush=True)
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
    P = ctypes.POINTER
    lib.fs_default_config.argtypes = [P(fs_config)]
    lib.fs_default_config.restype = None
    lib.fs_create.argtypes = [P(vp), ctypes.c_int, vp, P(fs_config)]
    lib.fs_destroy.argtypes = [vp]
    lib.fs_destroy.restype = None
    lib.fs_last_error.argtypes = [vp]
    lib.fs_last_error.restype = ctypes.c_char_p
    lib.fs_preprocess.argtypes = [vp, P(fs_gaussians), P(fs_camera), P(fs_projected)]
    lib.fs_bin_sort.argtypes = [vp, P(fs_projected), P(fs_camera), i64, P(fs_bins)]
    lib.fs_render_fwd.argtypes = [vp, P(fs_projected), P(fs_bins), P(fs_camera), vp, vp, vp]
    lib.fs_l1_grad.argtypes = [vp, vp, vp, i32, i32, vp, vp]
    lib.fs_render_fwd_loss.argtypes = [vp, P(fs_projected), P(fs_bins), P(fs_camera), vp, vp, vp, vp, vp, vp]
    lib.fs_error_mask_fused.argtypes = [vp, i32, i32, i32, f32, vp, vp]
    lib.fs_set_score_record.argtypes = [vp, i32]
    lib.fs_set_backward_mode.argtypes = [vp, i32]
    lib.fs_set_record_mode.argtypes = [vp, i32]
    lib.fs_render_bwd.argtypes = [vp, P(fs_gaussians), P(fs_camera), P(fs_projected), P(fs_bins), vp, vp, vp, P(fs_grads)]
    lib.fs_error_mask.argtypes = [vp, vp, vp, i32, i32, i32, f32, vp, vp]
    lib.fs_error_mask_noalloc.argtypes = [vp, vp, vp, i32, i32, i32, f32, vp, vp]
    lib.fs_score_accumulate.argtypes = [vp, P(fs_projected), P(fs_bins), P(fs_camera), vp, vp, vp, vp]
    lib.fs_score_record_rows.argtypes = [vp, P(fs_bins), P(fs_camera), vp]
    lib.fs_mask_score_fused.argtypes = [vp, P(fs_projected), P(fs_bins), P(fs_camera), vp, ctypes.c_int32, ctypes.c_float, vp, vp, vp]
    lib.fs_photo_loss.argtypes = [vp, vp, vp, i32, i32, f32, vp, vp]
    lib.fs_prune_score_accumulate.argtypes = [vp, vp, i64, vp, vp]
    lib.fs_prune_score_normalize.argtypes = [vp, vp, i64, vp]
    lib.fs_densify_accumulate.argtypes = [vp, vp, vp, vp, i64, vp, vp, vp]
    lib.fs_select.argtypes = [vp, i64, vp, vp, vp, vp, vp, vp, vp, P(fs_select_params), vp, vp, vp]
    lib.fs_compact.argtypes = [vp, vp, i64, vp, P(i64)]
    lib.fs_gather_rows.argtypes = [vp, vp, i64, vp, i64, vp]
    lib.fs_adam_step.argtypes = [vp, vp, vp, vp, vp, i64, f32, f32, f32, f32, i32, f32, i32]
    lib.fs_grad_accumulate.argtypes = [vp, vp, vp, i64]
    lib.fs_adam_interval.argtypes = [i32]
    lib.fs_activate.argtypes = [vp, i64, vp, vp, vp, vp, vp, vp]
    lib.fs_activate_bwd.argtypes = [vp, i64, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.fs_combine_masks.argtypes = [vp, i64, vp, vp, vp, vp, vp, vp]
    lib.fs_counts_add.argtypes = [vp, vp, vp, i64]
    lib.fs_split_children.argtypes = [vp, vp, vp, vp, vp, i64, vp, f32, vp, vp]
    lib.fs_sample_by_score.argtypes = [vp, vp, vp, vp, i64, vp, P(i64)]
    lib.fs_activate_inv.argtypes = [vp, i64, vp, vp, f32, f32, vp, vp]
    lib.fs_measure_peaks.argtypes = [vp, i64, P(ctypes.c_double), P(ctypes.c_double)]
    lib.fs_profile_enable.argtypes = [vp, ctypes.c_uint32]
    lib.fs_profile_read.argtypes = [vp, i32, P(ctypes.c_char_p), P(ctypes.c_double), P(i64)]
    for name in EXPORTS:
        if name not in ("fs_default_config", "fs_destroy", "fs_last_error", "fs_adam_interval"):
            getattr(lib, name).restype = ctypes.c_int
    lib.fs_adam_interval.restype = ctypes.c_int32
    _lib = lib
    return lib


def default_config() -> fs_config:
    c = fs_config()
    load_library().fs_default_config(ctypes.byref(c))
    return c


def make_camera(cam) -> fs_camera:
    """From any object with width,height,fx,fy,cx,cy,R(3x3),t(3) (e.g. scenes.Camera)."""
    import numpy as np
    c = fs_camera()
    c.width, c.height = int(cam.width), int(cam.height)
    c.fx, c.fy, c.cx, c.cy = float(cam.fx), float(cam.fy), float(cam.cx), float(cam.cy)
    c.R = (ctypes.c_float * 9)(*[float(x) for x in np.asarray(cam.R, dtype=np.float32).reshape(9)])
    c.t = (ctypes.c_float * 3)(*[float(x) for x in np.asarray(cam.t, dtype=np.float32).reshape(3)])
    return c


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _chk(t, dtype, shape=None, name="tensor"):
    if not (t.is_cuda and t.is_contiguous() and t.dtype == dtype):
        raise ValueError(f"{name}: need a contiguous CUDA tensor of dtype {dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: shape {tuple(t.shape)} != {tuple(shape)}")
    return t


@dataclass
class Gaussians:
    """Device tensors of a scene (float32, contiguous)."""
    means: torch.Tensor
    scales: torch.Tensor
    quats: torch.Tensor
    opacities: torch.Tensor
    sh: torch.Tensor
    sh_degree: int

    @property
    def n(self) -> int:
        return int(self.means.shape[0])

    @staticmethod
    def from_scene(sc, device="cuda:0") -> "Gaussians":
        import numpy as np
        f = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)
        return Gaussians(f(sc.means), f(sc.scales), f(sc.quats), f(sc.opacities), f(sc.sh), int(sc.sh_degree))

    def struct(self) -> fs_gaussians:
        n, K = self.n, (self.sh_degree + 1) ** 2
        f = torch.float32
        _chk(self.means, f, (n, 3), "means"); _chk(self.scales, f, (n, 3), "scales")
        _chk(self.quats, f, (n, 4), "quats"); _chk(self.opacities, f, (n,), "opacities")
        _chk(self.sh, f, (n, K, 3), "sh")
        g = fs_gaussians()
        g.n, g.sh_degree = n, self.sh_degree
        g.means, g.scales, g.quats = self.means.data_ptr(), self.scales.data_ptr(), self.quats.data_ptr()
        g.opacities, g.sh = self.opacities.data_ptr(), self.sh.data_ptr()
        return g


@dataclass
class Projected:
    mean2d: torch.Tensor
    depth: torch.Tensor
    conic_opacity: torch.Tensor
    rgb: torch.Tensor
    rect: torch.Tensor           # int16 storage of the uint16 [n,4] rectangle
    tiles_touched: torch.Tensor  # int32 storage of uint32
    clamped: torch.Tensor

    def struct(self) -> fs_projected:
        p = fs_projected()
        p.mean2d, p.depth, p.conic_opacity = self.mean2d.data_ptr(), self.depth.data_ptr(), self.conic_opacity.data_ptr()
        p.rgb, p.rect, p.tiles_touched = self.rgb.data_ptr(), self.rect.data_ptr(), self.tiles_touched.data_ptr()
        p.clamped = self.clamped.data_ptr()
        return p


@dataclass
class Bins:
    """Result of fs_bin_sort: P and raw device pointers into ctx-owned memory (valid until the next
    fs_bin_sort on the same Context).  `copy_*` methods clone them into torch tensors for inspection."""
    num_pairs: int
    struct: fs_bins
    num_tiles: int
    device: torch.device

    def _copy(self, ptr, count, dtype):
        """Clone `count` elements at device address `ptr` into a new torch tensor (the ctx-owned
        memory is wrapped without a copy through the CUDA array interface, then cloned)."""
        if not count:
            return torch.empty(0, dtype=dtype, device=self.device)
        typestr = {torch.int64: "<i8", torch.int32: "<i4"}[dtype]

        class _Raw:
            __cuda_array_interface__ = {"shape": (count,), "typestr": typestr, "data": (int(ptr), False),
                                        "version": 2}
        return torch.as_tensor(_Raw(), device=self.device).clone()

    def copy_keys(self):
        return self._copy(self.struct.keys_sorted, self.num_pairs, torch.int64)

    def copy_gauss(self):
        return self._copy(self.struct.gauss_sorted, self.num_pairs, torch.int32)

    def copy_ranges(self):
        return self._copy(self.struct.tile_ranges, 2 * self.num_tiles, torch.int32).view(self.num_tiles, 2)

    def copy_order(self):
        return self._copy(self.struct.tile_order, self.num_tiles, torch.int32)


class Context:
    """Owns one fs_ctx bound to a torch device and (by default) torch's current stream on it."""

    def __init__(self, device="cuda:0", config: fs_config | None = None, stream: torch.cuda.Stream | None = None):
        self.lib = load_library()
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible: the FastGS HIP path has no CPU fallback")
        self.device = torch.device(device)
        self.config = config if config is not None else default_config()
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        h = ctypes.c_void_p()
        rc = self.lib.fs_create(ctypes.byref(h), self.device.index or 0, ctypes.c_void_p(self.stream.cuda_stream),
                                ctypes.byref(self.config))
        if rc != FS_OK:
            raise RuntimeError(f"fs_create failed: {_STATUS.get(rc, rc)}")
        self.handle = h

    def close(self):
        if getattr(self, "handle", None):
            self.lib.fs_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc, what):
        if rc != FS_OK:
            msg = self.lib.fs_last_error(self.handle)
            raise RuntimeError(f"{what}: {_STATUS.get(rc, rc)}: {msg.decode() if msg else ''}")

    # ---- measurement helpers --------------------------------------------------------------
    def fs_profile_enable(self, groups=None):
        """groups: iterable of names from KERNEL_GROUPS (None = all, () = off)."""
        mask = (1 << len(KERNEL_GROUPS)) - 1 if groups is None else sum(1 << KERNEL_GROUPS.index(g) for g in groups)
        self._check(self.lib.fs_profile_enable(self.handle, mask), "fs_profile_enable")

    def fs_profile_read(self) -> dict:
        """{group: (total_ms, launches)} accumulated since fs_profile_enable."""
        out = {}
        for k, nm in enumerate(KERNEL_GROUPS):
            name, ms, cnt = ctypes.c_char_p(), ctypes.c_double(), ctypes.c_int64()
            self._check(self.lib.fs_profile_read(self.handle, k, ctypes.byref(name), ctypes.byref(ms), ctypes.byref(cnt)),
                        "fs_profile_read")
            assert name.value.decode() == nm
            out[nm] = (ms.value, cnt.value)
        return out

    # ---- the calls of fastgs.h, same names ------------------------------------------------
    def fs_preprocess(self, g: Gaussians, cam: fs_camera, out: Projected | None = None) -> Projected:
        n, dev = g.n, self.device
        if out is None:
            out = Projected(torch.empty((n, 2), dtype=torch.float32, device=dev),
                            torch.empty(n, dtype=torch.float32, device=dev),
                            torch.empty((n, 4), dtype=torch.float32, device=dev),
                            torch.empty((n, 3), dtype=torch.float32, device=dev),
                            torch.empty((n, 4), dtype=torch.int16, device=dev),
                            torch.empty(n, dtype=torch.int32, device=dev),
                            torch.empty((n, 3), dtype=torch.uint8, device=dev))
        gs, ps = g.struct(), out.struct()
        self._check(self.lib.fs_preprocess(self.handle, ctypes.byref(gs), ctypes.byref(cam), ctypes.byref(ps)),
                    "fs_preprocess")
        return out

    def fs_bin_sort(self, proj: Projected, cam: fs_camera) -> Bins:
        b = fs_bins()
        ps = proj.struct()
        n = int(proj.depth.shape[0])
        self._check(self.lib.fs_bin_sort(self.handle, ctypes.byref(ps), ctypes.byref(cam), n, ctypes.byref(b)),
                    "fs_bin_sort")
        tiles = ((cam.width + 15) // 16) * ((cam.height + 15) // 16)
        return Bins(int(b.num_pairs), b, tiles, self.device)

    def fs_render_fwd(self, proj: Projected, bins: Bins, cam: fs_camera, image=None, final_T=None, n_contrib=None):
        H, W, dev = cam.height, cam.width, self.device
        if image is None:
            image = torch.empty((3, H, W), dtype=torch.float32, device=dev)
        if final_T is None:
            final_T = torch.empty((H, W), dtype=torch.float32, device=dev)
        if n_contrib is None:
            n_contrib = torch.empty((H, W), dtype=torch.int32, device=dev)
        ps = proj.struct()
        self._check(self.lib.fs_render_fwd(self.handle, ctypes.byref(ps), ctypes.byref(bins.struct), ctypes.byref(cam),
                                           _ptr(image), _ptr(final_T), _ptr(n_contrib)), "fs_render_fwd")
        return image, final_T, n_contrib

    def fs_render_fwd_loss(self, proj: Projected, bins: Bins, cam: fs_camera, target, image=None, final_T=None,
                           n_contrib=None, dL_dimage=None, loss_out=None, want_grad=True):
        H, W, dev = cam.height, cam.width, self.device
        _chk(target, torch.float32, (3, H, W), "target")
        if image is None:
            image = torch.empty((3, H, W), dtype=torch.float32, device=dev)
        if final_T is None:
            final_T = torch.empty((H, W), dtype=torch.float32, device=dev)
        if n_contrib is None:
            n_contrib = torch.empty((H, W), dtype=torch.int32, device=dev)
        if dL_dimage is None and want_grad:
            dL_dimage = torch.empty((3, H, W), dtype=torch.float32, device=dev)
        ps = proj.struct()
        self._check(self.lib.fs_render_fwd_loss(self.handle, ctypes.byref(ps), ctypes.byref(bins.struct), ctypes.byref(cam),
                                                _ptr(target), _ptr(image), _ptr(final_T), _ptr(n_contrib), _ptr(dL_dimage),
                                                _ptr(loss_out)), "fs_render_fwd_loss")
        return image, final_T, n_contrib, dL_dimage

    def fs_set_backward_mode(self, mode: int):
        self._check(self.lib.fs_set_backward_mode(self.handle, int(mode)), "fs_set_backward_mode")

    def fs_set_record_mode(self, mode: int):
        self._check(self.lib.fs_set_record_mode(self.handle, int(mode)), "fs_set_record_mode")

    def fs_set_score_record(self, on: bool):
        self._check(self.lib.fs_set_score_record(self.handle, 1 if on else 0), "fs_set_score_record")

    def fs_error_mask_fused(self, H, W, rule=FS_MASK_MEAN_STD, k=1.0, mask=None, threshold_out=None):
        if mask is None:
            mask = torch.empty((H, W), dtype=torch.uint8, device=self.device)
        if threshold_out is None:
            threshold_out = torch.empty(1, dtype=torch.float32, device=self.device)
        self._check(self.lib.fs_error_mask_fused(self.handle, int(H), int(W), int(rule), float(k), _ptr(mask),
                                                 _ptr(threshold_out)), "fs_error_mask_fused")
        return mask, threshold_out

    def fs_l1_grad(self, image, target, dL_dimage=None, loss_out=None):
        _, H, W = image.shape
        _chk(image, torch.float32, (3, H, W), "image"); _chk(target, torch.float32, (3, H, W), "target")
        if dL_dimage is None:
            dL_dimage = torch.empty_like(image)
        self._check(self.lib.fs_l1_grad(self.handle, _ptr(image), _ptr(target), H, W, _ptr(dL_dimage), _ptr(loss_out)),
                    "fs_l1_grad")
        return dL_dimage

    def fs_render_bwd(self, g: Gaussians, cam: fs_camera, proj: Projected, bins: Bins, final_T, n_contrib, dL_dimage,
                      out: dict | None = None, want_2d: bool = False, want_abs: bool = False) -> dict:
        n, K, dev = g.n, (g.sh_degree + 1) ** 2, self.device
        if out is None:
            e = lambda *s: torch.empty(s, dtype=torch.float32, device=dev)
            out = dict(means=e(n, 3), scales=e(n, 3), quats=e(n, 4), opacities=e(n), sh=e(n, K, 3), mean2d=e(n, 2))
            if want_2d:
                out["conic"] = e(n, 3)
                out["rgb"] = e(n, 3)
            if want_abs:
                out["mean2d_abs"] = e(n, 2)
        gr = fs_grads()
        gr.dmeans, gr.dscales, gr.dquats = out["means"].data_ptr(), out["scales"].data_ptr(), out["quats"].data_ptr()
        gr.dopacities, gr.dsh, gr.dmean2d = out["opacities"].data_ptr(), out["sh"].data_ptr(), out["mean2d"].data_ptr()
        gr.dconic = out["conic"].data_ptr() if "conic" in out else None
        gr.drgb = out["rgb"].data_ptr() if "rgb" in out else None
        gr.dmean2d_abs = out["mean2d_abs"].data_ptr() if "mean2d_abs" in out else None
        gs, ps = g.struct(), proj.struct()
        self._check(self.lib.fs_render_bwd(self.handle, ctypes.byref(gs), ctypes.byref(cam), ctypes.byref(ps),
                                           ctypes.byref(bins.struct), _ptr(final_T), _ptr(n_contrib), _ptr(dL_dimage),
                                           ctypes.byref(gr)), "fs_render_bwd")
        return out

    def fs_error_mask(self, image, target, rule=FS_MASK_MEAN_STD, k=1.0, mask=None, threshold_out=None):
        _, H, W = image.shape
        if mask is None:
            mask = torch.empty((H, W), dtype=torch.uint8, device=self.device)
        if threshold_out is None:
            threshold_out = torch.empty(1, dtype=torch.float32, device=self.device)
        self._check(self.lib.fs_error_mask(self.handle, _ptr(image), _ptr(target), H, W, int(rule), float(k), _ptr(mask),
                                           _ptr(threshold_out)), "fs_error_mask")
        return mask, threshold_out

    def fs_error_mask_noalloc(self, image, target, mask, threshold_out, rule=FS_MASK_MEAN_STD, k=1.0):
        """fs_error_mask on the library's static scratch; the outputs are the caller's (nothing is allocated)."""
        _, H, W = image.shape
        self._check(self.lib.fs_error_mask_noalloc(self.handle, _ptr(image), _ptr(target), H, W, int(rule), float(k),
                                                   _ptr(mask), _ptr(threshold_out)), "fs_error_mask_noalloc")
        return mask, threshold_out

    def fs_photo_loss(self, image, target, lam=0.2, dL_dimage=None, out3=None, want_grad=True):
        """Returns (out3, dL_dimage): out3 = device doubles {L1, SSIM, E}; dL_dimage is None if not wanted."""
        _, H, W = image.shape
        if out3 is None:
            out3 = torch.zeros(3, dtype=torch.float64, device=self.device)
        if dL_dimage is None and want_grad:
            dL_dimage = torch.empty_like(image)
        self._check(self.lib.fs_photo_loss(self.handle, _ptr(image), _ptr(target), H, W, float(lam),
                                           _ptr(dL_dimage) if dL_dimage is not None else None, _ptr(out3)), "fs_photo_loss")
        return out3, dL_dimage

    def fs_prune_score_accumulate(self, counts_view, E, acc):
        n = int(counts_view.shape[0])
        _chk(counts_view, torch.int32, (n,), "counts_view")
        _chk(acc, torch.float64, (n,), "acc")
        assert E.dtype == torch.float64 and E.numel() >= 1
        self._check(self.lib.fs_prune_score_accumulate(self.handle, _ptr(counts_view), n, _ptr(E), _ptr(acc)),
                    "fs_prune_score_accumulate")
        return acc

    def fs_prune_score_normalize(self, acc, s_p=None):
        n = int(acc.shape[0])
        if s_p is None:
            s_p = torch.empty(n, dtype=torch.float32, device=self.device)
        self._check(self.lib.fs_prune_score_normalize(self.handle, _ptr(acc), n, _ptr(s_p)), "fs_prune_score_normalize")
        return s_p

    def fs_measure_peaks(self, copy_bytes=1 << 30):
        """(streaming-copy GB/s, plain fp32 FMA TFLOP/s) measured on this context's device."""
        c, f = ctypes.c_double(0.0), ctypes.c_double(0.0)
        self._check(self.lib.fs_measure_peaks(self.handle, int(copy_bytes), ctypes.byref(c), ctypes.byref(f)), "fs_measure_peaks")
        return c.value, f.value

    def fs_adam_step(self, param, grad, m, v, step, lr, beta1=0.9, beta2=0.999, eps=1e-15, grad_scale=1.0,
                     zero_grad=False):
        for t, nm in ((param, "param"), (grad, "grad"), (m, "m"), (v, "v")):
            _chk(t, torch.float32, None, nm)
            assert t.numel() == param.numel()
        self._check(self.lib.fs_adam_step(self.handle, _ptr(param), _ptr(grad), _ptr(m), _ptr(v), param.numel(), float(lr),
                                          float(beta1), float(beta2), float(eps), int(step), float(grad_scale),
                                          int(bool(zero_grad))), "fs_adam_step")

    def fs_grad_accumulate(self, acc, grad):
        _chk(acc, torch.float32, None, "acc"); _chk(grad, torch.float32, None, "grad")
        assert acc.numel() == grad.numel()
        self._check(self.lib.fs_grad_accumulate(self.handle, _ptr(acc), _ptr(grad), acc.numel()), "fs_grad_accumulate")

    def fs_adam_interval(self, iteration):
        return int(self.lib.fs_adam_interval(int(iteration)))

    def fs_activate(self, raw_scales, raw_quats, raw_opacities):
        n = int(raw_opacities.shape[0])
        s, q, o = torch.empty_like(raw_scales), torch.empty_like(raw_quats), torch.empty_like(raw_opacities)
        self._check(self.lib.fs_activate(self.handle, n, _ptr(raw_scales), _ptr(raw_quats), _ptr(raw_opacities), _ptr(s),
                                         _ptr(q), _ptr(o)), "fs_activate")
        return s, q, o

    def fs_activate_bwd(self, raw_scales, raw_quats, raw_opacities, d_scales, d_quats, d_opacities, in_place=True):
        n = int(raw_opacities.shape[0])
        outs = (d_scales, d_quats, d_opacities) if in_place else tuple(torch.empty_like(t) for t in (d_scales, d_quats, d_opacities))
        self._check(self.lib.fs_activate_bwd(self.handle, n, _ptr(raw_scales), _ptr(raw_quats), _ptr(raw_opacities),
                                             _ptr(d_scales), _ptr(d_quats), _ptr(d_opacities), _ptr(outs[0]), _ptr(outs[1]),
                                             _ptr(outs[2])), "fs_activate_bwd")
        return outs

    def fs_densify_accumulate(self, dmean2d, dmean2d_abs, tiles_touched, grad_accum, abs_accum, denom):
        n = int(dmean2d.shape[0])
        self._check(self.lib.fs_densify_accumulate(self.handle, _ptr(dmean2d), _ptr(dmean2d_abs), _ptr(tiles_touched), n,
                                                   _ptr(grad_accum), _ptr(abs_accum), _ptr(denom)), "fs_densify_accumulate")

    def fs_select(self, grad_accum, abs_accum, denom, counts, scales, opacities, s_p, params: fs_select_params):
        n = int(grad_accum.shape[0])
        m = [torch.empty(n, dtype=torch.uint8, device=self.device) for _ in range(3)]
        self._check(self.lib.fs_select(self.handle, n, _ptr(grad_accum), _ptr(abs_accum), _ptr(denom), _ptr(counts),
                                       _ptr(scales), _ptr(opacities), _ptr(s_p), ctypes.byref(params), _ptr(m[0]),
                                       _ptr(m[1]), _ptr(m[2])), "fs_select")
        return tuple(m)

    def fs_combine_masks(self, clone, split, prune):
        """(keep, clone_eff, split_eff) uint8 [n]."""
        n = int(clone.shape[0])
        for t, nm in ((clone, "clone"), (split, "split"), (prune, "prune")):
            _chk(t, torch.uint8, (n,), nm)
        out = [torch.empty(n, dtype=torch.uint8, device=self.device) for _ in range(3)]
        self._check(self.lib.fs_combine_masks(self.handle, n, _ptr(clone), _ptr(split), _ptr(prune), _ptr(out[0]),
                                              _ptr(out[1]), _ptr(out[2])), "fs_combine_masks")
        return tuple(out)

    def fs_counts_add(self, total, view):
        n = int(total.shape[0])
        _chk(total, torch.int32, (n,), "total"); _chk(view, torch.int32, (n,), "view")
        self._check(self.lib.fs_counts_add(self.handle, _ptr(total), _ptr(view), n), "fs_counts_add")
        return total

    def fs_split_children(self, means, scales, quats, parents, normals, phi=1.6):
        """(child_means [2m,3], child_scales [2m,3]); normals [m,2,3] are the caller's N(0,1) draws."""
        n, m = int(means.shape[0]), int(parents.shape[0])
        _chk(means, torch.float32, (n, 3), "means"); _chk(scales, torch.float32, (n, 3), "scales")
        _chk(quats, torch.float32, (n, 4), "quats"); _chk(parents, torch.int32, (m,), "parents")
        _chk(normals, torch.float32, (m, 2, 3), "normals")
        cm = torch.empty((2 * m, 3), dtype=torch.float32, device=self.device)
        cs = torch.empty((2 * m, 3), dtype=torch.float32, device=self.device)
        self._check(self.lib.fs_split_children(self.handle, _ptr(means), _ptr(scales), _ptr(quats), _ptr(parents), m,
                                               _ptr(normals), float(phi), _ptr(cm), _ptr(cs)), "fs_split_children")
        return cm, cs

    def fs_sample_by_score(self, candidates, scores, exponentials):
        """uint8 [n] mask of floor(m / 2) of the m candidates; exponentials [n] are the caller's Exp(1) draws."""
        n = int(candidates.shape[0])
        _chk(candidates, torch.uint8, (n,), "candidates"); _chk(scores, torch.float32, (n,), "scores")
        _chk(exponentials, torch.float32, (n,), "exponentials")
        out = torch.empty(n, dtype=torch.uint8, device=self.device)
        cnt = ctypes.c_int64(0)
        self._check(self.lib.fs_sample_by_score(self.handle, _ptr(candidates), _ptr(scores), _ptr(exponentials), n,
                                                _ptr(out), ctypes.byref(cnt)), "fs_sample_by_score")
        return out, int(cnt.value)

    def fs_activate_inv(self, scales, opacities, lo=1e-4, hi=1.0 - 1e-4):
        n = int(opacities.shape[0])
        _chk(scales, torch.float32, (n, 3), "scales"); _chk(opacities, torch.float32, (n,), "opacities")
        rs, ro = torch.empty_like(scales), torch.empty_like(opacities)
        self._check(self.lib.fs_activate_inv(self.handle, n, _ptr(scales), _ptr(opacities), float(lo), float(hi), _ptr(rs),
                                             _ptr(ro)), "fs_activate_inv")
        return rs, ro

    def fs_compact(self, mask):
        """Returns the int32 tensor of selected positions (ascending)."""
        n = int(mask.shape[0])
        _chk(mask, torch.uint8, (n,), "mask")
        idx = torch.empty(max(n, 1), dtype=torch.int32, device=self.device)
        cnt = ctypes.c_int64(0)
        self._check(self.lib.fs_compact(self.handle, _ptr(mask), n, _ptr(idx), ctypes.byref(cnt)), "fs_compact")
        return idx[:cnt.value]

    def fs_gather_rows(self, src, indices):
        _chk(src, torch.float32, None, "src")
        count = int(indices.shape[0])
        row = int(src.numel() // max(1, src.shape[0]))
        dst = torch.empty((count,) + tuple(src.shape[1:]), dtype=torch.float32, device=self.device)
        self._check(self.lib.fs_gather_rows(self.handle, _ptr(src), row, _ptr(indices), count, _ptr(dst)), "fs_gather_rows")
        return dst

    def fs_score_accumulate(self, proj: Projected, bins: Bins, cam: fs_camera, final_T, n_contrib, mask, counts):
        _chk(counts, torch.int32, (int(proj.depth.shape[0]),), "counts")
        ps = proj.struct()
        self._check(self.lib.fs_score_accumulate(self.handle, ctypes.byref(ps), ctypes.byref(bins.struct),
                                                 ctypes.byref(cam), _ptr(final_T), _ptr(n_contrib), _ptr(mask),
                                                 _ptr(counts)), "fs_score_accumulate")
        return counts

    def fs_mask_score_fused(self, proj: Projected, bins: Bins, cam: fs_camera, n_contrib, counts, rule=FS_MASK_MEAN_STD,
                            k=1.0, mask=None, threshold_out=None):
        H, W = int(cam.height), int(cam.width)
        if mask is None:
            mask = torch.empty((H, W), dtype=torch.uint8, device=self.device)
        if threshold_out is None:
            threshold_out = torch.empty(1, dtype=torch.float32, device=self.device)
        _chk(mask, torch.uint8, (H, W), "mask")
        _chk(counts, torch.int32, (int(proj.depth.shape[0]),), "counts")
        ps = proj.struct()
        self._check(self.lib.fs_mask_score_fused(self.handle, ctypes.byref(ps), ctypes.byref(bins.struct), ctypes.byref(cam),
                                                 _ptr(n_contrib), int(rule), float(k), _ptr(mask), _ptr(threshold_out),
                                                 _ptr(counts)), "fs_mask_score_fused")
        return mask, threshold_out, counts

    def fs_score_record_rows(self, bins: Bins, cam: fs_camera, rows_per_tile=None):
        tiles = ((int(cam.height) + 15) // 16) * ((int(cam.width) + 15) // 16)
        if rows_per_tile is None:
            rows_per_tile = torch.empty(tiles, dtype=torch.int32, device=self.device)
        _chk(rows_per_tile, torch.int32, (tiles,), "rows_per_tile")
        self._check(self.lib.fs_score_record_rows(self.handle, ctypes.byref(bins.struct), ctypes.byref(cam),
                                                  _ptr(rows_per_tile)), "fs_score_record_rows")
        return rows_per_tile
