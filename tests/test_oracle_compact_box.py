"""Pins for the oracle's Compact Box mode (Sec. 4.4 and its supplement): the pairs are exactly the
tiles whose rectangle meets the support ellipse q <= beta * 2 ln(sigma / tau_alpha)."""
import copy

import numpy as np
import pytest

from helpers import brute_composite, one_gaussian_scene
from oracle import Config, Oracle, lib
from paper_2511_04283_amd import scenes
from paper_2511_04283_amd.scenes import Camera


def _cb(dtype, beta=1.0, **kw):
    return Oracle(dtype, Config(compact_box=True, cb_beta=beta, **kw))


def _pairs_matrix(o, sc, cam):
    proj, bins = o.preprocess(sc, cam), None
    bins = o.bin_sort(proj, cam)
    TX, TY = (cam.width + 15) // 16, (cam.height + 15) // 16
    m = np.zeros((sc.n, TX * TY), np.uint8)
    tiles = (bins.keys_sorted >> np.uint64(32)).astype(np.int64)
    m[bins.gauss_sorted.astype(np.int64), tiles] = 1
    assert m.sum() == bins.num_pairs       # no duplicates
    return proj, bins, m


def _whitened_distance2(mu, cov, x0, y0, x1, y1):
    """Independent statement of min over the rectangle of d^T cov^-1 d: map the plane by L^-1
    (cov = L L^T), where the ellipse is a circle round the origin, and take the squared distance
    from the origin to the image of the rectangle (a parallelogram): 0 inside, else the nearest of
    its four edge segments."""
    L = np.linalg.cholesky(cov)
    corners = np.array([[x0, y0], [x1, y0], [x1, y1], [x0, y1]], dtype=np.float64) - mu
    if x0 <= mu[0] <= x1 and y0 <= mu[1] <= y1:
        return 0.0
    w = np.linalg.solve(L, corners.T).T
    best = np.inf
    for k in range(4):
        p, q = w[k], w[(k + 1) % 4]
        e = q - p
        t = np.clip(-(p @ e) / (e @ e), 0.0, 1.0)
        c = p + t * e
        best = min(best, float(c @ c))
    return best


def test_pinned_log_accuracy():
    import ctypes
    _lib = lib()
    x = np.concatenate([np.exp(np.random.default_rng(0).uniform(-20, 20, 20000)), [1.0, 2.0, 0.5, 255.0, 1.0000001]])
    x = x.astype(np.float32)
    got = np.array([_lib.orc_log_c_f32(ctypes.c_float(v)) for v in x], dtype=np.float64)
    want = np.log(x.astype(np.float64))
    assert np.abs(got - want).max() <= 2e-7 * np.maximum(1.0, np.abs(want)).max()
    assert np.all(np.abs(got - want) <= 3e-7 * np.maximum(np.abs(want), 0.2))
    assert _lib.orc_log_c_f32(ctypes.c_float(1.0)) == 0.0


@pytest.mark.parametrize("seed,beta", [(1, 1.0), (2, 1.0), (3, 0.6), (4, 0.25)])
def test_pairs_equal_whitened_bruteforce(seed, beta):
    sc = scenes.tiny_scene(seed, 250, 200, 120, sh_degree=1, log_scale=(-2.4, 0.9), spread=1.3)
    cam = sc.cameras[0]
    checked = 0
    for dtype, margin in ((np.float64, 1e-9), (np.float32, 2e-4)):
        o = _cb(dtype, beta)
        proj, bins, m = _pairs_matrix(o, sc, cam)
        TX, TY = (cam.width + 15) // 16, (cam.height + 15) // 16
        near = 0
        for i in range(sc.n):
            a, b, c, sig = [float(v) for v in proj.conic_opacity[i]]
            if proj.tiles_touched[i] == 0 and a == 0.0:
                # culled before the ellipse test (behind the near plane, sigma <= tau_alpha, or no tile):
                # the ellipse test below is run on the 3-sigma oracle's projection in the next test
                continue
            conic = np.array([[a, b], [b, c]])
            cov = np.linalg.inv(conic)
            Q = beta * 2.0 * np.log(sig / o.cfg.alpha_min)
            mu = proj.mean2d[i].astype(np.float64)
            for ty in range(TY):
                for tx in range(TX):
                    d2 = _whitened_distance2(mu, cov, 16.0 * tx, 16.0 * ty, 16.0 * tx + 16, 16.0 * ty + 16)
                    if abs(d2 - Q) <= margin * max(Q, 1.0):
                        near += 1
                        continue
                    assert m[i, ty * TX + tx] == (d2 <= Q), (dtype, i, tx, ty, d2, Q)
                    checked += 1
            assert proj.tiles_touched[i] == m[i].sum()
        assert near < 20
    assert checked > 10000


def test_visibility_matches_three_sigma_projection_plus_ellipse():
    """Every Gaussian the Compact Box drops entirely either fails the ordinary visibility test or has
    an ellipse (taken from the 3-sigma oracle's projection) that meets no tile."""
    sc = scenes.tiny_scene(7, 300, 160, 96, sh_degree=0, log_scale=(-3.0, 0.5), spread=1.6)
    sc.opacities[::7] = 0.003     # below tau_alpha = 1/255: can never be blended
    cam = sc.cameras[0]
    p3 = Oracle(np.float64).preprocess(sc, cam)
    pc = _cb(np.float64).preprocess(sc, cam)
    TX, TY = (cam.width + 15) // 16, (cam.height + 15) // 16
    dropped = 0
    for i in range(sc.n):
        a, b, c, sig = [float(v) for v in p3.conic_opacity[i]]
        vis3 = a != 0.0
        if not vis3 and p3.tiles_touched[i] == 0:
            # near plane / degenerate: must stay invisible unless only the 3-sigma square missed the image
            pass
        if pc.tiles_touched[i] > 0:
            assert sig > 1 / 255
            assert np.array_equal(pc.conic_opacity[i], p3.conic_opacity[i]) or not vis3
            continue
        dropped += 1
        if vis3 and sig > 1 / 255:
            Q = 2 * np.log(sig * 255)
            cov = np.linalg.inv(np.array([[a, b], [b, c]]))
            d2 = min(_whitened_distance2(p3.mean2d[i].astype(np.float64), cov, 16.0 * tx, 16.0 * ty, 16.0 * tx + 16, 16.0 * ty + 16)
                     for ty in range(TY) for tx in range(TX))
            assert d2 > Q * (1 - 1e-9)
        assert not pc.conic_opacity[i].any() and not pc.rgb[i].any() and not pc.rect[i].any()
    assert dropped > 40 and (pc.tiles_touched > 0).sum() > 100


def test_isotropic_splat_is_circle_against_rectangle():
    """Closed form: an on-axis isotropic Gaussian has a circular support of radius
    sqrt(Q (s^2 f^2/z^2 + lowpass)); a tile is paired iff its rectangle is within that distance."""
    W, H, f, z, s, sig = 160, 128, 100.0, 5.0, 0.9, 0.8
    cam = Camera(W, H, f, f, 70.3, 66.1, np.eye(3), np.zeros(3))
    x, y = (70.3 - 70.3) * z / f, 0.0
    sc = one_gaussian_scene([x, y, z], [s, s, s], [1, 0, 0, 0], sig, [0.5, 0.5, 0.5], cam)
    for beta in (1.0, 0.5, 0.1):
        o = _cb(np.float64, beta)
        proj, bins, m = _pairs_matrix(o, sc, cam)
        r = np.sqrt(beta * 2 * np.log(sig * 255) * (s * s * f * f / (z * z) + 0.3))
        TX, TY = W // 16, H // 16
        for ty in range(TY):
            for tx in range(TX):
                ddx = max(16 * tx - 70.3, 0, 70.3 - 16 * tx - 16)
                ddy = max(16 * ty - 66.1, 0, 66.1 - 16 * ty - 16)
                assert m[0, ty * TX + tx] == (np.hypot(ddx, ddy) <= r), (beta, tx, ty)
        assert 0 < m.sum() < TX * TY


@pytest.mark.parametrize("seed", [21, 22])
def test_beta_one_image_equals_pairing_every_tile(seed):
    """At beta = 1 the ellipse is the set where alpha >= tau_alpha, so dropping the tiles outside it
    changes nothing: the image equals the tile-free composite over every visible Gaussian."""
    sc = scenes.tiny_scene(seed, 60, 40, 28, sh_degree=2, log_scale=(-2.3, 0.5))
    cam = sc.cameras[0]
    o3 = Oracle(np.float64)
    p3 = o3.preprocess(sc, cam)
    bimg, bT, nblend, cw, ca = brute_composite(p3, cam, o3.cfg, mask=np.ones((cam.height, cam.width), bool), use_rect=False)
    o = _cb(np.float64)
    proj, bins, img, fT, nc = o.forward(sc, cam)
    assert np.abs(img - bimg).max() < 1e-12
    assert np.abs(fT - bT).max() < 1e-12
    # the per-Gaussian counts agree with the tile-free ones too
    for mode, want in ((0, cw), (1, ca)):
        om = _cb(np.float64, score_mode=mode)
        cnt = om.score(proj, bins, cam, np.ones((cam.height, cam.width), np.uint8), np.zeros(sc.n, np.int32))
        assert np.array_equal(cnt, want)
    # fp32 build: same image within rounding
    img32 = _cb(np.float32).forward(sc, cam)[2]
    assert np.abs(img32 - bimg).max() < 2e-5


def test_pairs_shrink_monotonically_with_beta_and_fewer_than_three_sigma_on_average():
    sc = scenes.tiny_scene(5, 400, 320, 208, sh_degree=0, log_scale=(-2.2, 0.9), spread=1.2)
    cam = sc.cameras[0]
    prev = None
    counts = []
    for beta in (1.0, 0.7, 0.4, 0.15):
        _, bins, m = _pairs_matrix(_cb(np.float32, beta), sc, cam)
        if prev is not None:
            assert (m <= prev).all()
        prev = m
        counts.append(int(m.sum()))
    assert counts[0] > counts[1] > counts[2] > counts[3] > 0
    p3 = Oracle(np.float32).preprocess(sc, cam)
    assert counts[0] < int(p3.tiles_touched.sum())


def test_sorted_order_and_ranges_hold_in_compact_box_mode():
    sc = scenes.tiny_scene(6, 300, 200, 120, sh_degree=0, log_scale=(-2.2, 0.8))
    cam = sc.cameras[0]
    o = _cb(np.float32)
    proj = o.preprocess(sc, cam)
    bins = o.bin_sort(proj, cam)
    k = bins.keys_sorted
    assert (k[1:] >= k[:-1]).all()
    r = bins.tile_ranges.astype(np.int64)
    assert (r[:, 1] - r[:, 0]).sum() == bins.num_pairs == int(proj.tiles_touched.sum())
    d = proj.depth.astype(np.float32).view(np.uint32)
    assert np.array_equal((k & np.uint64(0xFFFFFFFF)).astype(np.uint32), d[bins.gauss_sorted])


def test_gradients_by_finite_differences_in_compact_box_mode():
    from test_oracle_gradients import _fd_check, _to64
    sc = _to64(scenes.tiny_scene(105, 7, 32, 24, sh_degree=1, log_scale=(-2.0, 0.4)))
    cam = sc.cameras[0]
    w = np.random.default_rng(5).normal(size=(3, cam.height, cam.width))
    for beta in (1.0, 0.5):
        checked, worst, g = _fd_check(_cb(np.float64, beta), sc, cam, w=w)
        assert checked > 100
