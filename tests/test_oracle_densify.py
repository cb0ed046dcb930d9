"""Pins for the absolute positional gradient (supplement, "Implementation Details": absolute gradients
for splitting) and for the densify / prune selection rules (Sec. 4.2, Sec. 4.3)."""
import copy

import numpy as np
import pytest

import oracle
from oracle import Oracle
from paper_2511_04283_amd import scenes


def test_absolute_gradient_equals_sum_of_per_pixel_magnitudes():
    """Brute force: d(pixel loss)/d(mu_2D of Gaussian i) by central differences of the compositing
    stage alone (projected arrays perturbed, pair lists held fixed), pixel by pixel; the absolute
    gradient is the sum of the magnitudes, the ordinary one the plain sum."""
    o = Oracle(np.float64)
    sc = scenes.tiny_scene(11, 9, 32, 32, sh_degree=0, log_scale=(-1.9, 0.3))
    cam = sc.cameras[0]
    proj, bins, img, fT, nc = o.forward(sc, cam)
    w = np.random.default_rng(0).normal(size=(3, cam.height, cam.width))
    d_mean2d, _, _, _, d_abs = o.render_bwd(proj, bins, cam, w)
    h = 1e-6
    checked = 0
    for i in range(sc.n):
        if proj.tiles_touched[i] == 0:
            continue
        for ax in range(2):
            pp = copy.deepcopy(proj); pp.mean2d[i, ax] += h
            pm = copy.deepcopy(proj); pm.mean2d[i, ax] -= h
            ip, _, ncp = o.render_fwd(pp, bins, cam)
            im, _, ncm = o.render_fwd(pm, bins, cam)
            if not (np.array_equal(ncp, nc) and np.array_equal(ncm, nc)):
                continue                      # a blend / skip decision flipped: not differentiable there
            per_pixel = (w * (ip - im)).sum(0) / (2 * h)
            assert per_pixel.sum() == pytest.approx(d_mean2d[i, ax], rel=1e-5, abs=1e-8)
            assert np.abs(per_pixel).sum() == pytest.approx(d_abs[i, ax], rel=1e-5, abs=1e-8)
            checked += 1
    assert checked >= 12
    # contributions of both signs exist, so the two really differ
    assert (d_abs >= np.abs(d_mean2d) - 1e-12).all() and (d_abs > np.abs(d_mean2d) * 1.05).any()


def test_absolute_gradient_equals_plain_one_when_nothing_cancels():
    """One Gaussian, all loss weights positive, colour brighter than the background: to the right of the
    centre every pixel pulls the mean the same way, so restricted to those pixels |sum| = sum| |."""
    o = Oracle(np.float64)
    from paper_2511_04283_amd.scenes import Camera
    from helpers import one_gaussian_scene
    cam = Camera(48, 48, 40.0, 40.0, 24.0, 24.0)
    sc = one_gaussian_scene([0.0, 0.0, 4.0], [0.5, 0.5, 0.5], [1, 0, 0, 0], 0.7, [0.9, 0.8, 0.7], cam)
    proj, bins, *_ = o.forward(sc, cam)
    w = np.zeros((3, 48, 48)); w[:, :, 25:] = 1.0
    d_mean2d, _, _, _, d_abs = o.render_bwd(proj, bins, cam, w)
    assert abs(d_mean2d[0, 0]) > 1e-3
    assert d_abs[0, 0] == pytest.approx(abs(d_mean2d[0, 0]), rel=1e-12)
    assert d_abs[0, 1] > abs(d_mean2d[0, 1]) + 1e-6         # up and down still cancel in the plain sum


def test_selection_rules_truth_table():
    # columns: grad, abs grad, denom, counts (K=10), max scale, opacity, s_p
    rows = [
        (0.0004 * 4, 0.0, 4, 80, 0.01, 0.5, 0.1),    # clone: small, high gradient, s_d = 8 > 5
        (0.0004 * 4, 0.0, 4, 50, 0.01, 0.5, 0.1),    # s_d = 5 is not > 5: nothing
        (0.0001 * 4, 0.01 * 4, 4, 80, 0.01, 0.5, 0.1),  # small with only the abs gradient high: nothing
        (0.0, 0.0009 * 4, 4, 80, 0.5, 0.5, 0.1),     # split: big, abs gradient high
        (0.01 * 4, 0.0001 * 4, 4, 80, 0.5, 0.5, 0.1),   # big with only the plain gradient high: nothing
        (0.0, 0.0, 0, 0, 0.01, 0.05, 0.0),           # prune: opacity below 0.1 (denom 0 must not divide)
        (0.0, 0.0, 4, 0, 0.01, 0.5, 0.95),           # prune: s_p above 0.9
        (0.01, 0.01, 1, 90, 0.01, 0.1, 0.9),         # boundaries: opacity == 0.1 and s_p == 0.9 stay; clone
    ]
    a = np.array(rows, dtype=np.float64)
    clone, split, prune = oracle.densify_prune_masks(a[:, 0], a[:, 1], a[:, 2], a[:, 3], 10, a[:, 4], a[:, 5], a[:, 6],
                                                     tau_grad=0.0002, tau_abs=0.0004, tau_d=5.0, size_limit=0.1)
    assert clone.tolist() == [1, 0, 0, 0, 0, 0, 0, 1]
    assert split.tolist() == [0, 0, 0, 1, 0, 0, 0, 0]
    assert prune.tolist() == [0, 0, 0, 0, 0, 1, 1, 0]
    assert not (clone & split).any()
