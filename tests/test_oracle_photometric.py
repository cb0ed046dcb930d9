"""Pins for the oracle's SSIM / photometric loss (Sec. 4.3, Sec. 4.5) and pruning score (Sec. 4.3)."""
import numpy as np
import pytest
from scipy import ndimage

import oracle

C1, C2 = 0.01 ** 2, 0.03 ** 2


def _window():
    k = np.arange(-5, 6)
    w = np.exp(-k * k / (2 * 1.5 ** 2))
    return w / w.sum()


def _ssim_scipy(x, y):
    """The same definition through a library routine: separable zero-padded correlation."""
    w = _window()
    f = lambda a: ndimage.correlate1d(ndimage.correlate1d(a, w, axis=-1, mode="constant"), w, axis=-2, mode="constant")
    m1, m2 = f(x), f(y)
    s1, s2, s12 = f(x * x) - m1 * m1, f(y * y) - m2 * m2, f(x * y) - m1 * m2
    return ((2 * m1 * m2 + C1) * (2 * s12 + C2)) / ((m1 * m1 + m2 * m2 + C1) * (s1 + s2 + C2))


def test_ssim_matches_separable_library_correlation():
    rng = np.random.default_rng(0)
    x = rng.uniform(0, 1, (3, 37, 53))
    y = np.clip(x + rng.normal(0, 0.2, x.shape), 0, 1)
    mean, smap, _ = oracle.ssim(x, y)
    want = _ssim_scipy(x, y)
    assert np.abs(smap - want).max() < 1e-12
    assert mean == pytest.approx(want.mean(), abs=1e-14)
    assert 0.0 < mean < 0.9


def test_ssim_identity_symmetry_and_constant_images():
    rng = np.random.default_rng(1)
    x = rng.uniform(0, 1, (2, 30, 41))
    y = rng.uniform(0, 1, (2, 30, 41))
    assert oracle.ssim(x, x)[0] == pytest.approx(1.0, abs=1e-14)
    assert oracle.ssim(x, y)[0] == pytest.approx(oracle.ssim(y, x)[0], abs=1e-14)
    # constants a and b: away from the border the window sees constants, so variances vanish and
    # SSIM = (2ab + C1) / (a^2 + b^2 + C1); at the border the zero continuation lowers the local means
    a, b = 0.7, 0.4
    _, smap, _ = oracle.ssim(np.full((1, 24, 24), a), np.full((1, 24, 24), b))
    assert np.allclose(smap[0, 5:-5, 5:-5], (2 * a * b + C1) / (a * a + b * b + C1), atol=1e-13)
    # corner pixel: window mass m = (sum_{k>=0} w_k)^2; mu = m a, e11 = m a^2, ...
    w = _window()
    m = w[5:].sum() ** 2
    m1, m2 = m * a, m * b
    s1, s2, s12 = m * a * a - m1 * m1, m * b * b - m2 * m2, m * a * b - m1 * m2
    corner = ((2 * m1 * m2 + C1) * (2 * s12 + C2)) / ((m1 * m1 + m2 * m2 + C1) * (s1 + s2 + C2))
    assert smap[0, 0, 0] == pytest.approx(corner, abs=1e-13)
    # contrast / structure: y = -x + 1 has negative covariance: SSIM below that of an uncorrelated pair
    assert oracle.ssim(x, 1 - x)[0] < oracle.ssim(x, y)[0]


def test_ssim_gradient_by_finite_differences():
    rng = np.random.default_rng(2)
    x = rng.uniform(0.1, 0.9, (2, 17, 19))
    y = rng.uniform(0.1, 0.9, (2, 17, 19))
    _, _, g = oracle.ssim(x, y, want_grad=True)
    h = 1e-6
    idx = [(0, 0, 0), (1, 16, 18), (0, 8, 9), (1, 3, 17), (0, 16, 0), (1, 5, 5), (0, 10, 2)]
    for c, v, u in idx:
        xp = x.copy(); xp[c, v, u] += h
        xm = x.copy(); xm[c, v, u] -= h
        fd = (oracle.ssim(xp, y)[0] - oracle.ssim(xm, y)[0]) / (2 * h)
        assert g[c, v, u] == pytest.approx(fd, rel=2e-6, abs=1e-10)
    # the channel-threaded harness path returns the same numbers
    m1, s1, g1 = oracle.ssim(x, y, want_grad=True, threads=2)
    assert m1 == pytest.approx(oracle.ssim(x, y)[0], abs=1e-15) and np.abs(g1 - g).max() < 1e-17 + 1e-12 * np.abs(g).max()


def test_photometric_loss_and_gradient():
    rng = np.random.default_rng(3)
    x = rng.uniform(0, 1, (3, 20, 23))
    y = rng.uniform(0, 1, (3, 20, 23))
    for lam in (0.0, 0.2, 1.0):
        p = oracle.photometric(x, y, lam)
        assert p["L1"] == pytest.approx(np.abs(x - y).mean())
        assert p["E"] == pytest.approx((1 - lam) * p["L1"] + lam * (1 - p["ssim"]), abs=1e-15)
        h = 1e-6
        for c, v, u in [(0, 0, 0), (2, 19, 22), (1, 10, 11)]:
            xp = x.copy(); xp[c, v, u] += h
            xm = x.copy(); xm[c, v, u] -= h
            fd = (oracle.photometric(xp, y, lam, want_grad=False)["E"] - oracle.photometric(xm, y, lam, want_grad=False)["E"]) / (2 * h)
            assert p["grad"][c, v, u] == pytest.approx(fd, rel=5e-6, abs=1e-10)
    assert oracle.photometric(x, x, 0.2)["E"] == pytest.approx(0.0, abs=1e-14)


def test_prune_score_matches_numpy_and_is_normalised():
    rng = np.random.default_rng(4)
    counts = rng.integers(0, 5000, (10, 1000)).astype(np.int32)
    counts[:, 7] = 0
    E = rng.uniform(0.02, 0.3, 10)
    raw, sp = oracle.prune_score(counts, E)
    want = (counts.astype(np.float64) * E[:, None]).sum(0)
    assert np.allclose(raw, want, rtol=1e-14)
    assert sp.min() == 0.0 and sp.max() == 1.0 and sp[7] == 0.0
    assert np.allclose(sp, (want - want.min()) / (want.max() - want.min()), rtol=1e-13)
    # equal views weights: s_p is the normalised s_d; all-equal sums give zeros
    raw2, sp2 = oracle.prune_score(counts, np.full(10, 0.1))
    sd = counts.sum(0) / 10
    assert np.allclose(sp2, (sd - sd.min()) / (sd.max() - sd.min()), rtol=1e-12)
    assert not oracle.prune_score(np.full((3, 5), 4, np.int32), E[:3])[1].any()
