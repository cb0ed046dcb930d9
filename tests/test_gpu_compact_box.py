"""GPU parity with the Compact Box switched on (Sec. 4.4): the pairs come from the ellipse-tile test.
Same bars as the 3-sigma tests: integer outputs bit-exact against the fp32 oracle, images within
1e-4 relative, gradients within 1e-3 relative with the 2e-3 floor."""
import numpy as np
import pytest

from oracle import Config, Oracle
from paper_2511_04283_amd import scenes
from gpu_common import gpu_pipeline
from test_gpu_parity import check_all, oracle_pipeline

pytestmark = pytest.mark.gpu


def _ctx(beta=1.0, **kw):
    from paper_2511_04283_amd import binding as B
    cfg = B.default_config()
    cfg.compact_box = 1
    cfg.cb_beta = beta
    for k, v in kw.items():
        setattr(cfg, k, v)
    return B.Context("cuda:0", cfg)


def test_config1_everything_compact_box():
    sc = scenes.make_scene(1)
    cam = sc.cameras[0]
    tgt = scenes.target_image(1, 0, cam)
    c = _ctx()
    g = gpu_pipeline(c, sc, cam, target=tgt)
    r = oracle_pipeline(Oracle(np.float32, Config(compact_box=True)), sc, cam, target=tgt)
    r3 = Oracle(np.float32).preprocess(sc, cam)
    assert 0 < r["bins"].num_pairs < int(r3.tiles_touched.sum()) and r["counts"].sum() > 1000
    check_all(g, r, sc)
    c.close()


@pytest.mark.parametrize("deg,beta", [(0, 1.0), (3, 1.0), (1, 0.5), (2, 0.2)])
def test_tiny_scenes_ragged_image_compact_box(deg, beta):
    sc = scenes.tiny_scene(400 + deg, 9000, 203, 117, sh_degree=deg, log_scale=(-2.6, 0.8), spread=1.4)
    sc.sh[:, 0, :] = sc.sh[:, 0, :] * 3.0 - 1.0
    sc.opacities[::11] = 0.0035                            # sigma < 1/255: dropped by the Compact Box
    sc.opacities[5::11] = np.float32(1.0 / 255.0)         # exactly tau_alpha: ratio 1, dropped too
    cam = sc.cameras[0]
    tgt = np.random.default_rng(deg).uniform(0, 1, (3, cam.height, cam.width)).astype(np.float32)
    c = _ctx(beta)
    g = gpu_pipeline(c, sc, cam, target=tgt)
    r = oracle_pipeline(Oracle(np.float32, Config(compact_box=True, cb_beta=beta)), sc, cam, target=tgt)
    p = r["proj"]
    assert (p.tiles_touched == 0).any() and p.clamped.any()
    area = (p.rect[:, 2] - p.rect[:, 0]) * (p.rect[:, 3] - p.rect[:, 1])
    assert (p.tiles_touched < area).any()                  # boxes with corner tiles the ellipse misses
    L = r["bins"].tile_ranges[:, 1] - r["bins"].tile_ranges[:, 0]
    assert L.max() > (256 if beta >= 0.5 else 128)
    check_all(g, r, sc)
    c.close()


def test_config4_cut_two_views_on_one_context_compact_box():
    """Two views in a row on one context: the zeroed gradient records of the second call must not
    depend on what the first left in the scratch buffer."""
    sc = scenes.make_scene(4, 20000)
    c = _ctx()
    o = Oracle(np.float32, Config(compact_box=True))
    for v in (0, 4):
        cam0 = sc.cameras[v]
        cam = scenes.Camera(666 - 100 * v, 438, cam0.fx / 2, cam0.fy / 2, (666 - 100 * v) / 2.0, 219.0, cam0.R, cam0.t)
        tgt = scenes.target_image(4, v, cam)
        g = gpu_pipeline(c, sc, cam, target=tgt)
        r = oracle_pipeline(o, sc, cam, target=tgt)
        check_all(g, r, sc)
    c.close()


def test_huge_gaussian_and_ties_compact_box():
    cam = scenes.Camera(70, 50, 60.0, 60.0, 35.0, 25.0)
    n = 40
    means = np.tile([[0.0, 0.0, 3.0]], (n, 1)).astype(np.float32)
    means[:, 0] = np.linspace(-0.3, 0.3, n)
    sc = scenes.Scene("ties", 0, means, np.full((n, 3), 0.08, np.float32), np.tile([1.0, 0, 0, 0], (n, 1)).astype(np.float32),
                      np.full(n, 0.6, np.float32), np.random.default_rng(1).normal(0.5, 1.0, (n, 1, 3)).astype(np.float32), [cam], 0)
    sc.scales[0] = 5.0
    tgt = np.random.default_rng(2).uniform(0, 1, (3, cam.height, cam.width)).astype(np.float32)
    c = _ctx()
    g = gpu_pipeline(c, sc, cam, target=tgt)
    r = oracle_pipeline(Oracle(np.float32, Config(compact_box=True)), sc, cam, target=tgt)
    assert r["proj"].tiles_touched[0] == 5 * 4
    check_all(g, r, sc)
    c.close()


def test_bad_beta_is_rejected():
    import ctypes
    from paper_2511_04283_amd import binding as B
    lib = B.load_library()
    for beta in (0.0, -1.0, 1.5, float("nan")):
        cfg = B.default_config()
        cfg.compact_box = 1
        cfg.cb_beta = beta
        h = ctypes.c_void_p()
        assert lib.fs_create(ctypes.byref(h), 0, None, ctypes.byref(cfg)) == -1


@pytest.mark.parametrize("compact_box", [0, 1])
def test_lists_too_long_for_the_per_tile_sort_whole_path(compact_box):
    """Lists beyond 8192 entries: fs_bin_sort starts on the per-tile ordering, finds the longest list on the host
    and falls back to the radix sort, making the prefix sums it had skipped.  The whole path (ranges, image,
    gradients through the per-pair records, counts) against the oracle, with and without the Compact Box."""
    from paper_2511_04283_amd import binding as B
    cfg = B.default_config()
    cfg.compact_box = compact_box
    c = B.Context("cuda:0", cfg)
    sc = scenes.tiny_scene(77, 60000, 40, 33, sh_degree=0, log_scale=(-3.2, 0.7), spread=1.1)
    cam = sc.cameras[0]
    tgt = np.random.default_rng(3).uniform(0, 1, (3, cam.height, cam.width)).astype(np.float32)
    o = Oracle(np.float32, Config(compact_box=bool(compact_box)))
    r = oracle_pipeline(o, sc, cam, target=tgt)
    L = r["bins"].tile_ranges[:, 1].astype(np.int64) - r["bins"].tile_ranges[:, 0]
    assert L.max() > 8192
    g = gpu_pipeline(c, sc, cam, target=tgt)
    check_all(g, r, sc)
    c.close()


@pytest.mark.parametrize("compact_box", [0, 1])
def test_radix_ordering_whole_path(compact_box):
    """sort_mode = FS_SORT_RADIX: prefix sums, index-ordered emission, global radix sort -- and everything downstream
    of it (image, gradients through the per-pair records at their prefix-sum places, mask, counts) against the oracle."""
    from paper_2511_04283_amd import binding as B
    cfg = B.default_config()
    cfg.compact_box = compact_box
    cfg.sort_mode = B.FS_SORT_RADIX
    c = B.Context("cuda:0", cfg)
    sc = scenes.tiny_scene(78, 9000, 203, 117, sh_degree=2, log_scale=(-2.6, 0.8), spread=1.4)
    cam = sc.cameras[0]
    tgt = np.random.default_rng(4).uniform(0, 1, (3, cam.height, cam.width)).astype(np.float32)
    r = oracle_pipeline(Oracle(np.float32, Config(compact_box=bool(compact_box))), sc, cam, target=tgt)
    g = gpu_pipeline(c, sc, cam, target=tgt, want_abs=True)
    check_all(g, r, sc)
    c.close()
