"""GPU parity of the per-splat-parallel backward (fs_set_backward_mode(FS_BWD_PER_SPLAT)): the same inputs, outputs
and bars as the per-pixel backward -- gradients within 1e-3 relative with the 2e-3 floor of the fp32 oracle -- on
scenes that reach its branches: lists of one and of several batches, quadrant lists of more than one 64-entry chunk,
pixels that stop early, ragged images, the absolute gradient, the Compact Box; and against the per-pixel kernel."""
import numpy as np
import pytest

from oracle import Config, Oracle
from paper_2511_04283_amd import scenes
from gpu_common import assert_grads_close, gpu_pipeline
from test_gpu_parity import check_all, oracle_pipeline

pytestmark = pytest.mark.gpu


def _ctx(compact_box=False):
    from paper_2511_04283_amd import binding as B
    cfg = B.default_config()
    cfg.compact_box = int(compact_box)
    c = B.Context("cuda:0", cfg)
    c.fs_set_backward_mode(B.FS_BWD_PER_SPLAT)
    return c


def test_config1_everything_per_splat():
    sc = scenes.make_scene(1)
    cam = sc.cameras[0]
    tgt = scenes.target_image(1, 0, cam)
    c = _ctx()
    g = gpu_pipeline(c, sc, cam, target=tgt)
    r = oracle_pipeline(Oracle(np.float32), sc, cam, target=tgt)
    check_all(g, r, sc)
    c.close()


@pytest.mark.parametrize("deg,cb,want_abs", [(0, False, False), (3, False, True), (1, True, False), (2, True, True)])
def test_tiny_scenes_ragged_image_per_splat(deg, cb, want_abs):
    sc = scenes.tiny_scene(300 + deg, 9000 if cb else 3000, 203, 117, sh_degree=deg, log_scale=(-2.6, 0.8), spread=1.4)
    sc.sh[:, 0, :] = sc.sh[:, 0, :] * 3.0 - 1.0
    cam = sc.cameras[0]
    tgt = np.random.default_rng(deg).uniform(0, 1, (3, cam.height, cam.width)).astype(np.float32)
    c = _ctx(cb)
    g = gpu_pipeline(c, sc, cam, target=tgt, want_abs=want_abs)
    r = oracle_pipeline(Oracle(np.float32, Config(compact_box=cb)), sc, cam, target=tgt)
    L = r["bins"].tile_ranges[:, 1] - r["bins"].tile_ranges[:, 0]
    assert L.max() > 256                                   # several LDS batches per tile
    if want_abs:
        assert "mean2d_abs" in g["grads"] and np.abs(r["grads"]["mean2d_abs"]).max() > 0
    check_all(g, r, sc)
    c.close()


@pytest.mark.parametrize("case", ["long_lists", "opaque"])
def test_long_lists_and_early_stops_per_splat(case):
    """long_lists: tile lists of thousands of entries, quadrant lists of several 64-entry chunks per batch.
    opaque: most pixels stop long before the end of their list (states that stay untouched for whole batches)."""
    if case == "long_lists":
        sc = scenes.tiny_scene(812, 30000, 70, 50, sh_degree=0, log_scale=(-3.2, 0.7), spread=1.1)
    else:
        sc = scenes.tiny_scene(811, 9000, 150, 90, sh_degree=0, log_scale=(-1.6, 0.5), spread=1.0)
        sc.opacities[:] = 0.97
    cam = sc.cameras[0]
    tgt = np.random.default_rng(5).uniform(0, 1, (3, cam.height, cam.width)).astype(np.float32)
    c = _ctx()
    g = gpu_pipeline(c, sc, cam, target=tgt, want_score=False)
    r = oracle_pipeline(Oracle(np.float32), sc, cam, target=tgt)
    L = r["bins"].tile_ranges[:, 1] - r["bins"].tile_ranges[:, 0]
    assert L.max() > 1000
    check_all(g, r, sc)
    c.close()


def test_per_splat_against_per_pixel_config2_cut():
    """The two mappings on the same inputs: equal up to the order of the floating-point sums."""
    from paper_2511_04283_amd import binding as B
    sc = scenes.make_scene(2, 20000)
    cam = sc.cameras[0]
    tgt = scenes.target_image(2, 0, cam)
    a = B.Context("cuda:0")
    ga = gpu_pipeline(a, sc, cam, target=tgt, want_score=False, want_abs=True)
    a.close()
    b = _ctx()
    gb = gpu_pipeline(b, sc, cam, target=tgt, want_score=False, want_abs=True)
    b.close()
    assert_grads_close(gb["grads"], {k: v.astype(np.float64) for k, v in ga["grads"].items()}, rtol=2e-4, floor=1e-4)
    r = oracle_pipeline(Oracle(np.float32), sc, cam, target=tgt)
    check_all(gb, r, sc)


def test_per_splat_config3_full_against_the_oracle_and_the_per_pixel_kernel():
    """Benchmark size (500k Gaussians, 1600x1064, 1.36 M pairs), the launch configuration bench.py times: every
    gradient of the per-splat mapping against the oracle at the gradient tolerance, and against the per-pixel
    kernel's to a fifth of it."""
    from paper_2511_04283_amd import binding as B
    sc = scenes.make_scene(3)
    cam = sc.cameras[0]
    tgt = scenes.target_image(3, 0, cam)
    a = B.Context("cuda:0")
    ga = gpu_pipeline(a, sc, cam, target=tgt, want_score=False, want_abs=True)
    a.close()
    b = _ctx()
    gb = gpu_pipeline(b, sc, cam, target=tgt, want_score=False, want_abs=True)
    b.close()
    assert np.abs(ga["grads"]["means"]).max() > 0
    assert_grads_close(gb["grads"], {k: v.astype(np.float64) for k, v in ga["grads"].items()}, rtol=2e-4, floor=4e-4)
    o = Oracle(np.float32)
    proj = o.preprocess(sc, cam)
    bins = o.bin_sort(proj, cam)
    img, fT, nc = o.render_fwd_mt(proj, bins, cam, threads=14)
    _, dL = o.l1(img, tgt)
    ref = o.backward_mt(sc, cam, proj, bins, dL, threads=14)
    assert np.array_equal(gb["n_contrib"], nc)
    assert_grads_close(gb["grads"], ref)


def test_unknown_backward_mode_is_rejected():
    from paper_2511_04283_amd import binding as B
    c = B.Context("cuda:0")
    with pytest.raises(RuntimeError):
        c.fs_set_backward_mode(7)
    c.fs_set_backward_mode(B.FS_BWD_PER_SPLAT)
    c.fs_set_backward_mode(B.FS_BWD_PER_PIXEL)
    with pytest.raises(RuntimeError):
        c.fs_set_record_mode(3)
    for mode in (B.FS_RECORDS_SPARSE, B.FS_RECORDS_DENSE, B.FS_RECORDS_AUTO):
        c.fs_set_record_mode(mode)
    c.close()
