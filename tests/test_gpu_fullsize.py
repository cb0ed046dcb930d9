"""GPU parity at the benchmark's full sizes (configs 2-5), in the launch configuration bench.py
times.  The oracle is run in full (all tiles); several Python threads call its single-threaded
routines on disjoint tile subsets to keep the wall time of the test suite reasonable."""
import numpy as np
import pytest

from oracle import Config, Oracle
from paper_2511_04283_amd import scenes
from gpu_common import assert_grads_close, gpu_pipeline

pytestmark = pytest.mark.gpu
THREADS = 14


@pytest.fixture(scope="module")
def ctx():
    from paper_2511_04283_amd import binding as B
    c = B.Context("cuda:0")
    yield c
    c.close()


def _oracle_full(o, sc, cam, target, with_bwd=True, with_score=True):
    proj = o.preprocess(sc, cam)
    bins = o.bin_sort(proj, cam)
    img, fT, nc = o.render_fwd_mt(proj, bins, cam, threads=THREADS)
    out = dict(proj=proj, bins=bins, image=img, final_T=fT, n_contrib=nc)
    out["loss"], dL = o.l1(img, target)
    out["dL"] = dL
    if with_score:
        out["mask"], out["thr"], _ = o.error_mask(img, target, rule=0, k=1.0)
        out["counts"] = o.score_mt(proj, bins, cam, out["mask"], np.zeros(sc.n, np.int32), threads=THREADS)
    if with_bwd:
        out["grads"] = o.backward_mt(sc, cam, proj, bins, dL, threads=THREADS)
    return out


def _check(g, r, with_bwd=True, with_score=True):
    p, b = r["proj"], r["bins"]
    assert np.array_equal(g["tiles_touched"], p.tiles_touched)
    assert np.array_equal(g["rect"], p.rect)
    assert np.array_equal(g["clamped"], p.clamped)
    for k in ("mean2d", "conic_opacity", "rgb", "depth"):
        assert np.array_equal(g[k].view(np.uint32), getattr(p, k).view(np.uint32)), k
    assert g["num_pairs"] == b.num_pairs
    assert np.array_equal(g["keys_sorted"], b.keys_sorted)
    assert np.array_equal(g["gauss_sorted"], b.gauss_sorted)
    assert np.array_equal(g["tile_ranges"], b.tile_ranges)
    assert np.array_equal(g["n_contrib"], r["n_contrib"])
    err = np.abs(g["image"] - r["image"])
    assert (err <= 1e-4 * np.maximum(np.abs(r["image"]), 1e-2)).all(), float(err.max())
    assert np.abs(g["final_T"] - r["final_T"]).max() <= 1e-6
    assert g["loss"] == pytest.approx(r["loss"], rel=1e-6)
    assert np.array_equal(g["dL"], r["dL"])
    if with_score:
        assert np.float32(g["thr"]).view(np.uint32) == np.float32(r["thr"]).view(np.uint32)
        assert np.array_equal(g["mask"], r["mask"])
        assert np.array_equal(g["counts"], r["counts"])
        assert r["counts"].sum() > 0
    if with_bwd:
        assert_grads_close(g["grads"], r["grads"])


def test_config2_full(ctx, orc32):
    sc = scenes.make_scene(2)
    cam = sc.cameras[0]
    tgt = scenes.target_image(2, 0, cam)
    _check(gpu_pipeline(ctx, sc, cam, target=tgt), _oracle_full(orc32, sc, cam, tgt))


def test_config3_full_the_benchmark_workload(ctx, orc32):
    sc = scenes.make_scene(3)
    cam = sc.cameras[0]
    tgt = scenes.target_image(3, 0, cam)
    g = gpu_pipeline(ctx, sc, cam, target=tgt)
    r = _oracle_full(orc32, sc, cam, tgt)
    assert r["bins"].num_pairs == 1357789
    _check(g, r)


def test_config3_full_compact_box():
    """The benchmark workload with the Compact Box: fewer pairs, everything else to the same bar."""
    from paper_2511_04283_amd import binding as B
    sc = scenes.make_scene(3)
    cam = sc.cameras[0]
    tgt = scenes.target_image(3, 0, cam)
    cfg = B.default_config()
    cfg.compact_box = 1
    c = B.Context("cuda:0", cfg)
    g = gpu_pipeline(c, sc, cam, target=tgt)
    c.close()
    r = _oracle_full(Oracle(np.float32, Config(compact_box=True)), sc, cam, tgt)
    assert 0 < r["bins"].num_pairs < 1357789
    _check(g, r)


@pytest.fixture(scope="module")
def scene4():
    return scenes.make_scene(4)


@pytest.mark.parametrize("view", [0, 5, 9])
def test_config4_score_views(ctx, orc32, scene4, view):
    """Per view: forward, error mask (mean + 1 std) and counts, all bit-exact; view 0 also backward."""
    cam = scene4.cameras[view]
    tgt = scenes.target_image(4, view, cam)
    g = gpu_pipeline(ctx, scene4, cam, target=tgt, want_bwd=(view == 0))
    r = _oracle_full(orc32, scene4, cam, tgt, with_bwd=(view == 0))
    _check(g, r, with_bwd=(view == 0))


def test_config4_all_views_binning(ctx, orc32, scene4):
    """Integer stages of every one of the 10 views (keys, order, ranges), plus counts summed over
    views on the GPU being the sum of the per-view counts."""
    import torch
    from paper_2511_04283_amd import binding as B
    g = B.Gaussians.from_scene(scene4, ctx.device)
    total = torch.zeros(scene4.n, dtype=torch.int32, device=ctx.device)
    per_view_sum = np.zeros(scene4.n, np.int64)
    for v, cam in enumerate(scene4.cameras):
        fcam = B.make_camera(cam)
        proj = ctx.fs_preprocess(g, fcam)
        bins = ctx.fs_bin_sort(proj, fcam)
        p_o = orc32.preprocess(scene4, cam)
        b_o = orc32.bin_sort(p_o, cam)
        assert bins.num_pairs == b_o.num_pairs
        assert np.array_equal(bins.copy_keys().cpu().numpy().view(np.uint64), b_o.keys_sorted)
        assert np.array_equal(bins.copy_gauss().cpu().numpy().view(np.uint32), b_o.gauss_sorted)
        assert np.array_equal(bins.copy_ranges().cpu().numpy().view(np.uint32), b_o.tile_ranges)
        image, fT, nc = ctx.fs_render_fwd(proj, bins, fcam)
        tgt = torch.from_numpy(scenes.target_image(4, v, cam)).to(ctx.device)
        mask, thr = ctx.fs_error_mask(image, tgt)
        one = torch.zeros(scene4.n, dtype=torch.int32, device=ctx.device)
        ctx.fs_score_accumulate(proj, bins, fcam, fT, nc, mask, one)
        ctx.fs_score_accumulate(proj, bins, fcam, fT, nc, mask, total)
        per_view_sum += one.cpu().numpy()
    assert np.array_equal(total.cpu().numpy().astype(np.int64), per_view_sum) and per_view_sum.sum() > 0


def test_config5_full(ctx, orc32):
    sc = scenes.make_scene(5)
    cam = sc.cameras[0]
    tgt = scenes.target_image(5, 0, cam)
    g = gpu_pipeline(ctx, sc, cam, target=tgt)
    r = _oracle_full(orc32, sc, cam, tgt)
    assert r["bins"].num_pairs > 9_000_000
    _check(g, r)


def test_config5_wide_tail_27m_pairs(ctx, orc32):
    """Wide-tail variant of config 5 (27 M pairs): the integer stages in full; image, n_contrib, every gradient
    and the counts on a seeded 4 % sample of tiles.  The loss gradient is the L1 gradient inside the sampled tiles
    and zero elsewhere, so that the GPU's per-Gaussian sums over ALL tiles are the oracle's sums over the sample;
    likewise the count pass runs on a seeded mask that is empty outside the sample."""
    import torch
    from paper_2511_04283_amd import binding as B
    sc = scenes.make_scene(5, scale_sigma=1.2)
    cam = sc.cameras[0]
    p_o = orc32.preprocess(sc, cam)
    b_o = orc32.bin_sort(p_o, cam)
    T = b_o.tile_ranges.shape[0]
    tiles = np.sort(np.random.default_rng(7).choice(T, T // 25, replace=False)).astype(np.int32)
    TX = (cam.width + 15) // 16
    sel = np.zeros((cam.height, cam.width), bool)
    for t in tiles:
        sel[(t // TX) * 16:(t // TX) * 16 + 16, (t % TX) * 16:(t % TX) * 16 + 16] = True
    img, fT, nc = orc32.render_fwd_mt(p_o, b_o, cam, tile_list=tiles, threads=THREADS)
    tgt = scenes.target_image(5, 0, cam)
    _, dL_full = orc32.l1(img, tgt)
    dL = np.where(sel[None], dL_full, 0).astype(np.float32)
    mask = ((np.random.default_rng(8).uniform(size=sel.shape) < 0.2) & sel).astype(np.uint8)

    g = gpu_pipeline(ctx, sc, cam, dL=dL)
    assert b_o.num_pairs > 20_000_000 and g["num_pairs"] == b_o.num_pairs
    assert np.array_equal(g["rect"], p_o.rect)
    assert np.array_equal(g["keys_sorted"], b_o.keys_sorted)
    assert np.array_equal(g["gauss_sorted"], b_o.gauss_sorted)
    assert np.array_equal(g["tile_ranges"], b_o.tile_ranges)
    assert np.array_equal(g["n_contrib"][sel], nc[sel])
    err = np.abs(g["image"] - img)[:, sel]
    assert (err <= 1e-4 * np.maximum(np.abs(img[:, sel]), 1e-2)).all()
    # (both sides are handed the same loss gradient, so no sign of image - target is decided twice)
    ref = orc32.backward_mt(sc, cam, p_o, b_o, dL, tile_list=tiles, threads=THREADS)
    assert np.abs(ref["means"]).max() > 0
    assert_grads_close(g["grads"], ref)
    # counts
    gs = B.Gaussians.from_scene(sc, ctx.device)
    fcam = B.make_camera(cam)
    proj = ctx.fs_preprocess(gs, fcam)
    bins = ctx.fs_bin_sort(proj, fcam)
    image, final_T, n_contrib = ctx.fs_render_fwd(proj, bins, fcam)
    counts = torch.zeros(sc.n, dtype=torch.int32, device=ctx.device)
    ctx.fs_score_accumulate(proj, bins, fcam, final_T, n_contrib, torch.from_numpy(mask).to(ctx.device), counts)
    want = orc32.score_mt(p_o, b_o, cam, mask, np.zeros(sc.n, np.int32), tile_list=tiles, threads=THREADS)
    assert want.sum() > 1000
    assert np.array_equal(counts.cpu().numpy(), want)
