"""GPU parity: the HIP path (through the C ABI) against the fp32 CPU oracle on the same seeded
inputs.  Integer outputs (tile rectangles, keys, order, ranges, n_contrib, mask, counts) must be
bit-exact; images within 1e-4 relative; gradients within 1e-3 relative with the 2e-3 floor."""
import numpy as np
import pytest

from oracle import Config, Oracle
from paper_2511_04283_amd import scenes
from gpu_common import assert_grads_close, assert_image_close, gpu_pipeline

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    from paper_2511_04283_amd import binding as B
    c = B.Context("cuda:0")
    yield c
    c.close()


def oracle_pipeline(o, sc, cam, target=None, dL=None):
    proj, bins, img, fT, nc = o.forward(sc, cam)
    out = dict(proj=proj, bins=bins, image=img, final_T=fT, n_contrib=nc)
    if target is not None:
        out["loss"], dl = o.l1(img, target)
        out["dL"] = dl
        out["mask"], out["thr"], out["err"] = o.error_mask(img, target, rule=0, k=1.0)
        out["counts"] = o.score(proj, bins, cam, out["mask"], np.zeros(sc.n, np.int32))
    else:
        dl = dL
    if dl is not None:
        out["grads"] = o.backward(sc, cam, proj, bins, dl)
    return out


def check_all(g, r, sc, image_rtol=1e-4):
    p, b = r["proj"], r["bins"]
    # a1: integer decisions bit-exact; floats bit-exact too (same operation order)
    assert np.array_equal(g["tiles_touched"], p.tiles_touched)
    assert np.array_equal(g["rect"], p.rect)
    assert np.array_equal(g["clamped"], p.clamped)
    assert np.array_equal(g["depth"].view(np.uint32), p.depth.view(np.uint32))
    for k in ("mean2d", "conic_opacity", "rgb"):
        assert np.array_equal(g[k].view(np.uint32), getattr(p, k).view(np.uint32)), k
    # a2-a5
    assert g["num_pairs"] == b.num_pairs
    assert np.array_equal(g["keys_sorted"], b.keys_sorted)
    assert np.array_equal(g["gauss_sorted"], b.gauss_sorted)
    assert np.array_equal(g["tile_ranges"], b.tile_ranges)
    # a6
    assert np.array_equal(g["n_contrib"], r["n_contrib"])
    assert np.abs(g["final_T"] - r["final_T"]).max() <= 1e-6
    assert_image_close(g["image"], r["image"], image_rtol)
    if "loss" in r and "loss" in g:
        assert g["loss"] == pytest.approx(r["loss"], rel=1e-6)
        assert np.array_equal(g["dL"], r["dL"])
    if "mask" in r and "mask" in g:
        assert np.float32(g["thr"]).view(np.uint32) == np.float32(r["thr"]).view(np.uint32)
        assert np.array_equal(g["mask"], r["mask"])
        assert np.array_equal(g["counts"], r["counts"])
    if "grads" in r and "grads" in g:
        ref = dict(r["grads"])
        assert_grads_close(g["grads"], ref)


def test_config1_everything(ctx, orc32):
    sc = scenes.make_scene(1)
    cam = sc.cameras[0]
    tgt = scenes.target_image(1, 0, cam)
    g = gpu_pipeline(ctx, sc, cam, target=tgt)
    r = oracle_pipeline(orc32, sc, cam, target=tgt)
    assert r["bins"].num_pairs == 10642 and r["counts"].sum() > 1000
    check_all(g, r, sc)
    assert np.array_equal(g["image"], r["image"])     # same operation order: identical bits expected


@pytest.mark.parametrize("deg", [0, 1, 2, 3])
def test_tiny_scenes_all_sh_degrees_ragged_image(ctx, orc32, deg):
    # 203x117 is not a multiple of the tile size: ragged right and bottom tiles; wide spread -> culling
    sc = scenes.tiny_scene(300 + deg, 3000, 203, 117, sh_degree=deg, log_scale=(-2.6, 0.8), spread=1.4)
    sc.sh[:, 0, :] = sc.sh[:, 0, :] * 3.0 - 1.0          # some colours go negative: clamp path
    cam = sc.cameras[0]
    tgt = np.random.default_rng(deg).uniform(0, 1, (3, cam.height, cam.width)).astype(np.float32)
    g = gpu_pipeline(ctx, sc, cam, target=tgt)
    r = oracle_pipeline(orc32, sc, cam, target=tgt)
    assert (r["proj"].tiles_touched == 0).any() and r["proj"].clamped.any()
    L = r["bins"].tile_ranges[:, 1] - r["bins"].tile_ranges[:, 0]
    assert L.max() > 256                                   # several LDS batches per tile
    check_all(g, r, sc)


def test_config2_cut_20k(ctx, orc32):
    sc = scenes.make_scene(2, 20000)
    cam = sc.cameras[0]
    tgt = scenes.target_image(2, 0, cam)
    g = gpu_pipeline(ctx, sc, cam, target=tgt)
    r = oracle_pipeline(orc32, sc, cam, target=tgt)
    check_all(g, r, sc)


def test_both_score_modes_and_minmax_mask(ctx):
    from paper_2511_04283_amd import binding as B
    import torch
    sc = scenes.tiny_scene(77, 1500, 160, 96, sh_degree=1, log_scale=(-2.5, 0.6))
    cam = sc.cameras[0]
    tgt = np.random.default_rng(5).uniform(0, 1, (3, cam.height, cam.width)).astype(np.float32)
    for mode in (0, 1):
        cfg = B.default_config()
        cfg.score_mode = mode
        c = B.Context("cuda:0", cfg)
        o = Oracle(np.float32, Config(score_mode=mode))
        g = gpu_pipeline(c, sc, cam, target=tgt, mask_rule=1, mask_k=0.35, want_bwd=False)
        proj, bins, img, fT, nc = o.forward(sc, cam)
        mask, thr, _ = o.error_mask(img, tgt, rule=1, k=0.35)
        counts = o.score(proj, bins, cam, mask, np.zeros(sc.n, np.int32))
        assert np.float32(g["thr"]).view(np.uint32) == np.float32(thr).view(np.uint32)
        assert np.array_equal(g["mask"], mask) and 0.02 < mask.mean() < 0.9
        assert np.array_equal(g["counts"], counts) and counts.sum() > 0
        c.close()


def test_counts_accumulate_over_views(ctx, orc32):
    """Config-4 shape in small: several cameras, counts summed over views (bit-exact)."""
    import torch
    from paper_2511_04283_amd import binding as B
    sc = scenes.make_scene(4, 6000)
    views = sc.cameras[::3]
    g = B.Gaussians.from_scene(sc, ctx.device)
    counts = torch.zeros(sc.n, dtype=torch.int32, device=ctx.device)
    ref = np.zeros(sc.n, np.int32)
    for v, cam0 in enumerate(views):
        cam = scenes.Camera(333, 219, cam0.fx / 4, cam0.fy / 4, 333 / 2.0, 219 / 2.0, cam0.R, cam0.t)
        tgt = scenes.target_image(4, v, cam)
        fcam = B.make_camera(cam)
        proj = ctx.fs_preprocess(g, fcam)
        bins = ctx.fs_bin_sort(proj, fcam)
        image, fT, nc = ctx.fs_render_fwd(proj, bins, fcam)
        mask, thr = ctx.fs_error_mask(image, torch.from_numpy(tgt).to(ctx.device))
        ctx.fs_score_accumulate(proj, bins, fcam, fT, nc, mask, counts)
        r = oracle_pipeline(orc32, sc, cam, target=tgt)
        assert np.array_equal(mask.cpu().numpy(), r["mask"])
        ref += r["counts"]
    assert np.array_equal(counts.cpu().numpy(), ref) and ref.sum() > 0


def test_degenerate_inputs(ctx, orc32):
    from paper_2511_04283_amd import binding as B
    import torch
    cam = scenes.Camera(70, 50, 60.0, 60.0, 35.0, 25.0)
    # (1) no Gaussians at all; (2) every Gaussian culled: the image is the background
    empty = scenes.Scene("empty", 1, np.zeros((0, 3), np.float32), np.zeros((0, 3), np.float32), np.zeros((0, 4), np.float32),
                         np.zeros(0, np.float32), np.zeros((0, 4, 3), np.float32), [cam], 0)
    behind = scenes.tiny_scene(5, 40, 70, 50, sh_degree=1)
    behind.means = (behind.means - 100 * behind.cameras[0].R[2]).astype(np.float32)   # push behind the camera
    cfg = B.default_config()
    cfg.bg[0], cfg.bg[1], cfg.bg[2] = 0.25, 0.5, 0.75
    c = B.Context("cuda:0", cfg)
    for sc, cm in ((empty, cam), (behind, behind.cameras[0])):
        dL = np.ones((3, cm.height, cm.width), np.float32)
        g = gpu_pipeline(c, sc, cm, dL=dL)
        assert g["num_pairs"] == 0 and not g["tile_ranges"].any() and not g["n_contrib"].any()
        assert np.array_equal(g["final_T"], np.ones_like(g["final_T"]))
        assert np.allclose(g["image"], np.array([0.25, 0.5, 0.75], np.float32)[:, None, None])
        for k, v in g["grads"].items():
            assert not v.any(), k
    c.close()
    # (3) one huge Gaussian over every tile, plus equal-depth ties
    n = 40
    means = np.tile([[0.0, 0.0, 3.0]], (n, 1)).astype(np.float32)
    means[:, 0] = np.linspace(-0.3, 0.3, n)
    sc = scenes.Scene("ties", 0, means, np.full((n, 3), 0.08, np.float32), np.tile([1.0, 0, 0, 0], (n, 1)).astype(np.float32),
                      np.full(n, 0.6, np.float32), np.random.default_rng(1).normal(0.5, 1.0, (n, 1, 3)).astype(np.float32), [cam], 0)
    sc.scales[0] = 5.0
    tgt = np.random.default_rng(2).uniform(0, 1, (3, cam.height, cam.width)).astype(np.float32)
    g = gpu_pipeline(ctx, sc, cam, target=tgt)
    r = oracle_pipeline(orc32, sc, cam, target=tgt)
    assert r["proj"].tiles_touched[0] == 5 * 4
    check_all(g, r, sc)


def test_error_codes(ctx):
    import ctypes
    from paper_2511_04283_amd import binding as B
    lib = B.load_library()
    assert lib.fs_preprocess(None, None, None, None) == -1
    bad = B.default_config()
    bad.tile = 8
    h = ctypes.c_void_p()
    assert lib.fs_create(ctypes.byref(h), 0, None, ctypes.byref(bad)) == -1
    cam = B.make_camera(scenes.Camera(0, 10, 1.0, 1.0, 0.0, 0.0))
    g = B.fs_gaussians()
    p = B.fs_projected()
    assert lib.fs_preprocess(ctx.handle, ctypes.byref(g), ctypes.byref(cam), ctypes.byref(p)) == -1
    assert b"fs_preprocess" in lib.fs_last_error(ctx.handle)


@pytest.mark.parametrize("n,W,H,mode,lo,hi", [
    (3000, 203, 117, 1, 0, 2048),          # forced global radix sort
    (3000, 203, 117, 0, 0, 2048),          # per-tile LDS sort, 16 KB variant
    (40000, 70, 50, 0, 2049, 8192),        # lists that need the 64 KB variant
    (40000, 70, 50, 1, 2049, 8192),
    (45000, 40, 33, 0, 8193, 16384),       # a list that needs the 144 KB variant
    (90000, 40, 33, 0, 16385, 10 ** 9),    # lists beyond LDS: automatic fall-back to the radix sort
])
def test_pair_order_is_the_same_whichever_way_it_is_computed(orc32, n, W, H, mode, lo, hi):
    """Keys, order and ranges bit-exact for both orderings of fs_bin_sort, at list lengths that reach
    each of its code paths; image and n_contrib as well."""
    from paper_2511_04283_amd import binding as B
    cfg = B.default_config()
    cfg.sort_mode = mode
    c = B.Context("cuda:0", cfg)
    sc = scenes.tiny_scene(900 + n % 97, n, W, H, sh_degree=0, log_scale=(-3.2, 0.7), spread=1.1)
    sc.means[5:400:5, 2] = sc.means[5, 2]                  # equal depths: ties broken by index
    cam = sc.cameras[0]
    g = gpu_pipeline(c, sc, cam)
    p_o = orc32.preprocess(sc, cam)
    b_o = orc32.bin_sort(p_o, cam)
    L = b_o.tile_ranges[:, 1].astype(np.int64) - b_o.tile_ranges[:, 0]
    assert lo <= L.max() <= hi, int(L.max())
    assert g["num_pairs"] == b_o.num_pairs
    assert np.array_equal(g["keys_sorted"], b_o.keys_sorted)
    assert np.array_equal(g["gauss_sorted"], b_o.gauss_sorted)
    assert np.array_equal(g["tile_ranges"], b_o.tile_ranges)
    if n <= 45000:
        img, fT, nc = orc32.render_fwd_mt(p_o, b_o, cam, threads=8)
        assert np.array_equal(g["n_contrib"], nc)
        assert_image_close(g["image"], img)
    c.close()


def test_more_tiles_than_the_lds_counters_hold(ctx, orc32):
    """2016 x 2000 px = 126 x 125 = 15 750 tiles: beyond the per-tile LDS counters of the tile-bucketed
    ordering, so fs_bin_sort takes the radix path by itself; results as everywhere else."""
    sc = scenes.tiny_scene(31, 4000, 2016, 2000, sh_degree=0, log_scale=(-2.5, 0.8), spread=1.0)
    cam = sc.cameras[0]
    g = gpu_pipeline(ctx, sc, cam)
    p_o = orc32.preprocess(sc, cam)
    b_o = orc32.bin_sort(p_o, cam)
    assert b_o.tile_ranges.shape[0] == 126 * 125 and b_o.num_pairs > 10000
    assert g["num_pairs"] == b_o.num_pairs
    assert np.array_equal(g["keys_sorted"], b_o.keys_sorted)
    assert np.array_equal(g["gauss_sorted"], b_o.gauss_sorted)
    assert np.array_equal(g["tile_ranges"], b_o.tile_ranges)
    img, fT, nc = orc32.render_fwd_mt(p_o, b_o, cam, threads=8)
    assert np.array_equal(g["n_contrib"], nc)
    assert_image_close(g["image"], img)


def test_as_many_tiles_as_the_lds_counters_hold(orc32):
    """1920 x 2048 px = 120 x 128 = 15 360 tiles: the most the per-tile LDS counters of the tile-bucketed ordering take
    (60 KB of dynamic LDS beside the kernels' static arrays).  Two calls on one context: the second one enqueues its
    placement ahead of the read-back.  Keys, order and ranges bit-exact both times."""
    from paper_2511_04283_amd import binding as B
    c = B.Context("cuda:0")
    for seed, n in ((41, 5000), (42, 7000)):
        sc = scenes.tiny_scene(seed, n, 1920, 2048, sh_degree=0, log_scale=(-2.5, 0.8), spread=1.0)
        cam = sc.cameras[0]
        g = B.Gaussians.from_scene(sc, c.device)
        fcam = B.make_camera(cam)
        bins = c.fs_bin_sort(c.fs_preprocess(g, fcam), fcam)
        p_o = orc32.preprocess(sc, cam)
        b_o = orc32.bin_sort(p_o, cam)
        assert b_o.tile_ranges.shape[0] == 15360 and b_o.num_pairs > 10000
        assert bins.num_pairs == b_o.num_pairs
        assert np.array_equal(bins.copy_keys().cpu().numpy().view(np.uint64), b_o.keys_sorted)
        assert np.array_equal(bins.copy_gauss().cpu().numpy().view(np.uint32), b_o.gauss_sorted)
        assert np.array_equal(bins.copy_ranges().cpu().numpy().view(np.uint32), b_o.tile_ranges)
        order = bins.copy_order().cpu().numpy().astype(np.int64)
        assert np.array_equal(np.sort(order), np.arange(15360))
    c.close()


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("n,W,H", [(3000, 203, 117), (60000, 640, 400), (500, 1600, 1064)])
def test_tile_order_is_a_permutation_with_the_longest_lists_first(n, W, H, mode):
    """bins.tile_order (the order in which the render kernels take the tiles) holds every tile once, and list
    lengths, in units of 8 entries capped at 511 units, never increase along it -- from both orderings."""
    from paper_2511_04283_amd import binding as B
    cfg = B.default_config()
    cfg.sort_mode = mode
    c = B.Context("cuda:0", cfg)
    sc = scenes.tiny_scene(40 + n % 7, n, W, H, sh_degree=0, log_scale=(-3.0, 0.8), spread=1.1)
    g = B.Gaussians.from_scene(sc, c.device)
    fcam = B.make_camera(sc.cameras[0])
    bins = c.fs_bin_sort(c.fs_preprocess(g, fcam), fcam)
    order = bins.copy_order().cpu().numpy().astype(np.int64)
    r = bins.copy_ranges().cpu().numpy().view(np.uint32).astype(np.int64)
    T = ((W + 15) // 16) * ((H + 15) // 16)
    assert order.shape == (T,) and np.array_equal(np.sort(order), np.arange(T))
    units = np.minimum((r[:, 1] - r[:, 0])[order] >> 3, 511)
    assert (np.diff(units) <= 0).all() and units[0] > 0
    c.close()


@pytest.mark.parametrize("records", ["auto", "sparse"])
@pytest.mark.parametrize("compact_box", [0, 1])
def test_one_context_through_growing_and_shrinking_pair_counts(orc32, compact_box, records):
    """A context keeps its scratch buffers from call to call and grows them when a call needs more. One
    context therefore goes through: a first call, a much larger scene (buffers grow), smaller ones (buffers
    larger than needed), long lists after short ones and short after long (the LDS sort variants), lists beyond
    LDS (the radix path) between per-tile orderings, a scene without pairs, and another tile grid. From its second
    per-tile ordering on, fs_bin_sort enqueues placement and sorts before it has read the totals back, sized by the
    previous call: every transition above is one where that guess is right, too small, or too large. Keys, order,
    ranges and n_contrib bit-exact every time; on the small scenes the gradients as well (with the Compact Box the
    placement also zeroes the records of the candidates that are no pairs).  records: the layout of the backward
    pass's per-pair records -- chosen per call by the lists' mean length, or sparse throughout (its flag array, too, is
    kept from call to call, must grow, and must be all zeros again after every call)."""
    from paper_2511_04283_amd import binding as B
    cfg = B.default_config()
    cfg.compact_box = compact_box
    cfg.cb_beta = 0.7
    c = B.Context("cuda:0", cfg)
    if records == "sparse":
        c.fs_set_record_mode(B.FS_RECORDS_SPARSE)
    o = Oracle(np.float32, Config(compact_box=compact_box, cb_beta=0.7)) if compact_box else orc32
    cases = [(700, 2000, 203, 117, (-3.2, 0.7)),    # short lists
             (701, 30000, 203, 117, (-3.2, 0.7)),   # many more pairs: buffers grow
             (702, 9000, 203, 117, (-3.2, 0.7)),    # fewer again
             (703, 40000, 70, 50, (-3.2, 0.7)),     # lists beyond 2048 after short ones
             (704, 40000, 70, 50, (-3.2, 0.7)),     # ... and again
             (705, 1500, 70, 50, (-3.2, 0.7)),      # short after long
             (706, 0, 70, 50, (-3.2, 0.7)),         # nothing to order
             (707, 5000, 333, 219, (-3.0, 0.6)),    # another tile grid
             (708, 45000, 40, 33, (-3.2, 0.7)),     # a list beyond 8192 after short ones
             (709, 2500, 40, 33, (-3.2, 0.7)),      # short after that
             (710, 90000, 40, 33, (-3.2, 0.7)),     # lists beyond LDS: the radix path, whatever was enqueued ahead
             (711, 2500, 40, 33, (-3.2, 0.7)),      # per-tile again after the radix path
             (712, 2600, 40, 33, (-3.2, 0.7)),
             # the sort launches differ with the mix of list lengths: lists long throughout (more than 1024 entries on
             # average) get a launch for (2048, 4096] and one for (4096, 8192], a few long lists among short ones a
             # single launch for (2048, 8192]; what was enqueued ahead comes from the previous call's choice
             (715, 22000, 70, 50, (-3.2, 0.7)),           # long throughout, none beyond 4096
             (703, 40000, 70, 50, (-3.2, 0.7)),           # ... now some beyond 4096: only that launch is missing
             (713, 12000, 203, 117, (-3.6, 0.5), 0.25),   # a few long lists (up to 5989) among short ones
             (715, 22000, 70, 50, (-3.2, 0.7)),           # long throughout after the single launch
             (713, 12000, 203, 117, (-3.6, 0.5), 0.25),
             (709, 2500, 40, 33, (-3.2, 0.7))]
    seen_long = seen_huge = seen_radix = seen_few_long = False
    for seed, n, W, H, ls, *rest in cases:
        spread = rest[0] if rest else 1.1
        if n == 0:
            cam = scenes.Camera(W, H, 60.0, 60.0, W / 2.0, H / 2.0)
            sc = scenes.Scene("empty", 0, np.zeros((0, 3), np.float32), np.zeros((0, 3), np.float32),
                              np.zeros((0, 4), np.float32), np.zeros(0, np.float32), np.zeros((0, 1, 3), np.float32), [cam], 0)
        else:
            sc = scenes.tiny_scene(seed, n, W, H, sh_degree=0, log_scale=ls, spread=spread)
            cam = sc.cameras[0]
        small = 0 < n <= 9000
        dL = np.random.default_rng(seed).standard_normal((3, H, W)).astype(np.float32) if small else None
        g = gpu_pipeline(c, sc, cam, dL=dL)
        p_o = o.preprocess(sc, cam)
        b_o = o.bin_sort(p_o, cam)
        L = b_o.tile_ranges[:, 1].astype(np.int64) - b_o.tile_ranges[:, 0]
        seen_long |= bool(L.max() > 2048)
        seen_huge |= bool(8192 < L.max() <= 16384)
        seen_radix |= bool(L.max() > 16384)
        seen_few_long |= bool(L.max() > 4096 and b_o.num_pairs <= 1024 * L.size)
        assert g["num_pairs"] == b_o.num_pairs, (seed, n)
        assert np.array_equal(g["keys_sorted"], b_o.keys_sorted), (seed, n)
        assert np.array_equal(g["gauss_sorted"], b_o.gauss_sorted), (seed, n)
        assert np.array_equal(g["tile_ranges"], b_o.tile_ranges), (seed, n)
        if n <= 9000:
            img, fT, nc = o.render_fwd_mt(p_o, b_o, cam, threads=8)
            assert np.array_equal(g["n_contrib"], nc), (seed, n)
            assert_image_close(g["image"], img)
        if small:
            assert_grads_close(g["grads"], o.backward(sc, cam, p_o, b_o, dL))
    assert seen_long and seen_huge and seen_radix and seen_few_long
    c.close()


@pytest.mark.parametrize("W,H,rule,k", [(203, 117, 0, 1.0), (128, 96, 1, 0.35)])
def test_fused_forward_gives_what_the_separate_calls_give(ctx, orc32, W, H, rule, k):
    """fs_render_fwd_loss + fs_error_mask_fused against fs_render_fwd + fs_l1_grad + fs_error_mask (bit-exact
    image, n_contrib, dL, mask, threshold; the loss to rounding) and against the oracle."""
    import torch
    from paper_2511_04283_amd import binding as B
    sc = scenes.tiny_scene(700 + W, 4000, W, H, sh_degree=1, log_scale=(-2.6, 0.7), spread=1.2)
    cam = sc.cameras[0]
    tgt_np = np.random.default_rng(W).uniform(0, 1, (3, H, W)).astype(np.float32)
    g = B.Gaussians.from_scene(sc, ctx.device)
    fcam = B.make_camera(cam)
    tgt = torch.from_numpy(tgt_np).to(ctx.device)
    proj = ctx.fs_preprocess(g, fcam)
    bins = ctx.fs_bin_sort(proj, fcam)
    img_a, T_a, nc_a = ctx.fs_render_fwd(proj, bins, fcam)
    loss_a = torch.zeros(1, dtype=torch.float64, device=ctx.device)
    dL_a = ctx.fs_l1_grad(img_a, tgt, loss_out=loss_a)
    mask_a, thr_a = ctx.fs_error_mask(img_a, tgt, rule, k)
    loss_b = torch.zeros(1, dtype=torch.float64, device=ctx.device)
    img_b, T_b, nc_b, dL_b = ctx.fs_render_fwd_loss(proj, bins, fcam, tgt, loss_out=loss_b)
    mask_b, thr_b = ctx.fs_error_mask_fused(H, W, rule, k)
    mask_c, thr_c = ctx.fs_error_mask_fused(H, W, rule, k)           # the map may be used again
    for a, b in ((img_a, img_b), (T_a, T_b), (nc_a, nc_b), (dL_a, dL_b), (mask_a, mask_b), (mask_b, mask_c)):
        assert torch.equal(a, b)
    assert thr_a.item() == thr_b.item() == thr_c.item()
    assert loss_b.item() == pytest.approx(loss_a.item(), rel=1e-12)
    img_o = orc32.forward(sc, cam)[2]
    l_o, dL_o = orc32.l1(img_o, tgt_np)
    m_o, thr_o, _ = orc32.error_mask(img_o, tgt_np, rule=rule, k=k)
    assert loss_b.item() == pytest.approx(l_o, rel=1e-6) and np.array_equal(dL_b.cpu().numpy(), dL_o)
    assert np.array_equal(mask_b.cpu().numpy(), m_o) and 0.01 < m_o.mean() < 0.9
    # another call that uses the same scratch discards the pending map
    ctx.fs_l1_grad(img_a, tgt)
    with pytest.raises(RuntimeError):
        ctx.fs_error_mask_fused(H, W, rule, k)


@pytest.mark.parametrize("W,H,rule,k", [(203, 117, 0, 1.0), (128, 96, 1, 0.35), (100, 37, 0, 0.5), (64, 48, 1, 0.2)])
def test_mask_and_counts_in_one_call(ctx, orc32, W, H, rule, k):
    """fs_mask_score_fused against fs_error_mask_fused + fs_score_accumulate and against the oracle: mask, threshold
    and counts bit-exact -- with the forward pass's record (one kernel; widths that are and are not multiples of
    four take different store paths) and without it (the two kernels of the separate calls)."""
    import torch
    from paper_2511_04283_amd import binding as B
    sc = scenes.tiny_scene(900 + W, 5000, W, H, sh_degree=0, log_scale=(-2.7, 0.7), spread=1.2)
    cam = sc.cameras[0]
    tgt_np = np.random.default_rng(W + 1).uniform(0, 1, (3, H, W)).astype(np.float32)
    g = B.Gaussians.from_scene(sc, ctx.device)
    fcam = B.make_camera(cam)
    tgt = torch.from_numpy(tgt_np).to(ctx.device)
    p_o, b_o, img_o, _, _ = orc32.forward(sc, cam)
    m_o, thr_o, _ = orc32.error_mask(img_o, tgt_np, rule=rule, k=k)
    ref = orc32.score(p_o, b_o, cam, m_o, np.zeros(sc.n, np.int32))
    assert ref.sum() > 0 and 0.01 < m_o.mean() < 0.95
    proj = ctx.fs_preprocess(g, fcam)
    bins = ctx.fs_bin_sort(proj, fcam)
    for record in (True, False):
        ctx.fs_set_score_record(record)
        img, fT, nc, dL = ctx.fs_render_fwd_loss(proj, bins, fcam, tgt)
        mask_a, thr_a = ctx.fs_error_mask_fused(H, W, rule, k)
        cnt_a = torch.zeros(sc.n, dtype=torch.int32, device=ctx.device)
        ctx.fs_score_accumulate(proj, bins, fcam, fT, nc, mask_a, cnt_a)
        cnt_b = torch.full((sc.n,), 7, dtype=torch.int32, device=ctx.device)     # (the counts are added to)
        mask_b = torch.full((H, W), 9, dtype=torch.uint8, device=ctx.device)
        mask_b, thr_b, _ = ctx.fs_mask_score_fused(proj, bins, fcam, nc, cnt_b, rule, k, mask=mask_b)
        assert torch.equal(mask_a, mask_b) and thr_a.item() == thr_b.item(), record
        assert torch.equal(cnt_a + 7, cnt_b), record
        assert np.array_equal(mask_b.cpu().numpy(), m_o), record
        assert np.float32(thr_b.item()).view(np.uint32) == np.float32(thr_o).view(np.uint32), record
        assert np.array_equal(cnt_a.cpu().numpy(), ref), record
    ctx.fs_set_score_record(True)
    # without a pending error map the call is refused
    ctx.fs_l1_grad(img, tgt)
    with pytest.raises(RuntimeError):
        ctx.fs_mask_score_fused(proj, bins, fcam, nc, cnt_b, rule, k)


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("case", ["transparent", "opaque", "long_lists"])
def test_counts_from_the_forward_record_equal_the_walk_and_the_oracle(orc32, mode, case):
    """fs_score_accumulate from the per-pair record of the forward pass (either forward entry point) against
    fs_score_accumulate without a record (second walk over the lists) and the oracle, bit-exact, in both score
    modes; scenes: mostly transparent, opaque enough that pixels finish early and the tail of the lists is never
    reached, and lists of several batches.  Also: the record follows the latest forward pass, not an earlier one."""
    import torch
    from paper_2511_04283_amd import binding as B
    cfg = B.default_config()
    cfg.score_mode = mode
    c = B.Context("cuda:0", cfg)
    o = Oracle(np.float32, Config(score_mode=mode))
    if case == "transparent":
        sc = scenes.tiny_scene(810, 6000, 203, 117, sh_degree=1, log_scale=(-2.8, 0.7), spread=1.2)
    elif case == "opaque":
        sc = scenes.tiny_scene(811, 9000, 150, 90, sh_degree=0, log_scale=(-1.6, 0.5), spread=1.0)
        sc.opacities[:] = 0.97
    else:
        sc = scenes.tiny_scene(812, 30000, 70, 50, sh_degree=0, log_scale=(-3.2, 0.7), spread=1.1)
    cam = sc.cameras[0]
    H, W = cam.height, cam.width
    tgt_np = np.random.default_rng(5).uniform(0, 1, (3, H, W)).astype(np.float32)
    tgt = torch.from_numpy(tgt_np).to(c.device)
    g = B.Gaussians.from_scene(sc, c.device)
    fcam = B.make_camera(cam)
    proj = c.fs_preprocess(g, fcam)
    bins = c.fs_bin_sort(proj, fcam)
    p_o, b_o, img_o, T_o, nc_o = o.forward(sc, cam)
    L = b_o.tile_ranges[:, 1].astype(np.int64) - b_o.tile_ranges[:, 0]
    if case == "long_lists":
        assert L.max() > 600
    if case == "opaque":   # some pixels stop well before the end of their tile's list
        tl = np.repeat(np.repeat(L.reshape((H + 15) // 16, (W + 15) // 16), 16, 0), 16, 1)[:H, :W]
        assert (nc_o.astype(np.int64) + 256 < tl).mean() > 0.05
    m_o, _, _ = o.error_mask(img_o, tgt_np, rule=0, k=0.5)
    ref = o.score(p_o, b_o, cam, m_o, np.zeros(sc.n, np.int32))
    assert ref.sum() > 0

    # (1) record on (the default): fused forward, counts from the record
    img, fT, nc, dL = c.fs_render_fwd_loss(proj, bins, fcam, tgt)
    mask, thr = c.fs_error_mask_fused(H, W, 0, 0.5)
    assert np.array_equal(mask.cpu().numpy(), m_o) and np.array_equal(nc.cpu().numpy().view(np.uint32), nc_o)
    cnt_rec = torch.zeros(sc.n, dtype=torch.int32, device=c.device)
    c.fs_score_accumulate(proj, bins, fcam, fT, nc, mask, cnt_rec)
    c.fs_score_accumulate(proj, bins, fcam, fT, nc, mask, cnt_rec)          # accumulates; the record stays usable
    assert np.array_equal(cnt_rec.cpu().numpy(), 2 * ref)
    # (2) the plain forward pass keeps the record as well
    img2, fT2, nc2 = c.fs_render_fwd(proj, bins, fcam)
    assert torch.equal(img2, img) and torch.equal(nc2, nc)
    cnt_plain = torch.zeros(sc.n, dtype=torch.int32, device=c.device)
    c.fs_score_accumulate(proj, bins, fcam, fT2, nc2, mask, cnt_plain)
    assert np.array_equal(cnt_plain.cpu().numpy(), ref)
    # (3) record off: both forward passes give the same image, the count pass walks the lists
    c.fs_set_score_record(False)
    img3, fT3, nc3, dL3 = c.fs_render_fwd_loss(proj, bins, fcam, tgt)
    assert torch.equal(img3, img) and torch.equal(nc3, nc) and torch.equal(dL3, dL)
    cnt_off = torch.zeros(sc.n, dtype=torch.int32, device=c.device)
    c.fs_score_accumulate(proj, bins, fcam, fT3, nc3, mask, cnt_off)
    assert np.array_equal(cnt_off.cpu().numpy(), ref)
    img4, fT4, nc4 = c.fs_render_fwd(proj, bins, fcam)
    assert torch.equal(img4, img) and torch.equal(nc4, nc)
    cnt_off.zero_()
    c.fs_score_accumulate(proj, bins, fcam, fT4, nc4, mask, cnt_off)
    assert np.array_equal(cnt_off.cpu().numpy(), ref)
    # (4) record on again, another mask (every pixel): counts = blended pixels per Gaussian
    c.fs_set_score_record(True)
    c.fs_render_fwd_loss(proj, bins, fcam, tgt)
    ones = torch.ones((H, W), dtype=torch.uint8, device=c.device)
    cnt_all = torch.zeros(sc.n, dtype=torch.int32, device=c.device)
    c.fs_score_accumulate(proj, bins, fcam, fT, nc, ones, cnt_all)
    assert np.array_equal(cnt_all.cpu().numpy(), o.score(p_o, b_o, cam, np.ones((H, W), np.uint8), np.zeros(sc.n, np.int32)))
    # (5) the size of the record: per tile, the pairs with a counted pixel somewhere in the tile
    rows = c.fs_score_record_rows(bins, fcam).cpu().numpy()
    ones_np = np.ones((H, W), np.uint8)
    for t in range(rows.shape[0]):
        in_tile = o.score(p_o, b_o, cam, ones_np, np.zeros(sc.n, np.int32), tile_list=[t])
        assert rows[t] == np.count_nonzero(in_tile), t
    assert 0 < rows.sum() <= bins.num_pairs
    c.fs_set_score_record(False)
    c.fs_render_fwd(proj, bins, fcam)
    with pytest.raises(RuntimeError):
        c.fs_score_record_rows(bins, fcam)      # no record behind the latest forward pass
    c.close()


def test_pair_order_over_seeded_random_shapes(orc32):
    """Two dozen seeded shapes (Gaussian counts from 1 to 30 000, images from a single tile to 60 x 40 tiles, narrow
    and wide scale distributions, both box rules) through fs_preprocess + fs_bin_sort on one context per rule:
    pair count, keys, order and ranges bit-exact, tile order a permutation."""
    from paper_2511_04283_amd import binding as B
    rng = np.random.default_rng(20251104)
    for compact_box in (0, 1):
        cfg = B.default_config()
        cfg.compact_box = compact_box
        cfg.cb_beta = 0.8
        c = B.Context("cuda:0", cfg)
        o = Oracle(np.float32, Config(compact_box=bool(compact_box), cb_beta=0.8))
        for case in range(12):
            n = int(rng.choice([1, 2, 63, 64, 65, 257, 1000, 4097, 30000]))
            W = int(rng.integers(1, 960))
            H = int(rng.integers(1, 640))
            ls = (float(rng.uniform(-4.0, -1.5)), float(rng.uniform(0.2, 1.0)))
            sc = scenes.tiny_scene(1000 + 31 * case + compact_box, n, W, H, sh_degree=0, log_scale=ls,
                                   spread=float(rng.uniform(0.5, 1.6)))
            cam = sc.cameras[0]
            g = B.Gaussians.from_scene(sc, c.device)
            fcam = B.make_camera(cam)
            proj = c.fs_preprocess(g, fcam)
            bins = c.fs_bin_sort(proj, fcam)
            p_o = o.preprocess(sc, cam)
            b_o = o.bin_sort(p_o, cam)
            tag = (compact_box, case, n, W, H)
            assert bins.num_pairs == b_o.num_pairs, tag
            assert np.array_equal(bins.copy_keys().cpu().numpy().view(np.uint64), b_o.keys_sorted), tag
            assert np.array_equal(bins.copy_gauss().cpu().numpy().view(np.uint32), b_o.gauss_sorted), tag
            assert np.array_equal(bins.copy_ranges().cpu().numpy().view(np.uint32), b_o.tile_ranges), tag
            T = ((W + 15) // 16) * ((H + 15) // 16)
            assert np.array_equal(np.sort(bins.copy_order().cpu().numpy()), np.arange(T)), tag
        c.close()


@pytest.mark.parametrize("per_splat", [False, True])
@pytest.mark.parametrize("records", ["dense", "sparse"])
def test_whole_path_over_seeded_random_shapes(orc32, per_splat, records):
    """Ten seeded small shapes (1 to 2 500 Gaussians, all SH degrees, ragged images) through the whole path with
    both mappings of the backward pass and both layouts of its per-pair records: every output against the oracle
    (integers bit-exact, image 1e-4, gradients 1e-3 with the floor), the absolute gradient included."""
    from paper_2511_04283_amd import binding as B
    rng = np.random.default_rng(7 + int(per_splat))
    c = B.Context("cuda:0")
    if per_splat:
        c.fs_set_backward_mode(B.FS_BWD_PER_SPLAT)
    c.fs_set_record_mode(B.FS_RECORDS_SPARSE if records == "sparse" else B.FS_RECORDS_DENSE)
    for case in range(10):
        n = int(rng.choice([1, 33, 65, 100, 700, 2500]))
        W, H = int(rng.integers(17, 300)), int(rng.integers(17, 200))
        deg = int(rng.integers(0, 4))
        sc = scenes.tiny_scene(2000 + case, n, W, H, sh_degree=deg,
                               log_scale=(float(rng.uniform(-3.0, -1.2)), float(rng.uniform(0.3, 0.9))),
                               spread=float(rng.uniform(0.5, 1.4)))
        cam = sc.cameras[0]
        tgt = rng.uniform(0, 1, (3, H, W)).astype(np.float32)
        g = gpu_pipeline(c, sc, cam, target=tgt, want_abs=True)
        r = oracle_pipeline(orc32, sc, cam, target=tgt)
        check_all(g, r, sc)
    c.close()
