"""End-to-end training on a synthetic multi-view target through the C-ABI calls only: the loss falls, a
densify-and-prune cycle driven by the multi-view scores changes the Gaussian set consistently, and training
continues on the new set."""
import numpy as np
import pytest

from oracle import Oracle
from paper_2511_04283_amd import scenes

pytestmark = pytest.mark.gpu


def _views(sc, k):
    cam0 = sc.cameras[0]
    cams = []
    for j in range(k):
        a = np.deg2rad(-8 + 16 * j / max(1, k - 1))
        R = np.array([[np.cos(a), 0, np.sin(a)], [0, 1, 0], [-np.sin(a), 0, np.cos(a)]]) @ cam0.R
        cams.append(scenes.Camera(cam0.width, cam0.height, cam0.fx, cam0.fy, cam0.cx, cam0.cy, R, cam0.t))
    return cams


def test_training_with_a_densify_and_prune_cycle():
    import torch
    from paper_2511_04283_amd import binding as B
    from paper_2511_04283_amd.trainer import TrainConfig, Trainer
    ctx = B.Context("cuda:0")
    sc = scenes.tiny_scene(8, 600, 128, 96, sh_degree=1, log_scale=(-2.4, 0.4))
    cams = _views(sc, 4)
    o = Oracle(np.float32)
    targets = [torch.from_numpy(o.forward(sc, c)[2]).to(ctx.device) for c in cams]
    rng = np.random.default_rng(0)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a, np.float32))
    # start: perturbed copy with a third of the Gaussians missing and some near-transparent extras
    keep = rng.uniform(size=sc.n) > 0.33
    means = sc.means[keep] + rng.normal(0, 0.03, (keep.sum(), 3))
    op = sc.opacities[keep].copy()
    op[::9] = 0.02
    cfg = TrainConfig(lr=dict(means=2e-3, sh=5e-3, raw_scales=5e-3, raw_quats=1e-3, raw_opacities=2e-2), eps=1e-8,
                      tau_d=1.0, tau_grad=2e-6, tau_abs=1e-3, size_limit=1.0)
    tr = Trainer(ctx, t(means), t(sc.scales[keep]), t(sc.quats[keep]), t(op), t(sc.sh[keep] * 0.5), sc.sh_degree, cfg)
    losses = [tr.step(cams[i % 4], targets[i % 4]) for i in range(40)]
    assert np.mean(losses[-4:]) < 0.8 * np.mean(losses[:4])
    assert int(tr.denom.max().item()) > 0 and float(tr.grad_accum.max().item()) > 0

    n0 = tr.n
    counts, s_p = tr.score_views(cams, targets)
    assert counts.shape[0] == n0 and int(counts.sum().item()) > 0
    assert float(s_p.max().item()) == 1.0 and float(s_p.min().item()) == 0.0
    info = tr.densify_and_prune(cams, targets, early=False)
    assert info["before"] == n0 and info["after"] == info["kept"] + info["cloned"] == tr.n and info["split"] == 0
    assert info["cloned"] > 0 and info["kept"] < n0            # the near-transparent extras go, busy ones are cloned
    for k, v in tr.p.items():
        assert v.shape[0] == tr.n and tr.m[k].shape == v.shape and torch.isfinite(v).all()
    # clones are exact copies of their sources, appended after the survivors, with fresh optimiser state
    assert not tr.m["means"][info["kept"]:].any()
    g = tr.gaussians()
    assert float(g.opacities[:info["kept"]].min().item()) >= cfg.min_opacity * 0.999

    more = [tr.step(cams[i % 4], targets[i % 4]) for i in range(40)]
    assert np.isfinite(more).all() and np.mean(more[-4:]) < np.mean(losses[-4:]) * 1.05
    ctx.close()


def test_densify_splits_large_gaussians_and_samples_half_of_the_prune_candidates():
    """With a size limit inside the scale distribution the large, busy Gaussians are split (two children each, the
    parent removed); in the early phase only floor(m / 2) of the m prune candidates go."""
    import torch
    from paper_2511_04283_amd import binding as B
    from paper_2511_04283_amd.trainer import TrainConfig, Trainer
    ctx = B.Context("cuda:0")
    sc = scenes.tiny_scene(8, 600, 128, 96, sh_degree=1, log_scale=(-2.4, 0.4))
    cams = _views(sc, 4)
    o = Oracle(np.float32)
    targets = [torch.from_numpy(o.forward(sc, c)[2]).to(ctx.device) for c in cams]
    rng = np.random.default_rng(1)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a, np.float32))
    keep = rng.uniform(size=sc.n) > 0.33
    op = sc.opacities[keep].copy()
    op[::5] = 0.02
    cfg = TrainConfig(lr=dict(means=2e-3, sh=5e-3, raw_scales=5e-3, raw_quats=1e-3, raw_opacities=2e-2), eps=1e-8,
                      tau_d=1.0, tau_grad=2e-6, tau_abs=2e-6, size_limit=float(np.median(sc.scales.max(1))), seed=5)
    tr = Trainer(ctx, t(sc.means[keep] + rng.normal(0, 0.03, (keep.sum(), 3))), t(sc.scales[keep]), t(sc.quats[keep]),
                 t(op), t(sc.sh[keep] * 0.5), sc.sh_degree, cfg)
    for i in range(12):
        tr.step(cams[i % 4], targets[i % 4])
    n0 = tr.n
    # what the selection sees (the score pass is deterministic, so the trainer will see the same)
    counts, s_p = tr.score_views(cams, targets)
    g = tr.gaussians()
    prm = B.fs_select_params(tau_grad=cfg.tau_grad, tau_abs=cfg.tau_abs, tau_d=cfg.tau_d, size_limit=cfg.size_limit,
                             min_opacity=cfg.min_opacity, tau_p=cfg.tau_p, K=4)
    clone, split, prune = ctx.fs_select(tr.grad_accum, tr.abs_accum, tr.denom, counts, g.scales, g.opacities, s_p, prm)
    cand = int(prune.sum().item())
    assert cand >= 20 and int(split.sum().item()) > 0
    parents_scale = g.scales.clone()
    info = tr.densify_and_prune(cams, targets)            # iteration 12 < 15 000: the early phase
    assert info["pruned"] == cand // 2
    assert info["split"] > 0 and info["cloned"] > 0
    assert info["after"] == info["kept"] + info["cloned"] + 2 * info["split"] == tr.n
    assert info["kept"] == n0 - info["pruned"] - info["split"]
    # the two children of a parent share its scales divided by phi and sit at different places
    a0 = info["kept"] + info["cloned"]
    m = info["split"]
    g2 = tr.gaussians()
    c0, c1 = g2.scales[a0:a0 + m], g2.scales[a0 + m:a0 + 2 * m]
    assert torch.allclose(c0, c1, rtol=1e-6)
    assert float(c0.max().item()) <= float(parents_scale.max().item()) / 1.6 * 1.0001
    assert float(c0.max(1).values.min().item()) > cfg.size_limit / 1.6 * 0.999   # every parent was above the limit
    assert not torch.equal(tr.p["means"][a0:a0 + m], tr.p["means"][a0 + m:a0 + 2 * m])
    assert torch.equal(tr.p["sh"][a0:a0 + m], tr.p["sh"][a0 + m:a0 + 2 * m])
    assert not tr.m["means"][info["kept"]:].any()
    more = [tr.step(cams[i % 4], targets[i % 4]) for i in range(8)]
    assert np.isfinite(more).all()
    ctx.close()


def test_optimiser_schedule_accumulates_between_updates():
    """From iteration 15 000 on an update happens every 32 iterations, on the summed gradients."""
    import torch
    from paper_2511_04283_amd import binding as B
    from paper_2511_04283_amd.trainer import Trainer
    ctx = B.Context("cuda:0")
    sc = scenes.tiny_scene(9, 200, 64, 48, sh_degree=0, log_scale=(-2.2, 0.3))
    cam = sc.cameras[0]
    target = torch.rand(3, cam.height, cam.width, device=ctx.device)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a, np.float32))
    tr = Trainer(ctx, t(sc.means), t(sc.scales), t(sc.quats), t(sc.opacities), t(sc.sh), 0)
    tr.iteration = 15000 - 2
    snap = lambda: tr.p["means"].clone()
    p0 = snap(); tr.step(cam, target); p1 = snap(); tr.step(cam, target); p2 = snap()
    assert not torch.equal(p0, p1) and not torch.equal(p1, p2) and tr.updates == 2      # interval 1
    for _ in range(31):
        tr.step(cam, target)
    assert torch.equal(snap(), p2) and tr.updates == 2 and tr.pending == 31 and tr.acc["means"].any()
    tr.step(cam, target)
    assert not torch.equal(snap(), p2) and tr.updates == 3 and tr.pending == 0 and not tr.acc["means"].any()
    ctx.close()
