"""A FastGS training loop driven entirely through the C-ABI calls (Sec. 4 of the paper): training
iterations with the photometric loss and Adam, the multi-view score pass (VCD's s_d, VCP's s_p), and
densification by cloning and splitting plus pruning (before iteration 15 000: of half the candidates,
sampled by pruning score).  Orchestration only: every arithmetic step runs in the HIP kernels; PyTorch
supplies device memory (allocation, zero filling, concatenation of the per-Gaussian arrays) and the two
random streams the method draws from (standard normals for the split children, Exp(1) variates for the
sampling), which are handed to the library as inputs.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import torch

from . import binding as B

GROUPS = ("means", "sh", "raw_scales", "raw_quats", "raw_opacities")


@dataclass
class TrainConfig:
    lam: float = 0.2                      # weight of the SSIM term (Sec. 5.1)
    lr: dict = field(default_factory=lambda: dict(means=1.6e-4, sh=2.5e-3, raw_scales=5e-3, raw_quats=1e-3,
                                                  raw_opacities=5e-2))
    eps: float = 1e-15
    tau_d: float = 5.0                    # densify only where s_d exceeds it (supplement)
    tau_p: float = 0.9                    # prune where s_p exceeds it
    min_opacity: float = 0.1              # ... or where the opacity is below it
    tau_grad: float = 2e-4                # mean positional-gradient norm needed for cloning (pixel units)
    tau_abs: float = 4e-4                 # mean absolute positional gradient needed for splitting
    size_limit: float = 0.05              # clone below, split above this largest scale
    mask_rule: int = B.FS_MASK_MEAN_STD
    mask_k: float = 1.0
    split_phi: float = 1.6                # children's scales = parent's / phi (vanilla 3DGS: 0.8 x 2 children)
    early_until: int = 15000              # before this iteration only a sampled half of the prune candidates goes
    seed: int = 0                         # of the generator behind the normals and the exponentials


class Trainer:
    def __init__(self, ctx: B.Context, means, scales, quats, opacities, sh, sh_degree: int, cfg: TrainConfig | None = None):
        self.ctx, self.cfg, self.sh_degree = ctx, cfg or TrainConfig(), int(sh_degree)
        ctx.fs_set_score_record(False)   # training iterations are not followed by a count pass; score_views turns it on
        f = lambda t: t.detach().to(ctx.device, torch.float32).contiguous().clone()
        raw_s, raw_o = ctx.fs_activate_inv(f(scales), f(opacities), 1e-4, 1 - 1e-4)
        self.p = dict(means=f(means), sh=f(sh), raw_scales=raw_s, raw_quats=f(quats), raw_opacities=raw_o)
        self.rng = torch.Generator(device=ctx.device)
        self.rng.manual_seed(self.cfg.seed)
        self._reset_state()
        self.iteration = 0

    # -- state -----------------------------------------------------------------------
    @property
    def n(self) -> int:
        return int(self.p["means"].shape[0])

    def _reset_state(self):
        z = lambda t: torch.zeros_like(t)
        self.m = {k: z(v) for k, v in self.p.items()}
        self.v = {k: z(v) for k, v in self.p.items()}
        self.acc = {k: z(v) for k, v in self.p.items()}       # gradient sums between optimiser updates
        self.pending = 0
        self.updates = 0
        n, dev = self.n, self.ctx.device
        self.grad_accum = torch.zeros(n, device=dev)
        self.abs_accum = torch.zeros(n, device=dev)
        self.denom = torch.zeros(n, dtype=torch.int32, device=dev)

    def gaussians(self) -> B.Gaussians:
        s, q, o = self.ctx.fs_activate(self.p["raw_scales"], self.p["raw_quats"], self.p["raw_opacities"])
        return B.Gaussians(self.p["means"], s, q, o, self.p["sh"], self.sh_degree)

    # -- one training iteration on one view -------------------------------------------
    def step(self, cam, target) -> float:
        ctx, c = self.ctx, self.cfg
        fcam = B.make_camera(cam)
        g = self.gaussians()
        proj = ctx.fs_preprocess(g, fcam)
        bins = ctx.fs_bin_sort(proj, fcam)
        image, fT, nc = ctx.fs_render_fwd(proj, bins, fcam)
        out3, dL = ctx.fs_photo_loss(image, target, c.lam)
        gr = ctx.fs_render_bwd(g, fcam, proj, bins, fT, nc, dL, want_abs=True)
        ctx.fs_densify_accumulate(gr["mean2d"], gr["mean2d_abs"], proj.tiles_touched, self.grad_accum, self.abs_accum,
                                  self.denom)
        ctx.fs_activate_bwd(self.p["raw_scales"], self.p["raw_quats"], self.p["raw_opacities"], gr["scales"], gr["quats"],
                            gr["opacities"])
        grads = dict(means=gr["means"], sh=gr["sh"], raw_scales=gr["scales"], raw_quats=gr["quats"],
                     raw_opacities=gr["opacities"])
        # optimiser schedule: an update every fs_adam_interval iterations, on the sum of the gradients since the last
        interval = ctx.fs_adam_interval(self.iteration)
        self.iteration += 1
        self.pending += 1
        last = self.pending >= interval
        for k in GROUPS:
            if interval == 1:
                src = grads[k]
            else:
                ctx.fs_grad_accumulate(self.acc[k], grads[k])
                src = self.acc[k]
            if last:
                ctx.fs_adam_step(self.p[k], src, self.m[k], self.v[k], self.updates + 1, c.lr[k], eps=c.eps,
                                 zero_grad=(interval != 1))
        if last:
            self.updates += 1
            self.pending = 0
        return float(out3[2].item())

    # -- multi-view consistency scores (Sec. 4.2, 4.3) ----------------------------------
    def score_views(self, cams, targets):
        """Returns (counts int32 [n] summed over the views, s_p float32 [n]); s_d = counts / len(cams)."""
        ctx, c = self.ctx, self.cfg
        g = self.gaussians()
        n, dev = self.n, ctx.device
        counts = torch.zeros(n, dtype=torch.int32, device=dev)
        acc = torch.zeros(n, dtype=torch.float64, device=dev)
        ctx.fs_set_score_record(True)   # (off during the training iterations, which no count pass follows)
        for cam, target in zip(cams, targets):
            fcam = B.make_camera(cam)
            proj = ctx.fs_preprocess(g, fcam)
            bins = ctx.fs_bin_sort(proj, fcam)
            # forward pass with the error map and the per-pair record of counted pixels fused into it
            image, fT, nc, _ = ctx.fs_render_fwd_loss(proj, bins, fcam, target, want_grad=False)
            view = torch.zeros(n, dtype=torch.int32, device=dev)
            ctx.fs_mask_score_fused(proj, bins, fcam, nc, view, c.mask_rule, c.mask_k)   # mask, then the view's counts
            out3, _ = ctx.fs_photo_loss(image, target, c.lam, want_grad=False)
            ctx.fs_prune_score_accumulate(view, out3[2:3], acc)
            ctx.fs_counts_add(counts, view)
        ctx.fs_set_score_record(False)
        return counts, ctx.fs_prune_score_normalize(acc)

    # -- densify (clone, split) and prune; Adam state of the survivors is kept, new Gaussians start at zero ------
    def densify_and_prune(self, cams, targets, prune: bool = True, early: bool | None = None) -> dict:
        """One densification step.  Rows afterwards: the kept Gaussians (neither pruned nor split), the clones, the
        first children of the split parents, their second children.  `early` (default: iteration < early_until):
        only half of the prune candidates, sampled by their pruning score, are removed."""
        ctx, c = self.ctx, self.cfg
        dev = ctx.device
        counts, s_p = self.score_views(cams, targets)
        g = self.gaussians()
        prm = B.fs_select_params(tau_grad=c.tau_grad, tau_abs=c.tau_abs, tau_d=c.tau_d, size_limit=c.size_limit,
                                 min_opacity=c.min_opacity, tau_p=c.tau_p, K=len(cams))
        clone, split, prune_mask = ctx.fs_select(self.grad_accum, self.abs_accum, self.denom, counts, g.scales, g.opacities,
                                                 s_p, prm)
        n_before = self.n
        if not prune:
            prune_mask = torch.zeros_like(prune_mask)
        elif early if early is not None else self.iteration < c.early_until:
            expo = torch.empty(n_before, dtype=torch.float32, device=dev).exponential_(1.0, generator=self.rng)
            prune_mask, _ = ctx.fs_sample_by_score(prune_mask, s_p, expo)
        keep_m, clone_m, split_m = ctx.fs_combine_masks(clone, split, prune_mask)
        keep, clone_idx, split_idx = ctx.fs_compact(keep_m), ctx.fs_compact(clone_m), ctx.fs_compact(split_m)
        m = int(split_idx.shape[0])
        normals = torch.randn((m, 2, 3), dtype=torch.float32, device=dev, generator=self.rng)
        child_means, child_scales = ctx.fs_split_children(self.p["means"], g.scales, g.quats, split_idx, normals, c.split_phi)
        child_opac = ctx.fs_gather_rows(g.opacities, split_idx)
        child_raw_scales, _ = ctx.fs_activate_inv(child_scales, torch.cat([child_opac, child_opac]), 1e-4, 1 - 1e-4)
        children = dict(means=child_means, raw_scales=child_raw_scales)
        n_new = int(clone_idx.shape[0]) + 2 * m
        for d in (self.p, self.m, self.v, self.acc):
            for k in GROUPS:
                kept = ctx.fs_gather_rows(d[k], keep)
                if d is self.p:
                    par = ctx.fs_gather_rows(d[k], split_idx)       # children inherit what the split does not change
                    new = [ctx.fs_gather_rows(d[k], clone_idx), children.get(k, torch.cat([par, par]))]
                else:
                    new = [torch.zeros((n_new,) + tuple(d[k].shape[1:]), device=dev)]
                d[k] = torch.cat([kept] + new).contiguous()
        n = self.n
        self.grad_accum = torch.zeros(n, device=dev)
        self.abs_accum = torch.zeros(n, device=dev)
        self.denom = torch.zeros(n, dtype=torch.int32, device=dev)
        return dict(before=n_before, kept=int(keep.shape[0]), cloned=int(clone_idx.shape[0]), split=m,
                    pruned=int(n_before - keep.shape[0] - m), after=n)
