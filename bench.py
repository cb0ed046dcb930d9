#!/usr/bin/env python3
"""Benchmark of the FastGS rasterizer hot path on one MI355X.

One step = one pass of the whole hot path over one synthetic view of the workload: projection,
pair ordering, forward compositing, the L1 term, backward, error mask and the per-Gaussian count pass
(fs_preprocess, fs_bin_sort, fs_render_fwd_loss, fs_render_bwd, fs_error_mask_fused, fs_score_accumulate;
--separate-calls for the unfused entry points), inputs resident in HBM.  The headline workload is
benchmark config 3 (500k Gaussians, SH degree 3, 1600x1064).

Prints ONE JSON line (see the keys below).  `--gpus N` with N > 1 is refused: this build is
single-GPU by construction.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# Algorithmic work per unit: flops per examined list entry ("evaluation")
# and per blended (Gaussian, pixel) pair, for the forward and backward compositing kernels.
FWD_FLOPS_PER_EVAL = 11     # dx, dy, q (2 mul + 2 fma + mul), -0.5*q
FWD_FLOPS_PER_BLEND = 26    # exp (mul, rint, sub, 5 fma, ldexp) 14; alpha 2; T 2; w 1; colour 3 fma 6; + min
BWD_FLOPS_PER_EVAL = 11
BWD_FLOPS_PER_BLEND = 66    # exp 14; alpha 2; 1/(1-a), T, w 4; colour/alpha grads 17; conic/mean grads 20; 9-value sum 9
PEAK_FP32_TFLOPS = 157.3    # MI355X vector fp32 (packed FMA), 256 CU x 4 SIMD x 16 lanes x 2 x 2 x 2.4 GHz
PEAK_HBM_GBS = 8000.0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=3, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--compact-box", action="store_true",
                    help="pairs from the Compact Box (ellipse-tile test, Sec. 4.4) instead of the 3-sigma square")
    ap.add_argument("--cb-beta", type=float, default=1.0)
    ap.add_argument("--separate-calls", action="store_true",
                    help="fs_render_fwd + fs_l1_grad + fs_error_mask instead of fs_render_fwd_loss + fs_error_mask_fused")
    ap.add_argument("--radix-sort", action="store_true", help="order the pairs with the global radix sort (sort_mode)")
    ap.add_argument("--abs-grad", action="store_true",
                    help="also accumulate the absolute positional gradient in the backward pass (split criterion)")
    ap.add_argument("--per-splat-bwd", action="store_true",
                    help="run the backward pass in its per-splat-parallel mapping (fs_set_backward_mode), for comparison")
    ap.add_argument("--train-iteration", action="store_true",
                    help="time a whole training iteration: activations + the hot path + chain rule + Adam on every group")
    ap.add_argument("--photo-loss", action="store_true",
                    help="train on (1-0.2) L1 + 0.2 (1-SSIM) (fs_photo_loss) instead of the L1 term alone (fs_l1_grad)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy (reference for the FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2511_04283_amd import binding as B
    from paper_2511_04283_amd import scenes

    sc = scenes.make_scene(args.config)
    cam = sc.cameras[0]
    target_np = scenes.target_image(args.config, 0, cam)
    dev = torch.device("cuda:0")
    cfg0 = B.default_config()
    cfg0.compact_box = 1 if args.compact_box else 0
    cfg0.cb_beta = args.cb_beta
    cfg0.sort_mode = B.FS_SORT_RADIX if args.radix_sort else B.FS_SORT_AUTO
    ctx = B.Context(dev, cfg0)
    if args.per_splat_bwd:
        ctx.fs_set_backward_mode(B.FS_BWD_PER_SPLAT)
    g = B.Gaussians.from_scene(sc, dev)
    fcam = B.make_camera(cam)
    target = torch.from_numpy(target_np).to(dev)
    n, H, W, K = sc.n, cam.height, cam.width, (sc.sh_degree + 1) ** 2

    # every output is allocated once, before the timed region
    e = lambda *s, dt=torch.float32: torch.empty(s, dtype=dt, device=dev)
    proj = B.Projected(e(n, 2), e(n), e(n, 4), e(n, 3), e(n, 4, dt=torch.int16), e(n, dt=torch.int32), e(n, 3, dt=torch.uint8))
    image, final_T, n_contrib = e(3, H, W), e(H, W), e(H, W, dt=torch.int32)
    dL = e(3, H, W)
    loss = torch.zeros(1, dtype=torch.float64, device=dev)
    out3 = torch.zeros(3, dtype=torch.float64, device=dev)
    grads = dict(means=e(n, 3), scales=e(n, 3), quats=e(n, 4), opacities=e(n), sh=e(n, K, 3), mean2d=e(n, 2))
    if args.abs_grad:
        grads["mean2d_abs"] = e(n, 2)
    mask, thr = e(H, W, dt=torch.uint8), e(1)
    counts = torch.zeros(n, dtype=torch.int32, device=dev)
    state = {}

    if args.train_iteration:
        raw = dict(scales=torch.log(g.scales), quats=g.quats.clone(), opac=torch.logit(g.opacities.clamp(1e-4, 1 - 1e-4)))
        params = dict(means=g.means, sh=g.sh, scales=raw["scales"], quats=raw["quats"], opacities=raw["opac"])
        adam_m = {k: torch.zeros_like(v) for k, v in params.items()}
        adam_v = {k: torch.zeros_like(v) for k, v in params.items()}
        state["it"] = 0

    # the L1 term and the error map are fused into the forward kernel unless asked otherwise (same outputs)
    fused = not (args.separate_calls or args.photo_loss)

    def step():
        if args.train_iteration:
            state["it"] += 1
            s_, q_, o_ = ctx.fs_activate(raw["scales"], raw["quats"], raw["opac"])
            g.scales, g.quats, g.opacities = s_, q_, o_
        ctx.fs_preprocess(g, fcam, proj)
        bins = ctx.fs_bin_sort(proj, fcam)
        if fused:
            ctx.fs_render_fwd_loss(proj, bins, fcam, target, image, final_T, n_contrib, dL, loss)
        else:
            ctx.fs_render_fwd(proj, bins, fcam, image, final_T, n_contrib)
            if args.photo_loss:
                ctx.fs_photo_loss(image, target, 0.2, dL, out3)
            else:
                ctx.fs_l1_grad(image, target, dL, loss)
        ctx.fs_render_bwd(g, fcam, proj, bins, final_T, n_contrib, dL, grads)
        if args.train_iteration:
            ctx.fs_activate_bwd(raw["scales"], raw["quats"], raw["opac"], grads["scales"], grads["quats"], grads["opacities"])
            for k in params:
                ctx.fs_adam_step(params[k], grads[k], adam_m[k], adam_v[k], state["it"], 1e-5)
        if fused:
            ctx.fs_error_mask_fused(H, W, B.FS_MASK_MEAN_STD, 1.0, mask, thr)
        else:
            ctx.fs_error_mask(image, target, B.FS_MASK_MEAN_STD, 1.0, mask, thr)
        counts.zero_()
        ctx.fs_score_accumulate(proj, bins, fcam, final_T, n_contrib, mask, counts)
        state["bins"] = bins

    if args.calibrate_copy:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device=dev)   # 256 MiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # timed region: K steps; the dominant kernel (backward compositing) is also timed on its own
    # with HIP events recorded on the stream it is launched on
    ctx.fs_profile_enable(["render_bwd", "render_fwd"])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    timed = ctx.fs_profile_read()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    # the training iteration alone (no mask / score pass): preprocess, bin_sort, render_fwd, loss, render_bwd
    def train_iter():
        ctx.fs_preprocess(g, fcam, proj)
        b_ = ctx.fs_bin_sort(proj, fcam)
        if fused:
            ctx.fs_render_fwd_loss(proj, b_, fcam, target, image, final_T, n_contrib, dL, loss)
        else:
            ctx.fs_render_fwd(proj, b_, fcam, image, final_T, n_contrib)
            if args.photo_loss:
                ctx.fs_photo_loss(image, target, 0.2, dL, out3)
            else:
                ctx.fs_l1_grad(image, target, dL, loss)
        ctx.fs_render_bwd(g, fcam, proj, b_, final_T, n_contrib, dL, grads)
    ctx.fs_profile_enable(())
    ctx.fs_set_score_record(False)    # no count pass follows these forward passes
    train_iter()
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    for _ in range(args.steps):
        train_iter()
    torch.cuda.synchronize()
    fwd_bwd_ms = (time.perf_counter() - t2) * 1e3 / args.steps
    ctx.fs_set_score_record(True)

    # the multi-view score pass of VCD (Sec. 4.2): K views x (preprocess, bin_sort, render_fwd, error_mask,
    # score_accumulate), counts summed over the views -- for workloads that come with several cameras
    score_pass = None
    if len(sc.cameras) > 1:
        cams = [B.make_camera(c) for c in sc.cameras]
        tgts = [torch.from_numpy(scenes.target_image(args.config, v, c)).to(dev) for v, c in enumerate(sc.cameras)]

        def views():
            counts.zero_()
            for fc, tg in zip(cams, tgts):
                ctx.fs_preprocess(g, fc, proj)
                b_ = ctx.fs_bin_sort(proj, fc)
                if fused:
                    ctx.fs_render_fwd_loss(proj, b_, fc, tg, image, final_T, n_contrib, want_grad=False)
                    ctx.fs_error_mask_fused(fc.height, fc.width, B.FS_MASK_MEAN_STD, 1.0, mask, thr)
                else:
                    ctx.fs_render_fwd(proj, b_, fc, image, final_T, n_contrib)
                    ctx.fs_error_mask(image, tg, B.FS_MASK_MEAN_STD, 1.0, mask, thr)
                ctx.fs_score_accumulate(proj, b_, fc, final_T, n_contrib, mask, counts)
        views()
        torch.cuda.synchronize()
        t3 = time.perf_counter()
        reps = max(1, args.steps // 4)
        for _ in range(reps):
            views()
        torch.cuda.synchronize()
        sp_ms = (time.perf_counter() - t3) * 1e3 / reps
        score_pass = {"views": len(cams), "ms": round(sp_ms, 4), "ms_per_view": round(sp_ms / len(cams), 4),
                      "gaussians_with_s_d_above_5": int((counts.to(torch.float32) / len(cams) > 5.0).sum().item())}

    # untimed: per-kernel breakdown of the same steps
    ctx.fs_profile_enable(None)
    for _ in range(max(3, args.steps // 2)):
        step()
    prof = ctx.fs_profile_read()
    ctx.fs_profile_enable(())
    kernels_ms = {k: (ms / c if c else 0.0) for k, (ms, c) in prof.items()}

    # units of work of one step (exact, from the path's own outputs)
    P = state["bins"].num_pairs
    ranges = state["bins"].copy_ranges().to(torch.int64)
    tile_len = ranges[:, 1] - ranges[:, 0]
    evals_bwd = int(n_contrib.to(torch.int64).sum().item())          # entries walked back per pixel
    evals_fwd_bound = int(P) * 256                                    # upper bound: every pixel walks its whole list
    cfgA = B.default_config()
    cfgA.compact_box, cfgA.cb_beta = cfg0.compact_box, cfg0.cb_beta
    cfgA.score_mode = B.FS_SCORE_ALPHA
    ctxA = B.Context(dev, cfgA)
    projA = ctxA.fs_preprocess(g, fcam)
    binsA = ctxA.fs_bin_sort(projA, fcam)
    imA, TA, ncA = ctxA.fs_render_fwd(projA, binsA, fcam)
    blends_t = torch.zeros(n, dtype=torch.int32, device=dev)
    ctxA.fs_score_accumulate(projA, binsA, fcam, TA, ncA, torch.ones((H, W), dtype=torch.uint8, device=dev), blends_t)
    blends = int(blends_t.to(torch.int64).sum().item())               # blended (Gaussian, pixel) pairs
    ctxA.close()

    bwd_ms = timed["render_bwd"][0] / max(1, timed["render_bwd"][1])
    fwd_ms = timed["render_fwd"][0] / max(1, timed["render_fwd"][1])
    bwd_flops = BWD_FLOPS_PER_EVAL * evals_bwd + BWD_FLOPS_PER_BLEND * blends
    fwd_flops = FWD_FLOPS_PER_EVAL * evals_fwd_bound + FWD_FLOPS_PER_BLEND * blends
    dominant = max(kernels_ms, key=kernels_ms.get)
    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"traffic_cfg{args.config}.json")
    if os.path.exists(tpath) and not args.compact_box and not args.per_splat_bwd:
        with open(tpath) as f:
            traffic = json.load(f).get("render_bwd_bytes_per_launch")
    achieved = bwd_flops / (bwd_ms * 1e-3) / 1e12 if bwd_ms > 0 else 0.0
    roofline = {"kernel": "k_render_bwd_splat" if args.per_splat_bwd else "k_render_bwd", "bound": "alu",
                "achieved": round(achieved, 3), "peak": PEAK_FP32_TFLOPS,
                "unit": "TFLOP/s", "frac": round(achieved / PEAK_FP32_TFLOPS, 4), "traffic": traffic,
                "avg_launch_ms": round(bwd_ms, 4), "flops_per_launch": bwd_flops,
                "dominant_group_by_time": dominant}

    out = {
        "metric": "rasterizer fwd+bwd iters/s at 500k Gaussians, 1600x1064" if args.config == 3
                  else f"rasterizer fwd+bwd iters/s (config {args.config})",
        "value": round(1e3 / ms_per_step, 3), "unit": "iters/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": sc.name + (f"+compact_box(beta={args.cb_beta:g})" if args.compact_box else ""),
                   "gaussians": n, "sh_degree": sc.sh_degree, "image": [W, H],
                   "pairs": int(P), "max_tile_list": int(tile_len.max().item()),
                   "step": ("activate+" if args.train_iteration else "") + "preprocess+bin_sort+" +
                           ("render_fwd_loss(render_fwd+l1_grad+error map fused)" if fused else
                            "render_fwd+" + ("photo_loss" if args.photo_loss else "l1_grad")) + "+render_bwd+" +
                           ("activate_bwd+adam+" if args.train_iteration else "") +
                           ("error_mask_fused" if fused else "error_mask") + "+score_accumulate"},
        "roofline": roofline,
        "kernels_ms": {k: round(v, 4) for k, v in kernels_ms.items()},
        "gaussian_pixel_evals_per_s": round((evals_fwd_bound + evals_bwd) / (ms_per_step * 1e-3), 1),
        "render_fwd": {"avg_launch_ms": round(fwd_ms, 4),
                       "achieved_tflops": round(fwd_flops / (fwd_ms * 1e-3) / 1e12, 3) if fwd_ms > 0 else 0.0},
        "work": {"evals_fwd_upper_bound": evals_fwd_bound, "evals_bwd": evals_bwd, "blends": blends},
        "fwd_bwd_only": {"ms": round(fwd_bwd_ms, 4), "iters_per_s": round(1e3 / fwd_bwd_ms, 2),
                         "calls": "preprocess+bin_sort+render_fwd+loss+render_bwd (no mask, no score pass)"},
        "loss": float(out3[2].item()) if args.photo_loss else float(loss.item()),
        "score_pass": score_pass,
    }

    copy_gbs, fma_tf = ctx.fs_measure_peaks(1 << 30)
    out["measured_peaks"] = {"copy_GBps": round(copy_gbs, 1), "fp32_fma_TFLOPs_unpacked": round(fma_tf, 2),
                             "note": "1 GiB device copy (read + write) and chains of independent v_fma_f32, same process"}
    if not args.no_cpu_baseline and not args.train_iteration:   # (the oracle leg times the hot path on the untouched scene)
        from oracle import Config, Oracle
        o = Oracle(np.float32, Config(compact_box=args.compact_box, cb_beta=args.cb_beta))
        c0 = time.perf_counter()
        p_o, b_o, img_o, T_o, nc_o = o.forward(sc, cam)
        if args.photo_loss:
            import oracle as _orc
            ph = _orc.photometric(img_o, target_np, 0.2)
            l_o, dL_o = ph["E"], ph["grad"]
        else:
            l_o, dL_o = o.l1(img_o, target_np)
        o.backward(sc, cam, p_o, b_o, dL_o)
        m_o, thr_o, _ = o.error_mask(img_o, target_np)
        o.score(p_o, b_o, cam, m_o, np.zeros(n, np.int32))
        c1 = time.perf_counter()
        out["cpu_baseline"] = {"value": round(1.0 / (c1 - c0), 5), "unit": "iters/s", "cores": 1, "kind": "oracle",
                               "sample": f"one full step of {sc.name} (all tiles, same arrays), single thread, "
                                         f"{c1 - c0:.1f} s", "host_cores_visible": os.cpu_count()}
        out["cpu_baseline"]["loss_matches_gpu"] = bool(abs(l_o - out["loss"]) <= (1e-5 if args.photo_loss else 1e-6) * max(1.0, abs(l_o)))
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
