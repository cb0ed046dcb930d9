#!/usr/bin/env python3
"""Benchmark of the FastGS rasterizer hot path on one MI355X.

One step = one pass of the whole hot path over one synthetic view of the workload: projection,
pair ordering, forward compositing, the L1 term, backward, error mask and the per-Gaussian count pass
(fs_preprocess, fs_bin_sort, fs_render_fwd_loss, fs_render_bwd, fs_mask_score_fused = error mask + count pass;
--separate-calls for the unfused entry points), inputs resident in HBM.  The headline workload is
benchmark config 3 (500k Gaussians, SH degree 3, 1600x1064); --config N times another one.

Prints ONE JSON line.  `roofline` describes the kernel group that takes the most time in the step
(`rooflines` every group with a work model): achieved = algorithmic flops or bytes per launch / the group's
average duration, measured with HIP events on the stream the kernels are launched on.  `--gpus N` with N > 1 is
refused: this build is single-GPU by construction.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# Algorithmic work per unit: flops per examined list entry ("evaluation") and per blended (Gaussian, pixel) pair,
# for the forward and backward compositing kernels.
FWD_FLOPS_PER_EVAL = 11     # dx, dy, q (2 mul + 2 fma + mul), -0.5*q
FWD_FLOPS_PER_BLEND = 26    # exp (mul, rint, sub, 5 fma, ldexp) 14; alpha 2; T 2; w 1; colour 3 fma 6; + min
BWD_FLOPS_PER_EVAL = 11
BWD_FLOPS_PER_BLEND = 66    # exp 14; alpha 2; 1/(1-a), T, w 4; colour/alpha grads 17; conic/mean grads 20; 9-value sum 9
PEAK_FP32_TFLOPS = 157.3    # MI355X vector fp32 (packed FMA), 256 CU x 4 SIMD x 16 lanes x 2 x 2 x 2.4 GHz
PEAK_HBM_GBS = 8000.0
KERNEL_OF_GROUP = {"preprocess": "k_preprocess", "scan": "k_scan_*", "emit_pairs": "k_tile_pairs (count) + k_tile_sum + k_tile_scan",
                   "order_pairs": "k_tile_pairs (placement) + k_tile_sort", "tile_ranges": "k_tile_ranges + k_tile_order",
                   "render_fwd": "k_render_fwd", "l1_grad": "k_fold_tile_stats", "photo_loss": "k_ssim_*",
                   "render_bwd": "k_render_bwd", "preprocess_bwd": "k_preprocess_bwd", "error_mask": "k_err_*",
                   "score": "k_score_bits"}


def kernel_source_digest() -> str:
    """Digest of the HIP sources: a traffic summary under profiles/ only applies to the kernels it was measured on."""
    from paper_2511_04283_amd.build import source_digest
    return source_digest()


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=3, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--wide-tail", action="store_true",
                    help="config 5 with the wide scale distribution (27 M pairs instead of 10 M)")
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
    if args.wide_tail and args.config != 5:
        print("bench.py: --wide-tail is a variant of --config 5", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2511_04283_amd import binding as B
    from paper_2511_04283_amd import scenes

    sc = scenes.make_scene(args.config, scale_sigma=1.2) if args.wide_tail else scenes.make_scene(args.config)
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
        raw_s, raw_o = ctx.fs_activate_inv(g.scales, g.opacities, 1e-4, 1 - 1e-4)
        raw = dict(scales=raw_s, quats=g.quats.clone(), opac=raw_o)
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
        counts.zero_()
        if fused:
            ctx.fs_mask_score_fused(proj, bins, fcam, n_contrib, counts, B.FS_MASK_MEAN_STD, 1.0, mask, thr)
        else:
            ctx.fs_error_mask(image, target, B.FS_MASK_MEAN_STD, 1.0, mask, thr)
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

    # untimed: per-kernel-group breakdown of the same steps (a pair of HIP events per group and call, recorded on the
    # stream the kernels are launched on), which also names the group that dominates the step
    ctx.fs_profile_enable(None)
    for _ in range(max(3, args.steps // 2)):
        step()
    prof = ctx.fs_profile_read()
    kernels_ms = {k: (ms / c if c else 0.0) for k, (ms, c) in prof.items()}
    dominant = max(kernels_ms, key=kernels_ms.get)

    # timed region: K steps; only the dominant group keeps its events, and its average launch duration over exactly
    # these steps is what `roofline` is computed from
    ctx.fs_profile_enable([dominant])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    timed = ctx.fs_profile_read()
    ctx.fs_profile_enable(())
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    kernels_ms[dominant] = timed[dominant][0] / max(1, timed[dominant][1])

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
                    ctx.fs_mask_score_fused(proj, b_, fc, n_contrib, counts, B.FS_MASK_MEAN_STD, 1.0, mask, thr)
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

    # units of work of one step (exact, from the path's own outputs)
    step()   # (the work counts describe view 0; the forward pass of this step leaves its record for the count pass)
    torch.cuda.synchronize()
    bins = state["bins"]
    state["rows_per_tile"] = ctx.fs_score_record_rows(bins, fcam) if int(bins.num_pairs) > 0 else None
    P, R = int(bins.num_pairs), int(bins.struct.num_records)
    ranges = bins.copy_ranges().to(torch.int64)
    tile_len = ranges[:, 1] - ranges[:, 0]
    tiles = int(tile_len.shape[0])
    pixels = H * W
    n_vis = int((proj.tiles_touched != 0).sum().item())
    # list entries a pixel examines for certain: those up to the last one it blends (the forward pass goes on to the
    # entry that ends the pixel, or to the end of the list; the backward pass starts from exactly here)
    evals = int(n_contrib.to(torch.int64).sum().item())
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
    # pairs blended at one or more pixels of their tile: those that receive a gradient record in the sparse layout
    # (in this score mode a pair has a row in the forward pass's record exactly then)
    pairs_blended = int(ctxA.fs_score_record_rows(binsA, fcam).to(torch.int64).sum().item()) if int(binsA.num_pairs) > 0 else 0
    ctxA.close()
    del projA, imA, TA, ncA, blends_t
    # pairs of the tiles that hold at least one mask pixel (what the count pass has to read)
    th, tw = (H + 15) // 16, (W + 15) // 16
    mpad = torch.zeros((th * 16, tw * 16), dtype=torch.uint8, device=dev)
    mpad[:H, :W] = mask
    tile_has_mask = mpad.view(th, 16, tw, 16).amax(dim=(1, 3)).reshape(-1) != 0
    pairs_masked_tiles = int(tile_len[tile_has_mask].sum().item())
    # ... and, of those, the pairs the record holds a row for (counted at some pixel of their tile)
    if state.get("rows_per_tile") is not None:
        rows_masked_tiles = int(state["rows_per_tile"].to(torch.int64)[tile_has_mask].sum().item())
    else:
        rows_masked_tiles = pairs_masked_tiles

    # algorithmic work per launch of each kernel group (the design doc section 7 states the per-unit figures)
    g_in = 4 * (3 + 3 + 4 + 1 + 3 * K)            # bytes of one Gaussian's parameters (236 at degree 3)
    g_proj = 8 + 4 + 16 + 12 + 8 + 4 + 3           # bytes of one projected splat (fs_projected)
    copies = 256                                   # workgroups of the counting / placement kernels
    # (the library's own rule for FS_RECORDS_AUTO: sparse per-pair gradient records when the lists are long on average)
    sparse_records = P >= 320 * tiles
    work = {
        "preprocess": ("hbm", n * (12 + g_proj) + n_vis * (g_in - 12)),
        "emit_pairs": ("hbm", n * 16 + n_vis * 4 + 3 * 4 * tiles * copies + 16 * tiles),
        "order_pairs": ("hbm", n * 8 + n_vis * (44 + 64) + P * 8 + P * (8 + 12) + 4 * tiles * copies),
        "render_fwd": ("alu", FWD_FLOPS_PER_EVAL * evals + FWD_FLOPS_PER_BLEND * blends),
        "render_bwd": ("alu", BWD_FLOPS_PER_EVAL * evals + BWD_FLOPS_PER_BLEND * blends),
        "preprocess_bwd": ("hbm", (48 * pairs_blended + 2 * R if sparse_records else 48 * R) + n * 8 + n_vis * (g_in + 3) + n * (g_in + 8)),
        "error_mask": ("hbm", pixels * (24 + 4 + 4 + 1)),     # (separate calls only; fused: part of the count pass)
        "score": ("hbm", rows_masked_tiles * (32 + 4) + 8 * tiles + (pixels * (4 + 1) if fused else pixels)),
    }
    if args.radix_sort or args.per_splat_bwd or args.compact_box:
        for k in ("emit_pairs", "order_pairs"):      # (the models above describe the default ordering)
            work.pop(k, None)
    rooflines = {}
    for grp, (bound, amount) in work.items():
        ms = kernels_ms.get(grp, 0.0)
        if ms <= 0:
            continue
        if bound == "alu":
            ach, peak, unit = amount / (ms * 1e-3) / 1e12, PEAK_FP32_TFLOPS, "TFLOP/s"
        else:
            ach, peak, unit = amount / (ms * 1e-3) / 1e9, PEAK_HBM_GBS, "GB/s"
        rooflines[grp] = {"kernel": KERNEL_OF_GROUP[grp], "bound": bound, "achieved": round(ach, 3), "peak": peak, "unit": unit,
                          "frac": round(ach / peak, 4), "avg_launch_ms": round(ms, 4),
                          ("flops_per_launch" if bound == "alu" else "bytes_per_launch"): int(amount)}
    # HBM traffic per launch from the rocprofv3 --pmc summary under profiles/, if one exists for this workload AND
    # was measured on these very kernel sources; otherwise null
    traffic, traffic_note = None, None
    wl = f"cfg{args.config}" + ("_wide_tail" if args.wide_tail else "")
    tpath = os.path.join(ROOT, "profiles", f"traffic_{wl}.json")
    plain = not (args.compact_box or args.per_splat_bwd or args.radix_sort or args.separate_calls or args.photo_loss or
                 args.abs_grad or args.train_iteration)
    if os.path.exists(tpath) and plain:
        with open(tpath) as f:
            tj = json.load(f)
        if tj.get("kernel_source_digest") == kernel_source_digest():
            traffic = tj.get("bytes_per_launch", {}).get(dominant)
        else:
            traffic_note = "profiles/traffic summary was measured on other kernel sources: not used"
    roofline = dict(rooflines.get(dominant, {"kernel": KERNEL_OF_GROUP.get(dominant, dominant), "bound": "hbm", "achieved": None,
                                             "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": None}))
    roofline["group"] = dominant
    roofline["traffic"] = traffic
    if traffic_note:
        roofline["traffic_note"] = traffic_note
    if args.per_splat_bwd and dominant == "render_bwd":
        roofline["kernel"] = "k_render_bwd_splat"

    out = {
        "metric": "rasterizer fwd+bwd iters/s at 500k Gaussians, 1600x1064" if args.config == 3
                  else f"rasterizer fwd+bwd iters/s (config {args.config}{', wide tail' if args.wide_tail else ''})",
        "value": round(1e3 / ms_per_step, 3), "unit": "iters/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": sc.name + ("+wide_tail(scale_sigma=1.2)" if args.wide_tail else "") +
                               (f"+compact_box(beta={args.cb_beta:g})" if args.compact_box else ""),
                   "gaussians": n, "visible": n_vis, "sh_degree": sc.sh_degree, "image": [W, H],
                   "pairs": P, "max_tile_list": int(tile_len.max().item()),
                   "backward_records": "sparse" if sparse_records else "dense", "pairs_blended_somewhere": pairs_blended,
                   "step": ("activate+" if args.train_iteration else "") + "preprocess+bin_sort+" +
                           ("render_fwd_loss(render_fwd+l1_grad+error map fused)" if fused else
                            "render_fwd+" + ("photo_loss" if args.photo_loss else "l1_grad")) + "+render_bwd+" +
                           ("activate_bwd+adam+" if args.train_iteration else "") +
                           ("mask_score_fused" if fused else "error_mask+score_accumulate")},
        "roofline": roofline,
        "rooflines": rooflines,
        "kernels_ms": {k: round(v, 4) for k, v in kernels_ms.items()},
        "gaussian_pixel_evals_per_s": round(2 * evals / (ms_per_step * 1e-3), 1),
        "work": {"evals": evals, "blends": blends, "pairs_times_256_upper_bound": P * 256,
                 "note": "evals = list entries up to each pixel's last blended one, counted once for the forward and "
                         "once for the backward pass in gaussian_pixel_evals_per_s"},
        "fwd_bwd_only": {"ms": round(fwd_bwd_ms, 4), "iters_per_s": round(1e3 / fwd_bwd_ms, 2),
                         "calls": "preprocess+bin_sort+render_fwd+loss+render_bwd (no mask, no score pass)"},
        "loss": float(out3[2].item()) if args.photo_loss else float(loss.item()),
        "score_pass": score_pass,
    }

    copy_gbs, fma_tf = ctx.fs_measure_peaks(1 << 30)
    out["measured_peaks"] = {"copy_GBps": round(copy_gbs, 1), "fp32_fma_TFLOPs_unpacked": round(fma_tf, 2),
                             "note": "1 GiB device copy (read + write) and chains of independent v_fma_f32, same process"}
    if not args.no_cpu_baseline and not args.train_iteration:   # (the oracle leg times the hot path on the untouched scene)
        out["cpu_baseline"] = cpu_baseline(args, sc, cam, target_np, out["loss"], tiles)
    print(json.dumps(out))
    return 0


def cpu_baseline(args, sc, cam, target_np, gpu_loss, tiles):
    """The oracle as it stands, single thread, on the same arrays.  Configs 1-3: one whole step.  Configs 4 and 5: the
    projection and the ordering on everything, compositing / backward / count pass on every 16th tile, the tile part
    scaled by 16 (stated in `sample`): a bounded sample, so that the default run stays within minutes."""
    import numpy as np
    import oracle as _orc
    from oracle import Config, Oracle
    o = Oracle(np.float32, Config(compact_box=args.compact_box, cb_beta=args.cb_beta))
    n = sc.n
    if args.config <= 3:
        c0 = time.perf_counter()
        p_o, b_o, img_o, T_o, nc_o = o.forward(sc, cam)
        if args.photo_loss:
            ph = _orc.photometric(img_o, target_np, 0.2)
            l_o, dL_o = ph["E"], ph["grad"]
        else:
            l_o, dL_o = o.l1(img_o, target_np)
        o.backward(sc, cam, p_o, b_o, dL_o)
        m_o, thr_o, _ = o.error_mask(img_o, target_np)
        o.score(p_o, b_o, cam, m_o, np.zeros(n, np.int32))
        dt = time.perf_counter() - c0
        return {"value": round(1.0 / dt, 5), "unit": "iters/s", "cores": 1, "kind": "oracle",
                "sample": f"one full step of {sc.name} (all tiles, same arrays), single thread, {dt:.1f} s",
                "host_cores_visible": os.cpu_count(),
                "loss_matches_gpu": bool(abs(l_o - gpu_loss) <= (1e-5 if args.photo_loss else 1e-6) * max(1.0, abs(l_o)))}
    every = 16
    tl = np.arange(0, tiles, every, dtype=np.int32)
    c0 = time.perf_counter()
    p_o = o.preprocess(sc, cam)
    b_o = o.bin_sort(p_o, cam)
    c1 = time.perf_counter()
    img_o, T_o, nc_o = o.render_fwd(p_o, b_o, cam, tile_list=tl)
    _, dL_o = o.l1(img_o, target_np)
    o.backward(sc, cam, p_o, b_o, dL_o, tile_list=tl)
    m_o, thr_o, _ = o.error_mask(img_o, target_np)
    o.score(p_o, b_o, cam, m_o, np.zeros(n, np.int32), tile_list=tl)
    c2 = time.perf_counter()
    est = (c1 - c0) + every * (c2 - c1)
    return {"value": round(1.0 / est, 5), "unit": "iters/s", "cores": 1, "kind": "oracle", "extrapolated": True,
            "sample": f"{sc.name}: projection and ordering of everything ({c1 - c0:.1f} s), compositing + backward + count "
                      f"pass on every {every}th tile ({c2 - c1:.1f} s, scaled by {every}), single thread",
            "host_cores_visible": os.cpu_count()}


if __name__ == "__main__":
    sys.exit(main())
