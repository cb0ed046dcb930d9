"""Helpers of the GPU parity tests: run the HIP path through the C-ABI binding and bring every
output back as numpy, next to the fp32 oracle's outputs for the same seeded inputs."""
import numpy as np


def gpu_pipeline(ctx, sc, cam, target=None, dL=None, mask_rule=0, mask_k=1.0, want_bwd=True, want_score=True,
                 want_abs=False):
    import torch
    from paper_2511_04283_amd import binding as B
    g = B.Gaussians.from_scene(sc, ctx.device)
    fcam = B.make_camera(cam)
    proj = ctx.fs_preprocess(g, fcam)
    bins = ctx.fs_bin_sort(proj, fcam)
    image, final_T, n_contrib = ctx.fs_render_fwd(proj, bins, fcam)
    out = dict(
        mean2d=proj.mean2d.cpu().numpy(), depth=proj.depth.cpu().numpy(), conic_opacity=proj.conic_opacity.cpu().numpy(),
        rgb=proj.rgb.cpu().numpy(), rect=proj.rect.cpu().numpy().view(np.uint16).astype(np.int32),
        tiles_touched=proj.tiles_touched.cpu().numpy().view(np.uint32), clamped=proj.clamped.cpu().numpy(),
        num_pairs=bins.num_pairs, keys_sorted=bins.copy_keys().cpu().numpy().view(np.uint64),
        gauss_sorted=bins.copy_gauss().cpu().numpy().view(np.uint32),
        tile_ranges=bins.copy_ranges().cpu().numpy().view(np.uint32),
        image=image.cpu().numpy(), final_T=final_T.cpu().numpy(), n_contrib=n_contrib.cpu().numpy().view(np.uint32))
    if target is not None or dL is not None:
        if dL is None:
            tgt = torch.from_numpy(target).to(ctx.device)
            loss = torch.zeros(1, dtype=torch.float64, device=ctx.device)
            dLt = ctx.fs_l1_grad(image, tgt, loss_out=loss)
            out["loss"] = float(loss.item())
            out["dL"] = dLt.cpu().numpy()
        else:
            dLt = torch.from_numpy(np.ascontiguousarray(dL, dtype=np.float32)).to(ctx.device)
        if want_bwd:
            gr = ctx.fs_render_bwd(g, fcam, proj, bins, final_T, n_contrib, dLt, want_2d=True, want_abs=want_abs)
            out["grads"] = {k: v.cpu().numpy() for k, v in gr.items()}
        if want_score and target is not None:
            mask, thr = ctx.fs_error_mask(image, tgt, rule=mask_rule, k=mask_k)
            counts = torch.zeros(sc.n, dtype=torch.int32, device=ctx.device)
            ctx.fs_score_accumulate(proj, bins, fcam, final_T, n_contrib, mask, counts)
            out["mask"] = mask.cpu().numpy()
            out["thr"] = np.float32(thr.item())
            out["counts"] = counts.cpu().numpy()
            # the count pass has two implementations: from the record the forward pass left (above, the default)
            # and by a second walk over the tile lists (when no record is kept); both must give the same counts
            ctx.fs_set_score_record(False)
            try:
                image2, final_T2, n_contrib2 = ctx.fs_render_fwd(proj, bins, fcam)
                walked = torch.zeros(sc.n, dtype=torch.int32, device=ctx.device)
                ctx.fs_score_accumulate(proj, bins, fcam, final_T2, n_contrib2, mask, walked)
            finally:
                ctx.fs_set_score_record(True)
            assert torch.equal(image2, image) and torch.equal(n_contrib2, n_contrib)
            assert torch.equal(walked, counts), "count pass: record and walk disagree"
    return out


def assert_image_close(got, ref, rtol=1e-4):
    """The image bar: |got - ref| <= 1e-4 * |ref| per value, with |ref| floored at 1e-2 (colours are O(1); the floor
    keeps near-black pixels from demanding more than fp32 can give)."""
    err = np.abs(np.asarray(got, np.float64) - np.asarray(ref, np.float64))
    assert (err <= rtol * np.maximum(np.abs(ref), 1e-2)).all(), float(err.max())


def assert_grads_close(got: dict, ref: dict, rtol=1e-3, floor=2e-3):
    """|got - ref| <= rtol*|ref| + min(floor, floor*max|ref|) per gradient tensor (the benchmark's
    1e-3 relative / 2e-3 absolute-floor bar, never looser than its literal statement)."""
    worst = {}
    for k, r in ref.items():
        if k not in got:
            continue
        g = got[k].astype(np.float64)
        r = np.asarray(r, dtype=np.float64)
        assert g.shape == r.shape, (k, g.shape, r.shape)
        scale = np.abs(r).max() if r.size else 0.0
        atol = min(floor, floor * scale)
        err = np.abs(g - r)
        bad = err > rtol * np.abs(r) + atol
        worst[k] = float((err / (rtol * np.abs(r) + atol + 1e-300)).max()) if r.size else 0.0
        assert not bad.any(), (k, int(bad.sum()), r.size, float(err.max()), scale,
                               np.argwhere(bad)[:5].tolist(), g[bad][:5], r[bad][:5])
    return worst
