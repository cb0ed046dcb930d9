"""The entry point that allocates nothing (fs_error_mask_noalloc: error map and partial sums in a static device
array of the library) against fs_error_mask, through the C ABI: two calls in a row, the second on a smaller image,
both rules; the size limit is an error, not a fault."""
import ctypes

import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def test_noalloc_error_mask_matches_the_allocating_entry_point():
    import torch
    from paper_2511_04283_amd import binding as B
    ctx = B.Context("cuda:0")
    dev = ctx.device
    rng = np.random.default_rng(4283)
    for (H, W), rule, k in (((1064, 1600), B.FS_MASK_MEAN_STD, 1.0), ((117, 203), B.FS_MASK_MINMAX_TAU, 0.35),
                            ((33, 41), B.FS_MASK_MEAN_STD, 0.5)):
        img = torch.from_numpy(rng.uniform(0, 1, (3, H, W)).astype(np.float32)).to(dev)
        tgt = torch.from_numpy(rng.uniform(0, 1, (3, H, W)).astype(np.float32)).to(dev)
        want_mask, want_thr = ctx.fs_error_mask(img, tgt, rule, k)
        mask = torch.full((H, W), 7, dtype=torch.uint8, device=dev)
        thr = torch.zeros(1, dtype=torch.float32, device=dev)
        free0 = torch.cuda.mem_get_info(dev)[0]
        ctx.fs_error_mask_noalloc(img, tgt, mask, thr, rule, k)
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info(dev)[0] == free0          # no device memory was taken
        assert torch.equal(mask, want_mask)
        assert thr.cpu().numpy().view(np.uint32)[0] == want_thr.cpu().numpy().view(np.uint32)[0]
        assert 0 < int(mask.sum().item()) < H * W
    # beyond the static array: a clear error before anything is launched
    lib = B.load_library()
    small = torch.zeros((3, 4, 4), dtype=torch.float32, device=dev)
    m = torch.zeros(16, dtype=torch.uint8, device=dev)
    rc = lib.fs_error_mask_noalloc(ctx.handle, ctypes.c_void_p(small.data_ptr()), ctypes.c_void_p(small.data_ptr()), 4096,
                                   2048, 0, ctypes.c_float(1.0), ctypes.c_void_p(m.data_ptr()), None)
    assert rc == -4 and b"FS_NOALLOC_MAX_PIXELS" in lib.fs_last_error(ctx.handle)
    ctx.close()
