"""Writes tests/golden/oracle_digest.json from the fp32 CPU oracle alone (no GPU code is
imported).  The digest pins the oracle's bit-level behaviour across machines and edits: a change
of its arithmetic, of a compiler flag that alters rounding, or of the scene generator shows up as
a digest mismatch in test_oracle_golden.py.   Run:  python tests/golden/make_golden.py"""
import hashlib
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import Config, Oracle  # noqa: E402
from paper_2511_04283_amd import scenes  # noqa: E402


def sha(a):
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()[:32]


def digest(cfg, n=None, compact_box=False):
    sc = scenes.make_scene(cfg, n)
    cam = sc.cameras[0]
    o = Oracle(np.float32, Config(compact_box=compact_box))
    proj, bins, img, fT, nc = o.forward(sc, cam)
    tgt = scenes.target_image(cfg, 0, cam)
    mask, thr, _ = o.error_mask(img, tgt, rule=0, k=1.0)
    counts = o.score(proj, bins, cam, mask, np.zeros(sc.n, np.int32))
    return {
        "scene": sc.name, "n": sc.n, "inputs": sha(np.concatenate([sc.means.ravel(), sc.scales.ravel(), sc.quats.ravel(), sc.opacities, sc.sh.ravel()])),
        "num_pairs": bins.num_pairs, "rect": sha(proj.rect), "mean2d": sha(proj.mean2d), "conic_opacity": sha(proj.conic_opacity),
        "rgb": sha(proj.rgb), "keys_sorted": sha(bins.keys_sorted), "gauss_sorted": sha(bins.gauss_sorted),
        "tile_ranges": sha(bins.tile_ranges), "image": sha(img), "final_T": sha(fT), "n_contrib": sha(nc),
        "threshold_bits": int(np.float32(thr).view(np.uint32)), "mask": sha(mask), "counts": sha(counts),
        "counts_sum": int(counts.sum()),
    }


if __name__ == "__main__":
    out = {"cfg1": digest(1), "cfg2_n20000": digest(2, 20000), "cfg1_compact_box": digest(1, None, True),
           "cfg2_n20000_compact_box": digest(2, 20000, True)}
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_digest.json"), "w") as f:
        json.dump(out, f, indent=1, sort_keys=True)
    print(json.dumps(out, indent=1, sort_keys=True))
