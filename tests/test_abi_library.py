"""CPU-side checks of the boundary: the shared library loads and exports every symbol that
include/fastgs.h declares (no compute call is made: there is no GPU here)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "fastgs.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fs_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    from paper_2511_04283_amd import binding as B
    names = _declared()
    assert {"fs_preprocess", "fs_bin_sort", "fs_render_fwd", "fs_render_bwd", "fs_score_accumulate"} <= set(names)
    lib = B.load_library()
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(B.EXPORTS)


def test_default_config_and_struct_layouts_match_header():
    from paper_2511_04283_amd import binding as B
    c = B.default_config()
    assert c.tile == 16 and c.score_mode == 0
    assert abs(c.alpha_min - 1 / 255) < 1e-9 and abs(c.alpha_max - 0.99) < 1e-7 and abs(c.T_min - 1e-4) < 1e-10
    assert ctypes.sizeof(B.fs_config) == 56 and ctypes.sizeof(B.fs_camera) == 72
    assert ctypes.sizeof(B.fs_gaussians) == 56 and ctypes.sizeof(B.fs_projected) == 56
    assert ctypes.sizeof(B.fs_bins) == 88 and ctypes.sizeof(B.fs_grads) == 72 and ctypes.sizeof(B.fs_select_params) == 28


def test_null_context_is_rejected_without_touching_a_gpu():
    from paper_2511_04283_amd import binding as B
    lib = B.load_library()
    assert lib.fs_preprocess(None, None, None, None) == -1
    assert lib.fs_bin_sort(None, None, None, 0, None) == -1
    assert lib.fs_last_error(None) == b"null context"
    assert lib.fs_set_score_record(None, 1) == -1 and lib.fs_set_backward_mode(None, 0) == -1
    assert lib.fs_set_record_mode(None, 0) == -1


def test_no_product_code_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2511_04283_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "fastgs_oracle" not in text, f
