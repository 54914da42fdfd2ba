"""The C-ABI library loads on a machine without a GPU and exports every declared symbol."""
import ctypes
import os
import re

from paper_2102_08124_amd import binding as tm

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "tmask.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tmask_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    lib = tm.load_library()
    names = _declared_functions()
    assert set(names) == set(tm.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n


def test_version_and_error_text_without_gpu():
    assert tm.tmask_version() >= 100
    lib = tm.load_library()
    # host-side validation needs no device: a NULL descriptor array is rejected before any HIP call
    rc = lib.tmask_approx(None, 1, 0, 2, 4, 0, None, 0, None)
    assert rc == tm.TMASK_ERR_NULL
    assert b"NULL" in lib.tmask_last_error()
    rc = lib.tmask_approx(ctypes.cast(ctypes.c_void_p(8), ctypes.POINTER(tm.tmask_mat)), 1, 0, 3, 6, 0, None, 0, None)
    assert rc == tm.TMASK_ERR_NM
    assert lib.tmask_workspace_bytes(None, 1, 2, 4) == 0


def test_struct_layouts_match_header():
    assert ctypes.sizeof(tm.tmask_mat) == 56
    assert ctypes.sizeof(tm.tmask_pack_desc) == 80
    assert ctypes.sizeof(tm.tmask_fused_desc) == 88
    assert ctypes.sizeof(tm.tmask_flip_desc) == 56
    assert ctypes.sizeof(tm.tmask_dense_desc) == 64
    assert tm.tmask_mask_dense_desc is tm.tmask_dense_desc          # same layout, writable mask on the C side
    assert ctypes.sizeof(tm.tmask_violation_desc) == 56
    assert ctypes.sizeof(tm.tmask_score_out) == 56
