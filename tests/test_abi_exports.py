"""The C-ABI library loads and exports every symbol include/gmeta.h declares (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "gmeta.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gm_[a-z_]+)\s*\(", text)))


def _lib_path():
    from paper_2401_04338_amd import LIB_PATH
    if not os.path.exists(LIB_PATH):
        from paper_2401_04338_amd.build import build
        build(verbose=False)
    return LIB_PATH


def test_header_declares_the_entry_points():
    syms = _declared_symbols()
    for s in ["gm_create", "gm_destroy", "gm_last_error", "gm_workspace_bytes", "gm_meta_step",
              "gm_scatter_add", "gm_gather_pool", "gm_index_prep"]:
        assert s in syms


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(_lib_path())
    for s in _declared_symbols():
        assert hasattr(lib, s), s


def test_binding_names_match_header():
    from paper_2401_04338_amd import EXPORTS
    assert sorted(EXPORTS) == _declared_symbols()


def test_workspace_bytes_is_host_only_and_monotone():
    """gm_workspace_bytes touches no GPU: callable here; more tasks/steps never need less."""
    from paper_2401_04338_amd.binding import _model_desc, load_library
    import ctypes as C
    lib = load_library()
    d = _model_desc(8, [1000] * 8, 16, 13, [141, 64, 32, 1], 0)
    a = lib.gm_workspace_bytes(C.byref(d), 4, 128, 128, 1024, 1024, 1, 2)
    b = lib.gm_workspace_bytes(C.byref(d), 8, 256, 256, 2048, 2048, 1, 2)
    c = lib.gm_workspace_bytes(C.byref(d), 8, 256, 256, 2048, 2048, 3, 2)
    assert 0 < a < b < c
    bad = _model_desc(8, [1000] * 8, 16, 13, [140, 64, 32, 1], 0)   # d_0 != F*D + n_dense
    assert lib.gm_workspace_bytes(C.byref(bad), 4, 128, 128, 1024, 1024, 1, 2) == 0
