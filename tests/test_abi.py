"""The C-ABI library loads without a GPU and exports every symbol the header declares."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "ivf_gp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ivf_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_boundary():
    syms = declared_symbols()
    for name in ("ivf_load_index", "ivf_search", "ivf_encode", "ivf_free_index", "ivf_last_error"):
        assert name in syms


def test_library_exports_every_declared_symbol():
    import paper_1802_02422_amd as ivf
    if not os.path.exists(ivf.library_path()):
        from paper_1802_02422_amd.build import build_library
        build_library()
    lib = ctypes.CDLL(ivf.library_path())
    for name in declared_symbols():
        assert hasattr(lib, name), name


def test_binding_has_the_same_names():
    import paper_1802_02422_amd as ivf
    for name in declared_symbols():
        assert hasattr(ivf, name), name


def test_host_only_entry_points():
    import paper_1802_02422_amd as ivf
    from oracle import ivf_oracle as orc
    import numpy as np
    for P, L, tau in ((16, 8, 0.5), (64, 64, 0.25), (128, 64, 0.2), (256, 64, 0.2), (1, 1, 1e-6), (7, 3, 1.0),
                      (40, 24, 0.3)):
        assert ivf.ivf_num_kept(P, L, tau) == orc.num_kept(float(np.float32(tau)), P, L)
    assert ivf.ivf_num_kept(256, 64, 0.2) == 3277


def test_missing_library_fails_loudly(monkeypatch):
    import paper_1802_02422_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "_LIB_PATH", "/nonexistent/libivf_gp.so")
    with pytest.raises(b.IvfError):
        b.load_library()
