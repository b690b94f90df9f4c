"""The C-ABI library loads and exports every symbol include/ones.h declares (no GPU)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "ones.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ones_[a-z_]+)\s*\(", text)))


def test_header_declares_the_boundary():
    names = _declared()
    for must in ("ones_init", "ones_generation", "ones_best", "ones_set_jobs", "ones_export",
                 "ones_workspace_bytes", "ones_destroy", "ones_strerror"):
        assert must in names


def test_library_exports_every_declared_symbol():
    from paper_2108_03645_amd import ones
    if not os.path.exists(ones.library_path()):
        pytest.skip("libones.so not built here (python paper_2108_03645_amd/build.py)")
    lib = ctypes.CDLL(ones.library_path())
    for name in _declared():
        assert hasattr(lib, name), name
    assert sorted(ones.EXPORTS) == _declared()


def test_host_side_argument_checks_need_no_gpu():
    """Validation happens before any device work, so it can be exercised on the CPU."""
    from paper_2108_03645_amd import ones
    if not os.path.exists(ones.library_path()):
        pytest.skip("libones.so not built here")
    L = ones.load()
    bad = ones.ones_config(4, 4, 18, 0, 0.1, 0.5)                  # population not a multiple of 4
    assert L.ones_workspace_bytes(ctypes.byref(bad)) == 0
    ok = ones.ones_config(64, 40, 1024, 1, 0.1, 0.5)
    need = L.ones_workspace_bytes(ctypes.byref(ok))
    # P + K genome rows of 64 padded slots, a score per row, the survivor list
    assert need >= (1024 + 256) * 64 * 4 + (1024 + 256) * 8 + 256 * 4
    assert L.ones_padded_jobs(0) == 64 and L.ones_padded_jobs(64) == 64 and L.ones_padded_jobs(65) == 128
    h = ctypes.c_void_p()
    assert L.ones_init(ctypes.byref(h), ctypes.byref(bad), None, None, 0, None) == -1
    assert L.ones_init(None, ctypes.byref(ok), None, None, 0, None) == -1
    assert L.ones_init(ctypes.byref(h), ctypes.byref(ok), None, None, 0, None) == -1   # jobs missing
    assert h.value is None
    assert L.ones_generation(None, 1) == -1 and L.ones_best(None, None, None, None) == -1
    assert b"power" in L.ones_strerror(-2)
    L.ones_destroy(None)
