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


def test_job_table_validation_needs_no_gpu():
    """ones_init checks the job table and the workspace before it touches the device."""
    from paper_2108_03645_amd import ones
    from pyref import make_jobs
    if not os.path.exists(ones.library_path()):
        pytest.skip("libones.so not built here")
    L = ones.load()
    cfg = ones.ones_config(16, 8, 64, 0, 0.1, 0.5)
    h = ctypes.c_void_p()

    def init(jobs, workspace=0x1000, nbytes=1):
        js, keep = ones.make_jobs(jobs)
        return L.ones_init(ctypes.byref(h), ctypes.byref(cfg), ctypes.byref(js), ctypes.c_void_p(workspace), nbytes, None)

    good = make_jobs(8)
    assert init(good) == -5                                    # valid table, workspace of one byte
    assert init(good, workspace=0x1001, nbytes=1 << 30) == -5  # misaligned workspace
    assert init(good, workspace=0) == -1
    for field, value, code in [("bmin", 48, -2), ("bmax", None, -3), ("gpu_max_batch", 0, -2),
                               ("a", float("nan"), -4), ("remaining", float("inf"), -4), ("d", -1.0, -1),
                               ("c", 1e101, -3)]:
        bad = make_jobs(8)
        arr = getattr(bad, field)
        if field == "bmax":
            arr[3] = 1 << 30
            bad.gpu_max_batch[3] = 1                           # 2^30 GPUs: beyond the 2^20 a job may hold
        else:
            arr[3] = value
        assert init(bad) == code, field
        bad.active[3] = 0                                      # an empty slot's values are ignored
        assert init(bad) == -5, field
    lo_above_hi = make_jobs(8, bmin=512, bmax=256)
    assert init(lo_above_hi) == -3
    assert h.value is None
    for call in (lambda: L.ones_set_jobs(None, None), lambda: L.ones_set_progress(None, None, None, None),
                 lambda: L.ones_set_crossover(None, 0), lambda: L.ones_set_processed_time(None, None),
                 lambda: L.ones_set_new_jobs_first(None, 1), lambda: L.ones_placement(None, None, None),
                 lambda: L.ones_export(None, None, None, None, None), lambda: L.ones_export_remaining(None, None),
                 lambda: L.ones_generation_static(None, 1), lambda: L.ones_set_wait_limit(None, 5)):
        assert call() == -1
    assert b"static scratch" in L.ones_strerror(-7)
