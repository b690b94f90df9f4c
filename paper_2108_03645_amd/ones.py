"""Python binding of libones (include/ones.h): argument marshalling only.  Every step of
the search runs in the library's HIP kernels; PyTorch supplies the device workspace and the
stream.  There is no CPU fallback: without the built library or without a GPU this raises."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libones.so")
_lib = None


class OnesError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"libones error {code}: {message}")
        self.code = code


class ones_config(C.Structure):
    _fields_ = [("n_gpus", C.c_int32), ("n_slots", C.c_int32), ("population", C.c_int32),
                ("seed", C.c_uint64), ("mutation_rate", C.c_double), ("crossover_rate", C.c_double)]


class ones_jobs(C.Structure):
    _fields_ = [("job_id", C.c_void_p), ("active", C.c_void_p), ("bmin", C.c_void_p),
                ("bmax", C.c_void_p), ("gpu_max_batch", C.c_void_p), ("a", C.c_void_p),
                ("c", C.c_void_p), ("d", C.c_void_p), ("remaining", C.c_void_p)]


_JOB_DTYPES = {"job_id": np.int64, "active": np.uint8, "bmin": np.int32, "bmax": np.int32,
               "gpu_max_batch": np.int32, "a": np.float64, "c": np.float64, "d": np.float64,
               "remaining": np.float64}

EXPORTS = ["ones_workspace_bytes", "ones_init", "ones_set_jobs", "ones_generation", "ones_generation_static", "ones_set_wait_limit", "ones_best",
           "ones_export", "ones_placement", "ones_update_limits", "ones_set_new_jobs_first", "ones_set_processed_time", "ones_set_crossover",
           "ones_set_progress", "ones_export_remaining", "ones_padded_jobs",
           "ones_profile_enable", "ones_profile_read",
           "ones_destroy", "ones_strerror"]


class ones_limit_inputs(C.Structure):
    _fields_ = [("state", C.c_void_p), ("bmin", C.c_void_p), ("bcap", C.c_void_p), ("gpu_max_batch", C.c_void_p),
                ("last_batch", C.c_void_p), ("finished_epoch", C.c_void_p), ("elapsed", C.c_void_p)]


_LIMIT_DTYPES = {"state": np.uint8, "bmin": np.int32, "bcap": np.int32, "gpu_max_batch": np.int32,
                 "last_batch": np.int32, "finished_epoch": np.uint8, "elapsed": np.float64}


def update_limits(limit, sigma, **arrays):
    """ones_update_limits (Section 3.3.2): returns the new limits.  arrays: state, bmin, bcap,
    gpu_max_batch, last_batch, finished_epoch, elapsed, one entry per slot.  Host code only."""
    out = np.array(limit, np.int32)
    keep = [np.ascontiguousarray(arrays[k], dtype=dt) for k, dt in _LIMIT_DTYPES.items()]
    if any(a.shape != out.shape for a in keep):
        raise ValueError("one entry per slot in every array")
    inp = ones_limit_inputs(*[a.ctypes.data for a in keep])
    _check(load().ones_update_limits(len(out), C.byref(inp), float(sigma), out.ctypes.data))
    return out


def library_path() -> str:
    return _LIB_PATH


def load():
    """Load libones.so; raises if it has not been built (python -m paper_2108_03645_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise OnesError(-100, f"{_LIB_PATH} is missing: build it with paper_2108_03645_amd/build.py")
    # PyTorch bundles its own HIP runtime (same soname as ROCm's).  Import it first so that
    # libones binds to the runtime that owns the workspace and the stream instead of
    # bringing up a second one.
    import torch  # noqa: F401
    L = C.CDLL(_LIB_PATH)
    L.ones_workspace_bytes.argtypes = [C.POINTER(ones_config)]
    L.ones_workspace_bytes.restype = C.c_size_t
    L.ones_init.argtypes = [C.POINTER(C.c_void_p), C.POINTER(ones_config), C.POINTER(ones_jobs),
                            C.c_void_p, C.c_size_t, C.c_void_p]
    L.ones_set_jobs.argtypes = [C.c_void_p, C.POINTER(ones_jobs)]
    L.ones_generation.argtypes = [C.c_void_p, C.c_int32]
    L.ones_generation_static.argtypes = [C.c_void_p, C.c_int32]
    L.ones_set_wait_limit.argtypes = [C.c_void_p, C.c_uint32]
    L.ones_best.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(C.c_double)]
    L.ones_export.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(C.c_int64)]
    L.ones_placement.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
    L.ones_set_new_jobs_first.argtypes = [C.c_void_p, C.c_int32]
    L.ones_set_processed_time.argtypes = [C.c_void_p, C.c_void_p]
    L.ones_set_crossover.argtypes = [C.c_void_p, C.c_int32]
    L.ones_update_limits.argtypes = [C.c_int32, C.POINTER(ones_limit_inputs), C.c_double, C.c_void_p]
    L.ones_set_progress.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    L.ones_export_remaining.argtypes = [C.c_void_p, C.c_void_p]
    L.ones_padded_jobs.argtypes = [C.c_int32]
    L.ones_padded_jobs.restype = C.c_int32
    L.ones_profile_enable.argtypes = [C.c_void_p, C.c_int32]
    L.ones_profile_read.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int64),
                                    C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    L.ones_destroy.argtypes = [C.c_void_p]
    L.ones_destroy.restype = None
    L.ones_strerror.argtypes = [C.c_int]
    L.ones_strerror.restype = C.c_char_p
    _lib = L
    return L


def _check(rc: int):
    if rc != 0:
        raise OnesError(rc, load().ones_strerror(rc).decode())


def make_config(cluster) -> ones_config:
    return ones_config(int(cluster.n_gpus), int(cluster.n_slots), int(cluster.population),
                       int(cluster.seed) & (2**64 - 1), float(cluster.mutation_rate),
                       float(cluster.crossover_rate))


def make_jobs(jobs):
    """Returns (struct, keepalive list) for any object carrying the nine job arrays."""
    keep = [np.ascontiguousarray(getattr(jobs, k), dtype=dt) for k, dt in _JOB_DTYPES.items()]
    return ones_jobs(*[a.ctypes.data for a in keep]), keep


def workspace_bytes(cluster) -> int:
    cfg = make_config(cluster)
    return int(load().ones_workspace_bytes(C.byref(cfg)))


def padded_jobs(n_slots: int) -> int:
    return int(load().ones_padded_jobs(int(n_slots)))


class Search:
    """ones_init / ones_set_jobs / ones_generation / ones_best / ones_export on one GPU."""

    def __init__(self, cluster, jobs, device="cuda:0", stream=None):
        import torch
        if not torch.cuda.is_available():
            raise OnesError(-101, "no GPU visible: libones has no CPU path")
        L = load()
        self._torch = torch
        self.device = torch.device(device)
        self.n_slots = int(cluster.n_slots)
        self.n_gpus = int(cluster.n_gpus)
        self.population = int(cluster.population)
        self.jp = padded_jobs(self.n_slots)
        cfg = make_config(cluster)
        nbytes = int(L.ones_workspace_bytes(C.byref(cfg)))
        if nbytes == 0:
            raise OnesError(-1, "invalid configuration")
        with torch.cuda.device(self.device):
            self.stream = stream if stream is not None else torch.cuda.current_stream()
            self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        base = self.workspace.data_ptr()
        self._ws_ptr = (base + 255) & ~255
        self._h = C.c_void_p()
        js, keep = make_jobs(jobs)
        with torch.cuda.device(self.device):
            _check(L.ones_init(C.byref(self._h), C.byref(cfg), C.byref(js), C.c_void_p(self._ws_ptr),
                               nbytes, C.c_void_p(self.stream.cuda_stream)))

    def set_jobs(self, jobs):
        js, keep = make_jobs(jobs)
        with self._torch.cuda.device(self.device):
            _check(load().ones_set_jobs(self._h, C.byref(js)))

    def generation(self, n: int = 1):
        with self._torch.cuda.device(self.device):
            _check(load().ones_generation(self._h, int(n)))

    def generation_static(self, n: int = 1):
        """ones_generation_static: the same generations with the selection's scratch in the library's
        static device array (for callers that cannot allocate)."""
        with self._torch.cuda.device(self.device):
            _check(load().ones_generation_static(self._h, int(n)))

    def set_wait_limit(self, polls: int):
        _check(load().ones_set_wait_limit(self._h, int(polls)))

    def set_progress(self, alpha=None, beta=None, processed=None):
        """ones_set_progress: one entry per slot each; all None switches the sampling off."""
        with self._torch.cuda.device(self.device):
            if alpha is None and beta is None and processed is None:
                _check(load().ones_set_progress(self._h, None, None, None))
                return
            arrs = [np.ascontiguousarray(x, np.float64) for x in (alpha, beta, processed)]
            if any(a.shape != (self.n_slots,) for a in arrs):
                raise ValueError("alpha, beta, processed: one entry per slot")
            _check(load().ones_set_progress(self._h, *[a.ctypes.data for a in arrs]))

    def set_new_jobs_first(self, on=True):
        _check(load().ones_set_new_jobs_first(self._h, int(bool(on))))

    def set_crossover(self, per_gpu=False):
        _check(load().ones_set_crossover(self._h, 1 if per_gpu else 0))

    def set_processed_time(self, t_processed=None):
        if t_processed is None:
            _check(load().ones_set_processed_time(self._h, None))
            return
        t = np.ascontiguousarray(t_processed, np.float64)
        if len(t) != self.n_slots:
            raise ValueError("t_processed: one entry per slot")
        _check(load().ones_set_processed_time(self._h, t.ctypes.data))

    def export_remaining(self):
        y = np.zeros(max(self.n_slots, 1), np.float64)
        with self._torch.cuda.device(self.device):
            _check(load().ones_export_remaining(self._h, y.ctypes.data))
        return y[:self.n_slots]

    def best(self):
        b = np.zeros(self.n_slots, np.int32)
        g = np.zeros(self.n_slots, np.int32)
        f = C.c_double(0.0)
        with self._torch.cuda.device(self.device):
            _check(load().ones_best(self._h, b.ctypes.data, g.ctypes.data, C.byref(f)))
        return b, g, f.value

    def placement(self):
        """(slot of every GPU, -1 = idle; batch of every GPU's worker): Eq. 1 for the winner."""
        slot = np.zeros(max(self.n_gpus, 1), np.int32)
        batch = np.zeros(max(self.n_gpus, 1), np.int32)
        with self._torch.cuda.device(self.device):
            _check(load().ones_placement(self._h, slot.ctypes.data, batch.ctypes.data))
        return slot[:self.n_gpus], batch[:self.n_gpus]

    def export(self, genes=True):
        g = np.zeros((self.population, self.jp), np.int32) if genes else None
        fit = np.zeros(self.population, np.float64)
        sel = np.zeros(self.population // 4, np.int32)
        t = C.c_int64(0)
        with self._torch.cuda.device(self.device):
            _check(load().ones_export(self._h, g.ctypes.data if genes else None, fit.ctypes.data,
                                      sel.ctypes.data, C.byref(t)))
        return g, fit, sel, t.value

    def profile_enable(self, every: int = 1):
        """Bracket the kernels of every ``every``-th generation with HIP events (0 = off)."""
        _check(load().ones_profile_enable(self._h, int(every)))

    def profile_read(self):
        em, sm = C.c_double(0.0), C.c_double(0.0)
        en, sn = C.c_int64(0), C.c_int64(0)
        _check(load().ones_profile_read(self._h, C.byref(em), C.byref(en), C.byref(sm), C.byref(sn)))
        return {"evolve_ms": em.value, "evolve_launches": en.value,
                "select_ms": sm.value, "select_launches": sn.value}

    def synchronize(self):
        self.stream.synchronize()

    def close(self):
        if getattr(self, "_h", None):
            load().ones_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
