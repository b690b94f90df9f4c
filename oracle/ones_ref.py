"""ctypes wrapper around the CPU oracle (oracle/ones_ref.c).  Test infrastructure only:
imported by tests/, the smoke check and the benchmark's CPU-baseline leg, never by the
GPU library or its Python binding."""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libones_ref.so")
_SRC = os.path.join(_HERE, "ones_ref.c")
CFLAGS = ["-O2", "-ffp-contract=off", "-fopenmp", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc; returns the path of the shared object."""
    stale = (not os.path.exists(_SO)) or any(
        os.path.getmtime(os.path.join(_HERE, f)) > os.path.getmtime(_SO)
        for f in ("ones_ref.c", "ones_ref.h"))
    if force or stale:
        subprocess.check_call(["gcc", *CFLAGS, _SRC, "-o", _SO, "-lm"])
    return _SO


class _Config(C.Structure):
    _fields_ = [("n_gpus", C.c_int32), ("n_slots", C.c_int32), ("population", C.c_int32),
                ("seed", C.c_uint64), ("mutation_rate", C.c_double), ("crossover_rate", C.c_double)]


class _Jobs(C.Structure):
    _fields_ = [("job_id", C.c_void_p), ("active", C.c_void_p), ("bmin", C.c_void_p),
                ("bmax", C.c_void_p), ("gpu_max_batch", C.c_void_p), ("a", C.c_void_p),
                ("c", C.c_void_p), ("d", C.c_void_p), ("remaining", C.c_void_p)]


_DTYPES = {"job_id": np.int64, "active": np.uint8, "bmin": np.int32, "bmax": np.int32,
           "gpu_max_batch": np.int32, "a": np.float64, "c": np.float64, "d": np.float64,
           "remaining": np.float64}

class _LimitInputs(C.Structure):
    _fields_ = [("state", C.c_void_p), ("bmin", C.c_void_p), ("bcap", C.c_void_p), ("gpu_max_batch", C.c_void_p),
                ("last_batch", C.c_void_p), ("finished_epoch", C.c_void_p), ("elapsed", C.c_void_p)]


_LIMIT_DTYPES = {"state": np.uint8, "bmin": np.int32, "bcap": np.int32, "gpu_max_batch": np.int32,
                 "last_batch": np.int32, "finished_epoch": np.uint8, "elapsed": np.float64}

_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        L.ones_ref_init.argtypes = [C.POINTER(C.c_void_p), C.POINTER(_Config), C.POINTER(_Jobs)]
        L.ones_ref_set_jobs.argtypes = [C.c_void_p, C.POINTER(_Jobs)]
        L.ones_ref_generation.argtypes = [C.c_void_p, C.c_int32]
        L.ones_ref_best.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(C.c_double)]
        L.ones_ref_export.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(C.c_int64)]
        L.ones_ref_destroy.argtypes = [C.c_void_p]
        L.ones_ref_destroy.restype = None
        L.ones_ref_padded_jobs.argtypes = [C.c_int32]
        L.ones_ref_set_threads.argtypes = [C.c_int]
        L.ones_ref_set_threads.restype = None
        L.ones_ref_philox4x32_10.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        L.ones_ref_philox4x32_10.restype = None
        L.ones_ref_repair_genome.argtypes = [C.POINTER(_Config), C.POINTER(_Jobs), C.c_void_p,
                                             C.c_uint32, C.POINTER(C.c_int32)]
        L.ones_ref_score_genome.argtypes = [C.POINTER(_Config), C.POINTER(_Jobs), C.c_void_p,
                                            C.POINTER(C.c_double)]
        L.ones_ref_select.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
        L.ones_ref_select.restype = None
        L.ones_ref_compose_slot.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.POINTER(C.c_uint32),
                                            C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        L.ones_ref_initial_genome.argtypes = [C.POINTER(_Config), C.POINTER(_Jobs), C.c_int32,
                                              C.c_void_p, C.POINTER(C.c_uint32)]
        L.ones_ref_update_limits.argtypes = [C.c_int32, C.POINTER(_LimitInputs), C.c_double, C.c_void_p]
        L.ones_ref_set_new_jobs_first.argtypes = [C.c_void_p, C.c_int32]
        L.ones_ref_set_processed_time.argtypes = [C.c_void_p, C.c_void_p]
        L.ones_ref_set_crossover.argtypes = [C.c_void_p, C.c_int32]
        L.ones_ref_gpu_crossover.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_int32, C.c_int32,
                                             C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.ones_ref_gpu_crossover.restype = None
        L.ones_ref_repair_arrivals.argtypes = [C.POINTER(_Config), C.POINTER(_Jobs), C.c_void_p, C.c_uint32,
                                               C.c_void_p, C.c_void_p, C.POINTER(C.c_int32)]
        L.ones_ref_placement.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        L.ones_ref_set_progress.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.ones_ref_export_remaining.argtypes = [C.c_void_p, C.c_void_p]
        L.ones_ref_log.argtypes = [C.c_double]
        L.ones_ref_log.restype = C.c_double
        L.ones_ref_gamma_draw.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_double,
                                          C.POINTER(C.c_int)]
        L.ones_ref_gamma_draw.restype = C.c_double
        L.ones_ref_sampled_remaining.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_double, C.c_double,
                                                 C.c_double, C.POINTER(C.c_double)]
        L.ones_ref_sampled_remaining.restype = C.c_double
        _lib = L
    return _lib


def update_limits(limit, sigma, **arrays):
    """Section 3.3.2: returns the new limits; arrays: state, bmin, bcap, gpu_max_batch, last_batch,
    finished_epoch, elapsed (one entry per slot)."""
    out = np.array(limit, np.int32)
    keep = [np.ascontiguousarray(arrays[k], dtype=dt) for k, dt in _LIMIT_DTYPES.items()]
    if any(a.shape != out.shape for a in keep):
        raise ValueError("one entry per slot in every array")
    inp = _LimitInputs(*[a.ctypes.data for a in keep])
    _check(lib().ones_ref_update_limits(len(out), C.byref(inp), float(sigma), out.ctypes.data))
    return out


def log(x: float) -> float:
    return lib().ones_ref_log(float(x))


def gamma_draw(seed, j, t, which, shape):
    """(value, candidate draws used)"""
    n = C.c_int(0)
    v = lib().ones_ref_gamma_draw(int(seed), int(j), int(t), int(which), float(shape), C.byref(n))
    return v, n.value


def sampled_remaining(seed, j, t, alpha, beta, processed):
    """(Y, rho) of Eq. 7 for slot j in generation t"""
    rho = C.c_double(0.0)
    y = lib().ones_ref_sampled_remaining(int(seed), int(j), int(t), float(alpha), float(beta),
                                         float(processed), C.byref(rho))
    return y, rho.value


class RefError(RuntimeError):
    def __init__(self, code):
        super().__init__(f"oracle returned {code}")
        self.code = code


def _check(rc):
    if rc != 0:
        raise RefError(rc)


def _cfg(n_gpus, n_slots, population, seed, mutation_rate, crossover_rate):
    return _Config(int(n_gpus), int(n_slots), int(population), int(seed) & (2**64 - 1),
                   float(mutation_rate), float(crossover_rate))


def _jobs(jobs):
    """jobs: any object with the nine arrays as attributes.  Returns (struct, keepalive)."""
    keep = [np.ascontiguousarray(getattr(jobs, k), dtype=dt) for k, dt in _DTYPES.items()]
    return _Jobs(*[a.ctypes.data for a in keep]), keep


def set_threads(n: int):
    lib().ones_ref_set_threads(int(n))


def padded_jobs(n_slots: int) -> int:
    return lib().ones_ref_padded_jobs(int(n_slots))


def philox(ctr, key):
    c = np.asarray(ctr, np.uint32); k = np.asarray(key, np.uint32); o = np.zeros(4, np.uint32)
    lib().ones_ref_philox4x32_10(c.ctypes.data, k.ctypes.data, o.ctypes.data)
    return o


def repair_genome(n_gpus, jobs, genes, r, population=4):
    cfg = _cfg(n_gpus, len(genes), population, 0, 0.0, 0.0)
    js, keep = _jobs(jobs)
    g = np.ascontiguousarray(genes, np.int32).copy()
    rounds = C.c_int32(0)
    _check(lib().ones_ref_repair_genome(C.byref(cfg), C.byref(js), g.ctypes.data, int(r), C.byref(rounds)))
    return g, rounds.value


def repair_arrivals(n_gpus, jobs, genes, r, arrived, t_processed=None, population=4):
    """Repair with the jobs marked in arrived served first; t_processed orders the others."""
    cfg = _cfg(n_gpus, len(genes), population, 0, 0.0, 0.0)
    js, keep = _jobs(jobs)
    g = np.ascontiguousarray(genes, np.int32).copy()
    new = np.ascontiguousarray(arrived, np.uint8)
    times = None if t_processed is None else np.ascontiguousarray(t_processed, np.float64)
    if len(new) != len(g) or (times is not None and len(times) != len(g)):
        raise ValueError("arrived, t_processed: one entry per slot")
    rounds = C.c_int32(0)
    _check(lib().ones_ref_repair_arrivals(C.byref(cfg), C.byref(js), g.ctypes.data, int(r), new.ctypes.data,
                                          None if times is None else times.ctypes.data, C.byref(rounds)))
    return g, rounds.value


def gpu_crossover(seed, p0, t, n_gpus, c_a, c_b):
    """GPUs per job that each child inherits when the crossover scans the GPUs."""
    a = np.ascontiguousarray(c_a, np.int32)
    b = np.ascontiguousarray(c_b, np.int32)
    if len(a) != len(b):
        raise ValueError("one GPU count per job in both parents")
    n1, n2 = np.zeros(len(a), np.int32), np.zeros(len(a), np.int32)
    lib().ones_ref_gpu_crossover(int(seed), int(p0), int(t), int(n_gpus), len(a), a.ctypes.data, b.ctypes.data,
                                 n1.ctypes.data, n2.ctypes.data)
    return n1, n2


def score_genome(n_gpus, jobs, genes):
    cfg = _cfg(n_gpus, len(genes), 4, 0, 0.0, 0.0)
    js, keep = _jobs(jobs)
    g = np.ascontiguousarray(genes, np.int32)
    f = C.c_double(0.0)
    _check(lib().ones_ref_score_genome(C.byref(cfg), C.byref(js), g.ctypes.data, C.byref(f)))
    return f.value


def initial_genome(cluster, jobs, p):
    cfg = _cfg(cluster.n_gpus, cluster.n_slots, cluster.population, cluster.seed,
               cluster.mutation_rate, cluster.crossover_rate)
    js, keep = _jobs(jobs)
    g = np.zeros(int(cluster.n_slots), np.int32)
    r = C.c_uint32(0)
    _check(lib().ones_ref_initial_genome(C.byref(cfg), C.byref(js), int(p), g.ctypes.data, C.byref(r)))
    return g, r.value


def select(fit):
    f = np.ascontiguousarray(fit, np.float64)
    sel = np.zeros(len(f) // 4, np.int32)
    lib().ones_ref_select(f.ctypes.data, len(f), sel.ctypes.data)
    return sel


class RefSearch:
    """Same call sequence as the GPU binding's ``Search`` (init / set_jobs / generation /
    best / export), on host memory."""

    def __init__(self, cluster, jobs):
        self.n_slots = int(cluster.n_slots)
        self.n_gpus = int(cluster.n_gpus)
        self.population = int(cluster.population)
        self.jp = padded_jobs(self.n_slots)
        cfg = _cfg(cluster.n_gpus, cluster.n_slots, cluster.population, cluster.seed,
                   cluster.mutation_rate, cluster.crossover_rate)
        js, keep = _jobs(jobs)
        self._h = C.c_void_p()
        _check(lib().ones_ref_init(C.byref(self._h), C.byref(cfg), C.byref(js)))

    def set_jobs(self, jobs):
        js, keep = _jobs(jobs)
        _check(lib().ones_ref_set_jobs(self._h, C.byref(js)))

    def generation(self, n=1):
        _check(lib().ones_ref_generation(self._h, int(n)))

    def set_progress(self, alpha=None, beta=None, processed=None):
        """Alg. 1: per-slot Be(alpha, beta) and processed samples; all None switches it off."""
        if alpha is None and beta is None and processed is None:
            _check(lib().ones_ref_set_progress(self._h, None, None, None))
            return
        arrs = [np.ascontiguousarray(x, np.float64) for x in (alpha, beta, processed)]
        if any(a.shape != (self.n_slots,) for a in arrs):
            raise ValueError("alpha, beta, processed: one entry per slot")
        _check(lib().ones_ref_set_progress(self._h, *[a.ctypes.data for a in arrs]))

    def set_new_jobs_first(self, on=True):
        _check(lib().ones_ref_set_new_jobs_first(self._h, int(bool(on))))

    def set_crossover(self, per_gpu=False):
        _check(lib().ones_ref_set_crossover(self._h, int(bool(per_gpu))))

    def set_processed_time(self, t_processed=None):
        if t_processed is None:
            _check(lib().ones_ref_set_processed_time(self._h, None))
            return
        t = np.ascontiguousarray(t_processed, np.float64)
        if len(t) != self.n_slots:
            raise ValueError("t_processed: one entry per slot")
        _check(lib().ones_ref_set_processed_time(self._h, t.ctypes.data))

    def export_remaining(self):
        y = np.zeros(self.n_slots, np.float64)
        if self.n_slots:
            _check(lib().ones_ref_export_remaining(self._h, y.ctypes.data))
        return y

    def best(self):
        b = np.zeros(self.n_slots, np.int32); g = np.zeros(self.n_slots, np.int32)
        f = C.c_double(0.0)
        _check(lib().ones_ref_best(self._h, b.ctypes.data, g.ctypes.data, C.byref(f)))
        return b, g, f.value

    def placement(self):
        """(slot of every GPU, -1 = idle; batch of every GPU's worker)"""
        slot = np.zeros(max(self.n_gpus, 1), np.int32); batch = np.zeros(max(self.n_gpus, 1), np.int32)
        _check(lib().ones_ref_placement(self._h, slot.ctypes.data, batch.ctypes.data))
        return slot[:self.n_gpus], batch[:self.n_gpus]

    def export(self, genes=True):
        g = np.zeros((self.population, self.jp), np.int32) if genes else None
        fit = np.zeros(self.population, np.float64)
        sel = np.zeros(self.population // 4, np.int32)
        t = C.c_int64(0)
        _check(lib().ones_ref_export(self._h, g.ctypes.data if genes else None, fit.ctypes.data, sel.ctypes.data,
                                     C.byref(t)))
        return g, fit, sel, t.value

    def compose_slot(self, p):
        g = np.zeros(self.jp, np.int32)
        r = C.c_uint32(0); pa = C.c_int32(0); pb = C.c_int32(0)
        _check(lib().ones_ref_compose_slot(self._h, int(p), g.ctypes.data, C.byref(r), C.byref(pa), C.byref(pb)))
        return g, r.value, pa.value, pb.value

    def close(self):
        if self._h:
            lib().ones_ref_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
