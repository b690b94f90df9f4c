"""Seeded synthetic clusters for the ONES evolutionary search (paper Section 4.1 describes a
64-GPU testbed and a trace of 50 PyTorch job types; neither the trace nor the jobs exist
here, so these generators stand in for them).

This module only draws inputs: job tables (iteration-time parameters, batch-size windows,
remaining work) and the search hyper-parameters.  It contains none of the search's
arithmetic and is imported by the HIP binding's callers and by the CPU oracle's callers
alike, so that both sides provably see the same bytes (``sha256`` below).

Per-job draw order (fixed): a, c, d, remaining, window, per-GPU max batch.
"""
from __future__ import annotations

import hashlib
from dataclasses import dataclass, field

import numpy as np

# Search hyper-parameters shared by every configuration (Section 3.2.2 names the mutation
# rate theta; the pool is K elites + 2K crossover children + K mutants, so survivors = 25 %).
MUTATION_RATE = 0.1
CROSSOVER_RATE = 0.5


@dataclass
class Jobs:
    """Structure-of-arrays job table, one entry per slot (length ``n_slots``)."""
    job_id: np.ndarray         # int64   identity of the job held by the slot
    active: np.ndarray         # uint8   0 = empty slot
    bmin: np.ndarray           # int32   smallest allowed global batch (power of two)
    bmax: np.ndarray           # int32   batch-size limit R_j (power of two)
    gpu_max_batch: np.ndarray  # int32   per-GPU max batch (power of two)
    a: np.ndarray              # float64 s/sample   t(b,g) = a*b/g + c*log2(g) + d
    c: np.ndarray              # float64 s
    d: np.ndarray              # float64 s
    remaining: np.ndarray      # float64 remaining samples Y_j

    ARRAYS = ("job_id", "active", "bmin", "bmax", "gpu_max_batch", "a", "c", "d", "remaining")

    @property
    def n_slots(self) -> int:
        return int(self.job_id.shape[0])

    def copy(self) -> "Jobs":
        return Jobs(*(getattr(self, k).copy() for k in self.ARRAYS))

    def sha256(self) -> str:
        h = hashlib.sha256()
        for k in self.ARRAYS:
            h.update(np.ascontiguousarray(getattr(self, k)).tobytes())
        return h.hexdigest()


@dataclass
class Cluster:
    name: str
    n_gpus: int
    n_slots: int
    population: int
    generations: int
    seed: int
    mutation_rate: float = MUTATION_RATE
    crossover_rate: float = CROSSOVER_RATE
    epochs: int = 1            # > 1 only for the online sequence
    extra: dict = field(default_factory=dict)


def empty_jobs(n: int) -> Jobs:
    return Jobs(job_id=np.zeros(n, np.int64), active=np.zeros(n, np.uint8),
                bmin=np.ones(n, np.int32), bmax=np.ones(n, np.int32),
                gpu_max_batch=np.ones(n, np.int32), a=np.zeros(n), c=np.zeros(n),
                d=np.zeros(n), remaining=np.zeros(n))


def _draw_common(rng: np.random.Generator, n: int):
    a = rng.lognormal(-7.0, 0.5, n)          # exp(N(-7, 0.5)) s/sample
    c = rng.uniform(0.01, 0.05, n)
    d = rng.uniform(0.005, 0.02, n)
    return a, c, d


def _fixed_window_jobs(rng, n, lo_exp, hi_exp):
    a, c, d = _draw_common(rng, n)
    y = rng.uniform(1e5, 1e7, n)
    return a, c, d, y, np.full(n, 1 << lo_exp, np.int32), np.full(n, 1 << hi_exp, np.int32)


def _random_window_jobs(rng, n):
    """Parameters of the paper-scale jobs: random power-of-two windows inside [16, 4096]."""
    a, c, d = _draw_common(rng, n)
    y = rng.uniform(1e5, 1e7, n)
    lo = rng.integers(4, 13, n)
    hi = np.array([rng.integers(l, 13) for l in lo], dtype=np.int64) if n else np.zeros(0, np.int64)
    return a, c, d, y, (1 << lo).astype(np.int32), (1 << hi).astype(np.int32)


def _pack(n, a, c, d, y, bmin, bmax, m) -> Jobs:
    return Jobs(job_id=np.arange(1, n + 1, dtype=np.int64), active=np.ones(n, np.uint8),
                bmin=bmin, bmax=bmax, gpu_max_batch=np.asarray(m, np.int32),
                a=a, c=c, d=d, remaining=y)


def tiny(seed: int = 0):
    """16 GPUs, 8 jobs, pool 64, 10 generations; window [32,1024], 256 samples per GPU."""
    n = 8
    rng = np.random.default_rng(seed)
    a, c, d, y, bmin, bmax = _fixed_window_jobs(rng, n, 5, 10)
    return (Cluster("tiny", 16, n, 64, 10, seed),
            _pack(n, a, c, d, y, bmin, bmax, np.full(n, 256)))


def paper_scale(seed: int = 1):
    """64 GPUs (the paper's testbed size), 40 running jobs, pool 1024, 100 generations."""
    n = 40
    rng = np.random.default_rng(seed)
    a, c, d, y, bmin, bmax = _random_window_jobs(rng, n)
    return (Cluster("paper_scale", 64, n, 1024, 100, seed),
            _pack(n, a, c, d, y, bmin, bmax, np.full(n, 256)))


def large(seed: int = 3):
    """1024 GPUs, 512 jobs, pool 16384, 50 generations; per-GPU max batch in {64..512}."""
    n = 512
    rng = np.random.default_rng(seed)
    a, c, d, y, bmin, bmax = _fixed_window_jobs(rng, n, 5, 10)
    m = rng.choice(np.array([64, 128, 256, 512]), n)
    return (Cluster("large", 1024, n, 16384, 50, seed),
            _pack(n, a, c, d, y, bmin, bmax, m))


def stress(seed: int = 4, population: int = 65536, n_jobs: int = 2048, n_gpus: int = 4096):
    """4096 GPUs, 2048 jobs, pool 65536, 20 generations; Pareto(1.2, 1e5) remaining work,
    10 % of the jobs pinned at the minimum batch (window collapsed to one value)."""
    n = n_jobs
    rng = np.random.default_rng(seed)
    a, c, d = _draw_common(rng, n)
    u = 1.0 - rng.random(n)                    # (0, 1]
    y = 1e5 * u ** (-1.0 / 1.2)
    bmin = np.full(n, 32, np.int32)
    bmax = np.full(n, 1024, np.int32)
    pinned = rng.random(n) < 0.1
    bmax[pinned] = 32
    return (Cluster("stress", n_gpus, n, population, 20, seed,
                    extra={"pinned": int(pinned.sum())}),
            _pack(n, a, c, d, y, bmin, bmax, np.full(n, 256)))


def progress(n_slots: int, seed: int = 0):
    """Per-slot inputs of the probability sampling (Alg. 1): the samples a job has processed,
    ~ U(1e4, 1e7); alpha = processed / epoch size with the epoch size log-uniform in
    [1e4, 1e6], and beta (epochs still to come) ~ U(1, 60), both thresholded at 1 as in
    Section 3.2.1.  Returns (alpha, beta, processed)."""
    rng = np.random.default_rng([seed, 0xBE7A])
    processed = rng.uniform(1e4, 1e7, n_slots)
    epoch = np.exp(rng.uniform(np.log(1e4), np.log(1e6), n_slots))
    alpha = np.maximum(processed / epoch, 1.0)
    beta = np.maximum(rng.uniform(1.0, 60.0, n_slots), 1.0)
    return alpha, beta, processed


class OnlineSequence:
    """Online arrivals for the 64-GPU cluster: 64 slots, at most 60 busy, one scheduling
    epoch = 60 s, arrivals per epoch ~ Poisson(0.5), deferred first-in-first-out while 60
    slots are busy; a new job takes the lowest free slot with paper-scale parameters.

    ``advance(batch)`` applies the deployed schedule for one epoch: a running job with
    global batch B on ceil(B/m) GPUs processes 60*B/t samples, t = a*B/g + c*log2(g) + d;
    a job whose remaining work reaches zero frees its slot.  This is the simulated
    cluster, not the scheduler: the same code feeds either implementation.

    With ``limits`` (a function with the signature of ``update_limits``: the library's or the
    oracle's) the batch-size limits follow the policies of Section 3.3.2 instead of staying at
    the job's own maximum: a job starts on one GPU's batch, doubles its limit after every
    epoch it ran (penalised by its executed time, sigma = the arrival rate), is capped at its
    last batch when it gets pre-empted and halved for every further epoch it waits.

    ``progress()`` gives the inputs of the probability sampling (Alg. 1) the way a progress
    predictor would, without its training logs: a job has processed the fraction rho of its
    work; the predictor's Be(alpha, beta) is centred there and gets sharper with every epoch it
    has observed: alpha = 1 + k rho, beta = 1 + k (1 - rho), k = 8 (1 + epochs run).
    """
    EPOCH_S = 60.0
    MAX_BUSY = 60

    def __init__(self, seed: int = 2, n_slots: int = 64, epochs: int = 200, limits=None):
        self.cluster = Cluster("online", 64, n_slots, 2048, 20, seed, epochs=epochs)
        self.rng = np.random.default_rng(seed)
        self.jobs = empty_jobs(n_slots)
        self.jobs.gpu_max_batch[:] = 256
        self.limits = limits
        self.cap = np.zeros(n_slots, np.int32)          # the job's own largest batch
        self.elapsed = np.zeros(n_slots)                # executed seconds
        self.prev_batch = np.zeros(n_slots, np.int32)   # batch in the epoch before
        self.arrived = np.zeros(n_slots, np.uint8)      # arrived since the last limit update
        self.total = np.zeros(n_slots)                  # samples the job had to process when it arrived
        self.epochs_run = np.zeros(n_slots, np.int64)
        self.next_id = 1
        self.backlog = 0
        self.completed = 0
        # a few jobs are present at the first epoch so that the search never starts empty
        self._arrive(int(self.rng.poisson(0.5)) + 4)

    def _arrive(self, n_new: int):
        self.backlog += n_new
        while self.backlog > 0 and int(self.jobs.active.sum()) < self.MAX_BUSY:
            free = np.flatnonzero(self.jobs.active == 0)
            s = int(free[0])
            a, c, d, y, bmin, bmax = _random_window_jobs(self.rng, 1)
            j = self.jobs
            j.job_id[s], j.active[s] = self.next_id, 1
            j.a[s], j.c[s], j.d[s], j.remaining[s] = a[0], c[0], d[0], y[0]
            j.bmin[s], j.bmax[s], j.gpu_max_batch[s] = bmin[0], bmax[0], 256
            self.cap[s], self.elapsed[s], self.prev_batch[s], self.arrived[s] = bmax[0], 0.0, 0, 1
            self.total[s], self.epochs_run[s] = y[0], 0
            self.next_id += 1
            self.backlog -= 1
        if self.limits is not None:
            self._update_limits(np.zeros(self.jobs.n_slots, np.int32))

    def advance(self, batch: np.ndarray):
        """Run the cluster for one epoch under the schedule ``batch`` (global batch per
        slot, 0 = waiting), then admit this epoch's arrivals."""
        j = self.jobs
        for s in range(j.n_slots):
            b = int(batch[s])
            if not j.active[s] or b == 0:
                continue
            m = int(j.gpu_max_batch[s])
            g = max(1, -(-b // m))
            t = j.a[s] * b / g + j.c[s] * np.log2(g) + j.d[s]
            j.remaining[s] -= self.EPOCH_S * b / t
            if j.remaining[s] <= 0.0:
                j.active[s] = 0
                j.remaining[s] = 0.0
                self.completed += 1
            self.elapsed[s] += self.EPOCH_S
            self.epochs_run[s] += 1
        self._arrive(int(self.rng.poisson(0.5)))
        if self.limits is not None:
            self._update_limits(np.asarray(batch, np.int32))

    def progress(self):
        """(alpha, beta, processed) per slot for ``set_progress``; empty slots get Be(1, 1) and 0."""
        j = self.jobs
        live = j.active != 0
        processed = np.where(live, np.maximum(self.total - j.remaining, 0.0), 0.0)
        rho = np.where(live & (self.total > 0), processed / np.maximum(self.total, 1e-300), 0.0)
        k = 8.0 * (1.0 + self.epochs_run)
        alpha = np.where(live, 1.0 + k * rho, 1.0)
        beta = np.where(live, 1.0 + k * (1.0 - rho), 1.0)
        return alpha, beta, processed

    def _update_limits(self, batch):
        """Section 3.3.2: the limits the scheduler sees in the next epoch."""
        j = self.jobs
        ran = (batch > 0) & (j.active != 0)
        state = np.where(j.active == 0, 0, np.where(self.arrived != 0, 1, np.where(ran, 3, 2))).astype(np.uint8)
        just_preempted = (state == 2) & (self.prev_batch > 0)
        new = self.limits(j.bmax, 0.5 / self.EPOCH_S, state=state, bmin=np.maximum(j.bmin, 1),
                          bcap=np.maximum(self.cap, 1), gpu_max_batch=j.gpu_max_batch,
                          last_batch=np.where(just_preempted, self.prev_batch, 0), finished_epoch=ran.astype(np.uint8),
                          elapsed=self.elapsed)
        active = j.active != 0
        j.bmax[active] = new[active]
        self.prev_batch = np.where(ran, batch, 0).astype(np.int32)
        self.arrived[:] = 0


CONFIGS = {"tiny": tiny, "paper_scale": paper_scale, "large": large, "stress": stress}
