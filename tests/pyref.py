"""Independent, slow Python checks used to pin the C oracle: a big-integer Philox, an exact
rational evaluation of the cluster objective, a batch-size-domain capacity repair written
sequentially, and the invariant checker.  Nothing here is shared with oracle/ or the GPU
library; everything works on global batch sizes B (not exponents) and uses ceil-division."""
from __future__ import annotations

from fractions import Fraction
from types import SimpleNamespace

import numpy as np

M32 = (1 << 32) - 1


def philox4x32_10(ctr, key):
    """Philox4x32-10 after Salmon et al. (SC'11), with Python integers."""
    x = [int(v) for v in ctr]
    k = [int(v) for v in key]
    for _ in range(10):
        p0 = 0xD2511F53 * x[0]
        p1 = 0xCD9E8D57 * x[2]
        x = [(p1 >> 32) ^ x[1] ^ k[0], p1 & M32, (p0 >> 32) ^ x[3] ^ k[1], p0 & M32]
        k = [(k[0] + 0x9E3779B9) & M32, (k[1] + 0xBB67AE85) & M32]
    return x


def make_jobs(n, **kw):
    """Job table with defaults: active, window [32,1024], m=256, a=1e-3, c=0.02, d=0.01, Y=1e6."""
    d = dict(job_id=np.arange(1, n + 1, dtype=np.int64), active=np.ones(n, np.uint8),
             bmin=np.full(n, 32, np.int32), bmax=np.full(n, 1024, np.int32),
             gpu_max_batch=np.full(n, 256, np.int32), a=np.full(n, 1e-3), c=np.full(n, 0.02),
             d=np.full(n, 0.01), remaining=np.full(n, 1e6))
    for k, v in kw.items():
        d[k] = np.asarray(v, dtype=d[k].dtype) if np.ndim(v) else np.full(n, v, d[k].dtype)
    return SimpleNamespace(**d)


def random_jobs(rng, n, inactive_frac=0.1):
    lo = rng.integers(4, 13, n)
    hi = np.array([rng.integers(l, 13) for l in lo]) if n else np.zeros(0, np.int64)
    m = rng.choice(np.array([64, 128, 256, 512]), n)
    return make_jobs(n, active=(rng.random(n) >= inactive_frac).astype(np.uint8),
                     bmin=1 << lo, bmax=1 << hi, gpu_max_batch=m,
                     a=rng.lognormal(-7, 0.5, n), c=rng.uniform(0.01, 0.05, n),
                     d=rng.uniform(0.005, 0.02, n), remaining=rng.uniform(1e5, 1e7, n))


def random_genome(rng, jobs, wait_frac=0.3, wild=False):
    n = len(jobs.bmin)
    g = np.zeros(n, np.int32)
    for j in range(n):
        if rng.random() < wait_frac:
            continue
        if wild:                      # anywhere in [1, 2^14], also outside the window
            g[j] = 1 << rng.integers(0, 15)
        else:
            lo, hi = int(jobs.bmin[j]).bit_length() - 1, int(jobs.bmax[j]).bit_length() - 1
            g[j] = 1 << rng.integers(lo, hi + 1)
    return g


def gpus(b, m):
    return 0 if b == 0 else -(-int(b) // int(m))


def visiting_order(n, r):
    """Jobs in the order the repair visits them: column-major over 64 columns, rotated by r."""
    jp = 64 * max(1, -(-n // 64))
    rows = jp // 64
    return sorted(range(n), key=lambda j: (((j % 64) * rows + j // 64) - r) % jp)


def start_batch(jobs, j):
    """Batch a waiting job resumes with: the per-GPU max, pulled inside the window."""
    return max(int(jobs.bmin[j]), min(int(jobs.gpu_max_batch[j]), int(jobs.bmax[j])))


def proposal(jobs, j, b):
    """(new batch, extra GPUs) of the single step job j may ask for, or None."""
    if not jobs.active[j]:
        return None
    m = int(jobs.gpu_max_batch[j])
    if b == 0:
        nb = start_batch(jobs, j)
        return nb, gpus(nb, m)
    if b < int(jobs.bmax[j]):
        return 2 * b, gpus(2 * b, m) - gpus(b, m)
    return None


def repair(G, jobs, genes, r):
    """Sequential statement of the repair in the batch-size domain."""
    n = len(genes)
    B = [int(v) for v in genes]
    order = visiting_order(n, r)
    for j in range(n):
        if not jobs.active[j]:
            B[j] = 0
        elif B[j]:
            B[j] = min(max(B[j], int(jobs.bmin[j])), int(jobs.bmax[j]))
            B[j] = max(B[j], min(int(jobs.gpu_max_batch[j]), int(jobs.bmax[j])))
    total = 0
    for j in order:                               # admission: keep the longest prefix that fits
        total += gpus(B[j], jobs.gpu_max_batch[j])
        if total > G:
            B[j] = 0
    rounds = 0
    while True:
        idle = G - sum(gpus(B[j], jobs.gpu_max_batch[j]) for j in range(n))
        asks = []
        for j in order:
            pr = proposal(jobs, j, B[j])
            if pr is not None and pr[1] <= idle:
                asks.append((j, pr))
        if not asks:
            break
        rounds += 1
        spent = 0
        for j, (nb, cost) in asks:                # first come first served, no skipping
            spent += cost
            if spent > idle:
                break
            B[j] = nb
    return np.array(B, np.int32), rounds


def repair_arrivals(G, jobs, genes, r, arrived, t_processed=None):
    """The repair when jobs arrived (Section 3.2.2, refresh (3)), stated sequentially: the
    arrived jobs, in visiting order, each take their starting batch while the cluster has room;
    the others keep their GPUs in visiting order (or, with t_processed, least executed time
    first) while what is left has room; then the usual fill."""
    n = len(genes)
    B = [int(v) for v in genes]
    order = visiting_order(n, r)
    m = jobs.gpu_max_batch
    for j in range(n):
        if not jobs.active[j] or arrived[j]:
            B[j] = 0
        elif B[j]:
            B[j] = min(max(B[j], int(jobs.bmin[j])), int(jobs.bmax[j]))
            B[j] = max(B[j], min(int(m[j]), int(jobs.bmax[j])))
    asked = room = 0
    for j in order:
        if arrived[j] and jobs.active[j]:
            asked += gpus(start_batch(jobs, j), m[j])
            if asked <= G:
                B[j] = start_batch(jobs, j)
                room = asked
    others = [j for j in order if not arrived[j]]
    if t_processed is not None:
        others = sorted((j for j in range(n) if not arrived[j]), key=lambda j: (t_processed[j], j))
    total = 0
    for j in others:
        total += gpus(B[j], m[j])
        if total > G - room:
            B[j] = 0
    filled, rounds = repair(G, jobs, B, r)      # clamp, lift and admission change nothing any more
    return filled, rounds


def check_invariants(G, jobs, genes):
    """I1 window / inactive, I2 capacity (Eq. 4), I3 maximality.  Returns idle GPUs."""
    n = len(genes)
    used = 0
    for j in range(n):
        b = int(genes[j])
        if not jobs.active[j]:
            assert b == 0, f"inactive slot {j} runs"
            continue
        if b:
            assert b & (b - 1) == 0 and jobs.bmin[j] <= b <= jobs.bmax[j], (j, b)
            # a running job never sits below the free (no extra GPU) batch
            assert b >= min(int(jobs.gpu_max_batch[j]), int(jobs.bmax[j])), (j, b)
        used += gpus(b, jobs.gpu_max_batch[j])
    assert used <= G, f"capacity exceeded: {used} > {G}"
    idle = G - used
    for j in range(n):
        pr = proposal(jobs, j, int(genes[j]))
        assert pr is None or pr[1] > idle, f"job {j} could still take {pr} with {idle} idle"
    return idle


def exact_objective(jobs, genes):
    """Sum over running jobs of T_j * c_j in exact rational arithmetic, following the chain
    t = a*B/g + c*log2(g) + d, X = B/t, T = Y/X literally (g = ceil(B/m))."""
    total = Fraction(0)
    for j, b in enumerate(genes):
        b = int(b)
        if b == 0 or not jobs.active[j]:
            continue
        g = gpus(b, jobs.gpu_max_batch[j])
        log2g = g.bit_length() - 1
        assert 1 << log2g == g
        t = Fraction(float(jobs.a[j])) * b / g + Fraction(float(jobs.c[j])) * log2g + Fraction(float(jobs.d[j]))
        X = Fraction(b) / t
        T = Fraction(float(jobs.remaining[j])) / X
        total += T * g
    return total


# ---- probability sampling (Alg. 1, Eq. 7): second implementation with Python floats ----
import math as _math
import struct as _struct

LN2_HEAD = 0.6931471803691238          # ln 2 rounded to 32 significant bits
LN2_TAIL = 1.9082149292705877e-10      # ln 2 - LN2_HEAD


def series_log(x):
    """ln x = e ln 2 + 2 artanh((m-1)/(m+1)), series cut after the s^23 term."""
    bits = _struct.unpack("<Q", _struct.pack("<d", x))[0]
    e = ((bits >> 52) & 0x7FF) - 1023
    m = _struct.unpack("<d", _struct.pack("<Q", (bits & ((1 << 52) - 1)) | (1023 << 52)))[0]
    if m > 1.4142135623730951:
        m, e = m * 0.5, e + 1
    f = m - 1.0
    s = f / (2.0 + f)
    z = s * s
    p = 1.0 / 23.0
    for k in range(21, 2, -2):
        p = p * z + 1.0 / k
    s2 = 2.0 * s
    lm = s2 + s2 * (z * p)
    return e * LN2_HEAD + (e * LN2_TAIL + lm)


def gamma_draw(seed, j, t, which, shape):
    """Marsaglia-Tsang with a polar normal; candidate n reads Philox counter (n, j, t, which)."""
    key = (seed & M32, seed >> 32)
    d = shape - 1.0 / 3.0
    c = 1.0 / _math.sqrt(9.0 * d)
    for n in range(64):
        w = philox4x32_10((n, j, t, which), key)
        u1 = (w[0] + 0.5) * 2.0 ** -31 - 1.0
        u2 = (w[1] + 0.5) * 2.0 ** -31 - 1.0
        s = u1 * u1 + u2 * u2
        if s >= 1.0:
            continue
        x = u1 * _math.sqrt((-2.0 * series_log(s)) / s)
        t1 = 1.0 + c * x
        if t1 <= 0.0:
            continue
        v = (t1 * t1) * t1
        u = (((w[2] << 20) | (w[3] >> 12)) + 0.5) * 2.0 ** -52
        if series_log(u) < ((0.5 * (x * x) + d) - d * v) + d * series_log(v):
            return d * v, n + 1
    return d, 64


def sampled_remaining(seed, j, t, alpha, beta, processed, cap=1e100):
    ga, _ = gamma_draw(seed, j, t, 1, alpha)
    gb, _ = gamma_draw(seed, j, t, 2, beta)
    rho = ga / (ga + gb)
    ratio = min(1.0 / rho - 1.0, cap)
    return min(processed * ratio, cap), rho


def gpu_crossover(seed, p0, t, G, c_a, c_b):
    """Crossover that scans the GPUs (Section 3.2.2 on the encoding of Eq. 1), by intervals:
    job j of a parent holds the GPUs [start_j, start_j + c_j) below G.  Returns the GPU counts
    the two children inherit per job."""
    key = (seed & M32, seed >> 32)
    coin = []
    for block in range(-(-G // 128)):
        w = philox4x32_10((block, p0, t, 3), key)
        coin += [(w[b // 32] >> (b % 32)) & 1 for b in range(128)]
    coin = coin[:G]
    n1, n2 = [0] * len(c_a), [0] * len(c_a)
    for counts, heads_to in ((c_a, n1), (c_b, n2)):
        tails_to = n2 if heads_to is n1 else n1
        start = 0
        for j, c in enumerate(counts):
            mine = coin[min(start, G):min(start + int(c), G)]
            heads_to[j] += sum(mine)
            tails_to[j] += len(mine) - sum(mine)
            start += int(c)
    return n1, n2
