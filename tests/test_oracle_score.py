"""Pins for the oracle's fitness: paper Eq. 3 (sum over running jobs of T_j * c_j) with
T = Y / X (Eq. 5) and the parametric iteration time t(b,g) = a*b/g + c*log2(g) + d."""
import math
import os

import numpy as np
import pytest

from pyref import exact_objective, make_jobs, random_genome, random_jobs

GOLD = os.path.join(os.path.dirname(__file__), "golden", "score_hand_values.txt")


def test_hand_values(ref):
    n = 0
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        a, c, d, y, m, b, want = line.split()
        jobs = make_jobs(1, a=float(a), c=float(c), d=float(d), remaining=float(y),
                         gpu_max_batch=int(m), bmin=1, bmax=4096)
        got = ref.score_genome(64, jobs, [int(b)])
        assert got == pytest.approx(float(want), rel=1e-12)
        n += 1
    assert n == 3


@pytest.mark.parametrize("n", [1, 8, 40, 64, 65, 200, 512])
def test_matches_exact_rational_objective(ref, n):
    rng = np.random.default_rng(n)
    for _ in range(8):
        jobs = random_jobs(rng, n)
        genes = random_genome(rng, jobs)
        got = ref.score_genome(1 << 20, jobs, genes)
        want = exact_objective(jobs, genes)
        assert got == pytest.approx(float(want), rel=1e-12, abs=0.0)


def test_waiting_and_inactive_jobs_add_nothing(ref):
    rng = np.random.default_rng(7)
    jobs = random_jobs(rng, 100, inactive_frac=0.0)
    genes = random_genome(rng, jobs, wait_frac=0.0)
    full = ref.score_genome(10**6, jobs, genes)
    # dropping job k to "waiting" removes exactly its term
    for k in (0, 17, 63, 64, 99):
        g2 = genes.copy(); g2[k] = 0
        one = make_jobs(1, **{f: getattr(jobs, f)[k:k + 1] for f in
                              ("bmin", "bmax", "gpu_max_batch", "a", "c", "d", "remaining")})
        term = ref.score_genome(10**6, one, genes[k:k + 1])
        assert term > 0
        assert ref.score_genome(10**6, jobs, g2) == pytest.approx(full - term, rel=1e-12)
    assert ref.score_genome(10**6, jobs, np.zeros(100, np.int32)) == 0.0
    jobs.active[:] = 0
    assert ref.score_genome(10**6, jobs, genes) == 0.0


def test_monotonicity(ref):
    """Below the per-GPU max a larger batch is strictly better (Y(a + d/b)); above it the
    term does not decrease (Y(a + (c*log2 g + d)/m)); the term grows with Y, a, c, d."""
    rng = np.random.default_rng(11)
    for _ in range(50):
        jobs = random_jobs(rng, 1, inactive_frac=0.0)
        jobs.bmin[:] = 1; jobs.bmax[:] = 1 << 14
        mu = int(jobs.gpu_max_batch[0]).bit_length() - 1
        f = [ref.score_genome(1 << 20, jobs, [1 << g]) for g in range(15)]
        for g in range(mu):
            assert f[g + 1] < f[g]
        for g in range(mu, 14):
            assert f[g + 1] >= f[g]
        for field in ("remaining", "a", "c", "d"):
            j2 = make_jobs(1, **{k: getattr(jobs, k).copy() for k in
                                 ("bmin", "bmax", "gpu_max_batch", "a", "c", "d", "remaining")})
            getattr(j2, field)[0] *= 1.5
            for g in (0, mu, mu + 2):
                lhs, rhs = ref.score_genome(1 << 20, j2, [1 << g]), f[g]
                if field == "c" and g <= mu:
                    assert lhs == rhs           # one GPU: no synchronisation term
                else:
                    assert lhs > rhs


def test_time_vs_utilisation_tension(ref):
    """Section 3.2.1: more GPUs shorten a job's remaining time T_j but do not shrink its
    utilisation T_j * c_j, which is why the objective is not 'give every job all GPUs'."""
    jobs = make_jobs(1, bmin=1, bmax=1 << 14)
    util = [ref.score_genome(1 << 20, jobs, [256 << k]) for k in range(6)]
    time = [u / (1 << k) for k, u in enumerate(util)]
    assert all(time[k + 1] < time[k] for k in range(5))
    assert all(util[k + 1] > util[k] for k in range(5))


def test_close_to_correctly_rounded_sum(ref):
    rng = np.random.default_rng(5)
    jobs = random_jobs(rng, 2048, inactive_frac=0.0)
    genes = random_genome(rng, jobs, wait_frac=0.2)
    terms = []
    for j in range(2048):
        one = make_jobs(1, **{f: getattr(jobs, f)[j:j + 1] for f in
                              ("bmin", "bmax", "gpu_max_batch", "a", "c", "d", "remaining")})
        terms.append(ref.score_genome(1 << 20, one, genes[j:j + 1]))
    assert ref.score_genome(1 << 20, jobs, genes) == pytest.approx(math.fsum(terms), rel=1e-13)
