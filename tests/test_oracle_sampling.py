"""Pins for the oracle's probability sampling: Alg. 1 draws the progress rho_j of every job
from Be(alpha_j, beta_j) and scores the schedules with Y_j = Y_processed_j (1/rho_j - 1)
(Eq. 7).  The draws are pinned to the distributions' closed forms and distribution functions,
the logarithm to the C library's, and the arithmetic to a Python transcription."""
import math

import numpy as np
import pytest
from scipy import stats

import pyref
from pyref import make_jobs, random_jobs
from paper_2108_03645_amd import workloads

SEED = 0x5EED0123456789AB


def ulps(a, b):
    return abs(a - b) / np.spacing(abs(b)) if b != 0 else abs(a) / 5e-324


# ------------------------------------------------------------------ logarithm ----
def test_log_matches_libm_within_two_ulp(ref):
    rng = np.random.default_rng(1)
    xs = np.concatenate([
        rng.random(20000),                                   # the uniforms it is applied to
        np.exp(rng.uniform(-700, 700, 20000)),               # whole exponent range
        1.0 + rng.uniform(-1e-3, 1e-3, 5000), 1.0 + rng.uniform(-1e-9, 1e-9, 5000),
        math.sqrt(2) * (1.0 + rng.uniform(-1e-12, 1e-12, 2000)),   # where the reduction switches
        2.0 ** rng.integers(-1000, 1000, 2000).astype(np.float64)])
    worst = 0.0
    for x in xs:
        worst = max(worst, ulps(ref.log(float(x)), math.log(float(x))))
    assert worst <= 2.0


def test_log_special_values(ref):
    assert ref.log(1.0) == 0.0
    for k in (-1022, -52, -1, 1, 2, 10, 1023):
        assert ulps(ref.log(2.0 ** k), k * math.log(2.0)) <= 1.0
    assert ref.log(0.5) == -ref.log(2.0)
    assert ref.log(2.0 ** -1022) < ref.log(2.0 ** -1021)


def test_log_is_monotone_near_one(ref):
    xs = 1.0 + np.arange(-2000, 2001) * 2.0 ** -52
    ys = [ref.log(float(x)) for x in xs]
    assert all(b >= a for a, b in zip(ys, ys[1:]))


# ------------------------------------------------------------------ gamma ----
N = 20000


def gamma_sample(ref, shape, t=7, which=1, n=N):
    out = np.empty(n)
    tries = np.empty(n, np.int64)
    for j in range(n):
        out[j], tries[j] = ref.gamma_draw(SEED, j, t, which, shape)
    return out, tries


@pytest.mark.parametrize("shape", [1.0, 1.5, 2.7, 10.0, 100.0, 1e4])
def test_gamma_moments_and_distribution(ref, shape):
    x, tries = gamma_sample(ref, shape)
    assert (x > 0).all()
    # mean = variance = shape
    assert abs(x.mean() - shape) < 5 * math.sqrt(shape / N)
    assert abs(x.var() - shape) < 5 * shape * math.sqrt((2 + 6 / shape) / N)   # sd of the sample variance
    d = stats.kstest(x, stats.gamma(shape).cdf).statistic
    assert d < 1.63 / math.sqrt(N)                                             # 1 % critical value
    # the polar step keeps pi/4 of its points and the acceptance test nearly all of those
    assert 4 / math.pi <= tries.mean() < 1.45
    assert tries.max() < 30


def test_gamma_shape_one_is_exponential(ref):
    x, _ = gamma_sample(ref, 1.0, t=11)
    assert stats.kstest(x, stats.expon.cdf).statistic < 1.63 / math.sqrt(N)
    assert abs(np.mean(x > math.log(2.0)) - 0.5) < 4 * 0.5 / math.sqrt(N)       # median ln 2


def test_gamma_streams_are_distinct_and_repeatable(ref):
    a = ref.gamma_draw(SEED, 5, 9, 1, 3.0)
    assert a == ref.gamma_draw(SEED, 5, 9, 1, 3.0)
    others = {ref.gamma_draw(SEED, 5, 9, 2, 3.0), ref.gamma_draw(SEED, 6, 9, 1, 3.0),
              ref.gamma_draw(SEED, 5, 10, 1, 3.0), ref.gamma_draw(SEED + 1, 5, 9, 1, 3.0),
              ref.gamma_draw(SEED + (1 << 32), 5, 9, 1, 3.0)}
    assert a not in others and len(others) == 5
    # the two gammas of a Beta draw are independent
    x, _ = gamma_sample(ref, 2.0, which=1)
    y, _ = gamma_sample(ref, 2.0, which=2)
    assert abs(np.corrcoef(x, y)[0, 1]) < 4 / math.sqrt(N)


# ------------------------------------------------------------------ Beta, Eq. 7 ----
@pytest.mark.parametrize("alpha,beta", [(1.0, 1.0), (2.0, 5.0), (10.0, 3.0), (50.0, 50.0), (1.0, 7.0), (300.0, 2.0)])
def test_beta_moments_and_distribution(ref, alpha, beta):
    rho = np.array([ref.sampled_remaining(SEED, j, 3, alpha, beta, 1.0)[1] for j in range(N)])
    assert ((rho > 0) & (rho < 1)).all()
    mean = alpha / (alpha + beta)
    var = alpha * beta / ((alpha + beta) ** 2 * (alpha + beta + 1))
    assert abs(rho.mean() - mean) < 5 * math.sqrt(var / N)
    assert abs(rho.var() - var) < 0.08 * var
    assert stats.kstest(rho, stats.beta(alpha, beta).cdf).statistic < 1.63 / math.sqrt(N)


def test_be_1_1_is_uniform(ref):
    rho = np.array([ref.sampled_remaining(SEED, j, 4, 1.0, 1.0, 1.0)[1] for j in range(N)])
    counts = np.histogram(rho, bins=20, range=(0, 1))[0]
    assert stats.chisquare(counts).pvalue > 1e-3


def test_remaining_work_is_eq_7(ref):
    for j, (alpha, beta, proc) in enumerate([(2.0, 3.0, 1e5), (40.0, 1.0, 5e7), (1.0, 1.0, 0.0), (7.5, 2.25, 123.0)]):
        y, rho = ref.sampled_remaining(SEED, j, 2, alpha, beta, proc)
        assert y == pytest.approx(proc * (1 / rho - 1), rel=1e-15)
        assert y >= 0
    # expected remaining work: E[1/rho - 1] = beta / (alpha - 1)
    alpha, beta = 10.0, 3.0
    y = np.array([ref.sampled_remaining(SEED, j, 5, alpha, beta, 2.0)[0] for j in range(N)])
    sd = math.sqrt(beta * (alpha + beta - 1) / ((alpha - 2) * (alpha - 1) ** 2))   # sd of the beta-prime ratio
    assert abs(y.mean() / 2.0 - beta / (alpha - 1)) < 5 * sd / math.sqrt(N)


def test_remaining_work_is_capped(ref):
    y, rho = ref.sampled_remaining(SEED, 0, 1, 1.0, 1e100, 1e100)
    assert 0 < rho < 1e-90 and y == 1e100
    y, _ = ref.sampled_remaining(SEED, 0, 1, 1e100, 1.0, 1e100)
    assert 0 <= y <= 1e100 and math.isfinite(y)
    assert ref.sampled_remaining(SEED, 0, 1, 1.0, 1e100, 0.0)[0] == 0.0


def test_python_transcription_gives_the_same_bits(ref):
    rng = np.random.default_rng(3)
    for x in np.concatenate([rng.random(300), np.exp(rng.uniform(-700, 700, 300))]):
        assert ref.log(float(x)) == pyref.series_log(float(x))
    for i in range(300):
        shape = float(np.exp(rng.uniform(0, 8)))
        j, t, which = int(rng.integers(0, 2048)), int(rng.integers(1, 1 << 31)), int(rng.integers(1, 3))
        assert ref.gamma_draw(SEED, j, t, which, shape) == pyref.gamma_draw(SEED, j, t, which, shape)
    for i in range(200):
        a, b = float(np.exp(rng.uniform(0, 6))), float(np.exp(rng.uniform(0, 6)))
        proc = float(rng.uniform(0, 1e7))
        assert ref.sampled_remaining(SEED, i, 77, a, b, proc) == pyref.sampled_remaining(SEED, i, 77, a, b, proc)


# ------------------------------------------------------------------ inside the search ----
def progress_of(jobs, seed):
    rng = np.random.default_rng(seed)
    n = len(jobs.bmin)
    return rng.uniform(1, 30, n), rng.uniform(1, 30, n), rng.uniform(1e4, 1e7, n)


def jobs_with(jobs, remaining):
    d = {k: np.array(getattr(jobs, k)) for k in ("job_id", "active", "bmin", "bmax", "gpu_max_batch", "a", "c", "d")}
    return make_jobs(len(jobs.bmin), remaining=remaining, **d)


def test_every_generation_scores_the_whole_pool_with_one_fresh_draw(ref):
    cluster, jobs = workloads.paper_scale()
    s = ref.RefSearch(cluster, jobs)
    alpha, beta, proc = progress_of(jobs, 1)
    s.generation(2)
    assert np.array_equal(s.export_remaining(), jobs.remaining)
    s.set_progress(alpha, beta, proc)
    previous = None
    for step in range(3):
        s.generation(1)
        genes, fit, sel, t = s.export()
        y = s.export_remaining()
        want = [ref.sampled_remaining(cluster.seed, j, t, alpha[j], beta[j], proc[j])[0] for j in range(cluster.n_slots)]
        assert np.array_equal(y, want)
        assert previous is None or not np.array_equal(y, previous)
        previous = y
        scored = jobs_with(jobs, y)
        for p in list(range(0, cluster.population, 37)) + list(sel[:5]):      # survivors (slots < K) included
            assert fit[p] == ref.score_genome(cluster.n_gpus, scored, genes[p, :cluster.n_slots])
        order = np.lexsort((np.arange(cluster.population), fit))
        assert np.array_equal(sel, order[:cluster.population // 4])           # Alg. 1: smallest scores win
    # switching off restores the table's remaining work
    s.set_progress()
    assert np.array_equal(s.export_remaining(), jobs.remaining)
    s.generation(1)
    genes, fit, sel, t = s.export()
    assert fit[3] == ref.score_genome(cluster.n_gpus, jobs, genes[3, :cluster.n_slots])


def test_progress_survives_a_job_table_change(ref):
    cluster, jobs = workloads.paper_scale()
    s = ref.RefSearch(cluster, jobs)
    alpha, beta, proc = progress_of(jobs, 2)
    s.set_progress(alpha, beta, proc)
    s.generation(1)
    changed = jobs_with(jobs, np.array(jobs.remaining) * 0.5)
    s.set_jobs(changed)
    assert np.array_equal(s.export_remaining(), changed.remaining)            # until the next draw
    s.generation(1)
    t = s.export()[3]
    assert s.export_remaining()[0] == ref.sampled_remaining(cluster.seed, 0, t, alpha[0], beta[0], proc[0])[0]
    s.set_progress()
    assert np.array_equal(s.export_remaining(), changed.remaining)


def test_progress_arguments_are_checked(ref):
    cluster, jobs = workloads.tiny()
    s = ref.RefSearch(cluster, jobs)
    n = cluster.n_slots
    one, proc = np.ones(n), np.full(n, 1e5)
    for bad, code in [((np.full(n, 0.5), one, proc), -1), ((one, np.full(n, 0.99), proc), -1),
                      ((one, one, np.full(n, -1.0)), -1), ((np.full(n, np.nan), one, proc), -4),
                      ((one, np.full(n, np.inf), proc), -4), ((np.full(n, 1e101), one, proc), -3),
                      ((one, one, np.full(n, 1e101)), -3)]:
        with pytest.raises(ref.RefError) as e:
            s.set_progress(*bad)
        assert e.value.code == code
    fit = s.export()[1].copy()
    s.generation(1)                                                           # a rejected call changed nothing
    t = ref.RefSearch(cluster, jobs); t.generation(1)
    assert np.array_equal(s.export()[1], t.export()[1]) and not np.array_equal(fit, s.export()[1])
