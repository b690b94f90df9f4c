"""Pins for the oracle's whole generation step (paper Section 3.2.2: pool = K refreshed
survivors + K parent pairs' 2K crossover children + K mutants, scored with Eq. 3 / Eq. 8,
best K kept; Alg. 1: the smallest score wins)."""
import itertools
from types import SimpleNamespace

import numpy as np
import pytest
from scipy import stats

import pyref
from paper_2108_03645_amd import workloads as W
from pyref import check_invariants, exact_objective, make_jobs, philox4x32_10, random_jobs


def cluster(n_gpus, n_slots, population, seed=0, theta=0.1, chi=0.5):
    return SimpleNamespace(n_gpus=n_gpus, n_slots=n_slots, population=population, seed=seed,
                           mutation_rate=theta, crossover_rate=chi)


# ----------------------------------------------------------------- selection ------
def test_select_is_lexicographic_on_fitness_then_index(ref):
    rng = np.random.default_rng(0)
    for P in (4, 64, 1000, 4096):
        fit = rng.integers(0, max(2, P // 8), P).astype(np.float64)   # many ties
        want = np.lexsort((np.arange(P), fit))[:P // 4]
        assert ref.select(fit).tolist() == want.tolist()
    assert ref.select(np.zeros(64)).tolist() == list(range(16))


# ----------------------------------------------------------- brute force, tiny -----
def _tiny_feasible_states(cl, jobs):
    """All schedules of the tiny cluster that respect Eq. 4 and leave no single step that
    would still fit (what 'no idle GPU' of the refresh means when batch sizes are
    discrete).  After the free lift a running job holds 256, 512 or 1024."""
    out = []
    for state in itertools.product((0, 256, 512, 1024), repeat=cl.n_slots):
        used = sum(pyref.gpus(b, 256) for b in state)
        if used > cl.n_gpus:
            continue
        idle = cl.n_gpus - used
        if any((pr := pyref.proposal(jobs, j, b)) is not None and pr[1] <= idle
               for j, b in enumerate(state)):
            continue
        out.append(state)
    return out


def test_tiny_brute_force_optimum_bounds_the_search(ref):
    cl, jobs = W.tiny()
    states = _tiny_feasible_states(cl, jobs)
    assert len(states) > 100
    # the oracle's repair fixes exactly these states, for any rotation
    rng = np.random.default_rng(1)
    feasible = set(states)
    for state in itertools.islice(itertools.product((0, 256, 512, 1024), repeat=8), 0, 65536, 97):
        got, _ = ref.repair_genome(cl.n_gpus, jobs, list(state), int(rng.integers(0, 64)))
        assert tuple(got.tolist()) in feasible
        assert (tuple(got.tolist()) == state) == (state in feasible)
    best_exact = min(exact_objective(jobs, s) for s in states)
    f_star = float(best_exact)

    s = ref.RefSearch(cl, jobs)
    trace = []
    for t in range(cl.generations + 1):
        genes, fit, sel, gen = s.export()
        assert gen == t
        assert fit.min() >= f_star * (1 - 1e-12)
        for p in range(cl.population):
            assert tuple(genes[p, :8].tolist()) in feasible
            assert fit[p] == pytest.approx(float(exact_objective(jobs, genes[p, :8])), rel=1e-12)
        b, g, f = s.best()
        assert f == fit[sel[0]] == fit.min()
        assert b.tolist() == genes[sel[0], :8].tolist()
        assert g.tolist() == [pyref.gpus(x, 256) for x in b]
        trace.append(f)
        s.generation(1)
    assert all(trace[i + 1] <= trace[i] for i in range(len(trace) - 1))   # elites are kept
    # with more generations the search reaches the brute-force optimum and never beats it
    s.generation(150)
    b, _, f = s.best()
    assert f == pytest.approx(f_star, rel=1e-12)
    assert exact_objective(jobs, b) == best_exact


# ------------------------------------------------------- invariants every step -----
@pytest.mark.parametrize("name", ["paper_scale", "multirow"])
def test_pool_invariants_every_generation(ref, name):
    if name == "paper_scale":
        cl, jobs = W.paper_scale()
        gens = 6
    else:
        rng = np.random.default_rng(42)
        jobs = random_jobs(rng, 300)
        cl = cluster(500, 300, 128, seed=42)
        gens = 4
    s = ref.RefSearch(cl, jobs)
    for t in range(gens):
        genes, fit, sel, _ = s.export()
        assert not genes[:, cl.n_slots:].any()                # padding never runs
        for p in range(0, cl.population, 7):
            check_invariants(cl.n_gpus, jobs, genes[p, :cl.n_slots])
            assert fit[p] == pytest.approx(float(exact_objective(jobs, genes[p, :cl.n_slots])), rel=1e-12)
        assert sel.tolist() == np.lexsort((np.arange(cl.population), fit))[:cl.population // 4].tolist()
        s.generation(1)


# ------------------------------------------------------------------ operators ------
def _words(seed, p, t, n_slots):
    key = [seed & 0xFFFFFFFF, seed >> 32]
    out = []
    for j in range(n_slots):
        l, i = j % 64, j // 64
        out.append(philox4x32_10([(i // 4) * 64 + l, p, t, 0], key)[i % 4])
    return out


def _draw(seed, p, t):
    return philox4x32_10([0xFFFFFFFF, p, t, 0], [seed & 0xFFFFFFFF, seed >> 32])


def test_pool_layout_parents_and_rotation(ref):
    """Slots [0,K) are the survivors in rank order, [K,3K) crossover pairs, [3K,4K) mutants;
    parents are independent uniform draws among the K survivors."""
    rng = np.random.default_rng(5)
    jobs = random_jobs(rng, 150)
    cl = cluster(200, 150, 64, seed=0x1234567890ABCDEF)
    s = ref.RefSearch(cl, jobs)
    s.generation(2)
    genes, fit, sel, t = s.export()
    K, jp = 16, 192
    for p in range(64):
        g, r, pa, pb = s.compose_slot(p)
        w = _draw(cl.seed, p, t + 1)
        assert r == (w[2] * jp) >> 32
        if p < K:
            assert (pa, pb) == (sel[p], -1)
            assert g.tolist() == genes[sel[p]].tolist()
        elif p < 3 * K:
            p0 = K + 2 * ((p - K) // 2)
            w0 = _draw(cl.seed, p0, t + 1)
            assert (pa, pb) == (sel[(w0[0] * K) >> 32], sel[(w0[1] * K) >> 32])
        else:
            assert (pa, pb) == (sel[(w[0] * K) >> 32], -1)


def test_crossover_children_are_complementary(ref):
    rng = np.random.default_rng(6)
    jobs = random_jobs(rng, 200)
    cl = cluster(300, 200, 256, seed=77, chi=0.5)
    s = ref.RefSearch(cl, jobs)
    s.generation(1)
    genes, _, sel, t = s.export()
    K = 64
    T_x = 1 << 31
    swaps = total = 0
    for q in range(K):
        c0, _, pa, pb = s.compose_slot(K + 2 * q)
        c1, _, pa1, pb1 = s.compose_slot(K + 2 * q + 1)
        assert (pa, pb) == (pa1, pb1)
        A, B = genes[pa], genes[pb]
        words = _words(cl.seed, K + 2 * q, t + 1, 200)
        for j in range(200):
            swap = words[j] < T_x
            assert (c0[j], c1[j]) == ((B[j], A[j]) if swap else (A[j], B[j]))
            swaps += swap; total += 1
    assert abs(swaps / total - 0.5) < 4 * 0.5 / np.sqrt(total)      # fair coin


def test_crossover_rate_one_swaps_parents_and_zero_copies_them(ref):
    rng = np.random.default_rng(8)
    jobs = random_jobs(rng, 70)
    for chi in (1.0, 0.0):
        cl = cluster(90, 70, 64, seed=3, chi=chi)
        s = ref.RefSearch(cl, jobs)
        genes, _, sel, _ = s.export()
        for q in range(16):
            c0, _, pa, pb = s.compose_slot(16 + 2 * q)
            c1, _, _, _ = s.compose_slot(16 + 2 * q + 1)
            first, second = (genes[pb], genes[pa]) if chi == 1.0 else (genes[pa], genes[pb])
            assert c0.tolist() == first.tolist() and c1.tolist() == second.tolist()


def test_mutation_touches_each_job_independently_with_rate_theta(ref):
    jobs = make_jobs(192, bmin=32, bmax=1024)            # n_j = 7 outcomes: wait, 32..1024
    cl = cluster(100, 192, 512, seed=11, theta=0.1)
    s = ref.RefSearch(cl, jobs)
    genes, _, sel, t = s.export()
    K = 128
    T_mut = int(np.floor(0.1 * 2**32))
    redrawn = changed = total = 0
    outcomes = np.zeros(7, int)
    for p in range(3 * K, 4 * K):
        m, _, pa, _ = s.compose_slot(p)
        words = _words(cl.seed, p, t + 1, 192)
        for j in range(192):
            total += 1
            if words[j] < T_mut:
                redrawn += 1
                k = ((words[j] & 0xFFFF) * 7) >> 16
                assert m[j] == (0 if k == 0 else 32 << (k - 1))
                outcomes[k] += 1
                changed += m[j] != genes[pa][j]
            else:
                assert m[j] == genes[pa][j]
    assert abs(redrawn / total - 0.1) < 4 * np.sqrt(0.1 * 0.9 / total)
    assert stats.chisquare(outcomes).pvalue > 1e-4         # redraw uniform over {wait, 32..1024}
    assert 0.7 < changed / redrawn <= 1.0                   # about 1 - 1/n_j of redraws differ


def test_mutation_rate_zero_and_inactive_slots(ref):
    rng = np.random.default_rng(12)
    jobs = random_jobs(rng, 64, inactive_frac=0.3)
    cl = cluster(80, 64, 64, seed=5, theta=0.0)
    s = ref.RefSearch(cl, jobs)
    genes, _, _, _ = s.export()
    for p in range(48, 64):
        m, _, pa, _ = s.compose_slot(p)
        assert m.tolist() == genes[pa].tolist()
    s2 = ref.RefSearch(cluster(80, 64, 64, seed=5, theta=1.0), jobs)
    for p in range(48, 64):
        m, _, _, _ = s2.compose_slot(p)
        assert not m[np.flatnonzero(jobs.active == 0)].any()


def test_parent_ranks_and_rotations_are_uniform(ref):
    jobs = make_jobs(64)
    cl = cluster(64, 64, 4096, seed=99)
    s = ref.RefSearch(cl, jobs)
    _, _, sel, _ = s.export()
    rank = {int(v): i for i, v in enumerate(sel)}
    K = 1024
    pa_hist = np.zeros(8, int); pb_hist = np.zeros(8, int); r_hist = np.zeros(8, int)
    same = 0
    for p in range(K, 4 * K, 2):
        _, r, pa, pb = s.compose_slot(p)
        pa_hist[rank[pa] * 8 // K] += 1
        r_hist[r * 8 // 64] += 1
        if pb >= 0:
            pb_hist[rank[pb] * 8 // K] += 1
            same += pa == pb
    assert stats.chisquare(pa_hist).pvalue > 1e-4
    assert stats.chisquare(pb_hist).pvalue > 1e-4
    assert stats.chisquare(r_hist).pvalue > 1e-4
    assert same < 10                                    # repeats allowed but rare (1/K each)


def test_initial_population_is_uniform_over_wait_and_window(ref):
    jobs = make_jobs(130, bmin=[16] * 65 + [64] * 65, bmax=[128] * 65 + [64] * 65)
    cl = cluster(50, 130, 2048, seed=21)
    hist_a = np.zeros(5, int); hist_b = np.zeros(2, int)
    for p in range(0, 2048, 8):
        g, r = ref.initial_genome(cl, jobs, p)
        words = _words(cl.seed, p, 0, 130)
        assert r == (_draw(cl.seed, p, 0)[2] * 192) >> 32
        for j in range(130):
            n = 5 if j < 65 else 2
            k = (words[j] * n) >> 32
            lo = 16 if j < 65 else 64
            assert g[j] == (0 if k == 0 else lo << (k - 1))
            (hist_a if j < 65 else hist_b)[k] += 1
    assert stats.chisquare(hist_a).pvalue > 1e-4
    assert stats.chisquare(hist_b).pvalue > 1e-4


def test_no_variation_collapses_to_the_best_and_ties_break_by_index(ref):
    """theta = chi = 0: every pool member is a copy of a survivor, so nothing new appears,
    the best stays in slot 0, and once all survivors are copies of it the ranking is
    decided by the slot index alone."""
    rng = np.random.default_rng(13)
    jobs = random_jobs(rng, 40)
    cl = cluster(64, 40, 64, seed=2, theta=0.0, chi=0.0)
    s = ref.RefSearch(cl, jobs)
    genes0, fit0, sel0, _ = s.export()
    survivors0 = {genes0[p].tobytes() for p in sel0}
    for _ in range(30):
        s.generation(1)
        genes, fit, sel, _ = s.export()
        assert {genes[p].tobytes() for p in range(64)} <= survivors0
        assert sel[0] == 0 and fit[0] == fit0[sel0[0]]
    assert np.all(fit == fit[0])
    assert sel.tolist() == list(range(16))


def test_threads_do_not_change_the_result(ref):
    rng = np.random.default_rng(14)
    jobs = random_jobs(rng, 100)
    cl = cluster(128, 100, 256, seed=9)
    ref.set_threads(1)
    s1 = ref.RefSearch(cl, jobs); s1.generation(3); e1 = s1.export()
    ref.set_threads(4)
    try:
        s4 = ref.RefSearch(cl, jobs); s4.generation(3); e4 = s4.export()
    finally:
        ref.set_threads(1)
    for x, y in zip(e1, e4):
        assert np.array_equal(x, y)


def test_seed_and_generation_enter_the_stream(ref):
    rng = np.random.default_rng(15)
    jobs = random_jobs(rng, 64)
    a = ref.RefSearch(cluster(64, 64, 64, seed=1), jobs)
    b = ref.RefSearch(cluster(64, 64, 64, seed=1 << 32), jobs)      # high key word
    assert not np.array_equal(a.export()[0], b.export()[0])
    g1, r1, *_ = a.compose_slot(60)
    a.generation(1)
    g2, r2, *_ = a.compose_slot(60)
    assert (r1, g1.tolist()) != (r2, g2.tolist())


# --------------------------------------------------------------------- online ------
def test_set_jobs_resets_changed_slots_and_refresh_projects_elites(ref):
    rng = np.random.default_rng(16)
    jobs = random_jobs(rng, 64, inactive_frac=0.2)
    cl = cluster(64, 64, 128, seed=4)
    s = ref.RefSearch(cl, jobs)
    s.generation(3)
    before, _, sel_before, t0 = s.export()
    new = SimpleNamespace(**{k: getattr(jobs, k).copy() for k in vars(jobs)})
    new.job_id[5] = 1000                      # slot 5 changes hands
    new.active[5] = 1; new.bmin[5] = 64; new.bmax[5] = 256
    new.active[9] = 0                         # job in slot 9 finished
    new.bmax[11] = new.bmin[11]               # limit R_j of slot 11 shrinks
    new.remaining[:] *= 0.5                   # progress
    s.set_jobs(new)
    after, _, sel_after, t1 = s.export()
    assert t1 == t0 and sel_after.tolist() == sel_before.tolist()
    assert not after[:, 5].any()
    mask = np.ones(64, bool); mask[5] = False
    assert np.array_equal(after[:, mask], before[:, mask])
    s.generation(1)
    genes, fit, sel, t2 = s.export()
    assert t2 == t0 + 1
    for p in range(128):
        check_invariants(cl.n_gpus, new, genes[p, :64])
        assert fit[p] == pytest.approx(float(exact_objective(new, genes[p, :64])), rel=1e-12)
    assert not genes[:, 9].any()
    assert set(np.unique(genes[:, 11])) <= {0, int(new.bmin[11])}


def test_empty_cluster_and_no_slots(ref):
    s = ref.RefSearch(cluster(8, 0, 16), make_jobs(0))
    s.generation(2)
    genes, fit, sel, t = s.export()
    assert genes.shape == (16, 64) and not genes.any() and not fit.any()
    assert sel.tolist() == [0, 1, 2, 3] and t == 2
    jobs = make_jobs(10, active=0)
    s = ref.RefSearch(cluster(8, 10, 16), jobs)
    s.generation(1)
    genes, fit, sel, _ = s.export()
    assert not genes.any() and not fit.any() and sel.tolist() == [0, 1, 2, 3]
    assert s.best()[2] == 0.0


# ----------------------------------------------------------------- validation ------
def test_argument_validation(ref):
    ok = make_jobs(4)
    R = ref.RefSearch

    def code(cl, jobs):
        with pytest.raises(ref.RefError) as e:
            R(cl, jobs)
        return e.value.code

    assert code(cluster(-1, 4, 16), ok) == -1
    assert code(cluster(4, 4, 18), ok) == -1                 # population not a multiple of 4
    assert code(cluster(4, 4, 0), ok) == -1
    assert code(cluster(4, 2049, 16), make_jobs(2049)) == -1
    assert code(cluster(4, 4, 16, theta=1.5), ok) == -1
    assert code(cluster(4, 4, 16, chi=float("nan")), ok) == -1
    assert code(cluster(4, 4, 16), make_jobs(4, bmin=[32, 48, 32, 32])) == -2
    assert code(cluster(4, 4, 16), make_jobs(4, bmin=64, bmax=32)) == -3
    assert code(cluster(4, 4, 16), make_jobs(4, bmin=1, bmax=1 << 30, gpu_max_batch=2)) == -3
    assert code(cluster(4, 4, 16), make_jobs(4, a=float("inf"))) == -4
    assert code(cluster(4, 4, 16), make_jobs(4, remaining=[1, float("nan"), 1, 1])) == -4
    assert code(cluster(4, 4, 16), make_jobs(4, d=-1.0)) == -1
    assert code(cluster(4, 4, 16), make_jobs(4, c=1e101)) == -3
    # garbage in an inactive slot is ignored
    R(cluster(4, 4, 16), make_jobs(4, active=[1, 0, 1, 1], bmin=[32, 3, 32, 32], a=[1e-3, float("nan"), 1e-3, 1e-3]))


# ------------------------------------------------ the winner as a map onto the GPUs (Eq. 1) ----
def test_placement_hand_example(ref):
    """Job 0 can only run 256 samples on one GPU, job 1 only 512 on two (256 per GPU), job 2 only
    1024 on four.  On 4 GPUs the fill leaves no GPU idle when it can: the winner runs jobs 0 and 1
    (3 GPUs, job 2 does not fit beside either) or job 2 alone; the scores decide.  Job 2 is given
    so much work that running it alone scores worse, so the map is 0, 1, 1, idle."""
    jobs = make_jobs(3, bmin=[256, 512, 1024], bmax=[256, 512, 1024], gpu_max_batch=256,
                     remaining=[1e6, 1e6, 1e9])
    cl = SimpleNamespace(n_gpus=4, n_slots=3, population=16, seed=5, mutation_rate=0.1, crossover_rate=0.5)
    s = ref.RefSearch(cl, jobs)
    s.generation(30)
    batch, gpus, _ = s.best()
    assert batch.tolist() == [256, 512, 0] and gpus.tolist() == [1, 2, 0]
    slot, per_gpu = s.placement()
    assert slot.tolist() == [0, 1, 1, -1] and per_gpu.tolist() == [256, 256, 256, 0]
    # with 7 GPUs everything runs: 0 | 1 1 | 2 2 2 2
    cl7 = SimpleNamespace(n_gpus=7, n_slots=3, population=16, seed=5, mutation_rate=0.1, crossover_rate=0.5)
    s7 = ref.RefSearch(cl7, jobs)
    s7.generation(30)
    slot, per_gpu = s7.placement()
    assert slot.tolist() == [0, 1, 1, 2, 2, 2, 2] and per_gpu.tolist() == [256] * 7


def test_placement_satisfies_eq_2(ref):
    """B_j = sum_i b_j^i and c_j = sum_i min(1, b_j^i) recover the winner; one job per GPU; the
    workers of a job are adjacent and the jobs appear in slot order (reorder); idle GPUs last."""
    for maker in (W.tiny, W.paper_scale):
        cluster, jobs = maker()
        s = ref.RefSearch(cluster, jobs)
        for gens in (0, 3):
            s.generation(gens)
            batch, gpus, _ = s.best()
            slot, per_gpu = s.placement()
            assert len(slot) == cluster.n_gpus
            for j in range(cluster.n_slots):
                mine = per_gpu[slot == j]
                assert mine.sum() == batch[j] and np.minimum(1, mine).sum() == gpus[j]
            used = int(gpus.sum())
            assert (slot[:used] >= 0).all() and (slot[used:] == -1).all() and (per_gpu[used:] == 0).all()
            assert (np.diff(slot[:used]) >= 0).all()


def test_placement_needs_a_schedule_under_the_current_table(ref):
    cluster, jobs = W.tiny()
    s = ref.RefSearch(cluster, jobs)
    s.placement()
    s.set_jobs(jobs)
    with pytest.raises(ref.RefError) as e:
        s.placement()
    assert e.value.code == -1
    s.generation(1)
    s.placement()


# ------------------------------------------------ new jobs are served first (refresh (3)) ----
def changed(jobs, **edits):
    d = {k: np.array(getattr(jobs, k)) for k in ("job_id", "active", "bmin", "bmax", "gpu_max_batch", "a", "c", "d",
                                                  "remaining")}
    for k, (j, v) in edits.items():
        d[k][j] = v
    return make_jobs(len(jobs.bmin), **d)


def test_new_job_first_hand_example(ref):
    """Two GPUs.  Job 0 (window 256..512, 256 per GPU) holds both; then job 1 arrives in slot 1.
    Served first, it takes one GPU with its starting batch 256; job 0's 512 on two GPUs no longer
    fits the one GPU left and is dropped, and the fill gives it the idle GPU back with 256.
    Without the option job 0 keeps both GPUs in the survivors and job 1 has to win its GPU in
    the search."""
    cl = SimpleNamespace(n_gpus=2, n_slots=2, population=8, seed=3, mutation_rate=0.0, crossover_rate=0.5)
    alone = make_jobs(2, active=[1, 0], bmin=256, bmax=512, gpu_max_batch=256)
    both = changed(alone, active=(1, 1), job_id=(1, 77))
    for option in (True, False):
        s = ref.RefSearch(cl, alone)
        s.generation(3)
        assert s.best()[0].tolist() == [512, 0]
        s.set_new_jobs_first(option)
        s.set_jobs(both)
        s.generation(1)
        genes = s.export()[0][:, :2]
        if option:
            assert (genes == [256, 256]).all()                 # every candidate, survivors included
        else:
            assert (genes[:2] == [512, 0]).all()               # the refreshed survivors kept job 0's GPUs


def test_new_jobs_run_in_every_candidate_when_they_fit(ref):
    cluster, jobs = W.paper_scale()
    s = ref.RefSearch(cluster, jobs)
    s.set_new_jobs_first(True)
    s.generation(5)
    new_slots = [3, 17, 30]
    j2 = changed(jobs)
    for j in new_slots:
        j2.job_id[j] += 1000
    s.set_jobs(j2)
    s.generation(1)
    genes = s.export()[0]
    assert (genes[:, new_slots] > 0).all()
    for p in range(0, cluster.population, 41):
        check_invariants(cluster.n_gpus, j2, genes[p, :cluster.n_slots])
    # the generation after that is an ordinary one again
    t = ref.RefSearch(cluster, jobs); t.generation(5); t.set_jobs(j2); t.generation(1)
    assert not (t.export()[0][:, new_slots] > 0).all()         # without the option some candidates leave them waiting


def test_more_new_jobs_than_gpus(ref):
    """Eight one-GPU jobs arrive on a three-GPU cluster: exactly three of them run, nothing else."""
    cl = SimpleNamespace(n_gpus=3, n_slots=9, population=16, seed=8, mutation_rate=0.1, crossover_rate=0.5)
    before = make_jobs(9, active=[1] + [0] * 8, bmin=64, bmax=1024, gpu_max_batch=256)
    after = changed(before)
    after.active[1:] = 1
    after.job_id[1:] += 50
    s = ref.RefSearch(cl, before)
    s.set_new_jobs_first(True)
    s.generation(2)
    s.set_jobs(after)
    s.generation(1)
    genes = s.export()[0][:, :9]
    assert (genes[:, 0] == 0).all()                            # the old job had to make room
    assert ((genes[:, 1:] > 0).sum(axis=1) == 3).all() and (genes[:, 1:].max(axis=1) == 256).all()


def test_option_changes_nothing_without_new_jobs(ref):
    cluster, jobs = W.tiny()
    a, b = ref.RefSearch(cluster, jobs), ref.RefSearch(cluster, jobs)
    a.set_new_jobs_first(True)
    j2 = changed(jobs, remaining=(2, 5e6))                     # same jobs, new remaining work
    for s in (a, b):
        s.generation(2); s.set_jobs(j2); s.generation(2)
    assert all(np.array_equal(x, y) for x, y in zip(a.export()[:3], b.export()[:3]))
