"""Pins for the oracle's capacity repair: the paper's refresh + fill (Section 3.2.2) under
the exclusivity constraint Eq. 4 (a GPU hosts one worker, so the GPU counts of a schedule
sum to at most the cluster size)."""
import os

import numpy as np
import pytest

import pyref
from pyref import check_invariants, make_jobs, random_genome, random_jobs

GOLD = os.path.join(os.path.dirname(__file__), "golden", "repair_worked_example.txt")


def test_worked_example(ref):
    jobs = make_jobs(3)
    n = 0
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        r, *want = [int(x) for x in line.split()]
        got, _ = ref.repair_genome(4, jobs, [1024, 512, 0], r)
        assert got.tolist() == want, r
        assert pyref.repair(4, jobs, [1024, 512, 0], r)[0].tolist() == want
        n += 1
    assert n == 3


CASES = [(1, 1), (3, 4), (8, 16), (40, 64), (64, 64), (65, 100), (130, 200), (200, 37),
         (512, 1024), (700, 5000)]


@pytest.mark.parametrize("n,G", CASES)
def test_invariants_idempotence_and_sequential_statement(ref, n, G):
    rng = np.random.default_rng(1000 * n + G)
    jp = 64 * -(-n // 64)
    for it in range(12):
        jobs = random_jobs(rng, n)
        genes = random_genome(rng, jobs, wild=(it % 2 == 1))
        r = int(rng.integers(0, jp))
        got, rounds = ref.repair_genome(G, jobs, genes, r)
        check_invariants(G, jobs, got)                       # I1, I2 (Eq. 4), I3
        want, want_rounds = pyref.repair(G, jobs, genes, r)  # independent sequential statement
        assert got.tolist() == want.tolist()
        assert rounds == want_rounds
        for r2 in {0, r, int(rng.integers(0, jp)), jp - 1}:  # I4: fixed point for every rotation
            again, rounds2 = ref.repair_genome(G, jobs, got, r2)
            assert again.tolist() == got.tolist()
            assert rounds2 == 0


def test_rotation_is_validated(ref):
    jobs = make_jobs(3)
    with pytest.raises(ref.RefError):
        ref.repair_genome(4, jobs, [0, 0, 0], 64)
    with pytest.raises(ref.RefError):
        ref.repair_genome(4, jobs, [3, 0, 0], 0)           # not a power of two


def test_enough_gpus_means_everybody_at_the_limit(ref):
    """G >= sum of c(bmax): the only fixed point is every active job at its limit R_j."""
    rng = np.random.default_rng(3)
    for n in (5, 64, 150):
        jobs = random_jobs(rng, n)
        need = sum(pyref.gpus(jobs.bmax[j], jobs.gpu_max_batch[j]) for j in range(n) if jobs.active[j])
        for G in (need, need + 7):
            genes = random_genome(rng, jobs, wild=True)
            got, _ = ref.repair_genome(G, jobs, genes, int(rng.integers(0, 64)))
            assert got.tolist() == [int(b) if a else 0 for a, b in zip(jobs.active, jobs.bmax)]


def test_no_gpus_means_everybody_waits(ref):
    rng = np.random.default_rng(4)
    jobs = random_jobs(rng, 70)
    got, rounds = ref.repair_genome(0, jobs, random_genome(rng, jobs), 5)
    assert not got.any() and rounds == 0


def test_single_job_gets_the_largest_batch_that_fits(ref):
    for G in (1, 2, 3, 4, 7, 8, 100):
        for hi in (6, 8, 10, 12):
            jobs = make_jobs(1, bmin=16, bmax=1 << hi, gpu_max_batch=256)
            for start in (0, 16, 1 << hi):
                got, _ = ref.repair_genome(G, jobs, [start], 0)
                fits = [1 << g for g in range(4, hi + 1) if pyref.gpus(1 << g, 256) <= G]
                if start == 0 or pyref.gpus(max(start, min(256, 1 << hi)), 256) <= G:
                    assert got[0] == max(fits)
                else:   # the incoming batch does not fit: dropped, then resumed and grown
                    assert got[0] == max(fits)


def test_admission_keeps_a_prefix_of_the_rotated_order(ref):
    rng = np.random.default_rng(9)
    n, G = 150, 40
    jobs = random_jobs(rng, n, inactive_frac=0.0)
    jobs.bmin[:] = 1024; jobs.bmax[:] = 1024; jobs.gpu_max_batch[:] = 256   # every job: 4 GPUs or none
    genes = np.full(n, 1024, np.int32)
    for r in (0, 1, 77, 191):
        got, _ = ref.repair_genome(G, jobs, genes, r)
        order = pyref.visiting_order(n, r)
        assert [int(got[j]) for j in order] == [1024] * 10 + [0] * (n - 10)


def test_lift_is_free_and_improves_the_score(ref):
    """A running job below the per-GPU max is raised to it: same GPU count, smaller term."""
    jobs = make_jobs(4, bmin=32, bmax=1024, gpu_max_batch=256)
    got, _ = ref.repair_genome(4, jobs, [32, 64, 128, 256], 0)
    assert got.tolist() == [256, 256, 256, 256]
    assert ref.score_genome(4, jobs, got) < ref.score_genome(4, jobs, [32, 64, 128, 256])


def test_limit_below_the_incoming_batch_scales_down(ref):
    """Refresh step (2): B_j > R_j is cut to R_j."""
    jobs = make_jobs(2, bmin=32, bmax=[512, 128], gpu_max_batch=256)
    got, _ = ref.repair_genome(3, jobs, [1024, 1024], 0)
    assert got.tolist() == [512, 128]      # 2 GPUs + 1 GPU
    got, _ = ref.repair_genome(2, jobs, [1024, 1024], 0)
    assert got.tolist() == [512, 0]        # after the cut job 0 takes both GPUs, job 1 waits


# ---- refresh (3) of Section 3.2.2: arrived jobs first, room taken from the largest T_processed ----

def test_arrival_takes_the_gpus_of_the_longest_running_job(ref):
    """Four GPUs, all busy: jobs 0, 1, 2 hold 1, 2 and 1 GPUs (256 per GPU) and have executed 100,
    300 and 200 s; job 3 arrives and starts on one GPU.  Three GPUs are left for the others; in
    order of executed time job 0 keeps its GPU (1 of 3), job 2 its GPU (2 of 3), job 1 with two
    GPUs no longer fits (4 of 3) and waits.  One GPU is idle then and the fill hands it to the
    first job it visits that can use it: job 1 again (on one GPU) when the visit starts there
    (r = 1), job 0 (doubling) when it starts at job 0."""
    jobs = make_jobs(4, bmin=256, bmax=512, gpu_max_batch=256)
    got, _ = ref.repair_arrivals(4, jobs, [256, 512, 256, 0], 1, [0, 0, 0, 1], [100.0, 300.0, 200.0, 0.0])
    assert got.tolist() == [256, 256, 256, 256]
    got, _ = ref.repair_arrivals(4, jobs, [256, 512, 256, 0], 0, [0, 0, 0, 1], [100.0, 300.0, 200.0, 0.0])
    assert got.tolist() == [512, 0, 256, 256]
    # with job 0 the longest runner instead
    jobs = make_jobs(4, bmin=256, bmax=256, gpu_max_batch=256)
    jobs.bmax[:] = [512, 512, 256, 256]
    got, _ = ref.repair_arrivals(4, jobs, [512, 256, 256, 0], 0, [0, 0, 0, 1], [900.0, 300.0, 200.0, 0.0])
    assert got.tolist() == [256, 256, 256, 256]            # job 0 dropped from 2 GPUs, resumed on the idle one
    # five one-GPU jobs on four GPUs, no room to resume: the longest runner waits
    jobs = make_jobs(5, bmin=256, bmax=256, gpu_max_batch=256)
    for times, loser in [([5.0, 9.0, 1.0, 3.0, 0.0], 1), ([5.0, 2.0, 1.0, 30.0, 0.0], 3), ([7.0, 7.0, 7.0, 7.0, 0.0], 3)]:
        got, rounds = ref.repair_arrivals(4, jobs, [256, 256, 256, 256, 0], 2, [0, 0, 0, 0, 1], times)
        want = [256] * 5
        want[loser] = 0                                      # equal times: the higher slot gives way
        assert got.tolist() == want and rounds == 0
    # without times the rotated visiting order decides: with r = 2 the visit starts at job 2
    got, _ = ref.repair_arrivals(4, jobs, [256, 256, 256, 256, 0], 2, [0, 0, 0, 0, 1], None)
    assert got.tolist() == [256, 0, 256, 256, 256]          # 2, 3, 0 keep theirs; job 1 comes last


@pytest.mark.parametrize("n,G", CASES)
def test_arrivals_against_the_sequential_statement(ref, n, G):
    rng = np.random.default_rng(77 * n + G)
    jp = 64 * -(-n // 64)
    for it in range(10):
        jobs = random_jobs(rng, n)
        genes, _ = ref.repair_genome(G, jobs, random_genome(rng, jobs), int(rng.integers(0, jp)))  # a feasible schedule
        arrived = (rng.random(n) < (0.1 if it % 3 else 0.5)).astype(np.uint8)
        times = [None, rng.integers(0, 5, n) * 60.0, rng.uniform(0, 1e5, n)][it % 3]   # none, many ties, distinct
        r = int(rng.integers(0, jp))
        got, rounds = ref.repair_arrivals(G, jobs, genes, r, arrived, times)
        check_invariants(G, jobs, got)
        want, want_rounds = pyref.repair_arrivals(G, jobs, genes, r, arrived, times)
        assert got.tolist() == want.tolist() and rounds == want_rounds
        # the arrived jobs that run do so on their starting batch or more, and as many of them run as fit
        new = [j for j in range(n) if arrived[j] and jobs.active[j]]
        asks = sorted(pyref.gpus(pyref.start_batch(jobs, j), jobs.gpu_max_batch[j]) for j in new)
        if sum(asks) <= G:
            assert all(got[j] >= pyref.start_batch(jobs, j) for j in new)
        if not arrived.any():
            assert got.tolist() == genes.tolist()            # a feasible schedule is left alone


def test_admitted_jobs_form_a_prefix_of_the_time_order(ref):
    """One-GPU jobs with a fixed batch (nothing to fill with afterwards except restarts, and no
    GPU is idle): among the old jobs exactly the ones with the largest executed times wait."""
    rng = np.random.default_rng(5)
    n, G = 150, 100
    jobs = make_jobs(n, bmin=128, bmax=128, gpu_max_batch=128)
    for it in range(8):
        running = rng.permutation(n)[:G]
        genes = np.zeros(n, np.int32); genes[running] = 128
        waiting = np.setdiff1d(np.arange(n), running)
        arrived = np.zeros(n, np.uint8); arrived[waiting[: 5 + it]] = 1
        times = rng.permutation(n).astype(np.float64)        # distinct
        got, _ = ref.repair_arrivals(G, jobs, genes, int(rng.integers(0, 192)), arrived, times)
        assert (got[arrived == 1] == 128).all()
        kept = [j for j in running if got[j]]
        dropped = [j for j in running if not got[j]]
        assert len(dropped) == 5 + it
        assert max(times[kept]) < min(times[dropped])
        assert (got[waiting[5 + it:]] == 0).all()           # nobody else got in: no GPU was idle


def test_processed_time_in_the_search(ref):
    """Through the search context: the generation after a table change uses the times, only with
    the new-jobs-first option, and a NULL forgets them."""
    from types import SimpleNamespace
    cl = SimpleNamespace(n_gpus=4, n_slots=5, population=16, seed=11, mutation_rate=0.0, crossover_rate=0.5)
    before = make_jobs(5, active=[1, 1, 1, 1, 0], bmin=256, bmax=256, gpu_max_batch=256)
    after = make_jobs(5, bmin=256, bmax=256, gpu_max_batch=256)
    after.job_id[4] += 100
    for times, loser in [([5.0, 9.0, 1.0, 3.0, 0.0], 1), ([5.0, 2.0, 1.0, 30.0, 0.0], 3)]:
        s = ref.RefSearch(cl, before)
        s.generation(2)
        assert s.best()[0].tolist() == [256, 256, 256, 256, 0]
        s.set_new_jobs_first(True)
        s.set_processed_time(times)
        s.set_jobs(after)
        s.generation(1)
        genes = s.export()[0][:, :5]
        want = [256] * 5; want[loser] = 0
        assert (genes == want).all()                         # every candidate: the longest runner waits
        s.close()
    # forgotten times: the rotation decides again (five slots in 64 columns: mostly job 3 comes last)
    s = ref.RefSearch(cl, before)
    s.generation(2); s.set_new_jobs_first(True); s.set_processed_time([5.0, 9.0, 1.0, 3.0, 0.0]); s.set_processed_time(None)
    s.set_jobs(after); s.generation(1)
    genes = s.export()[0][:, :5]
    assert (genes[:, 4] == 256).all() and not (genes[:, 1] == 0).all()
    s.close()
    with pytest.raises(ref.RefError):
        t = ref.RefSearch(cl, before); t.set_processed_time([1.0, -2.0, 0.0, 0.0, 0.0])
    with pytest.raises(ref.RefError):
        t.set_processed_time([1.0, float("nan"), 0.0, 0.0, 0.0])
