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
