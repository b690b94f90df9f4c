"""ones_generation_static, the entry point that allocates nothing: same generations as
ones_generation, bit for bit, with the selection's scratch in the library's static device array.
Called through the C ABI; every GPU context on the device shares that array."""
import ctypes as C
import sys
from types import SimpleNamespace

import numpy as np
import pytest

from pyref import random_jobs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ones():
    from paper_2108_03645_amd import ones as binding
    binding.load()
    return binding


def cluster(n_gpus, n_slots, population, seed):
    return SimpleNamespace(n_gpus=n_gpus, n_slots=n_slots, population=population, seed=seed,
                           mutation_rate=0.1, crossover_rate=0.5)


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def same(a, b, where):
    ga, fa, sa, ta = a.export()
    gb, fb, sb, tb = b.export()
    assert ta == tb, where
    assert np.array_equal(ga, gb), f"{where}: genomes differ"
    assert np.array_equal(fa.view(np.uint64), fb.view(np.uint64)), f"{where}: scores differ"
    assert np.array_equal(sa, sb), f"{where}: survivor lists differ"


def test_static_scratch_matches_the_workspace_scratch_on_two_calls_in_a_row(ones, ref):
    """A pool that selects through the buckets (P = 8192, 200 slots), then a smaller one
    (P = 1024, 130 slots), then the first one again: the second call finds the first one's
    leftovers in the array and the third the second one's.  (Both have more than one row of job
    slots: a pool of one row runs its generations in a single launch that uses no scratch at all,
    whichever entry point is called; the third shape checks that.)"""
    lib = ones.load()
    shapes = [(300, 200, 8192, 11), (200, 130, 1024, 12), (64, 40, 512, 13)]
    pairs = []
    for n_gpus, n_slots, pop, seed in shapes:
        cl = cluster(n_gpus, n_slots, pop, seed)
        jobs = random_jobs(np.random.default_rng(seed), n_slots)
        pairs.append((ones.Search(cl, jobs), ones.Search(cl, jobs), ref.RefSearch(cl, jobs), cl, jobs))
    for rnd, which in enumerate([0, 1, 0, 1, 2, 0]):
        static, plain, cpu, cl, jobs = pairs[which]
        say(f"[no alloc] call {rnd}: P={cl.population} slots={cl.n_slots} seed={cl.seed}")
        assert lib.ones_generation_static(static._h, 3) == 0          # straight through the C ABI
        assert lib.ones_generation(plain._h, 3) == 0
        cpu.generation(3)
        same(static, plain, f"call {rnd}")
        same(static, cpu, f"call {rnd} against the oracle")
        assert static.best()[2] == plain.best()[2]
    # the two entry points mixed on one context, and a table change in between
    static, plain, cpu, cl, jobs = pairs[0]
    jobs.remaining = jobs.remaining * 0.5
    jobs.job_id[3] += 99
    for s in (static, plain, cpu):
        s.set_jobs(jobs)
    static.generation_static(1); plain.generation(1); cpu.generation(1)
    same(static, plain, "after a table change")
    static.generation(2); plain.generation_static(2); cpu.generation(2)
    same(static, plain, "entry points swapped")
    same(static, cpu, "entry points swapped, against the oracle")
    # sampled remaining work goes through the general selection every generation
    from paper_2108_03645_amd import workloads as W
    progress = W.progress(cl.n_slots, seed=3)
    for s in (static, plain, cpu):
        s.set_progress(*progress)
    static.generation_static(2); plain.generation(2); cpu.generation(2)
    same(static, plain, "sampled remaining work")
    same(static, cpu, "sampled remaining work, against the oracle")
    assert lib.ones_generation_static(static._h, 0) == 0
    assert lib.ones_generation_static(static._h, -1) == -1
    assert lib.ones_generation_static(None, 1) == -1
    for static, plain, cpu, _, _ in pairs:
        static.close(); plain.close(); cpu.close()


def test_static_scratch_rejects_a_population_beyond_its_size(ones):
    """P = 262144 needs 16 MiB of bucket keys alone: refused, nothing launched, the context stays usable."""
    cl = cluster(9, 6, 1 << 18, 5)
    jobs = random_jobs(np.random.default_rng(5), 6, inactive_frac=0.0)
    say(f"[no alloc] too large: P={cl.population}")
    s = ones.Search(cl, jobs)
    before = s.export(genes=False)
    lib = ones.load()
    rc = lib.ones_generation_static(s._h, 1)
    assert rc == -7 and b"static scratch" in lib.ones_strerror(rc)
    after = s.export(genes=False)
    assert before[3] == after[3] == 0 and np.array_equal(before[2], after[2])
    s.generation(1)
    assert s.export(genes=False)[3] == 1
    s.close()
