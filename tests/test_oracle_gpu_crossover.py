"""Pins for the oracle's uniform crossover over the GPUs: the paper's operator on its own
encoding (Section 3.2.2; Eq. 1 maps every GPU to the job whose worker it hosts)."""
from types import SimpleNamespace

import numpy as np
import pytest

import pyref
from pyref import check_invariants, make_jobs, random_jobs
from paper_2108_03645_amd import workloads as W


def test_hand_example(ref):
    """Six GPUs.  Parent A: job 0 on GPUs 0-3, job 1 on 4-5.  Parent B: job 1 on GPU 0, job 2 on
    1-2, GPUs 3-5 idle.  The coins come from Philox (recomputed here with Python integers); a head
    sends A's job to the first child and B's to the second."""
    seed, p0, t = 77, 12, 3
    w = pyref.philox4x32_10((0, p0, t, 3), (seed, 0))
    coin = [(w[0] >> i) & 1 for i in range(6)]
    gpu_a = [0, 0, 0, 0, 1, 1]
    gpu_b = [1, 2, 2, -1, -1, -1]
    want1, want2 = [0, 0, 0], [0, 0, 0]
    for i in range(6):
        first, second = (gpu_a[i], gpu_b[i]) if coin[i] else (gpu_b[i], gpu_a[i])
        if first >= 0:
            want1[first] += 1
        if second >= 0:
            want2[second] += 1
    n1, n2 = ref.gpu_crossover(seed, p0, t, 6, [4, 2, 0], [0, 1, 2])
    assert n1.tolist() == want1 and n2.tolist() == want2
    assert 0 < sum(coin) < 6                                  # the example exercises both outcomes


@pytest.mark.parametrize("G,n", [(1, 1), (6, 3), (64, 40), (100, 7), (127, 64), (128, 64), (129, 70), (1000, 333),
                                 (4096, 2048), (8192, 100)])
def test_every_gpu_goes_to_exactly_one_child(ref, G, n):
    rng = np.random.default_rng(G * 31 + n)
    for it in range(6):
        # parents that fill, underfill or (as after a table change) overfill the cluster
        scale = [0.5, 1.0, 1.7][it % 3]
        c_a = rng.multinomial(int(G * scale), rng.dirichlet(np.ones(n))).astype(np.int32)
        c_b = rng.multinomial(int(G * scale), rng.dirichlet(np.ones(n))).astype(np.int32)
        seed, p0, t = int(rng.integers(0, 2**63)), int(rng.integers(0, 2**20)), int(rng.integers(1, 2**31))
        n1, n2 = ref.gpu_crossover(seed, p0, t, G, c_a, c_b)
        # what lies inside the cluster: the leading GPUs in slot order
        inside = lambda c: np.diff(np.minimum(np.concatenate([[0], np.cumsum(c)]), G))
        assert (n1 + n2 == inside(c_a) + inside(c_b)).all()
        assert n1.sum() <= G and n2.sum() <= G                # Eq. 4 holds for both children as they are
        want1, want2 = pyref.gpu_crossover(seed, p0, t, G, c_a, c_b)
        assert n1.tolist() == want1 and n2.tolist() == want2
        # equal parents: both children equal them
        m1, m2 = ref.gpu_crossover(seed, p0, t, G, c_a, c_a)
        assert (m1 == inside(c_a)).all() and (m2 == inside(c_a)).all()
        # swapping the parents swaps the children
        s1, s2 = ref.gpu_crossover(seed, p0, t, G, c_b, c_a)
        assert (s1 == n2).all() and (s2 == n1).all()


def test_coins_are_fair_and_independent_of_the_neighbours(ref):
    """One job on all 4096 GPUs against an idle cluster: n1 is the number of heads."""
    G = 4096
    heads = np.array([ref.gpu_crossover(9, p0, 5, G, [G], [0])[0][0] for p0 in range(0, 800, 2)])
    z = (heads.mean() - G / 2) / np.sqrt(G / 4 / len(heads))
    assert abs(z) < 4.5
    assert abs(heads.var() / (G / 4) - 1) < 0.25              # binomial variance: coins are not tied together
    # per GPU: with one-GPU jobs n1[j] is the coin of GPU j
    ones = np.ones(G, np.int32)
    coins = np.array([ref.gpu_crossover(9, p0, 5, G, ones, np.zeros(G, np.int32))[0] for p0 in range(0, 600, 2)])
    freq = coins.mean(axis=0)
    assert abs(freq.mean() - 0.5) < 0.005 and freq.min() > 0.3 and freq.max() < 0.7
    # generation, slot and seed all enter the stream
    base = ref.gpu_crossover(9, 4, 5, G, ones, np.zeros(G, np.int32))[0]
    for args in [(10, 4, 5), (9, 6, 5), (9, 4, 6)]:
        assert (ref.gpu_crossover(*args, G, ones, np.zeros(G, np.int32))[0] != base).sum() > G // 3


def cluster(G, n, P, seed, theta=0.1):
    return SimpleNamespace(n_gpus=G, n_slots=n, population=P, seed=seed, mutation_rate=theta, crossover_rate=0.5)


def test_children_in_the_search_come_from_the_operator(ref):
    """compose of a crossover slot = the operator on the parents' GPU counts, rounded down to a
    power of two per job, at the job's local batch."""
    rng = np.random.default_rng(3)
    jobs = random_jobs(rng, 90)
    cl = cluster(200, 90, 64, seed=21)
    s = ref.RefSearch(cl, jobs)
    s.set_crossover(per_gpu=True)
    s.generation(2)
    genes, _, sel, t = s.export()
    K = cl.population // 4
    m = jobs.gpu_max_batch
    for p0 in range(K, 3 * K, 2):
        first, _, pa, pb = s.compose_slot(p0)
        second, _, pa2, pb2 = s.compose_slot(p0 + 1)
        assert (pa, pb) == (pa2, pb2) and pa in sel and pb in sel
        c_a = [pyref.gpus(genes[pa][j], m[j]) for j in range(90)]
        c_b = [pyref.gpus(genes[pb][j], m[j]) for j in range(90)]
        n1, n2 = pyref.gpu_crossover(cl.seed, p0, t + 1, cl.n_gpus, c_a, c_b)
        for child, counts in ((first, n1), (second, n2)):
            for j in range(90):
                if counts[j] == 0:
                    assert child[j] == 0
                else:
                    c = 1 << (counts[j].bit_length() - 1)
                    local = min(int(m[j]), int(jobs.bmax[j]))
                    assert child[j] == c * local
                # a child's job never has more GPUs than both parents together
                assert pyref.gpus(child[j], m[j]) <= c_a[j] + c_b[j] or child[j] == 0
    s.close()


@pytest.mark.parametrize("name", ["tiny", "paper_scale"])
def test_pool_invariants_with_the_crossover_over_gpus(ref, name):
    cl, jobs = W.CONFIGS[name]()
    a, b = ref.RefSearch(cl, jobs), ref.RefSearch(cl, jobs)
    a.set_crossover(per_gpu=True)
    best = []
    for gen in range(8):
        a.generation(1); b.generation(1)
        genes, fit, sel, _ = a.export()
        for p in range(0, cl.population, 7):
            check_invariants(cl.n_gpus, jobs, genes[p, :cl.n_slots])
        best.append(fit[sel[0]])
    assert all(x >= y for x, y in zip(best, best[1:]))        # elitism: the best score never gets worse
    ga, gb = a.export()[0], b.export()[0]
    K = cl.population // 4
    assert not np.array_equal(ga[K:3 * K], gb[K:3 * K])       # the operator really differs from the per-job one
    a.close(); b.close()


def test_mode_validation(ref):
    cl, jobs = W.tiny()
    s = ref.RefSearch(cl, jobs)
    with pytest.raises(ref.RefError):
        ref._check(ref.lib().ones_ref_set_crossover(s._h, 2))
    big = cluster(8193, 8, 16, seed=1)
    t = ref.RefSearch(big, make_jobs(8))
    with pytest.raises(ref.RefError) as e:
        t.set_crossover(per_gpu=True)
    assert e.value.code == -3
    t.set_crossover(per_gpu=False)
    ok = ref.RefSearch(cluster(8192, 8, 16, seed=1), make_jobs(8))
    ok.set_crossover(per_gpu=True)
    ok.generation(1)
    s.close(); t.close(); ok.close()


def test_parents_are_read_under_the_current_table(ref):
    """After a table change the parents' genes were written under the old table: a parent's job
    holds the GPUs that clamp and lift of the repair would give it under the new one (batch pulled
    into the new window and raised for free to the new per-GPU batch), an emptied slot none, and
    what does not fit the cluster lies beyond its last GPU."""
    rng = np.random.default_rng(8)
    n = 70
    jobs = random_jobs(rng, n)
    cl = cluster(60, n, 64, seed=5)
    s = ref.RefSearch(cl, jobs)
    s.set_crossover(per_gpu=True)
    s.generation(2)
    j2 = random_jobs(np.random.default_rng(9), n)             # other windows, per-GPU batches, empty slots
    j2.job_id[:] = jobs.job_id                                # same jobs: no slot is reset
    s.set_jobs(j2)
    genes, _, sel, t = s.export()
    K = cl.population // 4

    def gpus_under_new_table(b, j):
        if not j2.active[j] or b == 0:
            return 0
        b = min(max(int(b), int(j2.bmin[j])), int(j2.bmax[j]))
        b = max(b, min(int(j2.gpu_max_batch[j]), int(j2.bmax[j])))
        return pyref.gpus(b, j2.gpu_max_batch[j])

    lifted = 0
    for p0 in range(K, 3 * K, 2):
        first, _, pa, pb = s.compose_slot(p0)
        second = s.compose_slot(p0 + 1)[0]
        c_a = [gpus_under_new_table(genes[pa][j], j) for j in range(n)]
        c_b = [gpus_under_new_table(genes[pb][j], j) for j in range(n)]
        lifted += sum(1 for j in range(n) if genes[pa][j] and j2.active[j] and genes[pa][j] < min(j2.gpu_max_batch[j], j2.bmax[j]))
        n1, n2 = pyref.gpu_crossover(cl.seed, p0, t + 1, cl.n_gpus, c_a, c_b)
        for child, counts in ((first, n1), (second, n2)):
            for j in range(n):
                want = 0 if counts[j] == 0 else (1 << (counts[j].bit_length() - 1)) * min(int(j2.gpu_max_batch[j]), int(j2.bmax[j]))
                assert child[j] == want
    assert lifted > 0                                          # the case the lift matters for did occur
    s.generation(1)
    genes = s.export()[0]
    for p in range(cl.population):
        check_invariants(cl.n_gpus, j2, genes[p, :n])
    s.close()
