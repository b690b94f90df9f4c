"""GPU parity: libones (HIP, through the C ABI) against the CPU oracle on the same seeded
inputs.  Genomes and survivor lists must match bit for bit every generation; scores within
1e-12 relative (they are expected to be bit-identical too, which is asserted separately)."""
import sys
from types import SimpleNamespace

import numpy as np
import pytest

from paper_2108_03645_amd import workloads as W
from pyref import make_jobs, random_jobs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ones():
    from paper_2108_03645_amd import ones as binding
    binding.load()           # fails loudly if the library is not built
    return binding


def cluster(n_gpus, n_slots, population, seed=0, theta=0.1, chi=0.5):
    return SimpleNamespace(n_gpus=n_gpus, n_slots=n_slots, population=population, seed=seed,
                           mutation_rate=theta, crossover_rate=chi)


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def assert_same_state(gpu, cpu, where, genes=True):
    """genes=False leaves the genomes out (the scores and the survivor list still cover every candidate)."""
    g_genes, g_fit, g_sel, g_t = gpu.export(genes=genes)
    c_genes, c_fit, c_sel, c_t = cpu.export(genes=genes)
    assert g_t == c_t, where
    if genes:
        bad = np.flatnonzero((g_genes != c_genes).any(axis=1))
        assert bad.size == 0, f"{where}: genomes differ in {bad.size} slots, first {bad[:5]}"
    rel = np.abs(g_fit - c_fit) / np.maximum(np.abs(c_fit), 1e-300)
    assert rel.max() <= 1e-12 if rel.size else True, f"{where}: fitness off by {rel.max()}"
    assert np.array_equal(g_sel, c_sel), f"{where}: survivor lists differ"
    assert np.array_equal(g_fit.view(np.uint64), c_fit.view(np.uint64)), f"{where}: fitness bits differ"


def run_pair(ones, ref, cl, jobs, generations, every=1, label=""):
    say(f"[parity] {label}: G={cl.n_gpus} slots={cl.n_slots} P={cl.population} seed={cl.seed} gens={generations}")
    gpu = ones.Search(cl, jobs)
    cpu = ref.RefSearch(cl, jobs)
    assert_same_state(gpu, cpu, f"{label} generation 0")
    done = 0
    while done < generations:
        step = min(every, generations - done)
        gpu.generation(step)
        cpu.generation(step)
        done += step
        assert_same_state(gpu, cpu, f"{label} generation {done}")
    gb, gg, gf = gpu.best()
    cb, cg, cf = cpu.best()
    assert gb.tolist() == cb.tolist() and gg.tolist() == cg.tolist() and gf == cf
    gpu.close(); cpu.close()


def test_tiny_every_generation(ones, ref):
    cl, jobs = W.tiny()
    run_pair(ones, ref, cl, jobs, cl.generations, 1, "tiny")


def test_paper_scale(ones, ref):
    cl, jobs = W.paper_scale()
    run_pair(ones, ref, cl, jobs, cl.generations, 5, "paper_scale")


@pytest.mark.parametrize("n_slots,n_gpus,pop,seed", [
    (1, 3, 8, 1), (63, 40, 64, 2), (64, 64, 128, 3), (65, 100, 64, 4), (130, 90, 256, 5),
    (300, 500, 128, 6), (448, 300, 64, 7), (700, 5000, 64, 8), (1000, 1500, 128, 9),
    (1500, 800, 64, 10), (2048, 4096, 256, 11),
])
def test_ragged_shapes(ones, ref, n_slots, n_gpus, pop, seed):
    """Row counts 1..32 including odd ones, a ragged last row, inactive slots, mixed
    per-GPU batch sizes and windows."""
    rng = np.random.default_rng(seed)
    jobs = random_jobs(rng, n_slots)
    run_pair(ones, ref, cluster(n_gpus, n_slots, pop, seed=seed * 7919), jobs, 4, 1,
             f"ragged{n_slots}")


@pytest.mark.parametrize("rows", list(range(1, 33)))
def test_every_row_count(ones, ref, rows):
    rng = np.random.default_rng(100 + rows)
    n_slots = 64 * rows - int(rng.integers(0, 64))
    jobs = random_jobs(rng, n_slots)
    run_pair(ones, ref, cluster(int(n_slots * 1.3), n_slots, 32, seed=rows), jobs, 2, 1, f"rows{rows}")


def test_large_reduced_population(ones, ref):
    cl, jobs = W.large()
    cl.population = 2048
    run_pair(ones, ref, cl, jobs, 6, 2, "large/P=2048")


def test_stress_reduced_population(ones, ref):
    cl, jobs = W.stress(population=1024)
    run_pair(ones, ref, cl, jobs, 4, 2, "stress/P=1024")


@pytest.mark.parametrize("pop,n_jobs,n_gpus", [(4096 * 3 + 8, 6, 5), (4100, 6, 5), (5000, 9, 7), (8192, 12, 9),
                                               (20000, 5, 4)])
def test_selection_with_massive_ties(ones, ref, pop, n_jobs, n_gpus):
    """Pools larger than one LDS sort chunk with few distinct genomes, hence few distinct scores:
    single buckets overflow into the spill list and the scratch pool."""
    rng = np.random.default_rng(pop)
    jobs = make_jobs(n_jobs, bmin=256, bmax=512, remaining=rng.uniform(1e5, 1e7, n_jobs))
    run_pair(ones, ref, cluster(n_gpus, n_jobs, pop, seed=12), jobs, 4, 1, f"ties/P={pop}")


@pytest.mark.parametrize("pop", [4100, 8192, 20000, 40004])
def test_bucketed_selection_and_table_changes(ones, ref, pop):
    """Pools above one sort chunk select through survivor-quantile buckets while the job table
    stays the same and through the general sort right after it changed; alternate the two."""
    rng = np.random.default_rng(pop)
    jobs = random_jobs(rng, 130)
    cl = cluster(180, 130, pop, seed=pop)
    say(f"[parity] buckets: P={pop}")
    gpu = ones.Search(cl, jobs); cpu = ref.RefSearch(cl, jobs)
    ref.set_threads(8)
    try:
        for step in range(4):
            gpu.generation(2); cpu.generation(2)
            assert_same_state(gpu, cpu, f"buckets P={pop} step {step}")
            jobs.remaining = jobs.remaining * rng.uniform(0.5, 1.0, 130)     # progress: new table
            if step == 1:
                jobs.job_id[7] += 1000; jobs.active[9] ^= 1
            gpu.set_jobs(jobs); cpu.set_jobs(jobs)
            gpu.generation(1); cpu.generation(1)
            assert_same_state(gpu, cpu, f"buckets P={pop} step {step} after set_jobs")
    finally:
        ref.set_threads(1)
    gpu.close(); cpu.close()


@pytest.mark.parametrize("theta,chi", [(0.0, 0.0), (1.0, 1.0), (0.0, 1.0), (1.0, 0.5)])
def test_rate_extremes(ones, ref, theta, chi):
    rng = np.random.default_rng(21)
    jobs = random_jobs(rng, 100)
    run_pair(ones, ref, cluster(150, 100, 64, seed=5, theta=theta, chi=chi), jobs, 4, 1,
             f"theta={theta} chi={chi}")


def test_degenerate_clusters(ones, ref):
    run_pair(ones, ref, cluster(8, 0, 16), make_jobs(0), 2, 1, "no slots")
    run_pair(ones, ref, cluster(8, 10, 16), make_jobs(10, active=0), 2, 1, "all inactive")
    run_pair(ones, ref, cluster(0, 10, 16), make_jobs(10), 2, 1, "no GPUs")
    run_pair(ones, ref, cluster(1, 1, 4), make_jobs(1), 3, 1, "one job, one GPU, K=1")
    run_pair(ones, ref, cluster(1 << 20, 70, 8), make_jobs(70, bmin=1, bmax=1 << 28, gpu_max_batch=256),
             2, 1, "largest GPU counts")
    run_pair(ones, ref, cluster(40, 90, 8), make_jobs(90, bmin=2048, bmax=4096, gpu_max_batch=64),
             2, 1, "window above the per-GPU batch")
    run_pair(ones, ref, cluster(40, 90, 8), make_jobs(90, bmin=1, bmax=16, gpu_max_batch=512),
             2, 1, "window below the per-GPU batch")


def test_online_sequence(ones, ref):
    """Warm-started epochs: arrivals, completions, shrinking limits; both sides are driven by
    their own best schedule through the same cluster simulation."""
    sims = [W.OnlineSequence(epochs=40), W.OnlineSequence(epochs=40)]
    cl = sims[0].cluster
    cl.population = 512
    say(f"[parity] online: P={cl.population} epochs=40 gens/epoch=5")
    gpu = ones.Search(cl, sims[0].jobs)
    cpu = ref.RefSearch(cl, sims[1].jobs)
    for epoch in range(40):
        gpu.generation(5); cpu.generation(5)
        assert_same_state(gpu, cpu, f"online epoch {epoch}")
        gb, gg, gf = gpu.best(); cb, cg, cf = cpu.best()
        assert gb.tolist() == cb.tolist() and gg.tolist() == cg.tolist() and gf == cf
        sims[0].advance(gb); sims[1].advance(cb)
        assert sims[0].jobs.sha256() == sims[1].jobs.sha256()
        gpu.set_jobs(sims[0].jobs); cpu.set_jobs(sims[1].jobs)
        assert_same_state(gpu, cpu, f"online epoch {epoch} after set_jobs")
    assert sims[0].completed > 0
    gpu.close(); cpu.close()


@pytest.mark.parametrize("per_gpu", [False, True])
def test_online_sequence_with_limit_policies(ones, ref, per_gpu):
    """The online sequence with the batch-size limits of Section 3.3.2 (each side computes them
    with its own update_limits) and newly arrived jobs served first after every table change
    (refresh (3) of Section 3.2.2), the room for them taken from the longest runners; with the
    crossover over the jobs and over the GPUs."""
    sims = [W.OnlineSequence(epochs=40, limits=ones.update_limits), W.OnlineSequence(epochs=40, limits=ref.update_limits)]
    cl = sims[0].cluster
    cl.population = 512
    say(f"[parity] online with limit policies: P={cl.population} epochs=40 gens/epoch=5 per_gpu={per_gpu}")
    gpu = ones.Search(cl, sims[0].jobs)
    cpu = ref.RefSearch(cl, sims[1].jobs)
    gpu.set_new_jobs_first(True); cpu.set_new_jobs_first(True)
    gpu.set_crossover(per_gpu=per_gpu); cpu.set_crossover(per_gpu=per_gpu)
    limits_seen = set()
    for epoch in range(40):
        gpu.generation(5); cpu.generation(5)
        assert_same_state(gpu, cpu, f"online+policies epoch {epoch}")
        gb, gg, gf = gpu.best(); cb, cg, cf = cpu.best()
        assert gb.tolist() == cb.tolist() and gg.tolist() == cg.tolist() and gf == cf
        sims[0].advance(gb); sims[1].advance(cb)
        assert sims[0].jobs.sha256() == sims[1].jobs.sha256()
        limits_seen.update(sims[0].jobs.bmax[sims[0].jobs.active != 0].tolist())
        gpu.set_jobs(sims[0].jobs); cpu.set_jobs(sims[1].jobs)
        gpu.set_processed_time(sims[0].elapsed); cpu.set_processed_time(sims[1].elapsed)
        assert_same_state(gpu, cpu, f"online+policies epoch {epoch} after set_jobs")
    assert sims[0].completed > 0 and len(limits_seen) > 3      # the limits really moved
    gpu.close(); cpu.close()


def test_online_sequence_with_everything_on(ones, ref):
    """The whole loop at once: limit policies, new jobs first with executed times, the crossover
    over the GPUs, and the remaining work drawn per generation from the progress the simulated
    predictor reports (Alg. 1)."""
    sims = [W.OnlineSequence(epochs=30, limits=ones.update_limits), W.OnlineSequence(epochs=30, limits=ref.update_limits)]
    cl = sims[0].cluster
    cl.population = 1024
    say(f"[parity] online, everything on: P={cl.population} epochs=30 gens/epoch=4")
    gpu = ones.Search(cl, sims[0].jobs)
    cpu = ref.RefSearch(cl, sims[1].jobs)
    for s, sim in ((gpu, sims[0]), (cpu, sims[1])):
        s.set_new_jobs_first(True)
        s.set_crossover(per_gpu=True)
        s.set_progress(*sim.progress())
    for epoch in range(30):
        gpu.generation(4); cpu.generation(4)
        assert_same_state(gpu, cpu, f"online/all epoch {epoch}")
        assert np.array_equal(gpu.export_remaining(), cpu.export_remaining())
        gb, gg, gf = gpu.best(); cb, cg, cf = cpu.best()
        assert gb.tolist() == cb.tolist() and gg.tolist() == cg.tolist() and gf == cf
        sims[0].advance(gb); sims[1].advance(cb)
        assert sims[0].jobs.sha256() == sims[1].jobs.sha256()
        for s, sim in ((gpu, sims[0]), (cpu, sims[1])):
            s.set_jobs(sim.jobs)
            s.set_processed_time(sim.elapsed)
            s.set_progress(*sim.progress())
        assert_same_state(gpu, cpu, f"online/all epoch {epoch} after the updates")
    assert sims[0].completed > 0
    gpu.close(); cpu.close()


def test_set_jobs_rejects_bad_tables_and_keeps_state(ones, ref):
    rng = np.random.default_rng(31)
    jobs = random_jobs(rng, 64)
    cl = cluster(64, 64, 64, seed=3)
    gpu = ones.Search(cl, jobs); cpu = ref.RefSearch(cl, jobs)
    gpu.generation(2); cpu.generation(2)
    bad = SimpleNamespace(**{k: getattr(jobs, k).copy() for k in vars(jobs)})
    live = int(np.flatnonzero(jobs.active)[0])
    bad.bmin[live] = 48
    with pytest.raises(ones.OnesError) as e:
        gpu.set_jobs(bad)
    assert e.value.code == -2
    bad.bmin[live] = jobs.bmin[live]; bad.remaining[live] = float("nan")
    with pytest.raises(ones.OnesError) as e:
        gpu.set_jobs(bad)
    assert e.value.code == -4
    assert_same_state(gpu, cpu, "after rejected set_jobs")
    gpu.generation(1); cpu.generation(1)
    assert_same_state(gpu, cpu, "generation after rejected set_jobs")


def test_best_between_a_table_change_and_the_next_generation(ones, ref):
    """ones_best right after ones_set_jobs: no schedule exists under the new table yet; the call returns the
    last winner as stored (slots that changed hands already waiting) with the score it had under the old
    table, on both sides alike; ones_placement refuses in that state."""
    rng = np.random.default_rng(77)
    jobs = random_jobs(rng, 100, inactive_frac=0.0)
    cl = cluster(150, 100, 256, seed=9)
    gpu, cpu = ones.Search(cl, jobs), ref.RefSearch(cl, jobs)
    gpu.generation(4); cpu.generation(4)
    before = gpu.best()
    running = np.flatnonzero(before[0] > 0)
    assert running.size > 2
    jobs.job_id[running[:2]] += 500                                # two running jobs are replaced
    jobs.remaining = jobs.remaining * 0.5
    gpu.set_jobs(jobs); cpu.set_jobs(jobs)
    gb, cb = gpu.best(), cpu.best()
    assert gb[0].tolist() == cb[0].tolist() and gb[1].tolist() == cb[1].tolist() and gb[2] == cb[2]
    assert gb[2] == before[2] and (gb[0][running[:2]] == 0).all() and (gb[0][running[2:]] == before[0][running[2:]]).all()
    with pytest.raises(ones.OnesError) as e:
        gpu.placement()
    assert e.value.code == -1
    gpu.generation(1); cpu.generation(1)
    assert_same_state(gpu, cpu, "the generation after")
    assert gpu.best()[2] == cpu.best()[2] != before[2]
    gpu.close(); cpu.close()


def test_init_rejects_bad_arguments(ones):
    import torch
    jobs = make_jobs(4)
    with pytest.raises(ones.OnesError) as e:
        ones.Search(cluster(4, 4, 18), jobs)
    assert e.value.code == -1
    with pytest.raises(ones.OnesError) as e:
        ones.Search(cluster(4, 4, 16), make_jobs(4, bmin=64, bmax=32))
    assert e.value.code == -3
    # workspace too small / misaligned
    import ctypes as C
    cfg = ones.make_config(cluster(4, 4, 16))
    js, keep = ones.make_jobs(jobs)
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda:0")
    h = C.c_void_p()
    L = ones.load()
    ptr = (ws.data_ptr() + 255) & ~255
    assert L.ones_init(C.byref(h), C.byref(cfg), C.byref(js), C.c_void_p(ptr), 1024, None) == -5
    assert L.ones_init(C.byref(h), C.byref(cfg), C.byref(js), C.c_void_p(ptr + 4), 1 << 19, None) == -5
    assert h.value is None


def test_two_contexts_and_a_side_stream(ones, ref):
    import torch
    rng = np.random.default_rng(41)
    jobs = random_jobs(rng, 200)
    cl1, cl2 = cluster(256, 200, 64, seed=1), cluster(256, 200, 64, seed=2)
    side = torch.cuda.Stream()
    a = ones.Search(cl1, jobs)
    b = ones.Search(cl2, jobs, stream=side)
    ca, cb = ref.RefSearch(cl1, jobs), ref.RefSearch(cl2, jobs)
    for _ in range(3):
        a.generation(1); b.generation(1); ca.generation(1); cb.generation(1)
    assert_same_state(a, ca, "context a")
    assert_same_state(b, cb, "context b (side stream)")


# ---- pools of one job row: all generations of a call in one launch ----

@pytest.mark.parametrize("sampled", [False, True])
@pytest.mark.parametrize("n_slots,n_gpus,pop,seed,per_gpu,new_first", [
    (8, 16, 64, 0, False, False), (40, 64, 1024, 1, False, False), (64, 64, 2048, 2, False, True),
    (64, 200, 2048, 3, True, True), (33, 20, 68, 4, False, False), (5, 3, 4, 5, True, False), (17, 9, 8, 6, False, True),
    (60, 64, 1500, 7, True, False), (1, 1, 12, 8, False, False), (64, 4000, 600, 9, False, True)])
def test_single_launch_generations_with_mixed_call_lengths(ones, ref, n_slots, n_gpus, pop, seed, per_gpu, new_first,
                                                           sampled):
    """Calls of 1 and 2 generations take two launches per generation, longer ones a single launch
    for the whole call; the state one path leaves is the state the other starts from.  With table
    changes (the first generation of the next call refreshes the survivors), arrivals served first
    by executed time, both crossovers, and the remaining work fixed or drawn per generation (the
    draw of the last generation is what ones_export_remaining returns; switched off and on again
    half way)."""
    rng = np.random.default_rng(seed)
    cl = cluster(n_gpus, n_slots, pop, seed=seed + 77)
    jobs = random_jobs(rng, n_slots)
    say(f"[single launch] G={n_gpus} slots={n_slots} P={pop} seed={cl.seed} per_gpu={per_gpu} new_first={new_first} sampled={sampled}")
    gpu, cpu = ones.Search(cl, jobs), ref.RefSearch(cl, jobs)
    progress = W.progress(n_slots, seed=seed)
    for s in (gpu, cpu):
        s.set_crossover(per_gpu=per_gpu)
        s.set_new_jobs_first(new_first)
        if sampled:
            s.set_progress(*progress)
    assert_same_state(gpu, cpu, "initial population")
    for step, n in enumerate([5, 1, 3, 2, 20, 4, 1, 7, 3, 40]):
        gpu.generation(n); cpu.generation(n)
        assert_same_state(gpu, cpu, f"call {step} of {n} generations")
        assert np.array_equal(gpu.export_remaining().view(np.uint64), cpu.export_remaining().view(np.uint64)), f"call {step}"
        if sampled and step in (4, 6):                                # off before the call of 4, on again before the call of 7
            for s in (gpu, cpu):
                s.set_progress(*(progress if step == 6 else (None, None, None)))
        gb, cb = gpu.best(), cpu.best()
        assert gb[0].tolist() == cb[0].tolist() and gb[1].tolist() == cb[1].tolist() and gb[2] == cb[2]
        if step in (1, 3, 4, 6, 8):                                   # a new table before calls of 3, 20, 4, 7 and 40
            j2 = random_jobs(rng, n_slots) if step != 4 else jobs
            j2.job_id = np.where(rng.random(n_slots) < 0.6, jobs.job_id, jobs.job_id + 1000 * (step + 1))
            j2.remaining = j2.remaining * 0.9
            for s in (gpu, cpu):
                s.set_jobs(j2)
                if new_first and step != 6:
                    s.set_processed_time(rng_times(seed, step, n_slots))
            assert_same_state(gpu, cpu, f"table change after call {step}")
            jobs = j2
    assert all(np.array_equal(x, y) for x, y in zip(gpu.placement(), cpu.placement()))
    gpu.close(); cpu.close()


@pytest.mark.parametrize("name,calls,per_call", [("tiny", 10, 500), ("paper_scale", 8, 250)])
def test_single_launch_long_calls(ones, ref, name, calls, per_call):
    """Thousands of generations inside few launches: every exchange between the workgroups of a launch
    (scores, ranks) happens hundreds of times per call, and a single stale or early read would change the
    state the oracle reaches."""
    cl, jobs = W.CONFIGS[name]()
    say(f"[single launch] long calls: {name}, {calls} calls of {per_call} generations")
    ref.set_threads(host_threads())
    try:
        gpu, cpu = ones.Search(cl, jobs), ref.RefSearch(cl, jobs)
        for call in range(calls):
            if call == calls // 2:                   # a new table half way, so that the second half starts from a changed pool
                jobs.remaining = jobs.remaining * 0.7
                jobs.job_id[1] += 100
                gpu.set_jobs(jobs); cpu.set_jobs(jobs)
            gpu.generation(per_call); cpu.generation(per_call)
            assert_same_state(gpu, cpu, f"{name} after call {call}")
        gpu.close(); cpu.close()
    finally:
        ref.set_threads(1)


def rng_times(seed, step, n_slots):
    return np.random.default_rng([seed, step]).integers(0, 5, n_slots) * 60.0


def test_single_launch_waits_are_bounded(ones):
    """With a wait limit of 0 every workgroup gives up at its first wait for the others' results:
    the launch ends by itself, the next synchronising call reports the error and the context
    refuses further work."""
    cl, jobs = W.paper_scale()
    s = ones.Search(cl, jobs)
    s.generation(5)
    before = s.export(genes=False)
    assert before[3] == 5
    s.set_wait_limit(0)
    say("[single launch] wait limit 0")
    s.generation(5)                                  # asynchronous: the launch itself succeeds
    with pytest.raises(ones.OnesError) as e:
        s.best()
    assert e.value.code == -6 and b"gave up" in ones.load().ones_strerror(-6)
    for call in (lambda: s.generation(1), lambda: s.generation(5), s.best, s.export, s.placement):
        with pytest.raises(ones.OnesError) as e:
            call()
        assert e.value.code == -6
    s.close()
    # an untouched context is not affected
    s = ones.Search(cl, jobs)
    s.generation(5)
    assert np.array_equal(s.export(genes=False)[2], before[2])
    s.close()


# ---- the five configurations at their stated size and length ----

def host_threads():
    import os
    return min(16, os.cpu_count() or 1)


def test_online_config_at_full_size(ones, ref):
    """64 GPUs, 64 slots, pool 2048, 200 scheduling epochs of 20 warm-started generations each;
    every epoch the winner drives the simulated cluster and the job table is replaced.  The
    first epoch in which the two sides differ fails the test and is named."""
    sims = [W.OnlineSequence(), W.OnlineSequence()]
    cl = sims[0].cluster
    assert (cl.population, cl.n_slots, cl.n_gpus, cl.epochs, cl.generations) == (2048, 64, 64, 200, 20)
    say(f"[parity] online at full size: P={cl.population} epochs={cl.epochs} gens/epoch={cl.generations} seed={cl.seed}")
    ref.set_threads(host_threads())
    try:
        gpu = ones.Search(cl, sims[0].jobs)
        cpu = ref.RefSearch(cl, sims[1].jobs)
        busy = []
        for epoch in range(cl.epochs):
            gpu.generation(cl.generations); cpu.generation(cl.generations)
            assert_same_state(gpu, cpu, f"online, first divergent epoch {epoch} (after its generations)")
            gb, gg, gf = gpu.best(); cb, cg, cf = cpu.best()
            assert gb.tolist() == cb.tolist() and gg.tolist() == cg.tolist() and gf == cf, f"winner differs in epoch {epoch}"
            sims[0].advance(gb); sims[1].advance(cb)
            assert sims[0].jobs.sha256() == sims[1].jobs.sha256()
            busy.append(int(sims[0].jobs.active.sum()))
            gpu.set_jobs(sims[0].jobs); cpu.set_jobs(sims[1].jobs)
            assert_same_state(gpu, cpu, f"online, first divergent epoch {epoch} (after the table change)")
            if epoch % 50 == 49:
                say(f"[parity] online at full size: epoch {epoch + 1} done, {sims[0].completed} jobs completed")
        assert gpu.export(genes=False)[3] == cl.epochs * cl.generations
        assert sims[0].completed > 20 and min(busy) < max(busy)          # jobs came and went
        gpu.close(); cpu.close()
    finally:
        ref.set_threads(1)


@pytest.mark.parametrize("mode", ["plain", "sampled", "crossover over gpus"])
def test_large_config_at_full_length(ones, ref, mode):
    """1024 GPUs, 512 jobs, pool 16384: all 50 generations, every one compared in full."""
    cl, jobs = W.large()
    assert (cl.population, cl.n_slots, cl.n_gpus, cl.generations) == (16384, 512, 1024, 50)
    say(f"[parity] large at full length ({mode}): P={cl.population} gens={cl.generations} seed={cl.seed}")
    ref.set_threads(host_threads())
    try:
        gpu, cpu = ones.Search(cl, jobs), ref.RefSearch(cl, jobs)
        for s in (gpu, cpu):
            if mode == "sampled":
                s.set_progress(*W.progress(cl.n_slots, seed=cl.seed))
            s.set_crossover(per_gpu=mode == "crossover over gpus")
        assert_same_state(gpu, cpu, "large generation 0")
        for gen in range(1, cl.generations + 1):
            gpu.generation(1); cpu.generation(1)
            assert_same_state(gpu, cpu, f"large ({mode}) generation {gen}")
        gb, cb = gpu.best(), cpu.best()
        assert gb[0].tolist() == cb[0].tolist() and gb[1].tolist() == cb[1].tolist() and gb[2] == cb[2]
        gpu.close(); cpu.close()
    finally:
        ref.set_threads(1)


def test_stress_config_at_full_length(ones, ref):
    """4096 GPUs, 2048 jobs, pool 65536, the benchmark's launch configuration: all 20 generations.
    Scores (bit for bit) and survivor lists of every generation; the 512 MiB of genomes at
    generations 0, 1, 5, 10, 15 and 20."""
    cl, jobs = W.stress()
    assert (cl.population, cl.n_slots, cl.n_gpus, cl.generations) == (65536, 2048, 4096, 20)
    say(f"[parity] stress at full length: P={cl.population} gens={cl.generations} seed={cl.seed}")
    ref.set_threads(host_threads())
    try:
        gpu, cpu = ones.Search(cl, jobs), ref.RefSearch(cl, jobs)
        assert_same_state(gpu, cpu, "stress generation 0")
        for gen in range(1, cl.generations + 1):
            gpu.generation(1); cpu.generation(1)
            assert_same_state(gpu, cpu, f"stress generation {gen}", genes=gen in (1, 5, 10, 15, 20))
            say(f"[parity] stress at full length: generation {gen} matches")
        gb, cb = gpu.best(), cpu.best()
        assert gb[0].tolist() == cb[0].tolist() and gb[1].tolist() == cb[1].tolist() and gb[2] == cb[2]
        gpu.close(); cpu.close()
    finally:
        ref.set_threads(1)


def test_profile_hook_counts_launches(ones):
    cl = cluster(200, 130, 1024, seed=1)                 # two job rows: one evolve and one selection launch per generation
    jobs = random_jobs(np.random.default_rng(1), 130)
    s = ones.Search(cl, jobs)
    s.profile_enable(1)
    s.generation(7)
    prof = s.profile_read()
    assert prof["evolve_launches"] == 7 and prof["select_launches"] == 7
    assert prof["evolve_ms"] > 0 and prof["select_ms"] > 0
    s.profile_enable(3)                       # generations 0, 3, 6 of the next 8
    s.generation(8)
    assert s.profile_read()["evolve_launches"] == 3
    s.profile_enable(0)
    s.generation(1)
    assert s.profile_read()["evolve_launches"] == 0
    s.close()
    # a pool of at most 64 job slots and 2048 candidates runs a whole call in one launch
    cl, jobs = W.paper_scale()
    s = ones.Search(cl, jobs)
    s.profile_enable(1)
    s.generation(7)
    s.generation(3)
    prof = s.profile_read()
    assert prof["evolve_launches"] == 2 and prof["select_launches"] == 0 and prof["evolve_ms"] > 0
    s.generation(1)                           # a call of one or two generations takes two launches per generation
    prof = s.profile_read()
    assert prof["evolve_launches"] == 3 and prof["select_launches"] == 1
    s.close()


# ------------------------------------------------ probability sampling (Alg. 1, Eq. 7) ----
def test_sampled_remaining_work_matches_the_oracle_bit_for_bit(ones, ref):
    """Every slot's draw, over several generations, for shapes from 1 to 1e100."""
    n = 2048
    rng = np.random.default_rng(21)
    cl = cluster(256, n, 64, seed=0xFEEDFACE12345678)
    jobs = random_jobs(rng, n)
    alpha = np.exp(rng.uniform(0, 12, n)); beta = np.exp(rng.uniform(0, 12, n))
    proc = rng.uniform(0, 1e7, n)
    alpha[:8] = [1.0, 1.0, 1.0000000001, 1e100, 1e100, 1.0, 3.5, 1e6]
    beta[:8] = [1.0, 1e100, 1.0, 1.0, 1e100, 1.0000000001, 1e6, 3.5]
    proc[:8] = [0.0, 1e100, 1e100, 1e100, 1.0, 5.0, 1e100, 0.0]
    say(f"[sampling] draws: slots={n} seed={cl.seed:#x}")
    gpu = ones.Search(cl, jobs)
    gpu.set_progress(alpha, beta, proc)
    for step in range(4):
        gpu.generation(1 if step else 3)
        t = gpu.export(genes=False)[3]
        got = gpu.export_remaining()
        want = np.array([ref.sampled_remaining(cl.seed, j, t, alpha[j], beta[j], proc[j])[0] for j in range(n)])
        bad = np.flatnonzero(got.view(np.uint64) != want.view(np.uint64))
        assert bad.size == 0, f"generation {t}: {bad.size} draws differ, first slots {bad[:5]}"
    gpu.close()


@pytest.mark.parametrize("name", ["tiny", "paper_scale", "ragged", "buckets"])
def test_sampled_search_matches_the_oracle(ones, ref, name):
    """Sampling switched on after a few generations, a job-table change under it, switched
    off again: genomes, scores and survivor lists agree after every call."""
    if name == "tiny":
        cl, jobs = W.tiny()
    elif name == "paper_scale":
        cl, jobs = W.paper_scale()
    elif name == "ragged":
        cl = cluster(700, 333, 512, seed=31)
        jobs = random_jobs(np.random.default_rng(31), 333)
    else:
        cl = cluster(300, 200, 8192, seed=32)                  # large enough for the bucketed selection
        jobs = random_jobs(np.random.default_rng(32), 200)
    alpha, beta, proc = W.progress(cl.n_slots, seed=5)
    say(f"[sampling] search {name}: G={cl.n_gpus} slots={cl.n_slots} P={cl.population} seed={cl.seed}")
    gpu, cpu = ones.Search(cl, jobs), ref.RefSearch(cl, jobs)

    def both(call, where):
        call(gpu); call(cpu)
        assert_same_state(gpu, cpu, f"{name} {where}")
        assert np.array_equal(gpu.export_remaining().view(np.uint64), cpu.export_remaining().view(np.uint64)), where

    both(lambda s: s.generation(3), "fixed remaining work")
    both(lambda s: s.set_progress(alpha, beta, proc), "sampling on")
    for i in range(4):
        both(lambda s: s.generation(1), f"sampled generation {i}")
    both(lambda s: s.generation(5), "five sampled generations")
    # the progress moves on while draws made ahead of it are still waiting to be used
    alpha2, beta2, proc2 = W.progress(cl.n_slots, seed=6)
    both(lambda s: s.set_progress(alpha2, beta2, proc2), "new progress under sampling")
    both(lambda s: s.generation(2), "sampled generations with the new progress")
    # a slot changes hands and another job's window shrinks while sampling is on
    j2 = make_jobs(cl.n_slots, **{k: np.array(getattr(jobs, k)) for k in
                                  ("job_id", "active", "bmin", "bmax", "gpu_max_batch", "a", "c", "d", "remaining")})
    j2.job_id[0] += 1000
    j2.bmax[cl.n_slots - 1] = j2.bmin[cl.n_slots - 1]
    both(lambda s: s.set_jobs(j2), "table change under sampling")
    both(lambda s: s.generation(1), "first generation after the table change")
    both(lambda s: s.generation(2), "sampled generations after the table change")
    both(lambda s: s.set_progress(), "sampling off")
    both(lambda s: s.generation(1), "first generation with the table's remaining work")
    both(lambda s: s.generation(3), "fixed remaining work again")
    gb, cb = gpu.best(), cpu.best()
    assert gb[0].tolist() == cb[0].tolist() and gb[1].tolist() == cb[1].tolist() and gb[2] == cb[2]
    gpu.close(); cpu.close()


def test_set_progress_rejects_bad_arguments_and_keeps_state(ones, ref):
    cl, jobs = W.tiny()
    gpu, cpu = ones.Search(cl, jobs), ref.RefSearch(cl, jobs)
    n = cl.n_slots
    one, proc = np.ones(n), np.full(n, 1e5)
    for bad, code in [((np.full(n, 0.5), one, proc), -1), ((one, np.full(n, 0.99), proc), -1),
                      ((one, one, np.full(n, -1.0)), -1), ((np.full(n, np.nan), one, proc), -4),
                      ((one, np.full(n, np.inf), proc), -4), ((np.full(n, 1e101), one, proc), -3),
                      ((one, one, np.full(n, 1e101)), -3)]:
        with pytest.raises(ones.OnesError) as e:
            gpu.set_progress(*bad)
        assert e.value.code == code
    lib = ones.load()
    assert lib.ones_set_progress(gpu._h, one.ctypes.data, None, proc.ctypes.data) == -1
    assert lib.ones_export_remaining(gpu._h, None) == -1
    gpu.generation(2); cpu.generation(2)
    assert_same_state(gpu, cpu, "after rejected calls")
    gpu.close(); cpu.close()


def test_full_size_stress_with_sampled_remaining_work_matches_oracle(ones, ref):
    """The launch configuration of `bench.py --sampled`: pool 65536, 2048 jobs, remaining work
    drawn every generation (the survivors are scored again in place, general selection)."""
    import os
    cl, jobs = W.stress()
    alpha, beta, proc = W.progress(cl.n_slots, seed=cl.seed)
    ref.set_threads(min(16, os.cpu_count() or 1))
    say(f"[sampling] stress full size: P={cl.population} slots={cl.n_slots} seed={cl.seed}")
    try:
        gpu, cpu = ones.Search(cl, jobs), ref.RefSearch(cl, jobs)
        for s in (gpu, cpu):
            s.generation(1)
            s.set_progress(alpha, beta, proc)
        for i in range(2):
            gpu.generation(1); cpu.generation(1)
            assert_same_state(gpu, cpu, f"stress sampled generation {i + 1}")
        assert np.array_equal(gpu.export_remaining().view(np.uint64), cpu.export_remaining().view(np.uint64))
        gpu.close(); cpu.close()
    finally:
        ref.set_threads(1)


def test_shares_of_more_than_one_round(ones, ref):
    """A pool so large that a workgroup's share of the ranks exceeds what it lists free rows for at
    a time (more than 256 ranks per workgroup at 18 rows), with a table change in between."""
    import os
    cl = cluster(3000, 1100, 280000, seed=41)
    jobs = random_jobs(np.random.default_rng(41), 1100)
    ref.set_threads(min(16, os.cpu_count() or 1))
    say(f"[parity] large shares: P={cl.population} slots={cl.n_slots} seed={cl.seed}")
    try:
        gpu, cpu = ones.Search(cl, jobs), ref.RefSearch(cl, jobs)
        assert_same_state(gpu, cpu, "large shares generation 0")
        gpu.generation(1); cpu.generation(1)
        assert_same_state(gpu, cpu, "large shares generation 1")
        j2 = make_jobs(cl.n_slots, **{k: np.array(getattr(jobs, k)) for k in
                                      ("job_id", "active", "bmin", "bmax", "gpu_max_batch", "a", "c", "d", "remaining")})
        j2.job_id[5] += 7
        j2.remaining[:] = j2.remaining * 0.9
        gpu.set_jobs(j2); cpu.set_jobs(j2)
        gpu.generation(1); cpu.generation(1)
        assert_same_state(gpu, cpu, "large shares after a table change")
        gpu.generation(1); cpu.generation(1)
        assert_same_state(gpu, cpu, "large shares, bucketed generation")
        gpu.close(); cpu.close()
    finally:
        ref.set_threads(1)


def test_largest_population(ones, ref):
    """P = 2^20, the largest pool the interface accepts (few job slots, so that the oracle keeps up)."""
    import os
    cl = cluster(9, 6, 1 << 20, seed=43)
    jobs = random_jobs(np.random.default_rng(43), 6, inactive_frac=0.0)
    ref.set_threads(min(16, os.cpu_count() or 1))
    say(f"[parity] largest population: P={cl.population} slots={cl.n_slots} seed={cl.seed}")
    try:
        gpu, cpu = ones.Search(cl, jobs), ref.RefSearch(cl, jobs)
        assert_same_state(gpu, cpu, "largest population generation 0")
        gpu.generation(2); cpu.generation(2)
        assert_same_state(gpu, cpu, "largest population generation 2")
        alpha, beta, proc = W.progress(cl.n_slots, seed=43)
        gpu.set_progress(alpha, beta, proc); cpu.set_progress(alpha, beta, proc)
        gpu.generation(1); cpu.generation(1)
        assert_same_state(gpu, cpu, "largest population, sampled remaining work")
        gpu.close(); cpu.close()
    finally:
        ref.set_threads(1)


@pytest.mark.parametrize("n_slots,n_gpus,pop,seed", [(8, 16, 64, 0), (40, 64, 256, 1), (333, 700, 128, 2),
                                                     (2048, 4096, 64, 3), (1500, 100000, 64, 4), (5, 0, 16, 5),
                                                     (2048, 1 << 20, 16, 6)])
def test_placement_matches_the_oracle(ones, ref, n_slots, n_gpus, pop, seed):
    """Eq. 1 for the winner (slot and batch per GPU), from few GPUs to the largest cluster."""
    cl = cluster(n_gpus, n_slots, pop, seed=seed)
    jobs = random_jobs(np.random.default_rng(seed), n_slots)
    say(f"[placement] G={n_gpus} slots={n_slots} P={pop} seed={seed}")
    gpu, cpu = ones.Search(cl, jobs), ref.RefSearch(cl, jobs)
    for gens in (0, 2):
        gpu.generation(gens); cpu.generation(gens)
        gs, gb = gpu.placement()
        cs, cb = cpu.placement()
        assert np.array_equal(gs, cs) and np.array_equal(gb, cb)
        batch, gpus, _ = gpu.best()
        assert int((gs >= 0).sum()) == int(gpus.sum())
    gpu.set_jobs(jobs); cpu.set_jobs(jobs)
    with pytest.raises(ones.OnesError) as e:
        gpu.placement()
    assert e.value.code == -1
    gpu.generation(1); cpu.generation(1)
    assert np.array_equal(gpu.placement()[0], cpu.placement()[0])
    gpu.close(); cpu.close()


@pytest.mark.parametrize("n_slots,n_gpus,pop,seed,n_new", [(8, 3, 64, 0, 6), (40, 64, 1024, 1, 3), (333, 700, 512, 2, 40),
                                                           (2048, 4096, 256, 3, 300), (2048, 100, 64, 4, 500),
                                                           (200, 300, 8192, 5, 17)])
@pytest.mark.parametrize("times", ["none", "ties", "distinct"])
@pytest.mark.parametrize("per_gpu", [False, True])
def test_new_jobs_first_matches_the_oracle(ones, ref, n_slots, n_gpus, pop, seed, n_new, times, per_gpu):
    """The option of serving arrived jobs first: the generation after the table change and the
    ordinary ones that follow, with more and with fewer new jobs than GPUs; the others admitted
    in visiting order or by executed time (many equal times, or all distinct)."""
    rng = np.random.default_rng(seed)
    cl = cluster(n_gpus, n_slots, pop, seed=seed)
    jobs = random_jobs(rng, n_slots)
    say(f"[new first] G={n_gpus} slots={n_slots} P={pop} seed={seed} new={n_new} times={times} per_gpu={per_gpu}")
    gpu, cpu = ones.Search(cl, jobs), ref.RefSearch(cl, jobs)
    for s in (gpu, cpu):
        s.set_new_jobs_first(True)
        s.set_crossover(per_gpu=per_gpu)
        s.generation(3)
    assert_same_state(gpu, cpu, "before the arrivals")
    j2 = make_jobs(n_slots, **{k: np.array(getattr(jobs, k)) for k in
                               ("job_id", "active", "bmin", "bmax", "gpu_max_batch", "a", "c", "d", "remaining")})
    arrived = rng.choice(n_slots, size=min(n_new, n_slots), replace=False)
    j2.job_id[arrived] += 100000
    j2.active[arrived[: len(arrived) // 2]] = 1
    for step in range(2):
        gpu.set_jobs(j2); cpu.set_jobs(j2)
        if times != "none":
            t_processed = rng.integers(0, 4, n_slots) * 60.0 if times == "ties" else rng.permutation(n_slots) * 1.5
            gpu.set_processed_time(t_processed); cpu.set_processed_time(t_processed)
        assert_same_state(gpu, cpu, "after the table change")
        gpu.generation(1); cpu.generation(1)
        assert_same_state(gpu, cpu, "the generation that serves the new jobs")
        gpu.generation(2); cpu.generation(2)
        assert_same_state(gpu, cpu, "ordinary generations after it")
        j2.job_id[arrived[:3]] += 7                                   # a few of them are replaced again
    for s in (gpu, cpu):
        s.set_processed_time(None)
        s.set_jobs(jobs)
        s.generation(1)
    assert_same_state(gpu, cpu, "times forgotten")
    for s in (gpu, cpu):
        s.set_new_jobs_first(False)
        s.set_jobs(j2)
        s.generation(1)
    assert_same_state(gpu, cpu, "option off again")
    gpu.close(); cpu.close()


def test_set_processed_time_rejects_bad_arguments(ones, ref):
    cl, jobs = W.tiny()
    gpu, cpu = ones.Search(cl, jobs), ref.RefSearch(cl, jobs)
    good = np.arange(cl.n_slots, dtype=np.float64)
    for slot, value in [(2, -1.0), (0, float("nan")), (5, float("inf")), (1, 1e101)]:
        bad = good.copy(); bad[slot] = value
        with pytest.raises(ones.OnesError) as g:
            gpu.set_processed_time(bad)
        with pytest.raises(ref.RefError) as c:
            cpu.set_processed_time(bad)
        assert g.value.code == c.value.code
    gpu.generation(2); cpu.generation(2)
    assert_same_state(gpu, cpu, "after rejected times")
    gpu.close(); cpu.close()


# ---- uniform crossover over the GPUs of the paper's encoding (Section 3.2.2, Eq. 1) ----

@pytest.mark.parametrize("n_slots,n_gpus,pop,seed", [(1, 1, 8, 7), (8, 3, 64, 0), (40, 64, 1024, 1), (333, 700, 512, 2),
                                                     (700, 129, 256, 8), (64, 127, 8192, 6), (100, 8191, 128, 5),
                                                     (2048, 4096, 256, 3), (2048, 8192, 64, 4), (1500, 33, 64, 9)])
def test_crossover_over_gpus_matches_the_oracle(ones, ref, n_slots, n_gpus, pop, seed):
    """Ordinary generations, a table change (parents that overfill the cluster under the new
    table), sampled remaining work, and back to the crossover over the jobs."""
    rng = np.random.default_rng(seed)
    cl = cluster(n_gpus, n_slots, pop, seed=seed)
    jobs = random_jobs(rng, n_slots)
    say(f"[crossover over GPUs] G={n_gpus} slots={n_slots} P={pop} seed={seed}")
    gpu, cpu = ones.Search(cl, jobs), ref.RefSearch(cl, jobs)

    def both(f, where):
        f(gpu); f(cpu)
        assert_same_state(gpu, cpu, where)

    both(lambda s: s.set_crossover(per_gpu=True), "mode set")
    for gen in range(3):
        both(lambda s: s.generation(1), f"generation {gen + 1}")
    j2 = random_jobs(np.random.default_rng(seed + 100), n_slots)      # other windows and per-GPU batches
    j2.job_id[: n_slots // 2] = jobs.job_id[: n_slots // 2]           # half of the jobs stay
    both(lambda s: s.set_jobs(j2), "table change")
    both(lambda s: s.generation(1), "generation after the table change")
    both(lambda s: s.generation(2), "two more")
    alpha, beta, proc = W.progress(n_slots, seed=seed)
    both(lambda s: s.set_progress(alpha, beta, proc), "sampling on")
    both(lambda s: s.generation(2), "sampled generations")
    both(lambda s: s.set_progress(), "sampling off")
    both(lambda s: s.generation(1), "fixed remaining work again")
    both(lambda s: s.set_crossover(per_gpu=False), "back to the jobs")
    both(lambda s: s.generation(2), "crossover over the jobs again")
    gpu.close(); cpu.close()


def test_crossover_over_gpus_needs_a_small_enough_cluster(ones, ref):
    cl = cluster(8193, 16, 64, seed=1)
    jobs = random_jobs(np.random.default_rng(1), 16)
    gpu, cpu = ones.Search(cl, jobs), ref.RefSearch(cl, jobs)
    with pytest.raises(ones.OnesError) as g:
        gpu.set_crossover(per_gpu=True)
    with pytest.raises(ref.RefError) as c:
        cpu.set_crossover(per_gpu=True)
    assert g.value.code == c.value.code == -3
    assert ones.load().ones_set_crossover(gpu._h, 2) == -1
    gpu.generation(1); cpu.generation(1)
    assert_same_state(gpu, cpu, "after the rejected mode")
    gpu.close(); cpu.close()


def test_full_size_stress_with_the_crossover_over_gpus(ones, ref):
    """The benchmark's launch configuration (2048 jobs, 4096 GPUs, pool 65536) in this mode."""
    import os
    cl, jobs = W.stress()
    say(f"[parity] stress full size, crossover over GPUs: P={cl.population}")
    ref.set_threads(min(16, os.cpu_count() or 1))
    try:
        gpu, cpu = ones.Search(cl, jobs), ref.RefSearch(cl, jobs)
        for s in (gpu, cpu):
            s.set_crossover(per_gpu=True)
            s.generation(2)
        assert_same_state(gpu, cpu, "stress, crossover over GPUs, generation 2")
        gpu.close(); cpu.close()
    finally:
        ref.set_threads(1)


def test_crossover_over_gpus_on_degenerate_clusters(ones, ref):
    for cl, jobs, label in [(cluster(8, 0, 16), make_jobs(0), "no slots"),
                            (cluster(8, 10, 16), make_jobs(10, active=0), "all inactive"),
                            (cluster(0, 10, 16), make_jobs(10), "no GPUs"),
                            (cluster(1, 1, 4), make_jobs(1), "one job, one GPU, K=1"),
                            (cluster(8192, 70, 8), make_jobs(70, bmin=1, bmax=1 << 28, gpu_max_batch=256), "huge jobs"),
                            (cluster(40, 90, 8), make_jobs(90, bmin=2048, bmax=4096, gpu_max_batch=64),
                             "window above the per-GPU batch")]:
        say(f"[crossover over GPUs] {label}")
        gpu, cpu = ones.Search(cl, jobs), ref.RefSearch(cl, jobs)
        gpu.set_crossover(per_gpu=True); cpu.set_crossover(per_gpu=True)
        for gen in range(3):
            gpu.generation(1); cpu.generation(1)
            assert_same_state(gpu, cpu, f"{label} generation {gen + 1}")
        gpu.close(); cpu.close()


@pytest.mark.parametrize("block", range(4))
def test_random_configurations(ones, ref, block):
    """Seeded random shapes, rates and modes (crossover over jobs or GPUs, sampled remaining
    work, new jobs first, executed times), each with two table changes and a placement."""
    ref.set_threads(8)
    try:
        for case in range(20 * block, 20 * block + 20):
            rng = np.random.default_rng(10_000 + case)
            n_slots = int(rng.choice([rng.integers(1, 65), rng.integers(1, 400), rng.integers(1, 2049)]))
            n_gpus = int(rng.choice([rng.integers(0, 20), rng.integers(0, 300), rng.integers(0, 8193),
                                     rng.integers(0, 3 * n_slots + 1)]))
            pop = 4 * int(rng.choice([rng.integers(1, 17), rng.integers(1, 300), rng.integers(1, 1200),
                                      rng.integers(1000, 3000), rng.integers(1000, 6000)]))
            pop = min(pop, 2048) if n_slots > 512 else min(pop, 8192) if n_slots > 128 else pop
            cl = cluster(n_gpus, n_slots, pop, seed=int(rng.integers(0, 2**62)),
                         theta=float(rng.choice([0.0, 0.02, 0.1, 0.5, 1.0])), chi=float(rng.choice([0.0, 0.3, 0.5, 1.0])))
            per_gpu, sampled, new_first, times = (bool(rng.integers(0, 2)) for _ in range(4))
            jobs = random_jobs(rng, n_slots)
            tag = (f"random {case}: slots={n_slots} G={n_gpus} P={pop} theta={cl.mutation_rate} chi={cl.crossover_rate} "
                   f"per_gpu={per_gpu} sampled={sampled} new_first={new_first} times={times}")
            say(f"[parity] {tag}")
            gpu, cpu = ones.Search(cl, jobs), ref.RefSearch(cl, jobs)
            assert_same_state(gpu, cpu, tag + " initial population")
            for s in (gpu, cpu):
                s.set_crossover(per_gpu=per_gpu)
                s.set_new_jobs_first(new_first)
                if sampled:
                    s.set_progress(*W.progress(n_slots, seed=case))
            for step in range(3):
                n = int(rng.integers(1, 4))
                gpu.generation(n); cpu.generation(n)
                assert_same_state(gpu, cpu, tag + f" step {step}")
                assert gpu.best()[0].tolist() == cpu.best()[0].tolist()
                if step == 2:
                    assert all(np.array_equal(x, y) for x, y in zip(gpu.placement(), cpu.placement())), tag
                    break
                j2 = random_jobs(rng, n_slots) if rng.random() < 0.5 else jobs
                j2.job_id = np.where(rng.random(n_slots) < 0.7, jobs.job_id, jobs.job_id + 5000 * (step + 1))
                t_processed = rng.integers(0, 6, n_slots) * 60.0
                for s in (gpu, cpu):
                    s.set_jobs(j2)
                    if times:
                        s.set_processed_time(t_processed)
                assert_same_state(gpu, cpu, tag + f" table change {step}")
                jobs = j2
            gpu.close(); cpu.close()
    finally:
        ref.set_threads(1)


@pytest.mark.parametrize("block", range(2))
def test_random_selections_of_larger_pools(ones, ref, block):
    """Seeded random pools above the size one launch ranks (4100 to 72000 candidates), a third of
    them with a handful of distinct scores (6 to 11 jobs on a few GPUs): the sample sort and the
    quantile buckets with small, counted, sorted and oversized buckets, with the remaining work
    fixed or sampled, the scratch in the workspace or in the static array, a table change in
    between.  Scores and survivor lists are compared after every call."""
    ref.set_threads(8)
    try:
        for case in range(30 * block, 30 * block + 30):
            rng = np.random.default_rng(77_000 + case)
            ties = rng.random() < 0.3
            n_slots = int(rng.integers(3, 12)) if ties else int(rng.integers(1, 200))
            n_gpus = int(rng.integers(1, 12)) if ties else int(rng.integers(1, 400))
            pop = 4 * int(rng.choice([rng.integers(1025, 1100), rng.integers(1025, 4000), rng.integers(4000, 18000)]))
            cl = cluster(n_gpus, n_slots, pop, seed=int(rng.integers(0, 2**62)),
                         theta=float(rng.choice([0.02, 0.1, 0.5, 1.0])), chi=float(rng.choice([0.0, 0.3, 0.5, 1.0])))
            sampled, static, per_gpu = (bool(rng.integers(0, 2)) for _ in range(3))
            jobs = (make_jobs(n_slots, bmin=256, bmax=512, remaining=rng.uniform(1e5, 1e7, n_slots)) if ties
                    else random_jobs(rng, n_slots))
            tag = (f"selection {case}: slots={n_slots} G={n_gpus} P={pop} theta={cl.mutation_rate} chi={cl.crossover_rate} "
                   f"ties={ties} sampled={sampled} static={static} per_gpu={per_gpu}")
            say(f"[parity] {tag}")
            gpu, cpu = ones.Search(cl, jobs), ref.RefSearch(cl, jobs)
            assert_same_state(gpu, cpu, tag + " initial population", genes=False)
            for s in (gpu, cpu):
                s.set_crossover(per_gpu=per_gpu)
                if sampled:
                    s.set_progress(*W.progress(n_slots, seed=case))
            for step in range(3):
                n = int(rng.integers(1, 5))
                call = gpu.generation_static if static and rng.random() < 0.7 else gpu.generation
                try:
                    call(n)
                except ones.OnesError as e:                  # the pool's scratch does not fit the static array
                    assert e.code == -7 and call == gpu.generation_static
                    gpu.generation(n)
                cpu.generation(n)
                assert_same_state(gpu, cpu, tag + f" step {step}", genes=step == 2)
                if step == 1 and rng.random() < 0.5:
                    jobs.remaining = jobs.remaining * rng.uniform(0.5, 1.0, n_slots)
                    gpu.set_jobs(jobs); cpu.set_jobs(jobs)
            gb, cb = gpu.best(), cpu.best()
            assert gb[0].tolist() == cb[0].tolist() and gb[2] == cb[2], tag
            gpu.close(); cpu.close()
    finally:
        ref.set_threads(1)
