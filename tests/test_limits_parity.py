"""libones' ones_update_limits (host code, no device work) against the oracle's on random
cluster states.  Needs the built library but no GPU."""
import os

import numpy as np
import pytest


@pytest.fixture(scope="module")
def ones():
    from paper_2108_03645_amd import ones as binding
    if not os.path.exists(binding.library_path()):
        pytest.skip("libones.so not built here")
    binding.load()
    return binding


def random_state(rng, n):
    lo = rng.integers(2, 9, n)
    hi = lo + rng.integers(0, 8, n)
    return dict(state=rng.integers(0, 4, n), bmin=1 << lo, bcap=1 << hi, gpu_max_batch=1 << rng.integers(4, 10, n),
                last_batch=np.where(rng.random(n) < 0.5, 0, 1 << rng.integers(2, 14, n)),
                finished_epoch=rng.integers(0, 2, n), elapsed=rng.uniform(0, 20000, n))


@pytest.mark.parametrize("n", [0, 1, 7, 64, 500, 2048])
def test_random_states(ones, ref, n):
    rng = np.random.default_rng(n)
    for sigma in (0.0, 1e-4, 0.01, 3.0):
        arrays = random_state(rng, n)
        limit = (1 << rng.integers(0, 14, n)).astype(np.int32)
        got = ones.update_limits(limit, sigma, **arrays)
        want = ref.update_limits(limit, sigma, **arrays)
        assert np.array_equal(got, want)
        # a second epoch from the produced limits
        assert np.array_equal(ones.update_limits(got, sigma, **arrays), ref.update_limits(want, sigma, **arrays))


def test_rejections_agree_and_leave_the_limits_alone(ones, ref):
    rng = np.random.default_rng(9)
    n = 12
    good = random_state(rng, n)
    good["state"][:] = 3
    limit = np.full(n, 64, np.int32)
    for key, value, code in [("state", 4, -1), ("bmin", 24, -2), ("bcap", 1, -3), ("elapsed", -1.0, -1),
                             ("elapsed", np.inf, -4), ("last_batch", -5, None)]:
        bad = {k: np.array(v) for k, v in good.items()}
        bad[key] = bad[key].astype(np.float64 if isinstance(value, float) else bad[key].dtype)
        bad[key][5] = value
        if key == "last_batch":
            bad["state"][5] = 2
        before = limit.copy()
        with pytest.raises(ones.OnesError) as g:
            ones.update_limits(limit, 0.01, **bad)
        with pytest.raises(ref.RefError) as c:
            ref.update_limits(limit, 0.01, **bad)
        assert g.value.code == c.value.code and (code is None or g.value.code == code)
        assert np.array_equal(limit, before)
    with pytest.raises(ones.OnesError):
        ones.update_limits(limit, -0.5, **good)
    lib = ones.load()
    assert lib.ones_update_limits(3, None, 0.1, limit.ctypes.data) == -1
    assert lib.ones_update_limits(-1, None, 0.1, None) == -1
    assert lib.ones_update_limits(0, None, 0.1, None) == 0


def test_online_sequence_is_the_same_under_either_implementation(ones, ref):
    """The simulated cluster driven by the oracle's search, once with the library's limits and
    once with the oracle's: identical job tables at every epoch, and the limits do move."""
    from paper_2108_03645_amd import workloads as W
    sims = [W.OnlineSequence(epochs=25, limits=ones.update_limits), W.OnlineSequence(epochs=25, limits=ref.update_limits)]
    cl = sims[1].cluster
    cl.population = 128
    search = ref.RefSearch(cl, sims[1].jobs)
    search.set_new_jobs_first(True)
    seen = set()
    for epoch in range(25):
        search.generation(3)
        batch, _, _ = search.best()
        for sim in sims:
            sim.advance(batch)
        assert sims[0].jobs.sha256() == sims[1].jobs.sha256(), epoch
        j = sims[1].jobs
        live = j.active != 0
        assert np.all(j.bmax[live] >= j.bmin[live]) and np.all(j.bmax[live] <= sims[1].cap[live])
        seen.update(j.bmax[live].tolist())
        search.set_jobs(j)
    assert len(seen) > 3
    search.close()
