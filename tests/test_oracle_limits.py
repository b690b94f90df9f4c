"""Pins for the oracle's batch-size limit policies (Section 3.3.2: Start, Resume, Scale-up,
Scale-down), the producer of bmax_j between scheduling epochs."""
import math

import numpy as np
import pytest


def update(ref, limit, sigma=0.0, **kw):
    n = len(limit)
    base = dict(state=np.full(n, 3), bmin=np.full(n, 16), bcap=np.full(n, 4096), gpu_max_batch=np.full(n, 256),
                last_batch=np.zeros(n), finished_epoch=np.zeros(n), elapsed=np.zeros(n))
    base.update({k: np.asarray(v) for k, v in kw.items()})
    return ref.update_limits(limit, sigma, **base).tolist()


def test_start_limits_a_new_job_to_one_gpu(ref):
    assert update(ref, [0, 4096, 7], state=[1, 1, 1], gpu_max_batch=[256, 64, 512]) == [256, 64, 512]
    # ... inside the job's own window
    assert update(ref, [0, 0], state=[1, 1], gpu_max_batch=[256, 8], bmin=[16, 16], bcap=[128, 4096]) == [128, 16]


def test_resume_caps_at_the_batch_before_preemption_then_halves(ref):
    assert update(ref, [2048], state=[2], last_batch=[512]) == [512]        # first update after pre-emption
    assert update(ref, [256], state=[2], last_batch=[512]) == [256]         # "does not exceed"
    lim = [512]
    seen = []
    for _ in range(7):                                                       # rejected again and again
        lim = update(ref, lim, state=[2], last_batch=[0])
        seen.append(lim[0])
    assert seen == [256, 128, 64, 32, 16, 16, 16]                            # never below bmin


def test_scale_up_doubles_after_an_epoch(ref):
    assert update(ref, [128, 128], finished_epoch=[1, 0]) == [256, 128]
    assert update(ref, [4096], finished_epoch=[1]) == [4096]                 # the job's own cap


@pytest.mark.parametrize("sigma_t,want", [(0.0, 1024), (0.5, 512), (1.0, 512), (1.5, 256), (2.0, 256), (3.0, 256),
                                          (7.0, 128), (100.0, 16)])
def test_scale_down_is_the_printed_formula(ref, sigma_t, want):
    """R' = ceil(2R / ceil(sigma*T + 1)) with R = 512, rounded down to a power of two:
    sigma*T = 0.5 -> ceil(1024/2) = 512; 1.5 -> ceil(1024/3) = 342 -> 256; 7 -> 1024/8 = 128."""
    r = 512
    exact = math.ceil(2 * r / math.ceil(sigma_t + 1))
    assert 2 ** int(math.log2(max(exact, 16))) == want
    assert update(ref, [r], sigma=0.01, finished_epoch=[1], elapsed=[sigma_t / 0.01]) == [want]


def test_limits_never_grow_with_elapsed_time(ref):
    rng = np.random.default_rng(0)
    for _ in range(200):
        r = int(2 ** rng.integers(4, 13))
        ts = np.sort(rng.uniform(0, 5000, 6))
        outs = [update(ref, [r], sigma=0.003, finished_epoch=[1], elapsed=[t])[0] for t in ts]
        assert all(b <= a for a, b in zip(outs, outs[1:]))
        assert all(16 <= o <= 4096 and o & (o - 1) == 0 for o in outs)


def test_empty_slots_and_argument_checks(ref):
    assert update(ref, [300], state=[0]) == [0]
    for kw, code in [(dict(state=[4]), -1), (dict(bmin=[24]), -2), (dict(bmin=[512], bcap=[256]), -3),
                     (dict(elapsed=[-1.0]), -1), (dict(elapsed=[float("nan")]), -4)]:
        with pytest.raises(ref.RefError) as e:
            update(ref, [64], sigma=0.1, **kw)
        assert e.value.code == code
    with pytest.raises(ref.RefError):
        update(ref, [64], sigma=-1.0)
    with pytest.raises(ref.RefError):
        update(ref, [0], state=[3])                                          # a running job has a limit
