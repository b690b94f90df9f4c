"""Pins for the oracle's counter-based generator (Philox4x32-10, Salmon et al. SC'11)."""
import os

import numpy as np

from pyref import philox4x32_10

GOLD = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def _kat():
    rows = []
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(x, 16) for x in line.split()]
        rows.append((w[0:4], w[4:6], w[6:10]))
    return rows


def test_published_known_answers(ref):
    rows = _kat()
    assert len(rows) == 3
    for ctr, key, out in rows:
        assert ref.philox(ctr, key).tolist() == out
        assert philox4x32_10(ctr, key) == out


def test_against_big_integer_transcription(ref):
    rng = np.random.default_rng(123)
    for _ in range(500):
        ctr = rng.integers(0, 2**32, 4, dtype=np.uint64)
        key = rng.integers(0, 2**32, 2, dtype=np.uint64)
        assert ref.philox(ctr, key).tolist() == philox4x32_10(ctr, key)


def test_counter_words_are_all_used(ref):
    base = ref.philox([1, 2, 3, 4], [5, 6]).tolist()
    for i in range(4):
        c = [1, 2, 3, 4]
        c[i] ^= 1
        assert ref.philox(c, [5, 6]).tolist() != base
    assert ref.philox([1, 2, 3, 4], [5, 7]).tolist() != base
    assert ref.philox([1, 2, 3, 4], [4, 6]).tolist() != base
