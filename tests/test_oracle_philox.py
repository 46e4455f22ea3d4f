"""Pins for the oracle's Philox4x32-10: published known answers, a big-integer twin, bijection."""
import os

import numpy as np

from tests import pyref

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def _kat():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            v = [int(x, 16) for x in line.split()]
            rows.append((v[0:4], v[4:6], v[6:10]))
    return rows


def test_known_answers(oracle):
    rows = _kat()
    assert len(rows) == 3
    for ctr, key, want in rows:
        assert list(oracle.philox4x32_10(ctr, key)) == want
        assert pyref.philox4x32_10(ctr, key) == want


def test_matches_bigint_twin(oracle):
    rng = np.random.default_rng(7)
    for _ in range(20000):
        ctr = rng.integers(0, 2 ** 32, size=4, dtype=np.uint64)
        key = rng.integers(0, 2 ** 32, size=2, dtype=np.uint64)
        assert list(oracle.philox4x32_10(ctr, key)) == pyref.philox4x32_10(ctr, key)


def test_distinct_counters_give_distinct_blocks(oracle):
    seen = set()
    for c0 in range(1 << 12):
        seen.add(tuple(oracle.philox4x32_10([c0, 0, 3, 5], [11, 0])))
    assert len(seen) == 1 << 12


def test_bit_frequencies(oracle):
    # every output bit is set about half the time over consecutive counters
    n = 1 << 13
    words = np.array([oracle.philox4x32_10([c0, 0, 0, 0], [1, 2]) for c0 in range(n)], dtype=np.uint32)
    bits = ((words.reshape(-1)[:, None] >> np.arange(32, dtype=np.uint32)) & 1).mean(axis=0)
    assert np.all(np.abs(bits - 0.5) < 5 * 0.5 / np.sqrt(4 * n))
