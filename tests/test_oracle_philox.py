"""Pins for the oracle's Philox generator: the published known-answer vectors, the uniform
mapping's exactness in fp32, and uniformity."""
import os

import numpy as np
from scipy import stats

from oracle import philox

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def _kat_rows():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            w = [int(x, 16) for x in line.split()]
            rows.append((w[0:4], w[4:6], w[6:10]))
    return rows


def test_known_answer_vectors():
    rows = _kat_rows()
    assert len(rows) == 3
    for ctr, key, out in rows:
        got = philox.philox4x32_10(np.array(ctr), np.array(key))
        assert [int(x) for x in got] == out


def test_vectorised_matches_scalar_calls():
    rng = np.random.default_rng(1)
    ctr = rng.integers(0, 2**32, size=(50, 4), dtype=np.uint64)
    key = rng.integers(0, 2**32, size=(50, 2), dtype=np.uint64)
    batch = philox.philox4x32_10(ctr, key)
    for i in range(50):
        assert np.array_equal(batch[i], philox.philox4x32_10(ctr[i], key[i]))


def test_counter_fields_are_all_used():
    base = philox.uniform(7, 3, 5, 11, 1)
    assert base != philox.uniform(8, 3, 5, 11, 1)
    assert base != philox.uniform(7 + 2**32, 3, 5, 11, 1)      # high seed word is key[1]
    assert base != philox.uniform(7, 4, 5, 11, 1)
    assert base != philox.uniform(7, 3, 6, 11, 1)
    assert base != philox.uniform(7, 3, 5, 12, 1)
    assert base != philox.uniform(7, 3, 5, 11, 2)
    # the documented layout: counter = (position, step, sequence, stream), word 0
    w = philox.philox4x32_10(np.array([3, 5, 11, 1]), np.array([7, 0]))[0]
    assert base == philox.word_to_uniform(w)


def test_uniform_is_exact_in_fp32_and_open_interval():
    w = np.array([0, 1, 511, 512, 2**31, 2**32 - 1], dtype=np.uint32)
    u = philox.word_to_uniform(w)
    assert np.all(u > 0) and np.all(u < 1)
    assert np.array_equal(u.astype(np.float32).astype(np.float64), u)
    assert u[0] == 2.0 ** -24 and u[-1] == 1 - 2.0 ** -24
    assert u[2] == u[0] and u[3] > u[2]          # only the top 23 bits matter


def test_uniformity_chi_square():
    n = 1_000_000
    u = philox.uniform(0, np.arange(n) % 1000, np.arange(n) // 1000, 0, 1)
    counts, _ = np.histogram(u, bins=64, range=(0, 1))
    chi2 = np.sum((counts - n / 64) ** 2 / (n / 64))
    assert stats.chi2.sf(chi2, 63) > 1e-4
    assert abs(u.mean() - 0.5) < 4 * np.sqrt(1 / 12 / n)
    # streams are decorrelated
    v = philox.uniform(0, np.arange(n) % 1000, np.arange(n) // 1000, 0, 2)
    assert abs(np.corrcoef(u, v)[0, 1]) < 5e-3
