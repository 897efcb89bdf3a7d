"""Pins for the oracle's minibatch index sampler (no GPU).

The generator is pinned to the published known-answer vectors of Philox4x32-10
(tests/golden/philox4x32_10_kat.txt), the counter/key packing to a hand-built
counter, and the row mapping to exact uniformity properties.
"""
import os

import numpy as np
import pytest

from oracle.philox import philox4x32_10, sample_rows


def _read_kat(golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "philox4x32_10_kat.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            w = [int(v, 16) for v in line.split()]
            rows.append((w[0:4], w[4:6], w[6:10]))
    return rows


def test_philox_known_answers(golden_dir):
    kat = _read_kat(golden_dir)
    assert len(kat) == 3
    for ctr, key, want in kat:
        got = philox4x32_10(np.array(ctr, dtype=np.uint64), np.array(key, dtype=np.uint64))
        assert [int(v) for v in got] == want


def test_philox_vectorised_matches_scalar_calls():
    rng = np.random.default_rng(0)
    ctr = rng.integers(0, 2**32, size=(50, 4), dtype=np.uint64)
    key = rng.integers(0, 2**32, size=(50, 2), dtype=np.uint64)
    batch = philox4x32_10(ctr, key)
    for r in range(50):
        assert np.array_equal(batch[r], philox4x32_10(ctr[r], key[r]))


def test_philox_is_a_bijection_on_a_small_counter_slice():
    # For a fixed key the map counter -> output is a permutation: no collisions.
    ctr = np.zeros((4096, 4), dtype=np.uint64)
    ctr[:, 0] = np.arange(4096)
    out = philox4x32_10(ctr, np.array([7, 9], dtype=np.uint64))
    as_tuples = {tuple(int(v) for v in row) for row in out}
    assert len(as_tuples) == 4096


def test_sample_rows_counter_packing():
    # slot j of (seed, worker, t) is word j%4 of the block with counter
    # (j//4, t_lo, t_hi, worker) and key (seed_lo, seed_hi), top log2(n) bits.
    seed = (0x12345678 << 32) | 0x9ABCDEF0
    worker, t, batch, n = 5, (3 << 32) | 77, 11, 1 << 13
    got = sample_rows(seed, worker, t, batch, n)
    for j in range(batch):
        words = philox4x32_10(np.array([j // 4, 77, 3, worker], dtype=np.uint64),
                              np.array([0x9ABCDEF0, 0x12345678], dtype=np.uint64))
        assert got[j] == int(words[j % 4]) >> (32 - 13)
    assert got.min() >= 0 and got.max() < n


def test_sample_rows_prefix_property_and_independence_of_batch_size():
    a = sample_rows(3, 1, 10, 8, 4096)
    b = sample_rows(3, 1, 10, 32, 4096)
    assert np.array_equal(a, b[:8])


def test_sample_rows_differs_across_worker_iteration_seed():
    base = sample_rows(3, 0, 1, 64, 1 << 20)
    assert not np.array_equal(base, sample_rows(3, 1, 1, 64, 1 << 20))
    assert not np.array_equal(base, sample_rows(3, 0, 2, 64, 1 << 20))
    assert not np.array_equal(base, sample_rows(4, 0, 1, 64, 1 << 20))


def test_sample_rows_uniform_chi_square():
    n = 16
    counts = np.zeros(n)
    for t in range(1, 401):
        r = sample_rows(11, 2, t, 64, n)
        counts += np.bincount(r, minlength=n)
    total = counts.sum()
    chi2 = ((counts - total / n) ** 2 / (total / n)).sum()
    # 15 degrees of freedom: P(chi2 > 45) < 1e-4
    assert chi2 < 45.0


def test_sample_rows_lag_one_correlation_is_small():
    n = 1 << 16
    xs = np.concatenate([sample_rows(5, 0, t, 64, n) for t in range(1, 301)]).astype(np.float64)
    xs = (xs - xs.mean()) / xs.std()
    corr = float((xs[:-1] * xs[1:]).mean())
    assert abs(corr) < 0.03


def test_sample_rows_degenerate_and_invalid_sizes():
    assert np.array_equal(sample_rows(1, 0, 1, 5, 1), np.zeros(5, dtype=np.int64))
    assert set(sample_rows(1, 0, 1, 64, 2)) <= {0, 1}
    with pytest.raises(ValueError):
        sample_rows(1, 0, 1, 4, 12)
