"""Pins of the oracle's hand-off to Algorithm 2 (initialisation line: worker i imports its subset A_i
and runs with a batch size scaled by the capacity ratios): per-worker index lists against numpy's
stable argsort and bincount, partition invariants, a hand-worked example; batch sizes against
hand-worked vectors and the equal-time property that decides the reading."""
import numpy as np
import pytest

import oracle


def test_worker_shards_against_numpy_and_by_hand():
    assign = np.array([2, 0, -1, 1, 0, 2, 2, -1, 1, 0], dtype=np.int32)
    index, offset = oracle.worker_shards(assign, 3)
    assert offset.tolist() == [0, 3, 5, 8]
    assert index.tolist() == [1, 4, 9, 3, 8, 0, 5, 6]
    rng = np.random.default_rng(0)
    for N, K in ((1, 1), (17, 4), (1000, 16), (5000, 7)):
        a = rng.integers(-1, K, size=N).astype(np.int32)
        index, offset = oracle.worker_shards(a, K)
        taken = np.flatnonzero(a >= 0)
        ref = taken[np.argsort(a[taken], kind="stable")]
        assert np.array_equal(index, ref)
        assert np.array_equal(np.diff(offset), np.bincount(a[taken], minlength=K))
        # a partition of the assigned samples, ascending inside every worker
        assert sorted(index.tolist()) == taken.tolist()
        for k in range(K):
            part = index[offset[k]:offset[k + 1]]
            assert np.all(a[part] == k) and np.all(np.diff(part) > 0)
    with pytest.raises(ValueError):
        oracle.worker_shards(np.array([0, 3], dtype=np.int32), 3)
    with pytest.raises(ValueError):
        oracle.worker_shards(np.array([0, -2], dtype=np.int32), 3)


def test_batch_sizes_by_hand_and_equal_time():
    assert oracle.batch_sizes(64, [1, 1, 2, 4]).tolist() == [64, 64, 128, 256]
    assert oracle.batch_sizes(10, [2, 3]).tolist() == [10, 15]
    assert oracle.batch_sizes(10, [3, 2]).tolist() == [10, 7]          # 6.67 -> 7
    assert oracle.batch_sizes(3, [2, 1]).tolist() == [3, 2]            # 1.5 -> 2 (halves up)
    assert oracle.batch_sizes(1, [8, 1]).tolist() == [1, 1]            # 0.125 -> at least 1
    # proportional to capacity: every worker's time per iteration, batch_i / r_i, is that of worker 1
    # up to the rounding of its batch
    rng = np.random.default_rng(1)
    for _ in range(200):
        K = int(rng.integers(1, 17))
        r = rng.integers(1, 9, size=K)
        B = int(rng.integers(1, 513))
        b = oracle.batch_sizes(B, r)
        assert b[0] == B
        exact = B * r / r[0]
        assert np.all(np.abs(b - np.maximum(exact, 1.0)) <= 0.5 + 1e-12)
        assert np.all(np.abs(b / r - B / r[0]) <= np.maximum(0.5, 1.0 - exact) / r + 1e-12)
