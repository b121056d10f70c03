"""Pins of the oracle's quota rule (constraint line of Algorithm 1)."""
import os

import numpy as np
import pytest

import oracle
import synth_inputs as si


def _golden(golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "quota_vectors.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            n, r, cap = line.split(";")
            rows.append((int(n), [int(x) for x in r.split()], [int(x) for x in cap.split()]))
    return rows


def test_hand_worked_vectors(golden_dir):
    rows = _golden(golden_dir)
    assert len(rows) >= 7
    for n, r, cap in rows:
        assert oracle.quota(n, r).tolist() == cap, (n, r)


@pytest.mark.parametrize("seed", range(20))
def test_sum_and_closeness_to_real_valued_constraint(seed):
    rng = np.random.default_rng(seed)
    K = int(rng.integers(1, 17))
    r = rng.integers(1, 9, size=K)
    n = int(rng.integers(0, 6000))
    cap = oracle.quota(n, r)
    assert cap.sum() == n                                  # sum_j C_{l,j} = |V_l|
    real = n * r / r.sum()
    assert np.all(cap - real <= 1.0) and np.all(cap - real > -1.0)
    # the extras go to the largest capacities: no worker with a smaller r
    # got an extra while a larger-r worker did not
    extra = cap - np.floor(real).astype(np.int64)
    assert set(extra.tolist()) <= {0, 1}
    if extra.any() and not extra.all():
        assert r[extra == 1].min() >= r[extra == 0].max()


def test_equal_capacities_give_label_balanced_case():
    # Algorithm 3 (label-balanced) is Algorithm 1 with all r equal: C_l = |V_l| / N
    assert oracle.quota(1000, [1] * 8).tolist() == [125] * 8
    assert oracle.quota(1000, [3] * 8).tolist() == [125] * 8


def test_every_configured_workload_has_consistent_quotas():
    for w in si.WORKLOADS.values():
        r = w.r if w.r is not None else np.random.default_rng(w.seed).integers(1, 5, size=w.K)
        cap = oracle.quota(w.n_c, r)
        assert cap.sum() == w.n_c and len(cap) == w.K


def test_rejects_nonpositive_capacity():
    with pytest.raises(ValueError):
        oracle.quota(10, [1, 0, 2])
