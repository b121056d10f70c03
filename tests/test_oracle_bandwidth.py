"""Pins of the oracle's kernel bandwidth (Section 4, "Submodular functions":
sigma = sum_{v,v' in V} ||v - v'||_2 / n^2) against what the formula and the mathematics fix:
closed forms on a line, on a regular simplex and for two points, the library routine
scipy.spatial.distance.pdist, exact scaling and translation behaviour on dyadic inputs,
permutation invariance, the n^2 (not n(n-1)) denominator, distance not squared."""
import numpy as np
import pytest
from scipy.spatial.distance import pdist

import oracle
import synth_inputs as si


def to_bf16_bits(a):
    return (np.ascontiguousarray(a, dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)


def test_closed_forms():
    # two points at distance 5: ordered pairs (0, 5, 5, 0) over n^2 = 4
    X = np.array([[0, 0], [3, 4]], dtype=np.float32)
    assert oracle.bandwidth(X) == 2.5
    # one point: its only pair is with itself
    assert oracle.bandwidth(np.ones((1, 7), dtype=np.float32)) == 0.0
    # n points on a line at unit spacing: sum_{i,j} |i - j| = n (n^2 - 1) / 3
    for n in (2, 3, 10, 257):
        X = np.zeros((n, 3), dtype=np.float32)
        X[:, 1] = np.arange(n)
        assert oracle.bandwidth(X) == pytest.approx((n * n - 1) / (3.0 * n), rel=1e-14)
    # vertices of a regular simplex (scaled unit vectors): every pair at a sqrt(2), n (n - 1) of them
    n, a = 12, 4.0
    X = (a * np.eye(n)).astype(np.float32)
    assert oracle.bandwidth(X) == pytest.approx(a * np.sqrt(2.0) * (n - 1) / n, rel=1e-14)
    # the distance is not squared: a 3-4-5 triangle
    X = np.array([[0, 0], [3, 0], [0, 4]], dtype=np.float32)
    assert oracle.bandwidth(X) == pytest.approx(2 * (3 + 4 + 5) / 9.0, rel=1e-15)


def test_against_scipy_pdist():
    for seed, n, d in ((1, 50, 8), (2, 131, 33), (3, 300, 64)):
        X = si.make_class(seed=seed, n=n, d=d)
        ref = 2.0 * pdist(X.astype(np.float64)).sum() / (n * n)
        assert oracle.bandwidth(X) == pytest.approx(ref, rel=1e-12)
    Xb = si.make_class(seed=4, n=90, d=32, dtype="bf16")
    as_f32 = (Xb.astype(np.uint32) << 16).view(np.float32)
    ref = 2.0 * pdist(as_f32.astype(np.float64)).sum() / (90 * 90)
    assert oracle.bandwidth(Xb) == pytest.approx(ref, rel=1e-12)


def test_scaling_translation_permutation():
    rng = np.random.default_rng(5)
    X = rng.integers(-64, 64, size=(40, 6)).astype(np.float32) / 8.0      # dyadic: shifts and scalings are exact
    s = oracle.bandwidth(X)
    assert oracle.bandwidth(4.0 * X) == 4.0 * s                            # homogeneous of degree 1, exactly
    assert oracle.bandwidth(X + np.float32(16.5)) == s                     # translation invariant, exactly
    perm = rng.permutation(40)
    assert oracle.bandwidth(X[perm]) == pytest.approx(s, rel=1e-14)
    # duplicating every sample keeps the mean over ordered pairs (each pair class is counted 4 times over 4 n^2)
    assert oracle.bandwidth(np.concatenate([X, X])) == pytest.approx(s, rel=1e-14)


def test_bf16_inputs_are_read_as_their_exact_values():
    X = si.make_class(seed=6, n=64, d=16)
    bits = to_bf16_bits(X)
    back = (bits.astype(np.uint32) << 16).view(np.float32)
    assert oracle.bandwidth(bits) == oracle.bandwidth(back)
    assert oracle.bandwidth(bits) != oracle.bandwidth(X)
