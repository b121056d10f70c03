"""Pins of the oracle's similarity (Gaussian kernel on the L2 distance, Section 4
of arXiv 2211.00839) against facts fixed by mathematics, not by the oracle."""
import math

import numpy as np
import pytest

import oracle
import synth_inputs as si


def test_two_points_closed_form():
    # distance 5 (3-4-5 triangle), sigma^2 = 12.5  ->  exp(-25/25) = 1/e
    X = np.array([[0.0, 0.0], [3.0, 4.0]], dtype=np.float32)
    S32, S64 = oracle.similarity(X, 12.5, want64=True)
    assert S64[0, 1] == pytest.approx(math.exp(-1.0), rel=1e-15)
    assert S64[1, 0] == pytest.approx(math.exp(-1.0), rel=1e-15)
    assert S64[0, 0] == 1.0 and S64[1, 1] == 1.0
    assert S32[0, 1] == np.float32(math.exp(-1.0))


def test_scaled_unit_vectors_closed_form():
    # x_i = a e_i: every pair is at squared distance 2 a^2 -> exp(-a^2/sigma^2)
    n, a, sigma2 = 7, 1.5, 3.0
    X = (a * np.eye(n)).astype(np.float32)
    _, S64 = oracle.similarity(X, sigma2, want64=True)
    off = S64[~np.eye(n, dtype=bool)]
    assert np.allclose(off, math.exp(-a * a / sigma2), rtol=1e-15, atol=0)
    assert np.all(np.diag(S64) == 1.0)


def test_symmetry_range_diagonal_on_mixture():
    X = si.make_class(seed=11, n=60, d=16)
    S32, S64 = oracle.similarity(X, 16.0, want64=True)
    assert np.array_equal(S64, S64.T)          # computed pair by pair, never mirrored
    assert np.all(np.diag(S32) == np.float32(1.0))
    assert np.all(S64 > 0.0) and np.all(S64 <= 1.0)


def test_translation_and_joint_scaling_are_exact_on_dyadic_inputs():
    rng = np.random.default_rng(5)
    X = rng.integers(-8, 9, size=(20, 6)).astype(np.float32)
    base = oracle.similarity(X, 40.0, want64=True)[1]
    shifted = oracle.similarity(X + np.float32(3.0), 40.0, want64=True)[1]
    scaled = oracle.similarity(X * np.float32(2.0), 160.0, want64=True)[1]
    assert np.array_equal(base, shifted)
    assert np.array_equal(base, scaled)


def test_against_gram_identity_in_numpy():
    # an independent route: ||x||^2 + ||y||^2 - 2 x.y through numpy's matmul
    X = si.make_class(seed=3, n=50, d=32)
    sigma2 = 32.0
    _, S64 = oracle.similarity(X, sigma2, want64=True)
    Xd = X.astype(np.float64)
    sq = (Xd * Xd).sum(1)
    D = np.maximum(sq[:, None] + sq[None, :] - 2.0 * Xd @ Xd.T, 0.0)
    ref = np.exp(-D / (2.0 * sigma2))
    off = ~np.eye(len(X), dtype=bool)
    assert np.allclose(S64[off], ref[off], rtol=1e-12, atol=0)


def test_sigma_enters_as_two_sigma_squared():
    # one pair at squared distance 8: sigma2=4 -> exp(-1); sigma2=2 -> exp(-2)
    X = np.array([[0, 0], [2, 2]], dtype=np.float32)
    assert oracle.similarity(X, 4.0, want64=True)[1][0, 1] == pytest.approx(math.exp(-1.0), rel=1e-15)
    assert oracle.similarity(X, 2.0, want64=True)[1][0, 1] == pytest.approx(math.exp(-2.0), rel=1e-15)


def test_bf16_inputs_are_read_exactly():
    Xf = si.make_class(seed=9, n=24, d=16)
    bits = si.f32_to_bf16_bits(Xf)
    back = si.bf16_bits_to_f32(bits)
    assert np.array_equal(oracle.similarity(bits, 16.0), oracle.similarity(back, 16.0))
    # and rounding to bf16 did change the inputs, so the test is not vacuous
    assert not np.array_equal(back, Xf)


def test_bf16_rounding_helper_is_nearest_even():
    # 1 + 2^-8 is halfway between bf16 neighbours 1 and 1+2^-7: ties to even -> 1
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20], dtype=np.float32)
    got = si.bf16_bits_to_f32(si.f32_to_bf16_bits(x))
    assert got.tolist() == [1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7]


def test_rejects_bad_arguments():
    X = np.zeros((3, 2), dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.similarity(X, 0.0)
    with pytest.raises(TypeError):
        oracle.similarity(X.astype(np.float64), 1.0)
