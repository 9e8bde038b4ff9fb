"""Pins for the oracle's order-free RMSNorm (the producer of the inputs at positions 1 and 3 of
Section 2.1) -- CPU only.  Exact integer arithmetic in Python for the sum of squares, numpy's
float64 RMSNorm for the values, closed forms and invariants."""
from fractions import Fraction

import numpy as np

import oracle
import workloads as wl
from workloads import from_bf16_bits, to_bf16_bits


def _ulp_distance(a_bits, b_bits):
    """distance in bf16 steps between two finite bf16 bit patterns"""
    def key(b):
        b = b.astype(np.int32)
        return np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)
    return np.abs(key(a_bits) - key(b_bits))


def test_against_numpy_float64():
    gen = wl.rng(91)
    X = wl.activations_persistent(91, 64, 1024, 2)[0]
    gamma = to_bf16_bits((1.0 + 0.2 * gen.standard_normal(1024)).astype(np.float32))
    Y = oracle.rmsnorm(X, gamma, 1e-6)
    x, g = from_bf16_bits(X).astype(np.float64), from_bf16_bits(gamma).astype(np.float64)
    ref = x / np.sqrt((x * x).mean(axis=1, keepdims=True) + np.float64(np.float32(1e-6))) * g
    # the oracle rounds three times (r to single, x*r to bf16, the product with gamma to bf16), the
    # float64 formula never: the two agree to one step of 8 significant bits, and mostly exactly
    d = _ulp_distance(Y, to_bf16_bits(ref.astype(np.float32)))
    assert d.max() <= 1 and (d == 0).mean() > 0.6
    assert np.abs(from_bf16_bits(Y) - ref).max() <= 2.0 ** -7 * np.abs(ref).max()
    # with gamma = 1 only one rounding to 8 bits is left (after the single-precision product with r):
    # all but the values within 2^-24 of a rounding boundary must agree exactly
    ones = to_bf16_bits(np.ones(1024, np.float32))
    Y1 = oracle.rmsnorm(X, ones, 1e-6)
    ref1 = x / np.sqrt((x * x).mean(axis=1, keepdims=True) + np.float64(np.float32(1e-6)))
    d1 = _ulp_distance(Y1, to_bf16_bits(ref1.astype(np.float32)))
    assert d1.max() <= 1 and (d1 == 0).mean() > 0.999


def test_sum_of_squares_is_exact_when_nothing_is_truncated():
    """Values within 2^15 of each other: every term fits, so mean is the exact rational mean
    rounded once; checked through r on a row built to make x*r land on exact values."""
    vals = np.array([3.0, -1.5, 0.75, 2.0, 4.0, -0.5, 1.0, 6.0] * 4, np.float32)
    X = to_bf16_bits(vals[None, :])
    exact_mean = sum(Fraction(float(v)) ** 2 for v in vals) / len(vals)
    r = np.float32(1.0 / np.sqrt(float(exact_mean)))          # eps = 0
    gamma = to_bf16_bits(np.ones(32, np.float32))
    Y = oracle.rmsnorm(X, gamma, 0.0)
    expect = to_bf16_bits((vals * r).astype(np.float32)[None, :])
    assert np.array_equal(Y, expect)


def test_closed_forms_and_invariants():
    ones = to_bf16_bits(np.ones(64, np.float32))
    # a constant row normalises to its sign (power-of-two magnitude: no rounding anywhere)
    for c in (4.0, -0.125, 2.0 ** 60, 2.0 ** -60):
        Y = oracle.rmsnorm(to_bf16_bits(np.full((1, 64), c, np.float32)), ones, 0.0)
        assert (from_bf16_bits(Y) == np.sign(c)).all(), c
    # a single non-zero element: mean = v^2 / K, so y = sign * sqrt(K)
    x = np.zeros((1, 64), np.float32)
    x[0, 17] = -3.0
    Y = oracle.rmsnorm(to_bf16_bits(x), ones, 0.0)
    assert from_bf16_bits(Y)[0, 17] == -8.0 and np.count_nonzero(from_bf16_bits(Y)) == 1
    # gamma scales the already rounded value
    g2 = to_bf16_bits(np.full(64, 0.5, np.float32))
    X = wl.activations_diffuse(92, 8, 64)
    assert np.array_equal(from_bf16_bits(oracle.rmsnorm(X, g2, 1e-6)), from_bf16_bits(oracle.rmsnorm(X, ones, 1e-6)) * 0.5)
    # power-of-two change of units (eps = 0): nothing changes; order of the channels: only the order
    X2 = to_bf16_bits(from_bf16_bits(X) * np.float32(2.0 ** 9))
    assert np.array_equal(oracle.rmsnorm(X2, ones, 0.0), oracle.rmsnorm(X, ones, 0.0))
    perm = wl.rng(3).permutation(64)
    assert np.array_equal(oracle.rmsnorm(X[:, perm], ones, 1e-6), oracle.rmsnorm(X, ones, 1e-6)[:, perm])
    # an all-zero row stays zero when eps > 0; eps dominates tiny rows
    z = oracle.rmsnorm(np.zeros((1, 64), np.uint16), ones, 1e-6)
    assert (z == 0).all()
    tiny = to_bf16_bits(np.full((1, 64), 1e-30, np.float32))
    assert np.allclose(from_bf16_bits(oracle.rmsnorm(tiny, ones, 1e-6)), 1e-30 / np.sqrt(1e-6), rtol=2 ** -7)
    # huge dynamic range inside a row: terms 2^46 below the largest vanish, the result is finite
    wide = np.ones((1, 64), np.float32)
    wide[0, 0], wide[0, 1] = 2.0 ** 100, 2.0 ** -100
    Yw = from_bf16_bits(oracle.rmsnorm(to_bf16_bits(wide), ones, 0.0))
    assert np.isfinite(Yw).all() and Yw[0, 0] == 8.0


def test_nonfinite_rejected():
    X = to_bf16_bits(np.ones((2, 32), np.float32))
    X[0, 1] = 0x7F80
    try:
        oracle.rmsnorm(X, to_bf16_bits(np.ones(32, np.float32)))
    except oracle.OracleError:
        return
    raise AssertionError("a non-finite input must be refused")


def test_recipe_against_the_plain_double_precision_form():
    """The order-free recipe (fixed-point sum of squares, single-precision products) against the
    oracle's textbook RMSNorm: double accumulation, libm sqrt, roundings only where a model made of
    bf16 modules has them.  The plain form is itself pinned to numpy float64 here, so a slip in
    either shows."""
    X = wl.activations_persistent(191, 256, 4096, 2, jitter=0.2)[0]
    gamma = to_bf16_bits((1.0 + 0.2 * wl.rng(192).standard_normal(4096)).astype(np.float32))
    eps = 1e-6
    x, g = from_bf16_bits(X).astype(np.float64), from_bf16_bits(gamma).astype(np.float64)
    ref = x / np.sqrt((x * x).mean(axis=1, keepdims=True) + np.float64(np.float32(eps))) * g
    plain1 = oracle.rmsnorm_plain(X, gamma, eps)
    # a float64 value lands on a bf16 tie with probability ~2^-45: rounding through float32 is safe here
    d = _ulp_distance(plain1, to_bf16_bits(ref.astype(np.float32)))
    assert d.max() <= 1 and (d == 0).mean() > 0.9999
    Y = oracle.rmsnorm(X, gamma, eps)
    d1 = _ulp_distance(Y, plain1)                                   # one rounding against two
    assert d1.max() <= 1
    d2 = _ulp_distance(Y, oracle.rmsnorm_plain(X, gamma, eps, mid_round=True))   # same roundings, plain arithmetic
    assert d2.max() <= 2 and (d2 == 0).mean() >= 0.999
    ones = to_bf16_bits(np.ones(4096, np.float32))
    d3 = _ulp_distance(oracle.rmsnorm(X, ones, eps), oracle.rmsnorm_plain(X, ones, eps))
    assert d3.max() <= 1 and (d3 == 0).mean() >= 0.999
