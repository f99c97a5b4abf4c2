"""Pins for the oracle's squared norms (Table 1: update_norm; Sec. 5.3 of the
paper: divergence from ||h||, ||u_i|| and the exact ||w_s - w_r||).  CPU only."""
import math
from fractions import Fraction

import numpy as np

import oracle


def test_exactly_rounded_against_fsum_and_rationals():
    rng = np.random.default_rng(2)
    for scale in (1.0, 1e-20, 1e18):
        x = (rng.normal(0, 1, 3001) * scale).astype(np.float32)
        exact = math.fsum(float(v) * float(v) for v in x)      # squares are exact in binary64
        assert oracle.sum_sq(x) == exact
        as_rational = sum(Fraction(float(v)) ** 2 for v in x[:200])
        assert Fraction(oracle.sum_sq(x[:200].copy())) == Fraction(float(as_rational))


def test_cancellation_heavy_sum_is_still_exact():
    # one huge term and many tiny ones that a plain binary64 running sum would drop
    x = np.array([2.0 ** 40] + [1.0] * 5000 + [2.0 ** -30] * 5000, dtype=np.float32)
    expect = Fraction(2) ** 80 + 5000 + Fraction(5000, 2 ** 60)
    assert Fraction(oracle.sum_sq(x)) == Fraction(float(expect))


def test_known_values_and_scaling():
    assert oracle.sum_sq(np.ones(1000, np.float32)) == 1000.0
    assert oracle.sum_sq(np.array([3.0, -4.0], np.float32)) == 25.0
    assert oracle.sum_sq(np.zeros(0, np.float32)) == 0.0
    x = np.random.default_rng(4).normal(0, 1, 777).astype(np.float32)
    assert oracle.sum_sq(2 * x) == 4 * oracle.sum_sq(x)            # powers of two are exact
    # slices return rounded partial sums: a few units in the last place at most
    assert abs(oracle.sum_sq(x, threads=5) / oracle.sum_sq(x) - 1) < 1e-15


def test_difference_is_taken_exactly():
    a = np.array([1.0, 2.0 ** 24, 5.0], np.float32)
    b = np.array([2.0 ** -24, 1.0, 5.0], np.float32)          # a - b is not a binary32 number
    d0 = Fraction(1) - Fraction(1, 2 ** 24)
    d1 = Fraction(2) ** 24 - 1
    assert Fraction(oracle.sum_sq_diff(a, b)) == Fraction(float(d0 * d0 + d1 * d1))
    x = np.random.default_rng(6).normal(0, 1, 500).astype(np.float32)
    assert oracle.sum_sq_diff(x, x) == 0.0
    assert oracle.sum_sq_diff(x, np.zeros_like(x)) == oracle.sum_sq(x)
    assert abs(oracle.sum_sq_diff(x, np.zeros_like(x), threads=3) / oracle.sum_sq(x) - 1) < 1e-15


def test_two_update_divergence_of_the_paper():
    """Sec. 3.3: ||w2 - w0|| = ||(g + g^2) h0 + (1 + g) u1 + u2||, on dyadic data."""
    rng = np.random.default_rng(9)
    n, gamma, lr = 64, 0.5, 0.25
    w0 = rng.integers(-64, 65, n).astype(np.float32)
    h0 = rng.integers(-64, 65, n).astype(np.float32)
    g1 = rng.integers(-64, 65, n).astype(np.float32)
    g2 = rng.integers(-64, 65, n).astype(np.float32)
    w, h = w0.copy(), h0.copy()
    oracle.apply_ordered(w, h, [g1, g2], [0, 1], lr, gamma)
    lead = (gamma + gamma ** 2) * h0.astype(np.float64) + (1 + gamma) * (-lr * g1) + (-lr * g2)
    assert oracle.sum_sq_diff(w, w0) == float(np.sum(lead ** 2))      # exact: small dyadics
