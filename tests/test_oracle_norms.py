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


def test_bfloat16_squares_against_rationals_for_every_pattern():
    """All 65,536 bfloat16 bit patterns: the squared norm of a one-element vector
    is the square of the value the pattern denotes (sign, 8 exponent bits, 7
    fraction bits, read off the bits here), exactly; NaN patterns give NaN."""
    for bits in range(1 << 16):
        sign, exponent, fraction = bits >> 15, (bits >> 7) & 0xff, bits & 0x7f
        got = oracle.sum_sq(np.array([bits], dtype=np.uint16))
        if exponent == 0xff:
            assert math.isinf(got) if fraction == 0 else math.isnan(got), bits
            continue
        if exponent == 0:
            value = Fraction(fraction, 128) * Fraction(2) ** -126          # subnormal
        else:
            value = (1 + Fraction(fraction, 128)) * Fraction(2) ** (exponent - 127)
        value = -value if sign else value
        assert Fraction(got) == Fraction(float(value * value)), bits      # one rounding to binary64


def test_bfloat16_vector_norm_matches_the_widened_binary32_norm():
    import torch
    rng = np.random.default_rng(12)
    x = torch.from_numpy(rng.normal(0, 0.002, 5001).astype(np.float32)).to(torch.bfloat16)
    bits = x.view(torch.int16).numpy().view(np.uint16)
    widened = x.to(torch.float32).numpy()
    assert oracle.sum_sq(bits) == oracle.sum_sq(widened)
    assert oracle.sum_sq(bits) == math.fsum(float(v) * float(v) for v in widened)
    assert abs(oracle.sum_sq(bits, threads=4) / oracle.sum_sq(bits) - 1) < 1e-15


# ---- the divergence bound of Sec. 5.3 -----------------------------------------------------

def test_bound_has_the_papers_two_update_coefficients():
    """Two single updates: the bound is (g + g^2)||h0|| + (1 + g)||u1|| + ||u2||,
    the triangle inequality on the expression printed in Sec. 3.3."""
    gamma, lr = Fraction(1, 2), Fraction(1, 4)
    h, g1, g2 = Fraction(3), Fraction(5), Fraction(7)
    expect = (gamma + gamma ** 2) * h + (1 + gamma) * lr * g1 + lr * g2
    got = oracle.divergence_bound(float(h), [float(g1), float(g2)], None, [1, 1], float(lr), float(gamma))
    assert Fraction(got) == expect
    # squared, it is the printed form with every cross term at its Cauchy-Schwarz maximum
    a, b = gamma + gamma ** 2, 1 + gamma
    u1, u2 = lr * g1, lr * g2
    squared = (a * a * h * h + b * b * u1 * u1 + u2 * u2 + 2 * a * b * h * u1 + 2 * b * u1 * u2 + 2 * a * h * u2)
    assert Fraction(got) ** 2 == squared


def test_bound_dominates_the_exact_divergence_of_the_two_update_case():
    rng = np.random.default_rng(21)
    for trial in range(20):
        n, gamma, lr = 257, float(rng.uniform(0, 0.99)), float(rng.uniform(0.001, 0.5))
        w0 = rng.normal(0, 1, n).astype(np.float32)
        h0 = rng.normal(0, 0.1, n).astype(np.float32)
        g = [rng.normal(0, 1, n).astype(np.float32) for _ in range(2)]
        w, h = w0.copy(), h0.copy()
        oracle.apply_ordered(w, h, g, [0, 1], lr, gamma)
        exact = math.sqrt(oracle.sum_sq_diff(w, w0))
        bound = oracle.divergence_bound(math.sqrt(oracle.sum_sq(h0)), [math.sqrt(oracle.sum_sq(x)) for x in g],
                                        None, [1, 1], lr, gamma)
        assert exact <= bound * (1 + 1e-6)          # the model is stepped in binary32


def test_bound_dominates_grouped_batches_of_any_shape():
    rng = np.random.default_rng(22)
    for trial in range(30):
        M = int(rng.integers(1, 12))
        n, gamma, lr = 129, float(rng.uniform(0, 0.95)), float(rng.uniform(0.001, 0.3))
        groups, left = [], M
        while left > 0:
            ln = int(rng.integers(1, left + 1))
            groups.append(ln)
            left -= ln
        w0 = rng.normal(0, 1, n).astype(np.float32)
        h0 = rng.normal(0, 0.1, n).astype(np.float32)
        g = [rng.normal(0, 1, n).astype(np.float32) for _ in range(M)]
        wt = rng.uniform(-1.5, 1.5, M).astype(np.float32)
        order = list(rng.permutation(M))
        w, h = w0.copy(), h0.copy()
        oracle.apply_grouped(w, h, g, order, wt, groups, lr, gamma)
        exact = math.sqrt(oracle.sum_sq_diff(w, w0))
        in_sequence = [math.sqrt(oracle.sum_sq(g[j])) for j in order]
        bound = oracle.divergence_bound(math.sqrt(oracle.sum_sq(h0)), in_sequence, wt[order], groups, lr, gamma)
        assert exact <= bound * (1 + 1e-5), (trial, exact, bound)


def test_bound_is_tight_when_everything_points_the_same_way():
    """History and all updates positive multiples of one direction, positive
    weights and momentum: every triangle inequality is an equality."""
    v = np.array([3.0, 4.0, 12.0], dtype=np.float32)              # ||v|| = 13
    gamma, lr = 0.5, 0.25
    w0 = np.zeros(3, np.float32)
    h0 = 2.0 * v
    g = [-1.0 * v, -2.0 * v, -4.0 * v]                            # u = -lr g points along +v
    w, h = w0.copy(), h0.copy()
    oracle.apply_grouped(w, h, g, [0, 1, 2], np.ones(3, np.float32), [1, 2], lr, gamma)
    exact = math.sqrt(oracle.sum_sq_diff(w, w0))
    bound = oracle.divergence_bound(26.0, [13.0, 26.0, 52.0], np.ones(3, np.float32), [1, 2], lr, gamma)
    assert exact == bound                                         # small dyadic numbers: no rounding
    # one step more of momentum history, by hand: (g + g^2) 26 + (1 + g) 0.25*13 + 0.25*(26 + 52)
    assert bound == (0.5 + 0.25) * 26 + 1.5 * 3.25 + 19.5
