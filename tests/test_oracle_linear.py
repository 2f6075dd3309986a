"""Pins for the oracle's quantized Linear layer (Sec. IV-A: Y = R(R(R(W^T) R(X)) + R(B))): a
hand-worked case, an all-integer case fixed by integer arithmetic, and exact rational arithmetic
for the two output roundings.  CPU only."""
from fractions import Fraction

import numpy as np

import oracle
import workloads
from fmtdef import brute_force_round, positive_finite_values


def test_hand_worked_case():
    """1/6/9 keeps 10 significant bits.  X = [[1, 2]], W = [[1 + 2^-10, 3], [0.5, -1]],
    b = [2^-9 + 2^-20, 1].  R(W) = [[1, 3], [0.5, -1]] (1 + 2^-10 is a tie and goes to the even
    neighbour 1), so acc = [1 + 6, 0.5 - 2] = [7, -1.5].  R(b) = [2^-9, 1].  The fp32 sums are
    t = [7 + 2^-9, -0.5].  In [4, 8) the format's spacing is 2^-7, so 7 + 2^-9 rounds to 7."""
    X = np.array([[1.0, 2.0]], dtype=np.float32)
    W = np.array([[1 + 2.0 ** -10, 3.0], [0.5, -1.0]], dtype=np.float32)
    b = np.array([2.0 ** -9 + 2.0 ** -20, 1.0], dtype=np.float32)
    Y, T = oracle.linear(X, W, b, 6, 9, True)
    assert np.array_equal(T, np.array([[7 + 2.0 ** -9, -0.5]], dtype=np.float32))
    assert np.array_equal(Y, np.array([[7.0, -0.5]], dtype=np.float32))
    # without bias the value entering the last rounding is R(acc) itself
    Y0, T0 = oracle.linear(X, W, None, 6, 9, True)
    assert np.array_equal(T0, np.array([[7.0, -1.5]], dtype=np.float32)) and np.array_equal(Y0, T0)


def test_integer_case():
    rng = np.random.default_rng(1)
    X = rng.integers(-3, 4, (12, 20)).astype(np.float32)
    W = rng.integers(-3, 4, (9, 20)).astype(np.float32)
    b = rng.integers(-5, 6, 9).astype(np.float32)
    want = (X.astype(np.int64) @ W.astype(np.int64).T + b.astype(np.int64)).astype(np.float32)   # |.| < 2^9: representable
    for (e, m, d) in [(5, 10, True), (6, 9, False), (8, 7, True)]:
        Y, T = oracle.linear(X, W, b, e, m, d)
        assert np.array_equal(Y, want) and np.array_equal(T, want)


def test_epilogue_against_exact_rationals():
    rng = np.random.default_rng(2)
    acc = workloads.log2_normal((40, 30), -4, 6, 0.05, rng)
    bias = workloads.log2_normal(30, -4, 6, 0.1, rng)
    for (e, m, d) in [(5, 10, True), (5, 10, False), (6, 9, True), (8, 7, False)]:
        vals = positive_finite_values(e, m)
        Y, T = oracle.linear_epilogue(acc, bias, e, m, d)
        for i in range(acc.shape[0]):
            for j in range(acc.shape[1]):
                ra = brute_force_round(float(acc[i, j]), e, m, d, vals)
                rb = brute_force_round(float(bias[j]), e, m, d, vals)
                if np.isfinite(ra) and np.isfinite(rb):
                    t = np.float32(float(Fraction(ra) + Fraction(rb)))        # one fp32 rounding of the exact sum
                else:
                    t = np.float32(ra + rb)
                assert T[i, j] == t or (np.isnan(T[i, j]) and np.isnan(t))
                y = np.float32(brute_force_round(float(t), e, m, d, vals))
                assert Y[i, j] == y or (np.isnan(Y[i, j]) and np.isnan(y))
    # rounding twice differs from rounding the exact sum once somewhere (the formula really has two roundings)
    Y, T = oracle.linear_epilogue(acc, bias, 6, 9, True)
    once = oracle.quantize((acc.astype(np.float64) + bias.astype(np.float64)[None, :]).astype(np.float32), 6, 9, True)
    assert not np.array_equal(Y, once)
