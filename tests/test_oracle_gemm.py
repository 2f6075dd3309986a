"""Pins for the oracle's FMACS matrix product (Sec. III-B, Sec. IV-A): cases whose result is fixed
by hand or by exact integer arithmetic, the three operand layouts, and a numpy fp64 product of
independently quantized operands.  CPU only."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workloads
from fmtdef import brute_force_round, positive_finite_values


def test_hand_worked_2x2():
    """1/6/9 keeps 10 significant bits: 1 + 2^-10 rounds to 1 (tie to even), 1 + 3*2^-10 rounds
    to 1 + 2^-8 (tie to even), 3 stays 3.  C = Q(A) Q(B) by hand."""
    A = np.array([[1 + 2.0 ** -10, 3.0], [0.5, 1 + 3 * 2.0 ** -10]], dtype=np.float32)
    B = np.array([[2.0, 1.0], [1.0, -4.0]], dtype=np.float32)
    qa = np.array([[1.0, 3.0], [0.5, 1 + 2.0 ** -8]])
    want = (qa @ B.astype(np.float64)).astype(np.float32)
    got = oracle.gemm(A, B, 6, 9, True)
    assert np.array_equal(got, want)
    assert got[0, 0] == 5.0 and got[0, 1] == -11.0


@pytest.mark.parametrize("transA,transB", [(False, False), (False, True), (True, False), (True, True)])
def test_exact_integer_case_all_layouts(transA, transB):
    """Small integers times powers of two are values of every 16-bit format and all partial sums
    are exact, so the product must equal integer arithmetic exactly in every layout."""
    rng = np.random.default_rng(3)
    M, N, K = 13, 7, 29
    Ai = rng.integers(-15, 16, (M, K))
    Bi = rng.integers(-15, 16, (K, N))
    sa = rng.integers(-6, 7, (M, 1))
    sb = rng.integers(-6, 7, (1, N))
    A = (Ai * np.exp2(sa)).astype(np.float32)
    B = (Bi * np.exp2(sb)).astype(np.float32)
    want = ((Ai @ Bi) * np.exp2(sa) * np.exp2(sb)).astype(np.float32)
    Ain = np.ascontiguousarray(A.T) if transA else A
    Bin = np.ascontiguousarray(B.T) if transB else B
    for (e, m) in [(5, 10), (6, 9), (8, 7)]:
        got = oracle.gemm(Ain, Bin, e, m, True, transA=transA, transB=transB)
        assert np.array_equal(got, want)


def test_identity_and_permutation_return_quantized_operand():
    rng = np.random.default_rng(4)
    A = workloads.log2_normal((17, 12), -14, 6, 0.05, rng)
    I = np.eye(12, dtype=np.float32)
    P = I[rng.permutation(12)]
    for (e, m, d) in [(5, 10, True), (6, 9, False), (8, 7, True)]:
        qa = oracle.quantize(A, e, m, d)
        fin = np.where(np.isfinite(qa), qa, 0).astype(np.float32)   # inf * 0 would be NaN; keep the case finite
        Ain = np.where(np.isfinite(qa), A, 0).astype(np.float32)
        assert np.array_equal(oracle.gemm(Ain, I, e, m, d), fin)
        assert np.array_equal(oracle.gemm(Ain, P, e, m, d), fin @ P)


def test_outer_product_is_exact_and_products_are_not_rounded():
    """K = 1: C_ij = Q(a_i) Q(b_j) with the product itself NOT rounded to the format (FMACS keeps
    the exact product; Sec. IV-A says products are not rounded).  The exact product of two 10-bit
    significands has up to 20 bits and is still an fp32."""
    rng = np.random.default_rng(5)
    a = workloads.log2_normal((9, 1), -3, 2, 0, rng)
    b = workloads.log2_normal((1, 11), -3, 2, 0, rng)
    vals = positive_finite_values(6, 9)
    qa = [Fraction(brute_force_round(float(t), 6, 9, True, vals)) for t in a[:, 0]]
    qb = [Fraction(brute_force_round(float(t), 6, 9, True, vals)) for t in b[0]]
    got = oracle.gemm(a, b, 6, 9, True)
    some_unrepresentable = False
    for i in range(9):
        for j in range(11):
            p = qa[i] * qb[j]
            assert Fraction(float(got[i, j])) == p
            if float(oracle.quantize_one(np.float32(float(p)), 6, 9, True)) != float(p):
                some_unrepresentable = True
    assert some_unrepresentable


def test_exact_rational_dot_products():
    """Sums checked against exact rational arithmetic (then one rounding to fp32)."""
    rng = np.random.default_rng(6)
    K = 37
    A = workloads.log2_normal((3, K), -2, 3, 0.1, rng)
    B = workloads.log2_normal((K, 2), -2, 3, 0.1, rng)
    vals = positive_finite_values(5, 10)
    qa = [[Fraction(brute_force_round(float(t), 5, 10, False, vals)) for t in row] for row in A]
    qb = [[Fraction(brute_force_round(float(t), 5, 10, False, vals)) for t in row] for row in B]
    got = oracle.gemm(A, B, 5, 10, False)
    for i in range(3):
        for j in range(2):
            exact = sum(qa[i][k] * qb[k][j] for k in range(K))
            assert got[i, j] == np.float32(float(exact))       # float(Fraction) rounds correctly


@pytest.mark.parametrize("transA,transB", [(False, False), (False, True), (True, False)])
def test_matches_numpy_fp64_on_quantized_operands(transA, transB):
    rng = np.random.default_rng(7)
    M, N, K = 65, 33, 130
    A = (rng.standard_normal((M, K)) * 2.0 ** -10).astype(np.float32)
    B = (rng.standard_normal((K, N)) * 2.0 ** -10).astype(np.float32)
    Ain = np.ascontiguousarray(A.T) if transA else A
    Bin = np.ascontiguousarray(B.T) if transB else B
    for (e, m, d) in [(6, 9, True), (5, 10, False), (8, 7, False)]:
        ref = oracle.quantize(A, e, m, d).astype(np.float64) @ oracle.quantize(B, e, m, d).astype(np.float64)
        got = oracle.gemm(Ain, Bin, e, m, d, transA=transA, transB=transB)
        # numpy's blocked summation order differs; both are fp64 sums rounded to fp32
        assert np.max(np.abs(got - ref)) <= 2.0 ** -23 * np.max(np.abs(ref))
        rows = rng.integers(0, M, 20)
        cols = rng.integers(0, N, 20)
        samp = oracle.gemm_sampled(Ain, Bin, rows, cols, e, m, d, transA=transA, transB=transB)
        assert np.array_equal(samp, got[rows, cols])
    # rounding really happens: the unquantized product differs
    raw = (A.astype(np.float64) @ B.astype(np.float64)).astype(np.float32)
    assert not np.array_equal(raw, oracle.gemm(Ain, Bin, 6, 9, True, transA=transA, transB=transB))


def test_degenerate_shapes():
    A = np.zeros((4, 0), np.float32)
    B = np.zeros((0, 3), np.float32)
    assert np.array_equal(oracle.gemm(A, B, 6, 9, True), np.zeros((4, 3), np.float32))   # empty sum
    assert oracle.gemm(np.zeros((0, 5), np.float32), np.zeros((5, 3), np.float32), 6, 9, True).shape == (0, 3)


def test_nonfinite_operands_propagate():
    A = np.array([[1.0, np.inf], [np.nan, 1.0], [1e30, 1.0]], dtype=np.float32)
    B = np.array([[1.0, 0.0], [1.0, 1.0]], dtype=np.float32)
    got = oracle.gemm(A, B, 5, 10, True)
    assert np.isinf(got[0, 0]) and np.isinf(got[0, 1])
    assert np.isnan(got[1, 0]) and np.isnan(got[1, 1])
    # 1e30 overflows binary16 and becomes inf: inf*1 + 1*1 = inf, inf*0 + 1*1 = nan
    assert np.isinf(got[2, 0]) and np.isnan(got[2, 1])
