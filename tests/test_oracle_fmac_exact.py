"""Pins of oracle/fmac_exact.py (FMAC and FMAC-8 by their plain definition, exact rationals) against
things that are not itself, and of the fast C routines against it.  CPU only.

  * its value set against Table I and the code counts of Sec. III;
  * its rounding against numpy's IEEE binary16 conversion (1/5/10/d is binary16) and, for sums that
    are exact in double precision, its FMAC against "add in fp64, convert once" -- a single rounding by
    a library routine;
  * FMAC against hand-worked cases (a tie, a tie broken by a term 2^-60 of its size, the flush rule,
    signed zeros, overflow);
  * Algorithm 1 against hand-worked runs where every partial result can be written down;
  * oracle.fmac / oracle.fmac8_dot / oracle.gemm_fmac8 (C, fp64 with round-to-odd) against it on random
    and adversarial inputs, including 1/8/7 and 1/7/8 where the C routine's fp64 step is the one used.
"""
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workloads
from oracle import fmac_exact as fx

FORMATS = [(5, 10, True), (5, 10, False), (6, 9, True), (6, 9, False), (8, 7, True), (8, 7, False), (7, 8, True),
           (4, 3, True), (3, 2, False)]


def test_value_set_matches_table_1_and_code_counts(golden_dir):
    import os
    rows = [l.split() for l in open(os.path.join(golden_dir, "table1_formats.txt")) if l.strip() and not l.startswith("#")]
    assert rows, "golden table is empty"
    for e, m in [(5, 10), (6, 9), (8, 7)]:
        vals, beyond = fx.value_set(e, m)
        assert len(vals) == (2 ** e - 1) * 2 ** m            # codes 0 .. largest finite, per sign
        assert vals == sorted(set(vals))
        assert beyond == 2 * vals[-(1 << m)]                  # 2^(Emax+1): twice the smallest value of the top binade
    v5, _ = fx.value_set(5, 10)
    v6, _ = fx.value_set(6, 9)
    v8, _ = fx.value_set(8, 7)
    assert v5[1] == Fraction(1, 2 ** 24) and v5[1 << 10] == Fraction(1, 2 ** 14) and v5[-1] == 65504   # Table I, binary16
    assert v6[1] == Fraction(1, 2 ** 39) and v6[1 << 9] == Fraction(1, 2 ** 30) and v6[-1] == 2 ** 32 - 2 ** 22
    assert v8[1 << 7] == Fraction(1, 2 ** 126) and v8[-1] == (2 - Fraction(1, 128)) * 2 ** 127


def test_rounding_is_numpy_binary16_conversion():
    rng = np.random.default_rng(0)
    x = np.concatenate([workloads.log2_normal(4000, -8, 8, 0.02, rng), workloads.special_values(),
                        np.array([65504, 65519.99, 65520, 65536, 2.0 ** -25, 2.0 ** -25 * 1.0001, 2.0 ** -24 * 1.5], np.float32)])
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).astype(np.float32)
    for xi, wi in zip(x, want):
        got = fx.quantize(float(xi), 5, 10, True)
        assert (np.isnan(got) and np.isnan(wi)) or (got == wi and np.signbit(got) == np.signbit(wi)), (xi, got, wi)


def test_fmac_is_one_rounding_of_an_fp64_sum_when_that_sum_is_exact():
    """binary16 operands with exponents close enough that a + w*x is exact in fp64: converting that
    double to binary16 is one correctly rounded step done by numpy."""
    rng = np.random.default_rng(1)
    a = workloads.log2_normal(3000, 0, 4, 0.05, rng).astype(np.float16)
    w = workloads.log2_normal(3000, 0, 2, 0.05, rng).astype(np.float16)
    x = workloads.log2_normal(3000, 0, 2, 0.05, rng).astype(np.float16)
    checked = 0
    for ai, wi, xi in zip(a, w, x):
        s = np.float64(ai) + np.float64(wi) * np.float64(xi)
        if Fraction(float(s)) != Fraction(float(ai)) + Fraction(float(wi)) * Fraction(float(xi)):
            continue
        with np.errstate(over="ignore"):
            want = np.float16(s)
        got = fx.fmac(float(ai), float(wi), float(xi), 5, 10, True)
        assert got == float(want), (ai, wi, xi)
        checked += 1
    assert checked > 2500


def test_fmac_hand_worked_cases():
    f = (6, 9, True)
    ulp1 = 2.0 ** -9                                        # spacing of 1/6/9 in [1, 2)
    # exact tie between 1 and 1 + ulp: goes to the even code (1.0); between 1+ulp and 1+2ulp: up
    assert fx.fmac(1.0, 2.0 ** -5, 2.0 ** -5, *f) == 1.0
    assert fx.fmac(1.0 + ulp1, 2.0 ** -5, 2.0 ** -5, *f) == 1.0 + 2 * ulp1
    # a product far below the accumulator's last bit decides a tie only if it is seen exactly:
    # a = 1 + ulp/2 is not a value, so build the tie from a = 1 and w*x = ulp/2 + 2^-39*2^-30
    assert fx.fmac(1.0, 2.0 ** -5 + 2.0 ** -14, 2.0 ** -5, *f) == 1.0 + ulp1       # just above the tie
    # below 1 the spacing is 2^-10: -1 + 2^-11 is the tie between -1 (even code) and -(1 - 2^-10)
    assert fx.fmac(-1.0, 2.0 ** -5, 2.0 ** -6, *f) == -1.0
    assert fx.fmac(-1.0, 2.0 ** -5 + 2.0 ** -14, 2.0 ** -6, *f) == -(1.0 - 2.0 ** -10)   # 2^-20 past the tie
    # cancellation to an exact zero is +0; (-0) + (-0 * 1) is -0
    assert np.signbit(fx.fmac(-1.0, 1.0, 1.0, *f)) == False
    assert np.signbit(fx.fmac(-0.0, -0.0, 1.0, *f)) == True
    # a sum below half the smallest denormal rounds to a zero with the sum's sign
    r = fx.fmac(0.0, -(2.0 ** -30), 2.0 ** -30, *f)
    assert r == 0.0 and np.signbit(r)
    # flush: 1/6/9/n drops results below 2^-30, and keeps what rounds up to 2^-30
    assert fx.fmac(0.0, 2.0 ** -20, 2.0 ** -11, 6, 9, False) == 0.0
    assert fx.fmac(0.0, 2.0 ** -20, 2.0 ** -11, 6, 9, True) == 2.0 ** -31
    assert fx.fmac(2.0 ** -30 - 2.0 ** -39, 2.0 ** -20, 2.0 ** -20, 6, 9, False) == 2.0 ** -30   # tie to even, survives
    # overflow: maxN + half an ulp goes to infinity, anything less stays
    maxn = 2.0 ** 32 - 2.0 ** 22
    assert fx.fmac(maxn, 2.0 ** 10, 2.0 ** 11, *f) == np.inf
    assert fx.fmac(maxn, 2.0 ** 10, 2.0 ** 11 - 2.0 ** 2, *f) == maxn
    assert fx.fmac(np.inf, 1.0, 1.0, *f) == np.inf and np.isnan(fx.fmac(np.inf, -np.inf, 1.0, *f))


def test_algorithm_1_hand_worked():
    f = (6, 9, True)
    # 20 products of 1 * 1: a16 counts 1..8 exactly, master takes 8, 8, 4 -> 20
    assert fx.fmac8_dot([1.0] * 20, [1.0] * 20, *f) == 20.0
    # 1/6/9 has 10 significant bits: adding 1 to 1024 inside a group of 8 is lost (tie to even) every time,
    # while the fp32 master keeps units: groups (1024, then seven 1s) -> a16 = 1024; a group of eight 1s -> 8
    w = [1024.0] + [1.0] * 7 + [1.0] * 8
    assert fx.fmac8_dot(w, [1.0] * 16, *f) == 1032.0
    # the same numbers in another order: 1s first (a16 = 7), then 1024 -> 1031 is not a value: rounds to 1032 (even)
    w2 = [1.0] * 7 + [1024.0] + [1.0] * 8
    assert fx.fmac8_dot(w2, [1.0] * 16, *f) == 1040.0
    # the final rounding R(master): 1024 + 1 + 1 accumulates exactly in fp32 across groups, then rounds
    w3 = [1024.0] + [0.0] * 7 + [1.0] + [0.0] * 7 + [1.0]
    assert fx.fmac8_dot(w3, [1.0] * 17, *f) == 1026.0
    w4 = [1024.0] + [0.0] * 7 + [1.0]
    assert fx.fmac8_dot(w4, [1.0] * 9, *f) == 1024.0          # 1025 ties to the even code
    assert fx.fmac8_dot([], [], *f) == 0.0


@pytest.mark.parametrize("e,m,d", FORMATS)
def test_c_fmac_equals_the_definition(e, m, d):
    rng = np.random.default_rng(31 * e + m)
    c = oracle.format_constants(e, m)
    span = c["Emax"] - c["Emin"]
    n = 1200
    mid = (c["Emin"] + c["Emax"]) / 2
    a = oracle.quantize(workloads.log2_normal(n, mid, span / 4, 0.05, rng), e, m, d)
    w = oracle.quantize(workloads.log2_normal(n, mid / 2, span / 8, 0.05, rng), e, m, d)
    x = oracle.quantize(workloads.log2_normal(n, mid / 2, span / 8, 0.05, rng), e, m, d)
    # adversarial: products that land on or next to the accumulator's rounding boundary
    vals, _ = fx.value_set(e, m)
    for i in rng.integers(1 << m, len(vals) - 2, 150):
        half = (vals[i + 1] - vals[i]) / 2
        k = half.numerator.bit_length() - half.denominator.bit_length()
        kw, kx = (k + 1) // 2, k // 2
        if c["Emin"] <= kw <= c["Emax"] and c["Emin"] <= kx <= c["Emax"]:
            a = np.append(a, np.float32(vals[i]))
            w = np.append(w, np.float32(2.0 ** kw))
            x = np.append(x, np.float32(2.0 ** kx))
    for ai, wi, xi in zip(a, w, x):
        want = fx.fmac(ai, wi, xi, e, m, d)
        got = float(oracle.fmac(ai, wi, xi, e, m, d))
        assert (np.isnan(got) and np.isnan(want)) or (got == want and np.signbit(got) == np.signbit(want)), (ai, wi, xi, got, want)


@pytest.mark.parametrize("e,m,d", [(5, 10, True), (6, 9, True), (6, 9, False), (8, 7, False), (7, 8, True)])
def test_c_gemm_fmac8_equals_the_definition(e, m, d):
    rng = np.random.default_rng(e * m)
    c = oracle.format_constants(e, m)
    span = c["Emax"] - c["Emin"]
    A = workloads.log2_normal((6, 43), (c["Emin"] + c["Emax"]) / 4, span / 6, 0.05, rng)
    B = workloads.log2_normal((43, 5), (c["Emin"] + c["Emax"]) / 4, span / 6, 0.05, rng)
    want = fx.gemm_fmac8(A, B, e, m, d)
    got = oracle.gemm_fmac8(A, B, e, m, d)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))
    got_t = oracle.gemm_fmac8(np.ascontiguousarray(A.T), np.ascontiguousarray(B.T), e, m, d, transA=True, transB=True)
    assert np.array_equal(got_t[~nan].view(np.uint32), want[~nan].view(np.uint32))
