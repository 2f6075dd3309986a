"""Pins for the oracle's FMAC and FMAC-8 (Sec. III-B; Sec. IV-A, Algorithm 1) against exact rational
arithmetic: the fused a + w*x is formed as a Fraction and rounded once by the nearest-value search of
fmtdef.py; Algorithm 1 is re-run step by step with that exact FMAC.  CPU only."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workloads
from fmtdef import brute_force_round, consts, positive_finite_values

FORMATS = [(5, 10, True), (5, 10, False), (6, 9, True), (6, 9, False), (8, 7, True), (4, 3, True), (3, 2, False)]
_VALS = {}


def vals(e, m):
    if (e, m) not in _VALS:
        _VALS[(e, m)] = positive_finite_values(e, m)
    return _VALS[(e, m)]


def exact_round(q: Fraction, e, m, d):
    """Round an exact rational to the format (nearest, ties to even, overflow to inf, optional flush)."""
    if q == 0:
        return 0.0
    c = consts(e, m)
    v = vals(e, m)
    import bisect
    a = abs(q)
    beyond = Fraction(2) ** (c["Emax"] + 1)
    grid = v + [beyond]
    if a >= beyond:
        r = float("inf")
    else:
        hi = bisect.bisect_left(grid, a)
        lo = max(hi - 1, 0)
        dl, dh = abs(a - grid[lo]), abs(a - grid[hi])
        i = lo if dl < dh else hi if dh < dl else (lo if lo % 2 == 0 else hi)
        r = float("inf") if i == len(v) else float(v[i])
        if not d and 0 < r < 2.0 ** c["Emin"]:
            r = 0.0
    return r if q > 0 else -r


def exact_fmac(a, w, x, e, m, d):
    if np.isinf(a):                      # an overflowed accumulator stays infinite (operands are finite)
        return float(a)
    return exact_round(Fraction(float(a)) + Fraction(float(w)) * Fraction(float(x)), e, m, d)


def format_values(rng, e, m, d, n, spread):
    c = consts(e, m)
    centre = (c["Emin"] + c["Emax"]) / 2
    x = workloads.log2_normal(n, centre, spread, 0.05, rng)
    return oracle.quantize(x, e, m, d)


@pytest.mark.parametrize("e,m,d", FORMATS)
def test_fmac_against_exact_rationals(e, m, d):
    """Random operands across the format's whole range (far-apart exponents included)."""
    rng = np.random.default_rng(10 * e + m)
    c = consts(e, m)
    n = 1500
    a = format_values(rng, e, m, d, n, (c["Emax"] - c["Emin"]) / 4)
    w = format_values(rng, e, m, d, n, (c["Emax"] - c["Emin"]) / 8)
    x = format_values(rng, e, m, d, n, (c["Emax"] - c["Emin"]) / 8)
    for ai, wi, xi in zip(a, w, x):
        if not (np.isfinite(ai) and np.isfinite(wi) and np.isfinite(xi)):
            continue
        want = np.float32(exact_fmac(ai, wi, xi, e, m, d))
        got = oracle.fmac(ai, wi, xi, e, m, d)
        assert got == want or (np.isinf(got) and np.isinf(want) and got == want), (ai, wi, xi, got, want)
        if want == 0 and got == 0:
            exact = Fraction(float(ai)) + Fraction(float(wi)) * Fraction(float(xi))
            if exact != 0:
                assert np.signbit(got) == (exact < 0)


@pytest.mark.parametrize("e,m", [(5, 10), (6, 9), (8, 7)])
def test_fmac_ties_and_sticky_bits(e, m):
    """Adversarial sums: a is a value v, w*x brings it exactly onto the midpoint between v and its
    neighbour, or onto the midpoint plus / minus a far smaller term that only an exact sum sees."""
    c = consts(e, m)
    v = vals(e, m)
    rng = np.random.default_rng(e)
    idx = rng.integers(1 << m, len(v) - 2, 300)          # normal values
    for i in idx:
        lo, hi = v[i], v[i + 1]
        half = (hi - lo) / 2
        # half = 2^k: write it as w*x with w = 2^ceil(k/2), x = 2^floor(k/2) if those are format values
        k = half.numerator.bit_length() - half.denominator.bit_length()
        k = k if Fraction(2) ** k == half else k + 1
        assert Fraction(2) ** k == half
        kw, kx = (k + 1) // 2, k // 2
        if not (c["Emin"] <= kw <= c["Emax"] and c["Emin"] <= kx <= c["Emax"]):
            continue
        a, w, x = float(lo), 2.0 ** kw, 2.0 ** kx
        got = float(oracle.fmac(a, w, x, e, m, True))
        assert got == exact_fmac(a, w, x, e, m, True) == float(lo if i % 2 == 0 else hi)
        # just above the tie: w slightly larger (one ulp of the format) -> must go up
        w_up = float(v[v.index(Fraction(w)) + 1]) if Fraction(w) in v else None
        if w_up is not None:
            assert float(oracle.fmac(a, w_up, x, e, m, True)) == exact_fmac(a, w_up, x, e, m, True) == float(hi)


@pytest.mark.parametrize("e,m,d", [(5, 10, True), (6, 9, True), (6, 9, False), (8, 7, False), (4, 3, True)])
@pytest.mark.parametrize("n", [0, 1, 7, 8, 9, 16, 17, 40])
def test_fmac8_dot_follows_algorithm_1(e, m, d, n):
    """Algorithm 1 re-run with exact FMACs, fp32 master additions and the final R(.)."""
    rng = np.random.default_rng(100 * e + n)
    c = consts(e, m)
    w = format_values(rng, e, m, d, n, 3.0) if n else np.zeros(0, np.float32)
    x = format_values(rng, e, m, d, n, 3.0) if n else np.zeros(0, np.float32)
    w = np.where(np.isfinite(w), w, 1).astype(np.float32)
    x = np.where(np.isfinite(x), x, 1).astype(np.float32)
    A32 = np.float32(0)
    a16 = 0.0
    for i in range(n):
        if i % 8 == 0:
            A32 = np.float32(A32 + np.float32(a16))
            a16 = 0.0
        a16 = exact_fmac(a16, w[i], x[i], e, m, d)
    with np.errstate(over="ignore"):
        A32 = np.float32(A32 + np.float32(a16))
    want = np.float32(brute_force_round(float(A32), e, m, d, vals(e, m)))
    got = oracle.fmac8_dot(w, x, e, m, d)
    assert got == want or (np.isnan(got) and np.isnan(want)), (got, want)


def test_fmac8_differs_from_fmacs_and_matches_it_when_exact():
    """With small integers every partial sum is a value of the format, so FMAC-8 equals the exact
    product; with random data the 16-bit accumulator visibly loses accuracy against FMACS."""
    rng = np.random.default_rng(5)
    Ai = rng.integers(-3, 4, (9, 24)).astype(np.float32)
    Bi = rng.integers(-3, 4, (24, 7)).astype(np.float32)
    assert np.array_equal(oracle.gemm_fmac8(Ai, Bi, 6, 9, True), Ai @ Bi)
    A = rng.standard_normal((16, 256)).astype(np.float32)
    B = rng.standard_normal((256, 16)).astype(np.float32)
    f8 = oracle.gemm_fmac8(A, B, 6, 9, True).astype(np.float64)
    fs = oracle.gemm(A, B, 6, 9, True).astype(np.float64)
    rel = np.linalg.norm(f8 - fs) / np.linalg.norm(fs)
    assert 1e-5 < rel < 1e-2
    # the result is itself a value of the format (final R)
    assert np.array_equal(oracle.quantize(f8.astype(np.float32), 6, 9, True), f8.astype(np.float32))
    # layouts
    assert np.array_equal(oracle.gemm_fmac8(np.ascontiguousarray(A.T), np.ascontiguousarray(B.T), 6, 9, True,
                                            transA=True, transB=True), f8.astype(np.float32))
