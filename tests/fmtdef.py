"""Test-side restatement of the 1/e/m value set, written independently of the oracle.

Used only as a *pin*: the oracle rounds with frexp/ldexp/nearbyint; here the format is an
explicitly enumerated list of values (Sec. III, Def. III.1: x = M * 2^(E-p+1); normal numbers
have 2^(p-1) <= |M| <= 2^p - 1 with Emin <= E <= Emax, denormals have E = Emin and
|M| <= 2^(p-1) - 1) and rounding is a nearest-neighbour search with exact rationals.
"""
from __future__ import annotations

import bisect
from fractions import Fraction

import numpy as np


def consts(e: int, m: int):
    bias = 2 ** (e - 1) - 1
    return {"bias": bias, "Emax": bias, "Emin": 1 - bias}


def decode_codes(e: int, m: int) -> np.ndarray:
    """fp32 value of every (1+e+m)-bit code, in code order (NaN codes decode to NaN).
    Stored exponent field 0 = zero/denormal, all ones = infinity/NaN, else normal with
    the hidden bit (Sec. III)."""
    nbits = 1 + e + m
    codes = np.arange(1 << nbits, dtype=np.int64)
    sign = np.where((codes >> (e + m)) & 1, -1.0, 1.0)
    field = (codes >> m) & ((1 << e) - 1)
    mant = codes & ((1 << m) - 1)
    c = consts(e, m)
    val = np.where(field == 0,
                   np.ldexp(mant.astype(np.float64), c["Emin"] - m),
                   np.ldexp((mant + (1 << m)).astype(np.float64), (field - c["bias"] - m).astype(np.int64)))
    top = field == (1 << e) - 1
    val = np.where(top & (mant == 0), np.inf, val)
    val = np.where(top & (mant != 0), np.nan, val)
    out = (sign * val).astype(np.float32)
    # every finite value of a format with e <= 8, m <= 23 is exactly an fp32
    fin = np.isfinite(val)
    assert np.array_equal(out[fin].astype(np.float64), (sign * val)[fin])
    return out


def positive_finite_values(e: int, m: int) -> list:
    """All positive finite values of the format as exact Fractions, ascending; index = code."""
    c = consts(e, m)
    vals = [Fraction(0)]
    for k in range(1, 1 << m):
        vals.append(Fraction(k) * Fraction(2) ** (c["Emin"] - m))
    for E in range(c["Emin"], c["Emax"] + 1):
        for k in range(1 << m):
            vals.append(Fraction((1 << m) + k) * Fraction(2) ** (E - m))
    return vals


def brute_force_round(x: float, e: int, m: int, d: bool, vals=None) -> float:
    """Nearest value of the format to the fp32 x by search over the explicitly enumerated, sorted set;
    ties go to the value whose code is even; values at or beyond the midpoint between the
    largest finite value and 2^(Emax+1) become infinity; without denormals a result below
    2^Emin is replaced by zero.  Sign is carried separately."""
    import math
    if math.isnan(x):
        return float("nan")
    if math.isinf(x) or x == 0.0:
        return x
    c = consts(e, m)
    if vals is None:
        vals = positive_finite_values(e, m)
    a = abs(Fraction(x))
    beyond = Fraction(2) ** (c["Emax"] + 1)          # the value the code after maxN would have
    grid = vals + [beyond]
    if a >= beyond:
        best_i = len(vals)
    else:
        hi = bisect.bisect_left(grid, a)              # grid[hi-1] < a <= grid[hi]
        lo = max(hi - 1, 0)
        dl, dh = abs(a - grid[lo]), abs(a - grid[hi])
        if dl < dh:
            best_i = lo
        elif dh < dl:
            best_i = hi
        else:
            best_i = lo if lo % 2 == 0 else hi
    if best_i == len(vals):
        r = float("inf")
    else:
        r = vals[best_i]
        if not d and 0 < r < Fraction(2) ** c["Emin"]:
            r = Fraction(0)
        r = float(r)
    return math.copysign(r, x)
