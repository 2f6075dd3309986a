"""FMAC and FMAC-8 by their plain definition, in exact rational arithmetic -- TEST INFRASTRUCTURE ONLY.

This is the DEFINITION the other FMAC code is judged by (the C routines oracle_fmac / oracle_fmac8_dot
in fmt_oracle.c are the fast checker for large cases and are themselves pinned to this file):

  * the value set of a 1/e/m format is enumerated from Def. III.1 / Def. III.2 (Sec. III): denormals
    k * 2^(Emin-m), 0 < k < 2^m, and normals (2^m + k) * 2^(E-m), Emin <= E <= Emax, with the vanilla
    bias Emax = 2^(e-1) - 1, Emin = 1 - Emax (Table I);
  * rounding an exact rational q to the format is a search for the nearest element of that set, ties
    to the element whose code is even, magnitudes that are nearer to 2^(Emax+1) than to the largest
    finite value (or as near) become infinity, and with denormals flushed ("n") a result below 2^Emin
    becomes zero;
  * FMAC (Sec. III-B) is a + w*x formed EXACTLY as a rational and rounded once;
  * FMAC-8 (Sec. IV-A, Algorithm 1) keeps a 16-bit accumulator over 8 consecutive FMACs, adds it into
    a single-precision master accumulator at every k that is a multiple of 8 (one fp32 addition) and
    once more after the last k, and rounds the master to the format.

No float arithmetic decides anything here except the fp32 master additions the algorithm prescribes
(numpy float32 additions, correctly rounded).  Pure Python with Fractions: for small cases only.
Nothing in the GPU library, and nothing of fmt_oracle.c, is used or shared.
"""
from __future__ import annotations

import bisect
import math
from fractions import Fraction

import numpy as np

_SETS = {}


def value_set(e: int, m: int):
    """(values, beyond): the non-negative finite values of 1/e/m, ascending (index = code without the
    sign), and 2^(Emax+1), the value the code after the largest finite one would have."""
    key = (e, m)
    if key not in _SETS:
        emax = 2 ** (e - 1) - 1
        emin = 1 - emax
        vals = [Fraction(0)]
        vals += [Fraction(k) * Fraction(2) ** (emin - m) for k in range(1, 1 << m)]
        for E in range(emin, emax + 1):
            step = Fraction(2) ** (E - m)
            vals += [((1 << m) + k) * step for k in range(1 << m)]
        _SETS[key] = (vals, Fraction(2) ** (emax + 1))
    return _SETS[key]


def round_to_format(q: Fraction, e: int, m: int, d: bool, zero_sign: float = 1.0) -> float:
    """Nearest value of the format to the exact rational q (ties to the even code, overflow to
    infinity, optional flush).  A zero result carries the sign of q; q == 0 takes zero_sign."""
    if q == 0:
        return math.copysign(0.0, zero_sign)
    vals, beyond = value_set(e, m)
    a = abs(q)
    if a >= beyond:
        r = math.inf
    else:
        hi = bisect.bisect_left(vals, a)            # vals[hi-1] < a <= vals[hi], hi == len(vals) above the largest
        lo = hi - 1 if hi > 0 else 0
        upper = vals[hi] if hi < len(vals) else beyond
        dl, dh = a - vals[lo], upper - a
        i = lo if dl < dh else hi if dh < dl else (lo if lo % 2 == 0 else hi)
        r = math.inf if i == len(vals) else float(vals[i])   # every value of a format with e <= 8 is a double
        if not d and 0.0 < r < 2.0 ** (2 - 2 ** (e - 1)):
            r = 0.0
    return math.copysign(r, 1.0 if q > 0 else -1.0)


def quantize(x: float, e: int, m: int, d: bool) -> float:
    """Q_{e,m,d|n} of one fp32 value by the same search (any NaN gives NaN, infinities pass)."""
    x = float(x)
    if math.isnan(x) or math.isinf(x):
        return x
    return round_to_format(Fraction(x), e, m, d, zero_sign=math.copysign(1.0, x))


def fmac(a: float, w: float, x: float, e: int, m: int, d: bool) -> float:
    """o(a + w*x): the exact sum rounded once to the format (Sec. III-B).  a, w, x are values of the
    format.  Non-finite cases follow the arithmetic of the extended reals (inf - inf and 0 * inf are NaN)."""
    a, w, x = float(a), float(w), float(x)
    if not (math.isfinite(a) and math.isfinite(w) and math.isfinite(x)):
        return a + w * x                             # only infinities and NaN decide: no rounding is involved
    p_negative = (math.copysign(1.0, w) < 0) != (math.copysign(1.0, x) < 0)
    # an exact zero sum is -0 only when both terms are negative (zeros)
    both_negative = math.copysign(1.0, a) < 0 and p_negative
    return round_to_format(Fraction(a) + Fraction(w) * Fraction(x), e, m, d, zero_sign=-1.0 if both_negative else 1.0)


def fmac8_dot(w, x, e: int, m: int, d: bool) -> np.float32:
    """Algorithm 1 on two sequences of values of the format."""
    master = np.float32(0.0)
    a16 = 0.0
    with np.errstate(over="ignore", invalid="ignore"):
        for k in range(len(w)):
            if k % 8 == 0:
                master = np.float32(master + np.float32(a16))     # one single-precision addition
                a16 = 0.0
            a16 = fmac(a16, w[k], x[k], e, m, d)
        master = np.float32(master + np.float32(a16))
    out = quantize(float(master), e, m, d)
    return np.float32(np.nan) if math.isnan(out) else np.float32(out)


def gemm_fmac8(A, B, e: int, m: int, d: bool, transA: bool = False, transB: bool = False) -> np.ndarray:
    """C[i][j] = FMAC-8 dot product of row i of Q(op(A)) and column j of Q(op(B)); small shapes only."""
    A = np.asarray(A, dtype=np.float32)
    B = np.asarray(B, dtype=np.float32)
    opA = A.T if transA else A
    opB = B.T if transB else B
    M, K = opA.shape
    K2, N = opB.shape
    assert K == K2
    qa = [[quantize(opA[i, k], e, m, d) for k in range(K)] for i in range(M)]
    qb = [[quantize(opB[k, j], e, m, d) for k in range(K)] for j in range(N)]
    C = np.empty((M, N), dtype=np.float32)
    for i in range(M):
        for j in range(N):
            C[i, j] = fmac8_dot(qa[i], qb[j], e, m, d)
    return C
