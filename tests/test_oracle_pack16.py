"""Pins for the oracle's packed 16-bit storage (Sec. III encoding of the values Sec. IV-A's rounding
produces): oracle.pack16 / oracle.unpack16 against things other than themselves --
  * IEEE binary16 (1/5/10 "is" half precision, Sec. III): numpy's float16 in both directions, all
    2^16 codes;
  * bfloat16 (1/8/7 has fp32's exponent range, Sec. III): the upper half of the fp32 pattern, and
    torch's bfloat16 conversion;
  * any format: the value set enumerated from Def. III.1 in exact rationals -- codes in ascending
    order are the values in ascending order;
  * Table I's constants as codes of 1/6/9.
CPU only."""
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle

pytestmark = pytest.mark.filterwarnings("ignore:overflow encountered in cast")


def bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def edge_values(rng, n=200000):
    """fp32 inputs spread over all binades, with zeros, infinities, NaN and both signs."""
    u = rng.integers(0, 1 << 32, n, dtype=np.uint64).astype(np.uint32)
    x = u.view(np.float32).copy()
    x[:8] = [0.0, -0.0, np.inf, -np.inf, np.nan, 65504.0, 65520.0, -65520.0]
    return x


def test_binary16_unpack_is_numpy_half_all_codes():
    codes = np.arange(1 << 16, dtype=np.uint16)
    want = codes.view(np.float16).astype(np.float32)
    got = oracle.unpack16(codes, 5, 10)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(bits(got[~nan]), bits(want[~nan]))          # signed zeros and denormals included
    assert np.all(bits(got[nan]) == 0x7FC00000)


def test_binary16_pack_is_numpy_half():
    x = edge_values(np.random.default_rng(1))
    want = x.astype(np.float16).view(np.uint16)
    got = oracle.pack16(x, 5, 10, True)
    nan = np.isnan(x)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.all(got[nan] == 0x7E00)
    # flushed variant: results in the denormal range become zeros of the same sign
    got_n = oracle.pack16(x, 5, 10, False)
    den = (~nan) & ((want & 0x7C00) == 0)
    assert np.array_equal(got_n[~nan & ~den], want[~nan & ~den])
    assert np.array_equal(got_n[den], want[den] & 0x8000)
    assert int(den.sum()) > 1000


def test_bfloat16_is_the_upper_half_of_fp32():
    codes = np.arange(1 << 16, dtype=np.uint16)
    want = (codes.astype(np.uint32) << 16).view(np.float32)
    got = oracle.unpack16(codes, 8, 7)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(bits(got[~nan]), bits(want[~nan]))
    x = edge_values(np.random.default_rng(2))
    t = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = oracle.pack16(x, 8, 7, True)
    nanx = np.isnan(x)
    assert np.array_equal(got[~nanx], t[~nanx])
    assert np.all(got[nanx] == 0x7FC0)


@pytest.mark.parametrize("e,m", [(6, 9), (5, 2), (4, 3), (2, 1), (7, 8), (3, 12)])
def test_code_order_is_value_order_of_the_definition(e, m):
    """Def. III.1: x = M * 2^(E-p+1) with p = m + 1; denormals E = Emin, 0 < M < 2^m; normals
    Emin <= E <= Emax, 2^m <= M < 2^(m+1).  Enumerated exactly and sorted, the positive values are
    the codes 1, 2, ... up to the code below +infinity, in order."""
    bias = (1 << (e - 1)) - 1
    emin, emax = 1 - bias, bias
    vals = [Fraction(M) * Fraction(2) ** (emin - m) for M in range(1, 1 << m)]
    for E in range(emin, emax + 1):
        vals += [Fraction(M) * Fraction(2) ** (E - m) for M in range(1 << m, 1 << (m + 1))]
    assert vals == sorted(vals) and len(set(vals)) == len(vals)
    top = ((1 << e) - 1) << m
    assert len(vals) == top - 1
    codes = np.arange(1, top, dtype=np.uint16)
    got = oracle.unpack16(codes, e, m)
    want = np.array([float(v) for v in vals], dtype=np.float64)
    assert np.array_equal(got.astype(np.float64), want)
    neg = oracle.unpack16(codes | np.uint16(1 << (e + m)), e, m)
    assert np.array_equal(neg.astype(np.float64), -want)
    # zero, infinities, NaN
    sp = oracle.unpack16(np.array([0, 1 << (e + m), top, top | (1 << (e + m)), top + 1], dtype=np.uint16), e, m)
    assert bits(sp[:4]).tolist() == [0x00000000, 0x80000000, 0x7F800000, 0xFF800000] and np.isnan(sp[4])
    # and the encoder inverts it (every non-NaN code is a fixed point of pack o unpack)
    allc = np.arange(1 << (1 + e + m), dtype=np.uint32).astype(np.uint16)
    v = oracle.unpack16(allc, e, m)
    back = oracle.pack16(v, e, m, True)
    nan = np.isnan(v)
    assert np.array_equal(back[~nan], allc[~nan])
    assert np.all(back[nan] == (top | (1 << (m - 1))))


def test_table_I_constants_as_codes_of_1_6_9():
    """Table I: 1/6/9/d has Emin = -30, Emax = 31, smallest denormal 2^-39."""
    x = np.array([2.0 ** -39, 2.0 ** -30, (2 - 2.0 ** -9) * 2.0 ** 31, 1.0, -1.0, 2.0 ** 32, 2.0 ** -41], dtype=np.float32)
    got = oracle.pack16(x, 6, 9, True).tolist()
    assert got == [0x0001, 0x0200, 0x7DFF, 31 << 9, 0x8000 | (31 << 9), 0x7E00, 0x0000]
    assert oracle.pack16(x[:1], 6, 9, False).tolist() == [0x0000]      # flushed


def test_upper_bits_ignored_and_width_limit():
    v = oracle.unpack16(np.array([0x0033, 0xFF33], dtype=np.uint16), 4, 3)     # 8-bit codes
    assert bits(v)[0] == bits(v)[1]
    with pytest.raises(ValueError):
        oracle.pack16(np.zeros(1, np.float32), 8, 8, True)
    with pytest.raises(ValueError):
        oracle.unpack16(np.zeros(1, np.uint16), 6, 10)
