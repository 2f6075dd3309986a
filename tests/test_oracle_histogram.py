"""Pins for the oracle's per-tensor statistics (the denormal fraction of Sec. V plus binade
bins): hand-built tensors with known counts, closed-form counts on the exhaustive code set,
partition invariants and consistency with the quantizer.  CPU only."""
import numpy as np
import pytest

import oracle
import workloads
from fmtdef import consts, decode_codes

FORMATS16 = [(5, 10), (6, 9), (8, 7)]
CLASSES = ("zero", "underflow", "denormal", "normal", "overflow", "inf", "nan")


def test_one_element_per_binade():
    """x = 1.5 * 2^k for k = -60..30, one each: every bin count is fixed by hand."""
    ks = np.arange(-60, 31)
    x = (1.5 * np.exp2(ks.astype(np.float64))).astype(np.float32)
    h = oracle.histogram(x, 6, 9, exp_lo=-48)
    bins = h["bins"]
    assert bins[0] == 13                      # k = -60..-48 all clamp into the first bin
    assert np.all(bins[1:63] == 1)            # k = -47..14
    assert bins[63] == 16                     # k = 15..30
    assert h["total"] == ks.size and h["zero"] == 0 and h["nan"] == 0 and h["inf"] == 0
    # classes for 1/6/9: 1.5*2^k rounds to 0 iff 1.5*2^k < 2^-40 (k <= -41);
    # denormal result iff -40 <= k <= -31  (1.5*2^-40 -> 2^-39 = minD; 1.5*2^-31 stays below 2^-30)
    assert h["underflow"] == 20               # k = -60..-41
    assert h["denormal"] == 10                # k = -40..-31
    assert h["normal"] == 61                  # k = -30..30
    assert h["overflow"] == 0
    # a different window moves the bins, not the classes
    h2 = oracle.histogram(x, 6, 9, exp_lo=-60)
    assert np.all(h2["bins"][:63] == 1) and h2["bins"][63] == ks.size - 63
    for c in CLASSES:
        assert h2[c] == h[c]


def test_one_element_per_class():
    e, m = 5, 10
    x = np.array([0.0, -0.0,                  # zero x2
                  2.0 ** -26, -2.0 ** -25,     # underflow x2 (-2^-25 is the tie that goes to zero)
                  2.0 ** -24, 2.0 ** -15, -3 * 2.0 ** -24,   # denormal x3
                  2.0 ** -14, 1.0, -65504.0, 65519.0,        # normal x4
                  65520.0, -1e30,              # overflow x2
                  np.inf, -np.inf, np.inf,     # inf x3
                  np.nan], dtype=np.float32)   # nan x1
    h = oracle.histogram(x, e, m)
    assert [h[c] for c in CLASSES] == [2, 2, 3, 4, 2, 3, 1]
    assert h["total"] == x.size
    assert h["bins"].sum() == x.size - 2 - 1          # zeros and NaN are not binned
    assert h["bins"][63] == 2 + 2 + 3                 # binade 2^15 and above: -65504, 65519; 65520, -1e30; three infinities
    # 1/8/7 sees the same tensor with no underflow/overflow at all
    h8 = oracle.histogram(x, 8, 7)
    assert [h8[c] for c in CLASSES] == [2, 0, 0, 11, 0, 3, 1]   # all 11 finite non-zero inputs are normal


@pytest.mark.parametrize("e,m", FORMATS16)
def test_exhaustive_code_set_counts(e, m):
    """On the set of all 2^16 codes the class counts are closed-form."""
    v = decode_codes(e, m)
    h = oracle.histogram(v, e, m)
    nden = 2 * ((1 << m) - 1)
    nnorm = 2 * ((1 << e) - 2) * (1 << m)
    assert (h["zero"], h["denormal"], h["normal"], h["inf"], h["nan"]) == (2, nden, nnorm, 2, nden)
    assert h["underflow"] == 0 and h["overflow"] == 0 and h["total"] == 1 << 16
    # each normal binade holds 2 * 2^m codes
    c = consts(e, m)
    for E in range(max(c["Emin"], -47), min(c["Emax"], 14) + 1):
        assert h["bins"][E + 48] == 2 << m


@pytest.mark.parametrize("e,m", FORMATS16 + [(4, 3), (7, 12)])
def test_partition_and_quantizer_consistency(e, m):
    rng = np.random.default_rng(5 * e + m)
    x = np.concatenate([workloads.random_bits(100000, e * 100 + m), workloads.special_values(),
                        workloads.log2_normal(100000, -20, 8, 0.05, rng)])
    h = oracle.histogram(x, e, m)
    assert h["total"] == x.size == sum(h[c] for c in CLASSES)
    assert int(h["bins"].sum()) == h["total"] - h["zero"] - h["nan"]
    # classes against the quantizer's own outputs
    qd = oracle.quantize(x, e, m, True)
    qn = oracle.quantize(x, e, m, False)
    fin_in = np.isfinite(x)
    assert h["nan"] == int(np.isnan(x).sum())
    assert h["inf"] == int(np.isinf(x).sum())
    assert h["zero"] == int((x == 0).sum())
    assert h["underflow"] == int(((qd == 0) & (x != 0)).sum())
    assert h["overflow"] == int((np.isinf(qd) & fin_in).sum())
    assert h["denormal"] == int((qd.view(np.uint32) != qn.view(np.uint32)).sum())
    assert h["zero"] + h["underflow"] + h["denormal"] == int((qn == 0).sum())
    # bins are the binade of the input, whatever the format
    h2 = oracle.histogram(x, 8, 23)
    assert np.array_equal(h["bins"], h2["bins"])
    # bins recomputed with numpy's frexp
    ok = ~np.isnan(x) & (x != 0)
    with np.errstate(over="ignore"):
        ex = np.frexp(np.abs(x[ok]).astype(np.float64))[1] - 1
    ex = np.where(np.isinf(x[ok]), 10 ** 6, ex)
    b = np.clip(ex + 48, 0, 63)
    assert np.array_equal(np.bincount(b, minlength=64), h["bins"].astype(np.int64))


def test_expected_fractions_of_synthetic_distributions():
    """Statistical sanity (not a bit-level pin): for log2|x| ~ N(mu, s^2) the class fractions of
    the non-zero part follow from the normal CDF."""
    from math import erf, sqrt
    Phi = lambda z: 0.5 * (1 + erf(z / sqrt(2)))
    x = workloads.config1()["x"]
    n = x.size
    for (e, m) in [(5, 10), (6, 9)]:
        c = consts(e, m)
        h = oracle.histogram(x, e, m)
        nz = h["total"] - h["zero"]
        under = Phi((c["Emin"] - m - 1 + 14) / 6)
        den = Phi((c["Emin"] + 14) / 6) - under
        assert abs(h["underflow"] / nz - under) < 4 / np.sqrt(n)
        assert abs(h["denormal"] / nz - den) < 4 / np.sqrt(n)
    assert abs(oracle.histogram(x, 5, 10)["zero"] / n - 0.01) < 4 * np.sqrt(0.01 / n)
