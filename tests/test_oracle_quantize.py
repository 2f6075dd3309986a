"""Pins for the oracle's quantizer (roundfp of Sec. IV-A) against what the paper and the
mathematics fix: Table I, closed forms, the exhaustive code set of each 16-bit format, every
rounding boundary, IEEE binary16 / bfloat16 library conversions, and a brute-force search over
an explicitly enumerated value set.  CPU only."""
import os

import numpy as np
import pytest

import oracle
import workloads
from fmtdef import brute_force_round, consts, decode_codes, positive_finite_values

FORMATS16 = [(5, 10), (6, 9), (8, 7)]
VARIANTS = [(e, m, d) for (e, m) in FORMATS16 for d in (True, False)]


def bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def f32(b):
    return np.array(b, dtype=np.uint32).view(np.float32)


def same_bits(a, b):
    return np.array_equal(bits(a), bits(b))


# ---------------------------------------------------------------- Table I and closed forms

def test_table1_constants(golden_dir):
    """Emin, Emax and the smallest denormal printed in Table I (Sec. III-A)."""
    rows = [l.split() for l in open(os.path.join(golden_dir, "table1_formats.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for name, e, p, emin, emax, lg in rows:
        c = oracle.format_constants(int(e), int(p))
        assert c["Emin"] == int(emin) and c["Emax"] == int(emax), name
        if lg != "none":
            assert c["minD"] == 2.0 ** int(lg), name
            # and the quantizer really keeps that value, and drops half of it (tie to even -> 0)
            x = np.float32(2.0 ** int(lg))
            assert oracle.quantize_one(x, int(e), int(p), True) == x
            assert oracle.quantize_one(x / 2, int(e), int(p), True) == 0.0
            assert oracle.quantize_one(np.nextafter(x / 2, np.float32(1)), int(e), int(p), True) == x


CLOSED_FORMS = {
    # fp32 bit patterns worked out by hand from Def. III.1 / Table I:
    # maxN, minN, minD, max denormal, overflow threshold (first value that becomes inf), minD/2
    (5, 10): (0x477FE000, 0x38800000, 0x33800000, 0x387FC000, 0x477FF000, 0x33000000),
    (6, 9): (0x4F7FC000, 0x30800000, 0x2C000000, 0x307F8000, 0x4F7FE000, 0x2B800000),
    (8, 7): (0x7F7F0000, 0x00800000, 0x00010000, 0x007F0000, 0x7F7F8000, 0x00008000),
}


@pytest.mark.parametrize("e,m", FORMATS16)
def test_closed_form_bit_patterns(e, m):
    maxN, minN, minD, maxD, ovf, half = CLOSED_FORMS[(e, m)]
    c = oracle.format_constants(e, m)
    assert float(f32(maxN)) == c["maxN"] == (2 - 2.0 ** -m) * 2.0 ** c["Emax"]
    assert float(f32(minN)) == c["minN"] == 2.0 ** c["Emin"]
    assert float(f32(minD)) == c["minD"] == 2.0 ** (c["Emin"] - m)
    assert float(f32(maxD)) == c["minN"] - c["minD"]
    q = lambda b, d=True: bits(oracle.quantize(f32([b]), e, m, d))[0]
    # fixed points
    for b in (maxN, minN, minD, maxD):
        assert q(b) == b
    # overflow: just below the threshold -> maxN, at it -> inf
    assert q(ovf - 1) == maxN
    assert q(ovf) == 0x7F800000
    assert q(ovf | 0x80000000) == 0xFF800000
    # underflow: minD/2 is a tie between 0 (even) and minD (odd) -> 0, sign kept
    assert q(half) == 0
    assert q(half | 0x80000000) == 0x80000000
    assert q(half + 1) == minD
    # flushed variant: denormal results vanish, minN survives, and inputs that round UP to
    # minN survive as well (flush acts on the rounded value)
    assert q(maxD, False) == 0 and q(minD, False) == 0
    assert q(minN, False) == minN
    assert q(minN - 1, False) == minN
    assert q(minN - 1, True) == minN


def test_positive_code_counts():
    for (e, m), expect in zip(FORMATS16, (31743, 32255, 32639)):
        v = decode_codes(e, m)[: 1 << 15]
        assert int(np.sum(np.isfinite(v) & (v > 0))) == expect


# ---------------------------------------------------------------- exhaustive code sets

@pytest.mark.parametrize("e,m", FORMATS16)
def test_exhaustive_codes_are_fixed_points(e, m):
    """All 2^16 codes of the format, decoded from the definition: Q_d(v) = v bit for bit;
    Q_n(v) = v except that denormal codes give a zero of the same sign; NaN codes give NaN."""
    v = decode_codes(e, m)
    nan = np.isnan(v)
    assert int(nan.sum()) == 2 * ((1 << m) - 1)
    qd = oracle.quantize(v, e, m, True)
    assert same_bits(qd[~nan], v[~nan])
    assert np.all(bits(qd[nan]) == 0x7FC00000)
    qn = oracle.quantize(v, e, m, False)
    c = consts(e, m)
    den = (~nan) & (np.abs(v) > 0) & (np.abs(v) < 2.0 ** c["Emin"])
    assert int(den.sum()) == 2 * ((1 << m) - 1)
    assert same_bits(qn[~nan & ~den], v[~nan & ~den])
    assert same_bits(qn[den], np.copysign(np.float32(0), v[den]))
    # the oracle's own encoder inverts the decode
    codes = oracle.encode(qd[~nan], e, m)
    assert np.array_equal(codes, np.arange(1 << 16, dtype=np.uint32)[~nan])


@pytest.mark.parametrize("e,m,d", VARIANTS)
def test_every_rounding_boundary(e, m, d):
    """For each adjacent pair of non-negative codes (c, c+1): their midpoint is exactly an fp32
    and must go to the code with even last bit; the fp32 neighbours of the midpoint go to c and
    c+1.  Includes 0|minD (the underflow boundary) and maxN|2^(Emax+1) (the overflow one)."""
    c = consts(e, m)
    v = decode_codes(e, m)[: 1 << 15].astype(np.float64)
    last = ((1 << e) - 1) << m                       # code of +inf
    lo = v[:last].copy()                             # codes 0 .. maxN
    hi = v[1:last + 1].copy()
    hi[-1] = 2.0 ** (c["Emax"] + 1)                  # where the next code would sit
    mid64 = (lo + hi) / 2
    mid = mid64.astype(np.float32)
    assert np.array_equal(mid.astype(np.float64), mid64)
    codes = np.arange(last)
    expect_mid = np.where(codes % 2 == 0, lo, hi)
    below = np.nextafter(mid, np.float32(0))
    above = np.nextafter(mid, np.float32(np.inf))

    def finish(t):
        t = np.where(t >= 2.0 ** (c["Emax"] + 1), np.inf, t)
        if not d:
            t = np.where(t < 2.0 ** c["Emin"], 0.0, t)
        return t.astype(np.float32)

    for sgn in (1.0, -1.0):
        s = np.float32(sgn)
        assert same_bits(oracle.quantize(s * mid, e, m, d), s * finish(expect_mid))
        assert same_bits(oracle.quantize(s * below, e, m, d), s * finish(lo))
        assert same_bits(oracle.quantize(s * above, e, m, d), s * finish(hi))


# ---------------------------------------------------------------- library special cases

def _mixed_inputs(seed, n=200000):
    rng = np.random.default_rng(seed)
    parts = [workloads.random_bits(n, seed), workloads.special_values(),
             workloads.log2_normal(n, -14, 6, 0.01, rng),
             (rng.standard_normal(n) * 65504).astype(np.float32)]
    return np.concatenate(parts)


def test_binary16_matches_ieee_half():
    """1/5/10/d is IEEE half precision (Sec. III-A): numpy's float16 conversion is RNE with
    gradual underflow and overflow to infinity."""
    x = _mixed_inputs(11)
    nan = np.isnan(x)
    with np.errstate(over="ignore"):
        ref = x.astype(np.float16).astype(np.float32)
    got = oracle.quantize(x, 5, 10, True)
    assert same_bits(got[~nan], ref[~nan])
    assert np.all(np.isnan(got[nan]))


def test_bfloat16_matches_torch():
    """1/8/7 has bfloat16's layout (Sec. III-A); torch's CPU conversion is RNE and keeps
    denormals, so it pins 1/8/7/d including fp32-denormal inputs."""
    import torch
    x = _mixed_inputs(12)
    nan = np.isnan(x)
    ref = torch.from_numpy(x.copy()).to(torch.bfloat16).to(torch.float32).numpy()
    got = oracle.quantize(x, 8, 7, True)
    assert same_bits(got[~nan], ref[~nan])
    assert np.all(np.isnan(got[nan]))


def test_fp32_shape_is_identity():
    """e = 8 with 23 stored bits is IEEE single precision itself (the range remark in
    Sec. III-A), so rounding changes nothing but NaN payloads."""
    x = _mixed_inputs(13)
    nan = np.isnan(x)
    got = oracle.quantize(x, 8, 23, True)
    assert same_bits(got[~nan], x[~nan])
    assert np.all(bits(got[nan]) == 0x7FC00000)


# ---------------------------------------------------------------- brute force

@pytest.mark.parametrize("e,m", [(2, 1), (3, 2), (4, 3), (2, 3)])
@pytest.mark.parametrize("d", [True, False])
def test_tiny_formats_brute_force(e, m, d):
    """Dense grid through the whole range of a tiny format, against the nearest-value search."""
    c = consts(e, m)
    vals = positive_finite_values(e, m)
    knots = np.array([float(v) for v in vals] + [2.0 ** (c["Emax"] + 1)])
    frac = np.arange(8) / 8.0                         # 8 probes per gap, ties included (exact in fp32)
    grid64 = (knots[:-1, None] + (knots[1:] - knots[:-1])[:, None] * frac[None, :]).ravel()
    grid64 = np.concatenate([grid64, knots[-1] * np.array([1.0, 1.25, 4.0])])
    grid = grid64.astype(np.float32)
    assert np.array_equal(grid.astype(np.float64), grid64) and grid.size < 50000
    grid = np.concatenate([grid, -grid, workloads.special_values()])
    got = oracle.quantize(grid, e, m, d)
    for x, g in zip(grid, got):
        want = np.float32(brute_force_round(float(x), e, m, d, vals))
        if np.isnan(want):
            assert np.isnan(g)
        else:
            assert bits([g])[0] == bits([want])[0], (x, g, want)


@pytest.mark.parametrize("e,m,d", VARIANTS)
def test_real_formats_brute_force_sample(e, m, d):
    """A few thousand random and adversarial inputs per real format against the search."""
    rng = np.random.default_rng(100 * e + m)
    c = consts(e, m)
    vals = positive_finite_values(e, m)
    x = np.concatenate([
        workloads.random_bits(1500, 7 * e + m),
        workloads.special_values(),
        workloads.log2_normal(1500, c["Emin"] - m / 2, m, 0.0, rng),     # around the denormal range
        workloads.log2_normal(500, c["Emax"], 1.0, 0.0, rng),           # around overflow
    ])
    got = oracle.quantize(x, e, m, d)
    for xi, g in zip(x, got):
        want = np.float32(brute_force_round(float(xi), e, m, d, vals))
        if np.isnan(want):
            assert np.isnan(g)
        else:
            assert bits([g])[0] == bits([want])[0], (xi, g, want)


# ---------------------------------------------------------------- invariants

@pytest.mark.parametrize("e,m,d", VARIANTS + [(4, 3, True), (7, 16, False), (8, 23, True), (2, 1, True)])
def test_invariants(e, m, d):
    x = _mixed_inputs(1000 + 31 * e + m, n=100000)
    x = x[~np.isnan(x)]
    q = oracle.quantize(x, e, m, d)
    # idempotent
    assert same_bits(oracle.quantize(q, e, m, d), q)
    # odd, signed zeros included
    assert same_bits(oracle.quantize(-x, e, m, d), -q)
    # monotone non-decreasing
    order = np.argsort(x, kind="stable")
    qs = q[order]
    assert np.all(qs[1:] >= qs[:-1])
    # error bound: half a grid step at the input's binade (denormal-allowed rounding, finite results)
    qd = oracle.quantize(x, e, m, True).astype(np.float64)
    c = consts(e, m)
    fin = np.isfinite(qd) & np.isfinite(x) & (x != 0)
    E = np.floor(np.log2(np.abs(x[fin].astype(np.float64))))
    bound = np.exp2(np.maximum(E, c["Emin"]) - m - 1)
    assert np.all(np.abs(qd[fin] - x[fin].astype(np.float64)) <= bound)
    # flushed outputs are a subset of denormal-allowed outputs and differ exactly on denormal results
    qn = oracle.quantize(x, e, m, False)
    differs = bits(qn) != bits(qd.astype(np.float32))
    is_den = (np.abs(qd) > 0) & (np.abs(qd) < 2.0 ** c["Emin"])
    assert np.array_equal(differs, is_den)
    assert np.all(qn[differs] == 0)


def test_rejects_unsupported_formats():
    for e, m in [(1, 5), (9, 7), (5, 0), (5, 24)]:
        with pytest.raises(ValueError):
            oracle.quantize(np.ones(3, np.float32), e, m, True)
