"""GPU parity of fmt_gemm_fmac8 (Sec. IV-A, Algorithm 1) against the CPU oracle: the order of the
roundings is fixed by the algorithm, so the results must be identical bit for bit."""
import numpy as np
import pytest

import oracle
import workloads

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

VARIANTS = [(5, 10, True), (5, 10, False), (6, 9, True), (6, 9, False), (8, 7, True), (8, 7, False)]
LAYOUTS = [(False, False), (False, True), (True, False), (True, True)]


@pytest.fixture(scope="module")
def fmt():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    import paper_2103_15940_amd as lib
    return lib


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def run(fmt, A, B, f, tA=False, tB=False):
    Ain = np.ascontiguousarray(A.T) if tA else A
    Bin = np.ascontiguousarray(B.T) if tB else B
    C = fmt.fmt_gemm_fmac8(dev(Ain), dev(Bin), f, transA=tA, transB=tB)
    torch.cuda.synchronize()
    ref = oracle.gemm_fmac8(Ain, Bin, f[0], f[1], f[2], transA=tA, transB=tB)
    return C.cpu().numpy(), ref


def assert_bits(got, ref, what):
    g, r = got.view(np.uint32), ref.view(np.uint32)
    if not np.array_equal(g, r):
        bad = np.argwhere(g != r)
        i, j = bad[0]
        raise AssertionError("%s: %d outputs differ; first at (%d,%d): got %r want %r" %
                             (what, len(bad), i, j, got[i, j], ref[i, j]))


@pytest.mark.parametrize("tA,tB", LAYOUTS)
@pytest.mark.parametrize("e,m,d", VARIANTS)
def test_bit_exact_random(fmt, e, m, d, tA, tB):
    rng = np.random.default_rng(100 * e + m)
    M, N, K = 150, 70, 203                # ragged tiles; K not a multiple of 8 or of the stage
    A = rng.standard_normal((M, K)).astype(np.float32)
    B = (rng.standard_normal((K, N)) * 2.0 ** -3).astype(np.float32)
    got, ref = run(fmt, A, B, (e, m, d), tA, tB)
    assert_bits(got, ref, "1/%d/%d/%s" % (e, m, d))
    # results are values of the format
    assert np.array_equal(oracle.quantize(got, e, m, d).view(np.uint32), got.view(np.uint32))


@pytest.mark.parametrize("e,m,d", VARIANTS + [(4, 3, True), (7, 14, False), (3, 5, True), (6, 11, True), (6, 11, False),
                                             (2, 11, True), (6, 12, True), (7, 9, True)])
def test_bit_exact_wide_range(fmt, e, m, d):
    """Operands spread over the whole range of the format: accumulator and product exponents far
    apart (the sticky-bit cases), denormal and flushed accumulators, overflowing accumulators."""
    rng = np.random.default_rng(7 * e + m)
    c = oracle.format_constants(e, m)
    span = c["Emax"] - c["Emin"]
    A = workloads.log2_normal((90, 130), (c["Emin"] + c["Emax"]) / 4, span / 6, 0.05, rng)
    B = workloads.log2_normal((130, 75), (c["Emin"] + c["Emax"]) / 4, span / 6, 0.05, rng)
    got, ref = run(fmt, A, B, (e, m, d), False, True)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert_bits(np.where(nan, 0, got).astype(np.float32), np.where(nan, 0, ref).astype(np.float32), "wide range")


@pytest.mark.parametrize("e,m,d", [(5, 10, True), (6, 9, True), (6, 9, False), (6, 11, True)])
def test_single_and_double_precision_steps_agree(fmt, e, m, d, monkeypatch):
    """Formats with e <= 6 and m <= 11 run the fused step in single precision; forced onto the
    double-precision step they must give the same bits (and both equal the oracle)."""
    rng = np.random.default_rng(e + m)
    c = oracle.format_constants(e, m)
    span = c["Emax"] - c["Emin"]
    A = workloads.log2_normal((70, 96), (c["Emin"] + c["Emax"]) / 4, span / 5, 0.05, rng)
    B = workloads.log2_normal((96, 66), (c["Emin"] + c["Emax"]) / 4, span / 5, 0.05, rng)
    fast, ref = run(fmt, A, B, (e, m, d))
    monkeypatch.setenv("FMT_FMAC8_F64", "1")
    slow, _ = run(fmt, A, B, (e, m, d))
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(fast), nan) and np.array_equal(np.isnan(slow), nan)
    assert np.array_equal(fast[~nan].view(np.uint32), slow[~nan].view(np.uint32))
    assert np.array_equal(fast[~nan].view(np.uint32), ref[~nan].view(np.uint32))


@pytest.mark.parametrize("shape", [(1, 1, 1), (3, 5, 7), (64, 64, 8), (65, 63, 9), (10, 300, 40), (200, 17, 1000)])
def test_shapes(fmt, shape):
    M, N, K = shape
    rng = np.random.default_rng(M + 3 * N + 5 * K)
    A = rng.standard_normal((M, K)).astype(np.float32)
    B = rng.standard_normal((K, N)).astype(np.float32)
    got, ref = run(fmt, A, B, (6, 9, True))
    assert_bits(got, ref, str(shape))


def test_k_zero_and_nonfinite(fmt):
    C = fmt.fmt_gemm_fmac8(torch.empty((4, 0), device="cuda"), torch.empty((0, 6), device="cuda"), (6, 9, True))
    torch.cuda.synchronize()
    assert float(C.abs().sum()) == 0.0
    rng = np.random.default_rng(3)
    A = rng.standard_normal((20, 24)).astype(np.float32)
    B = rng.standard_normal((24, 20)).astype(np.float32)
    A[2, 3] = np.inf
    A[5, 7] = np.nan
    B[1, 4] = 1e30                     # overflows binary16
    got, ref = run(fmt, A, B, (5, 10, True))
    assert np.array_equal(np.isnan(got), np.isnan(ref))
    fin = ~np.isnan(ref)
    assert np.array_equal(got[fin].view(np.uint32), ref[fin].view(np.uint32))


def test_mlp_layer_shapes(fmt):
    """Configuration 2's first layer (256 x 784 -> 1024) forward with FMAC-8 in 1/6/9 and binary16."""
    cfg = workloads.config2()
    for f in [(6, 9, True), (5, 10, True)]:
        got, ref = run(fmt, cfg["X"], cfg["W"][0].T.copy(), f)
        assert_bits(got, ref, "mlp layer 1 %s" % (f,))


@pytest.mark.parametrize("f", [(6, 9, True), (5, 10, False)])
def test_bench_size_sampled(fmt, f):
    """The size the bench times (2048 x 2048 x 1024): every output is its own chain of K fused steps,
    so the oracle run on 48 sampled rows of A and 48 sampled columns of B gives those 48 x 48 outputs."""
    M, N, K = 2048, 2048, 1024
    rng = np.random.default_rng(17)
    A = rng.standard_normal((M, K)).astype(np.float32)
    B = (rng.standard_normal((K, N)) * 0.02).astype(np.float32)
    C = fmt.fmt_gemm_fmac8(dev(A), dev(B), f)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([rng.integers(0, M, 44), [0, 1, M - 2, M - 1]]))
    cols = np.unique(np.concatenate([rng.integers(0, N, 44), [0, 1, N - 2, N - 1]]))
    ref = oracle.gemm_fmac8(np.ascontiguousarray(A[rows]), np.ascontiguousarray(B[:, cols]), f[0], f[1], f[2])
    got = C.cpu().numpy()[np.ix_(rows, cols)]
    assert_bits(np.ascontiguousarray(got), ref, "sampled %s" % (f,))


def test_operand_of_more_than_2_to_the_32_elements(fmt):
    """A is (2^22 + 70) x 1024 (16 GiB), B 1024 x 8: sampled rows bit for bit against the oracle."""
    M, K, N = (1 << 22) + 70, 1024, 8
    f = (6, 9, True)
    g = torch.Generator(device="cuda")
    g.manual_seed(3)
    A = torch.randn((M, K), device="cuda", generator=g)
    B = torch.randn((K, N), device="cuda", generator=g) * 0.05
    C = fmt.fmt_gemm_fmac8(A, B, f)
    torch.cuda.synchronize()
    rng = np.random.default_rng(4)
    edge = [(1 << 31) // K, (1 << 32) // K]
    rows = np.unique(np.concatenate([np.arange(8), np.arange(M - 72, M), rng.integers(0, M, 60)] +
                                    [np.arange(r - 4, r + 4) for r in edge]))
    rows_d = torch.from_numpy(rows).cuda()
    ref = oracle.gemm_fmac8(A[rows_d].cpu().numpy(), B.cpu().numpy(), *f)
    assert_bits(C[rows_d].cpu().numpy(), ref, "sampled rows, M*K > 2^32")


@pytest.mark.parametrize("e,m,d", VARIANTS + [(7, 8, True), (7, 8, False), (4, 3, True)])
def test_against_the_plain_definition(fmt, e, m, d):
    """fmt_gemm_fmac8 compared directly with Algorithm 1 run in exact rational arithmetic
    (oracle/fmac_exact.py: the sum a + w*x as a Fraction, rounded once by a search over the enumerated
    value set) -- no fp64 construction in between.  Operands span the whole exponent range of the
    format, so accumulator and product are often far apart; 1/8/7 and 1/7/8 take the kernel's
    double-precision step, the others its single-precision one.  Small: the definition is slow."""
    from oracle import fmac_exact
    rng = np.random.default_rng(1000 + 10 * e + m + int(d))
    c = oracle.format_constants(e, m)
    span = c["Emax"] - c["Emin"]
    M, N, K = 16, 16, 40
    # two recipes: products mostly inside the range (accumulators wander through the denormal range and
    # far-apart exponents), and products that often overflow the accumulator or the final rounding
    for centre, sigma, min_finite in [(-span / 8, span / 6, M * N * 3 // 4), ((c["Emin"] + c["Emax"]) / 4, span / 5, 8)]:
        A = workloads.log2_normal((M, K), centre, sigma, 0.05, rng)
        B = workloads.log2_normal((K, N), centre, sigma, 0.05, rng)
        want = fmac_exact.gemm_fmac8(A, B, e, m, d)
        assert np.isfinite(want).sum() >= min_finite        # the case is not degenerate
        for tA, tB in LAYOUTS if (e, m, d) == (6, 9, True) else [(False, False)]:
            Ain = np.ascontiguousarray(A.T) if tA else A
            Bin = np.ascontiguousarray(B.T) if tB else B
            got = fmt.fmt_gemm_fmac8(dev(Ain), dev(Bin), (e, m, d), transA=tA, transB=tB)
            torch.cuda.synchronize()
            got = got.cpu().numpy()
            nan = np.isnan(want)
            assert np.array_equal(np.isnan(got), nan)
            assert_bits(np.where(nan, 0, got).astype(np.float32), np.where(nan, 0, want).astype(np.float32),
                        "definition, 1/%d/%d/%s layout %s" % (e, m, d, (tA, tB)))
