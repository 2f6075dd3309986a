"""GPU parity of fmt_linear (quantized fully connected layer, Sec. IV-A) against the CPU oracle.

The layer is Y = R(R(acc) + R(b)) with acc the fp32-accumulated product of the rounded operands.
Given acc everything is fixed bit for bit, so the tests are of two kinds:
 * operands whose products share a common power-of-two quantum per output column and whose sums
   stay below 2^24 quanta: every partial sum is exact in fp32 in ANY order, acc equals the oracle's
   fp64 sum exactly, and Y and the statistics of t must agree bit for bit, end to end;
 * real-valued operands: acc may differ from the fp64 sum in its last fp32 bits, which can move
   R(acc) by one step of the format for a small fraction of the outputs and nothing else.
"""
import numpy as np
import pytest

import oracle
import workloads

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

VARIANTS = [(5, 10, True), (5, 10, False), (6, 9, True), (6, 9, False), (8, 7, True), (8, 7, False)]
EXP_LO = -48


@pytest.fixture(scope="module")
def fmt():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    import paper_2103_15940_amd as lib
    return lib


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def exact_operands(rng, M, N, K, e, m, zero_rows=0.1):
    """X small integers; row j of W small integers times 2^s_j with s_j spread over (and beyond)
    the exponent range of the format: acc[i][j] is an integer multiple of a power of two with
    fewer than 24 bits, exact in fp32 whatever the order of the additions."""
    c = oracle.format_constants(e, m)
    lo = max(int(c["Emin"]) - m - 4, -100)        # stay clear of fp32's own denormals
    hi = min(int(c["Emax"]) - 3, 100)             # 7*2^hi is finite in the format, 49*K*2^hi in fp32
    X = rng.integers(-7, 8, (M, K)).astype(np.float32)
    s = rng.integers(lo, hi + 1, N)
    W = (rng.integers(-7, 8, (N, K)) * np.exp2(s.astype(np.float64))[:, None]).astype(np.float32)
    W[rng.random(N) < zero_rows] = 0.0            # acc = 0: t = R(b), the whole range of the bias
    mid = (c["Emin"] + c["Emax"]) / 2
    b = workloads.log2_normal(N, mid, (c["Emax"] - c["Emin"]) / 3.5, 0.05, rng)
    return X, W, b


def run(fmt, X, W, b, f, want_hist=True, out=None):
    h = fmt.new_hist(torch.device("cuda")) if want_hist else None
    Y = fmt.fmt_linear(dev(X), dev(W), None if b is None else dev(b), f, out=out, hist=h, exp_lo=EXP_LO)
    torch.cuda.synchronize()
    return Y.cpu().numpy(), (fmt.hist_to_dict(h) if want_hist else None)


def hist_of(T, f):
    return oracle.histogram(T, f[0], f[1], exp_lo=EXP_LO)


def assert_bits(got, ref, what):
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan), what + ": NaN positions differ"
    g = np.where(nan, np.float32(0), got).view(np.uint32)
    r = np.where(nan, np.float32(0), ref).view(np.uint32)
    if not np.array_equal(g, r):
        bad = np.argwhere(g != r)
        i, j = bad[0]
        raise AssertionError("%s: %d outputs differ; first at (%d,%d): got %r want %r" %
                             (what, len(bad), i, j, got[i, j], ref[i, j]))


def assert_hist(got, T, f, what):
    ref = hist_of(T, f)
    for k in ("total", "zero", "underflow", "denormal", "normal", "overflow", "inf", "nan"):
        assert int(got[k]) == int(ref[k]), "%s: class %s: got %d want %d" % (what, k, got[k], ref[k])
    assert np.array_equal(np.asarray(got["bins"], dtype=np.int64), np.asarray(ref["bins"], dtype=np.int64)), what


@pytest.mark.parametrize("e,m,d", VARIANTS + [(4, 3, True), (7, 14, False), (8, 23, True)])
def test_bit_exact_end_to_end(fmt, e, m, d):
    rng = np.random.default_rng(1000 * e + m + int(d))
    M, N, K = 203, 1190, 150                     # two column strips, ragged in every direction
    X, W, b = exact_operands(rng, M, N, K, e, m)
    Yo, To = oracle.linear(X, W, b, e, m, d)
    Y, h = run(fmt, X, W, b, (e, m, d))
    assert_bits(Y, Yo, "Y 1/%d/%d/%s" % (e, m, d))
    assert_hist(h, To, (e, m, d), "statistics of t")
    # the classes must be exercised, or the case proves little (t is a sum of two values of the
    # format, hence a multiple of minD: it cannot fall in the underflow class)
    ref = hist_of(To, (e, m, d))
    assert ref["zero"] > 0 and ref["normal"] > 0 and ref["inf"] > 0 and ref["underflow"] == 0
    if e < 8:
        assert ref["overflow"] > 0 and ref["nan"] > 0
        assert ref["denormal"] > 0 or not d


@pytest.mark.parametrize("shape", [(1, 1, 1), (3, 5, 7), (64, 1024, 32), (65, 1025, 33), (300, 7, 40),
                                   (37, 2051, 64), (1000, 130, 16)])
@pytest.mark.parametrize("bias", [True, False])
def test_shapes(fmt, shape, bias):
    M, N, K = shape
    e, m, d = 6, 9, True
    rng = np.random.default_rng(M + 3 * N + 5 * K)
    X, W, b = exact_operands(rng, M, N, K, e, m)
    if not bias:
        b = None
    Yo, To = oracle.linear(X, W, b, e, m, d)
    Y, h = run(fmt, X, W, b, (e, m, d))
    assert_bits(Y, Yo, "shape %r" % (shape,))
    assert_hist(h, To, (e, m, d), "shape %r" % (shape,))
    Y2, _ = run(fmt, X, W, b, (e, m, d), want_hist=False)     # the variant without statistics
    assert_bits(Y2, Yo, "no statistics, shape %r" % (shape,))


def run_prepared(fmt, X, W, b, f, want_hist=True):
    h = fmt.new_hist(torch.device("cuda")) if want_hist else None
    Xp, Wp = fmt.fmt_prepare(dev(X), f), fmt.fmt_prepare(dev(W), f)
    Y = fmt.fmt_linear_prepared(Xp, Wp, None if b is None else dev(b), hist=h, exp_lo=EXP_LO)
    torch.cuda.synchronize()
    return Y.cpu().numpy(), (fmt.hist_to_dict(h) if want_hist else None)


@pytest.mark.parametrize("e,m,d", VARIANTS + [(4, 3, True), (7, 14, False)])
def test_prepared_operands_bit_exact_end_to_end(fmt, e, m, d):
    """fmt_linear_prepared (the layer on operands rounded once with fmt_prepare) against the oracle, on
    operands whose partial sums are exact: output and statistics bit for bit, with and without bias."""
    rng = np.random.default_rng(2000 * e + m + int(d))
    for (M, N, K), bias in (((203, 1190, 150), True), ((65, 1025, 33), False), ((300, 7, 40), True)):
        X, W, b = exact_operands(rng, M, N, K, e, m)
        if not bias:
            b = None
        Yo, To = oracle.linear(X, W, b, e, m, d)
        Y, h = run_prepared(fmt, X, W, b, (e, m, d))
        assert_bits(Y, Yo, "Y 1/%d/%d/%s %r" % (e, m, d, (M, N, K)))
        assert_hist(h, To, (e, m, d), "statistics of t")
        Y2, _ = run_prepared(fmt, X, W, b, (e, m, d), want_hist=False)
        assert_bits(Y2, Yo, "no statistics")


def test_prepared_operands_config4_layer_equals_fmt_linear(fmt):
    """A config 4 layer (4096 tokens, 1024 -> 1024) through fmt_linear_prepared and through fmt_linear: the same
    product kernels on the same prepared planes, so the same bits and the same statistics."""
    L = workloads.config4()["layers"][1]
    f = (6, 9, True)
    X, W = dev(L["X"]), dev(L["W"])
    b = dev(np.random.default_rng(3).standard_normal(W.shape[0]).astype(np.float32) * 0.1)
    h1, h2 = fmt.new_hist(torch.device("cuda")), fmt.new_hist(torch.device("cuda"))
    Y1 = fmt.fmt_linear(X, W, b, f, hist=h1, exp_lo=EXP_LO)
    Y2 = fmt.fmt_linear_prepared(fmt.fmt_prepare(X, f), fmt.fmt_prepare(W, f), b, hist=h2, exp_lo=EXP_LO)
    torch.cuda.synchronize()
    assert torch.equal(Y1.view(torch.int32), Y2.view(torch.int32))
    assert torch.equal(h1, h2)


def test_strided_and_unaligned_output(fmt):
    """Leading dimensions larger than the rows, an output that is not 16-byte aligned and one whose
    leading dimension is odd (scalar accesses); the padding must stay untouched."""
    e, m, d = 5, 10, False
    rng = np.random.default_rng(77)
    M, N, K = 90, 333, 48
    X, W, b = exact_operands(rng, M, N, K, e, m)
    Yo, To = oracle.linear(X, W, b, e, m, d)
    Xp = torch.zeros((M, K + 5), dtype=torch.float32, device="cuda")
    Xp[:, :K] = dev(X)
    Wp = torch.zeros((N, K + 3), dtype=torch.float32, device="cuda")
    Wp[:, :K] = dev(W)
    for ldy, off in ((N + 7, 0), (N + 3, 1), (336, 0), (336, 3)):
        buf = torch.full((M * ldy + 8,), -7.5, dtype=torch.float32, device="cuda")
        out = buf[off:off + M * ldy].view(M, ldy)[:, :N]
        h = fmt.new_hist(torch.device("cuda"))
        fmt.fmt_linear(Xp[:, :K], Wp[:, :K], dev(b), (e, m, d), out=out, hist=h, exp_lo=EXP_LO)
        torch.cuda.synchronize()
        assert_bits(out.cpu().numpy(), Yo, "ldy %d offset %d" % (ldy, off))
        assert_hist(fmt.hist_to_dict(h), To, (e, m, d), "ldy %d offset %d" % (ldy, off))
        whole = buf.cpu().numpy()
        mask = np.ones(whole.size, dtype=bool)
        idx = off + (np.arange(M)[:, None] * ldy + np.arange(N)[None, :])
        mask[idx.ravel()] = False
        assert np.all(whole[mask] == np.float32(-7.5)), "padding overwritten"


def test_degenerate_sizes(fmt):
    f = (6, 9, True)
    cuda = torch.device("cuda")
    # K = 0: t = R(b) in every row
    b = np.array([1.0, -2.5, 3e-12, 1e12, 0.0, 1.0000001], dtype=np.float32)
    X = torch.empty((4, 0), dtype=torch.float32, device=cuda)
    W = torch.empty((6, 0), dtype=torch.float32, device=cuda)
    h = fmt.new_hist(cuda)
    Y = fmt.fmt_linear(X, W, dev(b), f, hist=h, exp_lo=EXP_LO)
    torch.cuda.synchronize()
    Yo, To = oracle.linear_epilogue(np.zeros((4, 6), dtype=np.float32), b, *f)
    assert_bits(Y.cpu().numpy(), Yo, "K = 0")
    assert_hist(fmt.hist_to_dict(h), To, f, "K = 0")
    # M = 0 and N = 0: nothing to do, the statistics are all zero
    for M, N in ((0, 5), (5, 0), (0, 0)):
        h = fmt.new_hist(cuda)
        h.fill_(-1)
        Y = fmt.fmt_linear(torch.empty((M, 3), dtype=torch.float32, device=cuda),
                           torch.empty((N, 3), dtype=torch.float32, device=cuda), None, f, hist=h)
        torch.cuda.synchronize()
        assert tuple(Y.shape) == (M, N)
        assert int(h.abs().sum().item()) == 0


def test_special_values(fmt):
    """Infinite and NaN sums: inf + (-inf) in the bias addition, overflowing accumulators."""
    f = (5, 10, True)
    X = np.array([[256.0, 0.0], [0.0, 256.0], [256.0, 256.0]], dtype=np.float32)
    W = np.array([[256.0, 0.0], [0.0, -256.0], [1.0, 1.0], [2.0 ** -25, 0.0]], dtype=np.float32)   # [out, in]
    b = np.array([-np.inf, np.inf, np.nan, 1.0], dtype=np.float32)
    # acc = [[65536, 0, 256, 2^-17], [0, -65536, 256, 0], [65536, -65536, 512, 2^-17]]: finite in fp32,
    # +-65536 rounds to +-infinity in binary16
    Yo, To = oracle.linear(X, W, b, *f)
    Y, h = run(fmt, X, W, b, f)
    assert_bits(Y, Yo, "special values")
    assert_hist(h, To, f, "special values")


@pytest.mark.parametrize("e,m,d", VARIANTS)
def test_real_operands_within_one_step(fmt, e, m, d):
    """MLP-shaped layer (784 -> 1024, batch 256; inputs U[0,1), Kaiming-normal weights): fp32
    accumulation differs from the fp64 sum by a few units of 2^-24 relative, which moves the
    rounding of acc by one step of the format for a small fraction of outputs, and never by more."""
    rng = np.random.default_rng(31 * e + m)
    M, N, K = 256, 1024, 784
    X = rng.random((M, K), dtype=np.float32)
    W = (rng.standard_normal((N, K)) * np.sqrt(2.0 / K)).astype(np.float32)
    b = (rng.standard_normal(N) * 0.1).astype(np.float32)
    Yo, To = oracle.linear(X, W, b, e, m, d)
    Y, h = run(fmt, X, W, b, (e, m, d))
    c = oracle.format_constants(e, m)
    def step_at(v):
        mag = np.maximum(np.abs(v.astype(np.float64)), float(c["minN"]))
        return np.exp2(np.floor(np.log2(mag)) - m)

    # R(acc) moves to a neighbouring value of the format at most (spacing at acc, twice that across
    # a binade boundary); the last rounding is monotone and adds at most one step at the result
    acc = oracle.gemm(X, W, e, m, d, transB=True)
    bound = 2 * step_at(acc) + 2 * step_at(Yo)
    diff = np.abs(Y.astype(np.float64) - Yo.astype(np.float64))
    assert np.all(diff <= bound * (1 + 1e-12)), "an output is further from the fp64-accumulated layer than one step"
    frac = np.count_nonzero(Y != Yo) / Y.size
    assert frac < 0.03, "too many outputs differ from the fp64-accumulated layer: %.4f" % frac
    assert np.array_equal(oracle.quantize(Y, e, m, d).view(np.uint32), Y.view(np.uint32))   # values of the format
    ref = hist_of(To, (e, m, d))
    assert int(h["total"]) == M * N == int(ref["total"])
    # an output that moved changes one class count and two bins of t at most; t may also move where
    # the last rounding hides it, so the bound is the same small fraction of the tensor
    slack = int(0.03 * M * N)
    for k in ("zero", "underflow", "denormal", "normal", "overflow", "inf", "nan"):
        assert abs(int(h[k]) - int(ref[k])) <= slack
    assert int(np.sum(np.abs(np.asarray(h["bins"], dtype=np.int64) - np.asarray(ref["bins"], dtype=np.int64)))) <= 2 * slack


def test_mlp_forward_config2(fmt):
    """The three layers of the 784-1024-1024-10 MLP at batch 256, chained on the GPU with ReLU
    between them; integer-valued operands make every layer exact, so the whole forward pass
    must match the oracle bit for bit."""
    e, m, d = 6, 9, True
    rng = np.random.default_rng(2)
    sizes = [784, 1024, 1024, 10]
    A = rng.integers(0, 4, (256, sizes[0])).astype(np.float32)
    A_ref = A.copy()
    act = dev(A)
    quantum = 1.0                                          # every activation is a multiple of it
    for li in range(3):
        W = (rng.integers(-3, 4, (sizes[li + 1], sizes[li])) * 2.0 ** -6).astype(np.float32)
        W[rng.random(W.shape) < 0.7] = 0.0                 # keep the sums small enough to stay exact
        b = (rng.integers(-8, 9, sizes[li + 1]) * 2.0 ** -4).astype(np.float32)
        quantum *= 2.0 ** -6
        # exactness in any order: the sum of the magnitudes of the products stays below 2^24 quanta
        assert (np.abs(A_ref).astype(np.float64) @ np.abs(W.T).astype(np.float64)).max() < 2.0 ** 24 * quantum
        Yo, To = oracle.linear(A_ref, W, b, e, m, d)
        h = fmt.new_hist(torch.device("cuda"))
        Y = fmt.fmt_linear(act, dev(W), dev(b), (e, m, d), hist=h, exp_lo=EXP_LO)
        torch.cuda.synchronize()
        assert_bits(Y.cpu().numpy(), Yo, "layer %d" % li)
        assert_hist(fmt.hist_to_dict(h), To, (e, m, d), "layer %d" % li)
        A_ref = np.maximum(Yo, 0)
        act = torch.clamp_min(Y, 0)


def test_config4_full_size_sampled(fmt):
    """Configuration 4's QKV layer (4096 tokens, 1024 -> 3072) at full size, the shape bench.py times
    (the product goes through the single scaled fp16 piece): 4000 sampled outputs of fmt_linear and of
    fmt_linear_pack16 against the oracle's fp64-accumulated layer, each within one step of the format
    as in the test above; the statistics cover all M*N values."""
    e, m, d = 6, 9, True
    layer = workloads.config4()["layers"][0]
    X, W = layer["X"], layer["W"]
    M, K = X.shape
    N = W.shape[0]
    rng = np.random.default_rng(44)
    b = (rng.standard_normal(N) * 0.05).astype(np.float32)
    rows, cols = rng.integers(0, M, 4000), rng.integers(0, N, 4000)
    acc = oracle.gemm_sampled(X, W, rows, cols, e, m, d, transB=True)
    Yo, _ = oracle.linear_epilogue(acc[None, :], b[cols], e, m, d)
    Yo = Yo[0]
    h = fmt.new_hist(torch.device("cuda"))
    Xd, Wd, bd = dev(X), dev(W), dev(b)
    Y = fmt.fmt_linear(Xd, Wd, bd, (e, m, d), hist=h, exp_lo=EXP_LO)
    C = fmt.fmt_linear_pack16(Xd, Wd, bd, (e, m, d))
    torch.cuda.synchronize()
    Yh = Y.cpu().numpy()
    got = Yh[rows, cols]
    c = oracle.format_constants(e, m)

    def step_at(v):
        mag = np.maximum(np.abs(v.astype(np.float64)), float(c["minN"]))
        return np.exp2(np.floor(np.log2(mag)) - m)

    bound = 2 * step_at(acc) + 2 * step_at(Yo)
    diff = np.abs(got.astype(np.float64) - Yo.astype(np.float64))
    assert np.all(diff <= bound * (1 + 1e-12))
    assert np.count_nonzero(got != Yo) / got.size < 0.03
    # every output is a value of the format, and the packed entry point stores exactly its code
    assert np.array_equal(oracle.quantize(Yh, e, m, d).view(np.uint32), Yh.view(np.uint32))
    assert np.array_equal(C.cpu().numpy().view(np.uint16), oracle.pack16(Yh, e, m, True))
    hd = fmt.hist_to_dict(h)
    assert int(hd["total"]) == M * N
    assert sum(int(hd[k]) for k in ("zero", "underflow", "denormal", "normal", "overflow", "inf", "nan")) == M * N


def test_output_of_more_than_2_to_the_32_elements(fmt):
    """Y is 65600 x 65600 (16 GiB; element offsets beyond 32 bits) with K = 64, exact operands: sampled
    rows (first, last, around the 2^31- and 2^32-element offsets, random) bit for bit against the oracle,
    for the fp32 output and for the 16-bit codes; the statistics count every output once."""
    M = N = 65600
    K = 64
    f = (6, 9, True)
    rng = np.random.default_rng(77)
    X, W, b = exact_operands(rng, M, N, K, 6, 9)
    Xd, Wd, bd = dev(X), dev(W), dev(b)
    edge = [(1 << 31) // N, (1 << 32) // N]
    rows = np.unique(np.concatenate([np.arange(4), np.arange(M - 4, M), rng.integers(0, M, 24)] +
                                    [np.arange(r - 2, r + 3) for r in edge]))
    rows_d = torch.from_numpy(rows).cuda()
    Yref, _ = oracle.linear(X[rows], W, b, *f)
    hist = fmt.new_hist(torch.device("cuda"))
    Y = fmt.fmt_linear(Xd, Wd, bd, f, hist=hist, exp_lo=EXP_LO)
    torch.cuda.synchronize()
    assert_bits(Y[rows_d].cpu().numpy(), Yref, "fp32 output, M*N > 2^32")
    h = fmt.hist_to_dict(hist)
    assert h["total"] == M * N == sum(h[k] for k in fmt.CLASS_NAMES[1:])
    del Y
    C = fmt.fmt_linear_pack16(Xd, Wd, bd, f)
    torch.cuda.synchronize()
    got = C[rows_d].cpu().numpy().view(np.uint16)
    assert np.array_equal(got, oracle.pack16(Yref, 6, 9, True)), "16-bit codes, M*N > 2^32"
