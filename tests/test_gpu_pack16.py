"""GPU parity of fmt_pack16 / fmt_unpack16 / fmt_linear_pack16 (through the C ABI) against the CPU
oracle: codes, values and statistics are integers or exact values -- everything bit for bit."""
import numpy as np
import pytest

import oracle
import workloads

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

VARIANTS = [(5, 10, True), (5, 10, False), (6, 9, True), (6, 9, False), (8, 7, True), (8, 7, False)]
NARROW = [(2, 1, True), (4, 3, False), (3, 12, True), (7, 8, True), (8, 1, False), (2, 13, False)]
EXP_LO = -48


@pytest.fixture(scope="module")
def fmt():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    import paper_2103_15940_amd as lib
    return lib


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def codes_of(t):
    return t.cpu().numpy().view(np.uint16)


def mixed(n, seed):
    rng = np.random.default_rng(seed)
    parts = [workloads.random_bits(n // 3, seed), workloads.log2_normal(n // 3, -14, 6, 0.01, rng)]
    rest = n - sum(p.size for p in parts)
    parts.append(np.resize(workloads.special_values(), rest))
    x = np.concatenate(parts)
    rng.shuffle(x)
    return x


def assert_codes(got, want, what):
    if not np.array_equal(got, want):
        bad = np.flatnonzero(got.ravel() != want.ravel())
        i = bad[0]
        raise AssertionError("%s: %d of %d codes differ; first at %d: got %04x want %04x" %
                             (what, bad.size, got.size, i, got.ravel()[i], want.ravel()[i]))


def assert_hist(fmtlib, hist, want, what):
    h = fmtlib.hist_to_dict(hist)
    for k in fmtlib.CLASS_NAMES:
        assert h[k] == want[k], "%s: class %s got %d want %d" % (what, k, h[k], want[k])
    assert np.array_equal(h["bins"], want["bins"]), what


@pytest.mark.parametrize("e,m,d", VARIANTS + NARROW)
def test_pack_matches_oracle(fmt, e, m, d):
    n = 3 * 4096 * 5 + 1234                                    # several tiles and a ragged tail
    x = mixed(n, 7 + e * 31 + m)
    hist = fmt.new_hist(torch.device("cuda"))
    c = fmt.fmt_pack16(dev(x), (e, m, d), hist=hist, exp_lo=EXP_LO)
    torch.cuda.synchronize()
    assert_codes(codes_of(c), oracle.pack16(x, e, m, d), "pack 1/%d/%d/%s" % (e, m, "d" if d else "n"))
    assert_hist(fmt, hist, oracle.histogram(x, e, m, exp_lo=EXP_LO), "pack statistics")
    c2 = fmt.fmt_pack16(dev(x), (e, m, d))                     # without statistics: another kernel variant
    torch.cuda.synchronize()
    assert np.array_equal(codes_of(c2), codes_of(c))


@pytest.mark.parametrize("e,m", [(5, 10), (6, 9), (8, 7), (2, 1), (4, 3), (3, 12), (7, 8), (2, 13)])
def test_unpack_every_code(fmt, e, m):
    codes = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)      # includes patterns with upper bits set
    y = fmt.fmt_unpack16(dev(codes.view(np.int16)), (e, m, True))
    torch.cuda.synchronize()
    got = y.cpu().numpy().view(np.uint32)
    want = oracle.unpack16(codes, e, m).view(np.uint32)
    assert np.array_equal(got, want)
    # and packing those values gives the codes back (non-NaN, upper bits clear)
    width = 1 + e + m
    clean = codes[: 1 << width] if width < 16 else codes
    v = oracle.unpack16(clean, e, m)
    back = codes_of(fmt.fmt_pack16(dev(v), (e, m, True)))
    ok = ~np.isnan(v)
    assert np.array_equal(back[ok], clean[ok])


def test_binary16_and_bfloat16_are_the_library_types(fmt):
    """1/5/10 codes are IEEE half patterns, 1/8/7 codes are bfloat16 patterns: torch's own casts on
    the GPU give the same bits (NaN aside)."""
    x = mixed(1 << 18, 99)
    xd = dev(x)
    ok = ~np.isnan(x)
    h = codes_of(fmt.fmt_pack16(xd, (5, 10, True)))
    assert np.array_equal(h[ok], xd.to(torch.float16).view(torch.int16).cpu().numpy().view(np.uint16)[ok])
    b = codes_of(fmt.fmt_pack16(xd, (8, 7, True)))
    assert np.array_equal(b[ok], xd.to(torch.bfloat16).view(torch.int16).cpu().numpy().view(np.uint16)[ok])


@pytest.mark.parametrize("off_x,off_c", [(0, 0), (1, 1), (2, 2), (3, 3), (1, 0), (0, 2), (3, 1), (0, 4), (1, 5)])
def test_alignment_and_small_sizes(fmt, off_x, off_c):
    """Every relative alignment of x and the codes (vector body with scalar head and tail, or the
    element-wise path), sizes from 0 up past one tile."""
    f = (6, 9, True)
    for n in [0, 1, 3, 4, 7, 8, 9, 15, 63, 64, 65, 1000, 4096, 4097, 8191 + 4096]:
        x = mixed(n + 16, n + off_x)[:n] if n else np.zeros(0, np.float32)
        xb = torch.zeros(n + 16, dtype=torch.float32, device="cuda")
        cb = torch.full((n + 16,), 0x5555, dtype=torch.int16, device="cuda")
        xb[off_x:off_x + n] = dev(x) if n else xb[off_x:off_x]
        fmt.fmt_pack16(xb[off_x:off_x + n], f, out=cb[off_c:off_c + n])
        torch.cuda.synchronize()
        got = codes_of(cb)
        assert_codes(got[off_c:off_c + n], oracle.pack16(x, *f), "n=%d" % n)
        assert np.all(got[:off_c] == 0x5555) and np.all(got[off_c + n:] == 0x5555), "wrote outside the range"
        # and back
        yb = torch.full((n + 16,), 7.0, dtype=torch.float32, device="cuda")
        fmt.fmt_unpack16(cb[off_c:off_c + n], f, out=yb[off_x:off_x + n])
        torch.cuda.synchronize()
        y = yb.cpu().numpy()
        want = oracle.unpack16(got[off_c:off_c + n], 6, 9)
        assert np.array_equal(y[off_x:off_x + n].view(np.uint32), want.view(np.uint32))
        assert np.all(y[:off_x] == 7.0) and np.all(y[off_x + n:] == 7.0)


def test_errors(fmt):
    x = torch.zeros(8, device="cuda")
    with pytest.raises(fmt.FmtError) as ei:
        fmt.fmt_pack16(x, (8, 8, True))
    assert ei.value.status == -1
    with pytest.raises(fmt.FmtError) as ei:
        fmt.fmt_unpack16(torch.zeros(8, dtype=torch.int16, device="cuda"), (5, 23, True))
    assert ei.value.status == -1


def exact_operands(rng, M, N, K, e, m):
    """Integer operands with a power-of-two scale per output column: the fp32 accumulation is exact
    in any order, so the layer's output is determined bit for bit (as in the fmt_linear tests)."""
    c = oracle.format_constants(e, m)
    lo = max(int(c["Emin"]) - m - 4, -100)
    hi = min(int(c["Emax"]) - 3, 100)
    X = rng.integers(-7, 8, (M, K)).astype(np.float32)
    s = rng.integers(lo, hi + 1, N)
    W = (rng.integers(-7, 8, (N, K)) * np.exp2(s.astype(np.float64))[:, None]).astype(np.float32)
    mid = (c["Emin"] + c["Emax"]) / 2
    b = workloads.log2_normal(N, mid, (c["Emax"] - c["Emin"]) / 3.5, 0.05, rng)
    return X, W, b


@pytest.mark.parametrize("e,m,d", VARIANTS + [(4, 3, True), (7, 8, False)])
@pytest.mark.parametrize("shape", [(65, 1025, 33), (300, 7, 40), (128, 512, 64)])
def test_linear_pack16_bit_exact(fmt, e, m, d, shape):
    M, N, K = shape
    rng = np.random.default_rng(5 + e + 10 * m + M)
    X, W, b = exact_operands(rng, M, N, K, e, m)
    Y, T = oracle.linear(X, W, b, e, m, d)
    hist = fmt.new_hist(torch.device("cuda"))
    C = fmt.fmt_linear_pack16(dev(X), dev(W), dev(b), (e, m, d), hist=hist, exp_lo=EXP_LO)
    torch.cuda.synchronize()
    assert_codes(codes_of(C), oracle.pack16(Y, e, m, True), "linear codes %s" % (shape,))
    assert_hist(fmt, hist, oracle.histogram(T, e, m, exp_lo=EXP_LO), "linear statistics")
    # the fp32 entry point gives the values of those codes
    Yf = fmt.fmt_linear(dev(X), dev(W), dev(b), (e, m, d)).cpu().numpy()
    nan = np.isnan(Yf)
    assert np.array_equal(oracle.unpack16(codes_of(C), e, m).view(np.uint32)[~nan], Yf.view(np.uint32)[~nan])


def test_linear_pack16_strided_output_and_no_bias(fmt):
    rng = np.random.default_rng(3)
    f = (6, 9, True)
    M, N, K = 70, 130, 96
    X, W, _ = exact_operands(rng, M, N, K, 6, 9)
    Y, _ = oracle.linear(X, W, None, *f)
    buf = torch.full((M, N + 6), 0x1234, dtype=torch.int16, device="cuda")
    out = buf[:, 3:3 + N]                                           # ldy = N + 6, 2-byte aligned only
    fmt.fmt_linear_pack16(dev(X), dev(W), None, f, out=out)
    torch.cuda.synchronize()
    got = codes_of(buf)
    assert_codes(got[:, 3:3 + N], oracle.pack16(Y, 6, 9, True), "strided")
    assert np.all(got[:, :3] == 0x1234) and np.all(got[:, 3 + N:] == 0x1234)
    # empty problems
    e0 = fmt.fmt_linear_pack16(torch.zeros((0, K), device="cuda"), dev(W), None, f)
    assert tuple(e0.shape) == (0, N)
    k0 = fmt.fmt_linear_pack16(torch.zeros((4, 0), device="cuda"), torch.zeros((5, 0), device="cuda"),
                               dev(np.array([1.0, -2.0, 0.0, 1e-12, 3e9], np.float32)), f)
    torch.cuda.synchronize()
    assert_codes(codes_of(k0), np.tile(oracle.pack16(np.array([1.0, -2.0, 0.0, 1e-12, 3e9], np.float32), 6, 9, True), (4, 1)),
                 "K = 0: the rounded bias")


def test_full_size_config5_sampled(fmt):
    """The bench's stream size (2^28 elements): codes of 2^20 sampled positions and the full statistics
    against the oracle's own pass over the tensor."""
    n = 1 << 28
    x = np.tile(workloads.config5(n=1 << 24), 16)
    xd = dev(x)
    hist = fmt.new_hist(torch.device("cuda"))
    c = fmt.fmt_pack16(xd, (6, 9, True), hist=hist, exp_lo=EXP_LO)
    torch.cuda.synchronize()
    rng = np.random.default_rng(0)
    idx = np.unique(np.concatenate([rng.integers(0, n, 1 << 20), np.arange(4096), np.arange(n - 4096, n)]))
    got = c[torch.from_numpy(idx).cuda()].cpu().numpy().view(np.uint16)
    assert_codes(got, oracle.pack16(x[idx], 6, 9, True), "sampled codes")
    h16 = oracle.histogram(x[: 1 << 24], 6, 9, exp_lo=EXP_LO)
    h = fmt.hist_to_dict(hist)
    for k in fmt.CLASS_NAMES:
        assert h[k] == 16 * h16[k], k
    assert np.array_equal(h["bins"], 16 * np.asarray(h16["bins"]))
