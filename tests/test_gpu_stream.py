"""GPU parity of fmt_quantize / fmt_histogram (through the C ABI) against the CPU oracle:
bit-exact values, bit-exact integer counts."""
import numpy as np
import pytest

import oracle
import workloads

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

VARIANTS = [(5, 10, True), (5, 10, False), (6, 9, True), (6, 9, False), (8, 7, True), (8, 7, False)]
OTHER = [(2, 1, True), (3, 2, False), (4, 3, True), (7, 16, False), (8, 23, True), (7, 23, True), (5, 23, False),
         (8, 1, False), (2, 22, True)]


@pytest.fixture(scope="module")
def fmt():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    import paper_2103_15940_amd as lib
    return lib


def bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def assert_same_values(got, want, what):
    g, w = bits(got), bits(want)
    if not np.array_equal(g, w):
        bad = np.flatnonzero(g != w)
        i = bad[0]
        raise AssertionError("%s: %d of %d elements differ; first at %d: got %08x want %08x" %
                             (what, bad.size, g.size, i, g[i], w[i]))


def assert_same_hist(fmtlib, hist, want, what):
    h = fmtlib.hist_to_dict(hist)
    for k in fmtlib.CLASS_NAMES:
        assert h[k] == want[k], "%s: class %s got %d want %d" % (what, k, h[k], want[k])
    assert np.array_equal(h["bins"], want["bins"]), "%s: bins differ\n%s\n%s" % (what, h["bins"], want["bins"])


def mixed(n, seed):
    rng = np.random.default_rng(seed)
    parts = [workloads.random_bits(n // 3, seed), workloads.log2_normal(n // 3, -14, 6, 0.01, rng)]
    rest = n - sum(p.size for p in parts)
    sp = workloads.special_values()
    parts.append(np.resize(sp, rest))
    x = np.concatenate(parts)
    rng.shuffle(x)
    return x


@pytest.mark.parametrize("e,m,d", VARIANTS + OTHER)
def test_quantize_and_fused_hist_bit_exact(fmt, e, m, d):
    n = (1 << 18) + 37                      # several workgroups' worth of tiles and a ragged tail
    x = mixed(n, 17 * e + m)
    xd = dev(x)
    hist = fmt.new_hist()
    y = fmt.fmt_quantize(xd, (e, m, d), hist=hist)
    y2 = fmt.fmt_quantize(xd, (e, m, d))   # store-only kernel
    torch.cuda.synchronize()
    want = oracle.quantize(x, e, m, d)
    assert_same_values(y.cpu().numpy(), want, "fused 1/%d/%d/%s" % (e, m, d))
    assert_same_values(y2.cpu().numpy(), want, "plain 1/%d/%d/%s" % (e, m, d))
    assert_same_hist(fmt, hist, oracle.histogram(x, e, m), "fused hist 1/%d/%d" % (e, m))
    h2 = fmt.fmt_histogram(xd, (e, m, d))
    torch.cuda.synchronize()
    assert_same_hist(fmt, h2, oracle.histogram(x, e, m), "hist-only 1/%d/%d" % (e, m))


@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 7, 63, 64, 65, 511, 2048, 2049, 8191, 8192 * 4 + 1, 70001])
def test_ragged_sizes(fmt, n):
    x = mixed(max(n, 8), n)[:n]
    xd = dev(x)
    for (e, m, d) in [(6, 9, True), (5, 10, False), (8, 7, True)]:
        hist = fmt.new_hist()
        y = fmt.fmt_quantize(xd, (e, m, d), hist=hist)
        torch.cuda.synchronize()
        assert_same_values(y.cpu().numpy(), oracle.quantize(x, e, m, d), "n=%d" % n)
        assert_same_hist(fmt, hist, oracle.histogram(x, e, m), "n=%d" % n)


def test_empty_input(fmt):
    xd = torch.empty(0, dtype=torch.float32, device="cuda")
    hist = torch.full((72,), 7, dtype=torch.int64, device="cuda")
    y = fmt.fmt_quantize(xd, (6, 9, True), hist=hist)
    torch.cuda.synchronize()
    assert y.numel() == 0 and int(hist.abs().sum()) == 0
    hist.fill_(5)
    fmt.fmt_histogram(xd, (6, 9, True), hist=hist)
    torch.cuda.synchronize()
    assert int(hist.abs().sum()) == 0


@pytest.mark.parametrize("ox,oy", [(0, 0), (1, 1), (3, 3), (1, 0), (0, 2), (2, 3)])
def test_misaligned_pointers(fmt, ox, oy):
    """Offsets in elements from a 256-byte aligned base: equal offsets take the vector path with a
    scalar head, unequal ones the dword fallback."""
    n = 50003
    x = mixed(n + 8, 5 + ox * 4 + oy)
    xb = dev(x)
    yb = torch.zeros(n + 8, dtype=torch.float32, device="cuda")
    xs, ys = xb[ox:ox + n], yb[oy:oy + n]
    hist = fmt.new_hist()
    fmt.fmt_quantize(xs, (6, 9, False), out=ys, hist=hist)
    h2 = fmt.fmt_histogram(xs, (6, 9, False))
    torch.cuda.synchronize()
    assert_same_values(ys.cpu().numpy(), oracle.quantize(x[ox:ox + n], 6, 9, False), "offsets %d,%d" % (ox, oy))
    want = oracle.histogram(x[ox:ox + n], 6, 9)
    assert_same_hist(fmt, hist, want, "fused")
    assert_same_hist(fmt, h2, want, "hist-only")
    # nothing outside [oy, oy+n) was written
    full = yb.cpu().numpy()
    assert np.all(full[:oy] == 0) and np.all(full[oy + n:] == 0)


def test_in_place(fmt):
    x = mixed(100000, 3)
    xd = dev(x)
    out = fmt.fmt_quantize(xd, (5, 10, True), out=xd)
    torch.cuda.synchronize()
    assert out.data_ptr() == xd.data_ptr()
    assert_same_values(xd.cpu().numpy(), oracle.quantize(x, 5, 10, True), "in place")


@pytest.mark.parametrize("exp_lo", [-192, -160, -149, -127, -126, -48, -24, 0, 64, 128])
def test_histogram_windows(fmt, exp_lo):
    """Windows that reach into the fp32-denormal binades use the per-binade rows."""
    den = (workloads.random_bits(60000, 9).view(np.uint32) & np.uint32(0x807FFFFF)).view(np.float32)   # fp32 denormals
    x = np.concatenate([mixed(60000, exp_lo + 500), den])
    xd = dev(x)
    hist = fmt.fmt_histogram(xd, (8, 7, True), exp_lo=exp_lo)
    h2 = fmt.new_hist()
    y = fmt.fmt_quantize(xd, (8, 7, True), hist=h2, exp_lo=exp_lo)
    torch.cuda.synchronize()
    want = oracle.histogram(x, 8, 7, exp_lo=exp_lo)
    assert_same_hist(fmt, hist, want, "exp_lo=%d" % exp_lo)
    assert_same_hist(fmt, h2, want, "fused exp_lo=%d" % exp_lo)
    assert_same_values(y.cpu().numpy(), oracle.quantize(x, 8, 7, True), "values")


@pytest.mark.parametrize("e,m", [(5, 10), (6, 9), (8, 7)])
def test_exhaustive_codes_and_boundaries(fmt, e, m):
    """Every code of the format, every midpoint between adjacent codes and the fp32 neighbours of
    each midpoint, both signs -- the same probes that pin the oracle, now through the GPU."""
    from fmtdef import decode_codes
    v = decode_codes(e, m)
    pos = v[: 1 << 15].astype(np.float64)
    last = ((1 << e) - 1) << m
    lo, hi = pos[:last].copy(), pos[1:last + 1].copy()
    hi[-1] = 2.0 ** (2 ** (e - 1))
    mid = ((lo + hi) / 2).astype(np.float32)
    probes = np.concatenate([v, mid, np.nextafter(mid, np.float32(0)), np.nextafter(mid, np.float32(np.inf))])
    probes = np.concatenate([probes, -probes])
    xd = dev(probes)
    for d in (True, False):
        hist = fmt.new_hist()
        y = fmt.fmt_quantize(xd, (e, m, d), hist=hist)
        torch.cuda.synchronize()
        got, want = y.cpu().numpy(), oracle.quantize(probes, e, m, d)
        nan = np.isnan(want)
        assert_same_values(got, want, "codes 1/%d/%d/%s" % (e, m, d))
        assert np.all(bits(got[nan]) == 0x7FC00000)
        assert_same_hist(fmt, hist, oracle.histogram(probes, e, m), "codes hist")


def test_config1_full(fmt):
    """Configuration 1: 2^20 values, log2|x| ~ N(-14, 6^2), 1 % zeros, 1/6/9 with denormals and flushed."""
    x = workloads.config1()["x"]
    xd = dev(x)
    ho = oracle.histogram(x, 6, 9)
    for d in (True, False):
        hist = fmt.new_hist()
        y = fmt.fmt_quantize(xd, (6, 9, d), hist=hist)
        torch.cuda.synchronize()
        assert_same_values(y.cpu().numpy(), oracle.quantize(x, 6, 9, d), "config1 d=%s" % d)
        assert_same_hist(fmt, hist, ho, "config1")


def test_config5_reduced_all_variants(fmt):
    """Configuration 5's heavy-tailed tensor at 2^23 elements: all six variants element by element."""
    x = workloads.config5(n=1 << 23)
    xd = dev(x)
    for (e, m, d) in VARIANTS:
        hist = fmt.new_hist()
        y = fmt.fmt_quantize(xd, (e, m, d), hist=hist)
        torch.cuda.synchronize()
        assert_same_values(y.cpu().numpy(), oracle.quantize(x, e, m, d), "config5 1/%d/%d/%s" % (e, m, d))
        assert_same_hist(fmt, hist, oracle.histogram(x, e, m), "config5 hist")


def test_repeated_calls_are_deterministic(fmt):
    x = workloads.config5(n=1 << 22)
    xd = dev(x)
    ref = None
    for _ in range(5):
        hist = fmt.fmt_histogram(xd, (5, 10, True))
        torch.cuda.synchronize()
        h = hist.cpu().numpy()
        if ref is None:
            ref = h
        assert np.array_equal(h, ref)


def test_non_default_stream(fmt):
    x = mixed(300000, 77)
    s = torch.cuda.Stream()
    xd = dev(x)
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        hist = fmt.new_hist()
        y = fmt.fmt_quantize(xd, (6, 9, True), hist=hist, stream=s)
    s.synchronize()
    assert_same_values(y.cpu().numpy(), oracle.quantize(x, 6, 9, True), "side stream")
    assert_same_hist(fmt, hist, oracle.histogram(x, 6, 9), "side stream")


def test_config5_full_size(fmt):
    """Configuration 5 at its full size (2^28 elements, the launch shape bench.py times): the
    integer statistics must equal the oracle's over the whole tensor, and the values are checked
    element by element on a 2^22-element sample made of 64 slices spread over the tensor
    (including its first and last elements)."""
    n = 1 << 28
    x = workloads.config5(n=n)
    xd = dev(x)
    y = torch.empty_like(xd)
    want_hist = oracle.histogram(x, 6, 9)                     # one pass of the oracle over 2^28 elements
    rng = np.random.default_rng(55)
    starts = np.concatenate([[0, n - (1 << 16)], rng.integers(0, n - (1 << 16), 62)])
    for (e, m, d) in [(6, 9, True), (6, 9, False)]:
        hist = fmt.new_hist()
        fmt.fmt_quantize(xd, (e, m, d), out=y, hist=hist)
        torch.cuda.synchronize()
        assert_same_hist(fmt, hist, want_hist, "config5 full 1/%d/%d" % (e, m))
        for s in starts:
            s = int(s)
            got = y[s:s + (1 << 16)].cpu().numpy()
            assert_same_values(got, oracle.quantize(x[s:s + (1 << 16)], e, m, d), "slice at %d" % s)
    # the other formats: statistics must satisfy the format-independent invariants at full size
    for (e, m) in [(5, 10), (8, 7)]:
        h = fmt.hist_to_dict(fmt.fmt_histogram(xd, (e, m, True)))
        assert h["total"] == n == sum(h[k] for k in fmt.CLASS_NAMES[1:])
        assert np.array_equal(h["bins"], want_hist["bins"])
        assert int(h["bins"].sum()) == n - h["zero"] - h["nan"]
        assert h["zero"] == want_hist["zero"] and h["nan"] == want_hist["nan"] and h["inf"] == want_hist["inf"]


def test_more_than_2_to_the_32_elements(fmt):
    """A tensor whose element indices do not fit 32 bits (2^32 + 12293 elements, 16 GiB): the tensor is
    a 2^24-element chunk repeated, so the statistics are 256 times the chunk's plus those of the ragged
    rest, and the values are checked on samples around every power-of-two index boundary and at the
    end.  Fused fp32 pass, statistics-only pass and the 16-bit code pass."""
    chunk_n = 1 << 24
    tail = 3 * 4096 + 5
    n = (1 << 32) + tail
    chunk = mixed(chunk_n, 1234)
    xd = dev(chunk).repeat(257)[:n]
    assert xd.numel() == n
    hc, ht = oracle.histogram(chunk, 6, 9), oracle.histogram(chunk[:tail], 6, 9)
    want = {k: 256 * hc[k] + ht[k] for k in fmt.CLASS_NAMES}
    want["bins"] = 256 * np.asarray(hc["bins"]) + np.asarray(ht["bins"])
    # sample positions: both ends, around 2^31 and 2^32, and random ones
    rng = np.random.default_rng(9)
    near = np.concatenate([np.arange(-2048, 2048) + b for b in (1 << 31, 1 << 32, (1 << 32) - (1 << 24))])
    idx = np.unique(np.concatenate([np.arange(4096), np.arange(n - 4096, n), near, rng.integers(0, n, 1 << 16)]))
    idx_d = torch.from_numpy(idx).cuda()
    src = chunk[idx % chunk_n]
    f = (6, 9, True)

    hist = fmt.new_hist()
    y = torch.empty_like(xd)
    fmt.fmt_quantize(xd, f, out=y, hist=hist)
    torch.cuda.synchronize()
    assert_same_hist(fmt, hist, want, "fused, n > 2^32")
    assert_same_values(y[idx_d].cpu().numpy(), oracle.quantize(src, *f), "sampled values, n > 2^32")
    del y

    assert_same_hist(fmt, fmt.fmt_histogram(xd, f), want, "statistics only, n > 2^32")

    hist = fmt.new_hist()
    c = fmt.fmt_pack16(xd, f, hist=hist)
    torch.cuda.synchronize()
    assert_same_hist(fmt, hist, want, "pack16, n > 2^32")
    got = c[idx_d].cpu().numpy().view(np.uint16)
    assert np.array_equal(got, oracle.pack16(src, *f)), "sampled codes, n > 2^32"
    back = fmt.fmt_unpack16(c, f)
    torch.cuda.synchronize()
    assert_same_values(back[idx_d].cpu().numpy(), oracle.quantize(src, *f), "unpacked values, n > 2^32")


@pytest.mark.parametrize("seed", range(40))
def test_seeded_random_cases(fmt, seed):
    """Format (any 2 <= e <= 8, 1 <= m <= 23, d or n), length, pointer offsets of input and output,
    histogram window and call (fused, values only, statistics only, 16-bit codes, in place) drawn from a
    seeded generator; everything bit for bit against the oracle, and nothing written outside the output."""
    rng = np.random.default_rng(5000 + seed)
    e, m, d = int(rng.integers(2, 9)), int(rng.integers(1, 24)), bool(rng.integers(0, 2))
    n = int(rng.choice([int(rng.integers(0, 64)), int(rng.integers(64, 20000)), int(rng.integers(20000, 400000))]))
    ox, oy = int(rng.integers(0, 4)), int(rng.integers(0, 4))
    exp_lo = int(rng.integers(-192, 129))
    x = mixed(n + 8, seed)[:n] if n else np.zeros(0, np.float32)
    xb = torch.zeros(n + 8, device="cuda")
    xb[ox:ox + n] = dev(x)
    xin = xb[ox:ox + n]
    want_h = oracle.histogram(x, e, m, exp_lo=exp_lo)
    want_y = oracle.quantize(x, e, m, d)
    what = "seed %d: 1/%d/%d/%s n=%d ox=%d oy=%d exp_lo=%d" % (seed, e, m, "d" if d else "n", n, ox, oy, exp_lo)
    kind = seed % 5
    if kind == 0:                                   # fused
        yb = torch.full((n + 8,), 7.0, device="cuda")
        hist = fmt.new_hist()
        fmt.fmt_quantize(xin, (e, m, d), out=yb[oy:oy + n], hist=hist, exp_lo=exp_lo)
        torch.cuda.synchronize()
        got = yb.cpu().numpy()
        assert_same_values(got[oy:oy + n], want_y, what)
        assert np.all(got[:oy] == 7.0) and np.all(got[oy + n:] == 7.0), what
        assert_same_hist(fmt, hist, want_h, what)
    elif kind == 1:                                 # values only
        yb = torch.full((n + 8,), 7.0, device="cuda")
        fmt.fmt_quantize(xin, (e, m, d), out=yb[oy:oy + n])
        torch.cuda.synchronize()
        got = yb.cpu().numpy()
        assert_same_values(got[oy:oy + n], want_y, what)
        assert np.all(got[:oy] == 7.0) and np.all(got[oy + n:] == 7.0), what
    elif kind == 2:                                 # statistics only
        hist = fmt.new_hist()
        fmt.fmt_histogram(xin, (e, m, d), hist=hist, exp_lo=exp_lo)
        torch.cuda.synchronize()
        assert_same_hist(fmt, hist, want_h, what)
        assert_same_values(xb.cpu().numpy()[ox:ox + n], x, what + ": input changed")
    elif kind == 3:                                 # in place, with statistics
        hist = fmt.new_hist()
        fmt.fmt_quantize(xin, (e, m, d), out=xin, hist=hist, exp_lo=exp_lo)
        torch.cuda.synchronize()
        assert_same_values(xb.cpu().numpy()[ox:ox + n], want_y, what)
        assert_same_hist(fmt, hist, want_h, what)
    else:                                           # 16-bit codes where the format has them
        if 1 + e + m > 16:
            e, m = 6, 9
            want_h = oracle.histogram(x, e, m, exp_lo=exp_lo)
        cb = torch.full((n + 8,), 0x5555, dtype=torch.int16, device="cuda")
        hist = fmt.new_hist()
        fmt.fmt_pack16(xin, (e, m, d), out=cb[oy:oy + n], hist=hist, exp_lo=exp_lo)
        torch.cuda.synchronize()
        got = cb.cpu().numpy().view(np.uint16)
        assert np.array_equal(got[oy:oy + n], oracle.pack16(x, e, m, d)), what
        assert np.all(got[:oy] == 0x5555) and np.all(got[oy + n:] == 0x5555), what
        assert_same_hist(fmt, hist, want_h, what)


def test_config2_every_tensor_of_a_step(fmt):
    """Config 2 call by call: one forward + backward step of the 784-1024-1024-10 MLP at batch 256 with
    loss scale 1024; fmt_quantize + statistics of EVERY tensor the step rounds -- the input, the three
    weight matrices, the three layer outputs, the loss-scaled gradient of the logits and the two
    back-propagated gradients (256 x 784 ... 256 x 10) -- against the oracle, bit for bit, in the three
    formats.  The step itself (products, ReLU, softmax) is harness glue in float64 on the host: parity is
    per call on identical inputs."""
    import oracle
    cfg = workloads.config2()
    X, W = cfg["X"], cfg["W"]
    tensors = [("X", X)] + [("W%d" % l, W[l]) for l in range(3)]
    acts = [X.astype(np.float64)]
    for l in range(3):
        z = acts[-1] @ W[l].astype(np.float64).T
        tensors.append(("Y%d" % l, z.astype(np.float32)))
        acts.append(np.maximum(z, 0) if l < 2 else z)
    z = acts[-1]
    p = np.exp(z - z.max(1, keepdims=True))
    p /= p.sum(1, keepdims=True)
    p[np.arange(z.shape[0]), cfg["labels"]] -= 1.0
    g = p / z.shape[0] * cfg["loss_scale"]
    tensors.append(("dY2", g.astype(np.float32)))
    for l in (2, 1):
        g = (g @ W[l].astype(np.float64)) * (acts[l] > 0)
        tensors.append(("dY%d" % (l - 1), g.astype(np.float32)))
    assert {t.shape for _, t in tensors} >= {(256, 784), (1024, 784), (256, 1024), (10, 1024), (256, 10)}
    for e, m, d in [(6, 9, True), (5, 10, True), (8, 7, False)]:
        for name, t in tensors:
            flat = np.ascontiguousarray(t).ravel()
            xd = torch.from_numpy(flat).cuda()
            hist = fmt.new_hist(xd.device)
            y = fmt.fmt_quantize(xd, (e, m, d), hist=hist)
            torch.cuda.synchronize()
            want = oracle.quantize(flat, e, m, d)
            assert np.array_equal(y.cpu().numpy().view(np.uint32), want.view(np.uint32)), (name, e, m, d)
            got, ho = fmt.hist_to_dict(hist), oracle.histogram(flat, e, m)
            assert all(got[k] == ho[k] for k in fmt.CLASS_NAMES), (name, e, m, d, got, ho)
            assert np.array_equal(got["bins"], ho["bins"]), (name, e, m, d)
