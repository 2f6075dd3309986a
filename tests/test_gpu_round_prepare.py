"""GPU parity of fmt_quantize_prepare_pair_batch: the rounding pass of Sec. IV-A over several tensors in one call --
the rounded fp32 copy and the statistics of Sec. V (what fmt_quantize gives) together with both prepared
orientations (what fmt_prepare_pair_batch gives), from one read of every tensor.  Rounded values and statistics
are compared bit for bit / count for count with the CPU oracle, the operands through the products they give
(bit-identical to those of fmt_prepare_pair_batch's operands, which have their own oracle tests, and within the
1e-5 relative Frobenius bound of the oracle's product); ragged, strided, unaligned and in-place tensors, windows
that reach below 2^-126, more tensors than one launch holds, repeated calls, and the argument errors."""
import numpy as np
import pytest

import oracle
import workloads

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

TOL = 1e-5
SHAPES = [(190, 260), (1, 1), (128, 32), (129, 33), (300, 1000), (64, 96), (512, 384), (5, 70), (33, 1), (1, 257)]


@pytest.fixture(scope="module")
def fmt():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    import paper_2103_15940_amd as lib
    return lib


@pytest.fixture(autouse=True)
def default_plans(monkeypatch):
    monkeypatch.delenv("FMT_GEMM_PLAN", raising=False)
    monkeypatch.delenv("FMT_GEMM_GROUP_TILE", raising=False)
    monkeypatch.delenv("FMT_GEMM_WINDOW", raising=False)


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def rel_err(got, ref):
    return float(np.linalg.norm(got.astype(np.float64) - ref.astype(np.float64)) /
                 max(np.linalg.norm(ref.astype(np.float64)), 1e-300))


def same_hist(fmtlib, hist, want):
    h = fmtlib.hist_to_dict(hist)
    return all(h[k] == want[k] for k in fmtlib.CLASS_NAMES) and np.array_equal(h["bins"], want["bins"])


def mixed_matrix(r, c, seed):
    """Every kind of fp32 pattern (random bits: NaN, infinities, fp32 denormals), a log-normal bulk and the
    special values, shuffled."""
    n = r * c
    rng = np.random.default_rng(seed)
    parts = [workloads.random_bits(n // 3, seed), workloads.log2_normal(n // 3, -14, 6, 0.01, rng)]
    rest = n - sum(p.size for p in parts)
    parts.append(np.resize(workloads.special_values(), rest))
    x = np.concatenate(parts)
    rng.shuffle(x)
    return x.reshape(r, c)


def wide_matrix(rng, f, r, c):
    k = oracle.format_constants(f[0], f[1])
    lo = max(k["Emin"] - f[1] - 2, -60)
    e = rng.integers(lo, lo + 40, (r, c))
    e[rng.random((r, c)) < 0.9] = lo + 30
    return (rng.standard_normal((r, c)) * np.exp2(e.astype(np.float64))).astype(np.float32)


def gram_products(fmt, ops):
    out = []
    for op, op_t in ops:
        out.append(fmt.fmt_gemm_prepared(op, op))
        out.append(fmt.fmt_gemm_prepared(op_t, op_t))
    return out


@pytest.mark.parametrize("exp_lo", [-48, -140])
@pytest.mark.parametrize("f", [(6, 9, True), (6, 9, False), (6, 8, True)])
def test_rounded_copy_and_statistics_match_the_oracle(fmt, f, exp_lo):
    xs = [mixed_matrix(r, c, 100 * i + f[1]) for i, (r, c) in enumerate(SHAPES)]
    dx = [dev(x) for x in xs]
    ys = [torch.full_like(x, 7.0) for x in dx]
    hs = [fmt.new_hist() for _ in dx]
    fmt.fmt_quantize_prepare_pair_batch(dx, f, ys, hs, exp_lo=exp_lo)
    torch.cuda.synchronize()
    for i, (x, y, h) in enumerate(zip(xs, ys, hs)):
        assert np.array_equal(bits(y.cpu().numpy()), bits(oracle.quantize(x, f[0], f[1], f[2]))), (i, x.shape)
        assert same_hist(fmt, h, oracle.histogram(x, f[0], f[1], exp_lo)), (i, x.shape)


@pytest.mark.parametrize("f", [(6, 9, True), (6, 8, False)])
def test_operands_equal_those_of_the_prepare_call(fmt, f):
    rng = np.random.default_rng(500 + f[1])
    xs = [wide_matrix(rng, f, r, c) for r, c in SHAPES]
    dx = [dev(x) for x in xs]
    ys = [torch.empty_like(x) for x in dx]
    hs = [fmt.new_hist() for _ in dx]
    ops = fmt.fmt_quantize_prepare_pair_batch(dx, f, ys, hs)
    ref = fmt.fmt_prepare_pair_batch(dx, f)
    got, want = gram_products(fmt, ops), gram_products(fmt, ref)
    torch.cuda.synchronize()
    for i, (g, w) in enumerate(zip(got, want)):
        assert torch.equal(g, w), i
    for i, x in enumerate(xs):
        assert rel_err(got[2 * i].cpu().numpy(), oracle.gemm(x, x, f[0], f[1], f[2], transB=True)) <= TOL, i
        assert rel_err(got[2 * i + 1].cpu().numpy(), oracle.gemm(x, x, f[0], f[1], f[2], transA=True)) <= TOL, i
        assert np.array_equal(bits(ys[i].cpu().numpy()), bits(oracle.quantize(x, f[0], f[1], f[2]))), i
        assert same_hist(fmt, hs[i], oracle.histogram(x, f[0], f[1], -48)), i


def test_forty_tensors_strided_unaligned_and_in_place(fmt):
    """More tensors than one launch holds (16); inputs and rounded copies that are views with a leading dimension
    beyond their columns and a base that is not 16-byte aligned; every fourth tensor rounded in place."""
    f = (6, 9, True)
    rng = np.random.default_rng(78)
    xs, dx, ys = [], [], []
    for i in range(40):
        r, c = int(rng.integers(1, 200)), int(rng.integers(1, 300))
        x = wide_matrix(rng, f, r, c)
        x[rng.random((r, c)) < 0.02] = 0.0
        xs.append(x)
        if i % 3 == 1:
            pad = torch.zeros(r, c + 5, device="cuda")
            pad[:, 1:c + 1] = dev(x)
            dx.append(pad[:, 1:c + 1])
        else:
            dx.append(dev(x))
        if i % 4 == 0:
            ys.append(dx[-1])
        elif i % 4 == 1:
            ys.append(torch.zeros(r, c + 3, device="cuda")[:, 3:])
        else:
            ys.append(torch.empty(r, c, device="cuda"))
    ref = fmt.fmt_prepare_pair_batch(dx, f)
    want = gram_products(fmt, ref)
    hs = [fmt.new_hist() for _ in dx]
    ops = fmt.fmt_quantize_prepare_pair_batch(dx, f, ys, hs)
    got = gram_products(fmt, ops)
    torch.cuda.synchronize()
    for i, (g, w) in enumerate(zip(got, want)):
        assert torch.equal(g, w), i
    for i, x in enumerate(xs):
        assert np.array_equal(bits(ys[i].cpu().numpy()), bits(oracle.quantize(x, f[0], f[1], f[2]))), i
        assert same_hist(fmt, hs[i], oracle.histogram(x, f[0], f[1], -48)), i


def test_repeated_calls_start_from_clean_records(fmt):
    """The partial statistics records in library scratch are summed and cleared by every call: a second, smaller
    call into the same buffers gives the second tensors' statistics."""
    f = (6, 9, True)
    a = [mixed_matrix(300, 500, 1), mixed_matrix(64, 64, 2)]
    b = [mixed_matrix(40, 70, 3)]
    hs = [fmt.new_hist(), fmt.new_hist()]
    da, db = [dev(x) for x in a], [dev(x) for x in b]
    fmt.fmt_quantize_prepare_pair_batch(da, f, [torch.empty_like(x) for x in da], hs)
    y = [torch.empty_like(db[0])]
    fmt.fmt_quantize_prepare_pair_batch(db, f, y, hs[:1])
    fmt.fmt_quantize(da[1], f, hist=hs[1])                     # and fmt_quantize shares the same scratch
    torch.cuda.synchronize()
    assert same_hist(fmt, hs[0], oracle.histogram(b[0], f[0], f[1], -48))
    assert same_hist(fmt, hs[1], oracle.histogram(a[1], f[0], f[1], -48))
    assert np.array_equal(bits(y[0].cpu().numpy()), bits(oracle.quantize(b[0], f[0], f[1], f[2])))


def test_config4_tensors_match_fmt_quantize_and_the_prepare_call(fmt):
    """The benchmark's twelve tensors (workloads.config4) at full size: rounded copies and statistics equal those of
    fmt_quantize (checked against the oracle at this size by the stream tests) and, on sampled rows, the oracle's
    directly; the products on the operands equal those on fmt_prepare_pair_batch's."""
    f = (6, 9, True)
    cfg = workloads.config4()
    host = [t for L in cfg["layers"] for t in (L["X"], L["W"], L["dY"])]
    tens = [dev(t) for t in host]
    ys = [torch.empty_like(t) for t in tens]
    hs = [fmt.new_hist() for _ in tens]
    ops = fmt.fmt_quantize_prepare_pair_batch(tens, f, ys, hs)
    ref = fmt.fmt_prepare_pair_batch(tens, f)
    rng = np.random.default_rng(3)
    for i, (t, y, h) in enumerate(zip(tens, ys, hs)):
        h2 = fmt.new_hist()
        y2 = fmt.fmt_quantize(t, f, hist=h2)
        assert torch.equal(y.view(torch.int32), y2.view(torch.int32)), i
        assert torch.equal(h, h2), i
        rows = rng.integers(0, host[i].shape[0], 8)
        assert np.array_equal(bits(y[torch.from_numpy(rows).cuda()].cpu().numpy()),
                              bits(oracle.quantize(np.ascontiguousarray(host[i][rows]), f[0], f[1], f[2]))), i
        assert same_hist(fmt, h, oracle.histogram(host[i], f[0], f[1], -48)), i

    def products(o):
        A, B = [], []
        for i in range(0, len(o), 3):
            (X, Xt), (W, Wt), (D, Dt) = o[i], o[i + 1], o[i + 2]
            A += [X, D, Dt]
            B += [W, Wt, Xt]
        return fmt.fmt_gemm_prepared_batch(A, B)

    got, want = products(ops), products(ref)
    torch.cuda.synchronize()
    for i, (g, w) in enumerate(zip(got, want)):
        assert torch.equal(g, w), i


def test_empty_and_argument_errors(fmt):
    f = (6, 9, True)
    assert fmt.fmt_quantize_prepare_pair_batch([], f, [], []) == []
    x, z = torch.randn(64, 96, device="cuda"), torch.randn(32, 48, device="cuda")
    h = [fmt.new_hist(), fmt.new_hist()]
    with pytest.raises(ValueError):
        fmt.fmt_quantize_prepare_pair_batch([x, z], f, [torch.empty_like(x)], h)
    with pytest.raises(ValueError):
        fmt.fmt_quantize_prepare_pair_batch([x], f, [torch.empty(64, 95, device="cuda")], h[:1])
    with pytest.raises(fmt.FmtError) as e:                      # a format whose operands are not exponent planes
        fmt.fmt_quantize_prepare_pair_batch([x], (5, 10, True), [torch.empty_like(x)], h[:1])
    assert e.value.status == -1
    with pytest.raises(fmt.FmtError) as e:                      # two tensors' statistics in one record
        fmt.fmt_quantize_prepare_pair_batch([x, z], f, [torch.empty_like(x), torch.empty_like(z)], [h[0], h[0]])
    assert e.value.status == -6
    big = torch.empty(64 * 96 + 8, device="cuda")
    big[:64 * 96] = x.reshape(-1)
    xin = big[:64 * 96].view(64, 96)
    with pytest.raises(fmt.FmtError) as e:                      # a rounded copy shifted over its own input
        fmt.fmt_quantize_prepare_pair_batch([xin], f, [big[8:8 + 64 * 96].view(64, 96)], h[:1])
    assert e.value.status == -6
    with pytest.raises(fmt.FmtError) as e:                      # a rounded copy over another tensor's input
        fmt.fmt_quantize_prepare_pair_batch([x, z], f, [torch.empty_like(x), x[:32, :48]], h)
    assert e.value.status in (-6, -3)
    torch.cuda.synchronize()
