"""GPU parity of fmt_gemm_prepared_batch: several products on prepared operands handed over in one call, the
small ones sharing kernel launches (Sec. IV-A: a layer's three products are all known once its tensors are
rounded; Sec. III-B: every product is an FMACS sum).  Checked against the CPU oracle -- bit for bit where every
partial sum is exact, within the 1e-5 relative Frobenius bound otherwise -- and against fmt_gemm_prepared on the
same operands, for every piece scheme, mixed and ragged shapes, members that run alone (split over k, long k),
more members than one launch holds, shared operands, and the argument errors."""
import numpy as np
import pytest

import oracle

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

TOL = 1e-5


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


def rel_err(got, ref):
    return float(np.linalg.norm(got.astype(np.float64) - ref.astype(np.float64)) /
                 max(np.linalg.norm(ref.astype(np.float64)), 1e-300))


def exact_operands(rng, f, M, N, K):
    """Small integers times per-row powers of two over the format's range: every partial sum is exact in fp32 in
    any order (also rows in the planes above and below the main one)."""
    c = oracle.format_constants(f[0], f[1])
    lo, hi = max(c["Emin"] + 1, -50), min(c["Emax"] - 6, 50)
    s, t = rng.integers(lo, hi, M), rng.integers(lo, hi, N)
    a = (rng.integers(-7, 8, (M, K)) * np.exp2(s.astype(np.float64))[:, None]).astype(np.float32)
    b = (rng.integers(-7, 8, (N, K)) * np.exp2(t.astype(np.float64))[:, None]).astype(np.float32)
    return a, b


SHAPES = [(190, 170, 260), (1, 1, 1), (128, 128, 32), (129, 257, 33), (300, 40, 1000), (64, 700, 96), (512, 384, 512),
          (5, 1000, 70)]


@pytest.mark.parametrize("tile", ["2", "4"])
@pytest.mark.parametrize("f", [(6, 9, True), (6, 8, False), (5, 10, True), (8, 7, False), (6, 12, True), (7, 16, False)])
def test_mixed_shapes_bit_identical_to_the_oracle(fmt, f, tile, monkeypatch):
    """Both workgroup tiles of the shared launch (128 x 128 and 256 x 256; the library picks one per launch, the
    variable forces it; three-piece formats have only the small one)."""
    monkeypatch.setenv("FMT_GEMM_GROUP_TILE", tile)
    rng = np.random.default_rng(100 + f[1])
    ab = [exact_operands(rng, f, *s) for s in SHAPES]
    A = [fmt.fmt_prepare(dev(a), f) for a, _ in ab]
    B = [fmt.fmt_prepare(dev(b), f) for _, b in ab]
    out = fmt.fmt_gemm_prepared_batch(A, B)
    torch.cuda.synchronize()
    for (a, b), c, shape in zip(ab, out, SHAPES):
        ref = oracle.gemm(a, b, f[0], f[1], f[2], transB=True)
        assert np.array_equal(c.cpu().numpy().view(np.uint32), ref.view(np.uint32)), shape


@pytest.mark.parametrize("f", [(6, 9, True), (5, 10, True), (8, 7, False), (6, 10, True), (4, 3, True)])
def test_random_operands_within_tolerance(fmt, f):
    """Normal operands with heavy tails (so that 1/6/9 fills the planes above and below): each result within the
    bound of the oracle."""
    rng = np.random.default_rng(f[0] * 31 + f[1])
    shapes = [(257, 130, 515), (100, 300, 64), (384, 256, 1024), (33, 33, 2048)]
    c = oracle.format_constants(f[0], f[1])
    lo, hi = max(-30, c["Emin"] - f[1]), min(12, c["Emax"] - 4)       # no overflow: the sums stay finite
    ab = []
    for M, N, K in shapes:
        a = (rng.standard_normal((M, K)) * np.exp2(rng.integers(lo, hi, (M, K)) * (rng.random((M, K)) < 0.02))).astype(np.float32)
        b = (rng.standard_normal((N, K)) * np.exp2(rng.integers(lo, hi, (N, K)) * (rng.random((N, K)) < 0.02))).astype(np.float32)
        ab.append((a, b))
    A = [fmt.fmt_prepare(dev(a), f) for a, _ in ab]
    B = [fmt.fmt_prepare(dev(b), f) for _, b in ab]
    out = fmt.fmt_gemm_prepared_batch(A, B)
    torch.cuda.synchronize()
    for (a, b), c in zip(ab, out):
        ref = oracle.gemm(a, b, f[0], f[1], f[2], transB=True)
        assert rel_err(c.cpu().numpy(), ref) <= TOL


@pytest.mark.parametrize("tile", ["2", "4"])
def test_same_tiles_same_bits_as_single_calls(fmt, tile, monkeypatch):
    """A product accumulates over k in the same order in a shared launch as in a launch of its own (when
    neither splits k), so the results agree bit for bit, whatever the data."""
    f = (6, 9, True)
    rng = np.random.default_rng(3)
    shapes = [(257, 130, 515), (384, 256, 1024), (100, 300, 64)]
    A = [fmt.fmt_prepare(dev(rng.standard_normal((M, K)).astype(np.float32)), f) for M, N, K in shapes]
    B = [fmt.fmt_prepare(dev(rng.standard_normal((N, K)).astype(np.float32)), f) for M, N, K in shapes]
    monkeypatch.setenv("FMT_GEMM_GROUP_TILE", tile)
    monkeypatch.setenv("FMT_GEMM_PLAN", "2,2,1,1")        # no member is split over k: all of them share the launch
    out = fmt.fmt_gemm_prepared_batch(A, B)
    for a, b, c in zip(A, B, out):
        single = fmt.fmt_gemm_prepared(a, b)
        torch.cuda.synchronize()
        assert torch.equal(single, c)


def test_members_that_run_alone_and_more_members_than_a_launch_holds(fmt):
    """40 products: 37 small ones (three launches of up to 16), one with k = 8192 (beyond the grouped kernels'
    4096), one that fmt_gemm_prepared splits over k (few tiles, long k), one more small one at the end; one
    operand B shared by all the small ones."""
    f = (6, 9, True)
    rng = np.random.default_rng(40)
    a_s, b_s = exact_operands(rng, f, 70, 90, 160)
    Bs = fmt.fmt_prepare(dev(b_s), f)
    pairs, A, B = [], [], []
    for i in range(37):
        a = np.roll(a_s, i, axis=0)
        pairs.append((a, b_s))
        A.append(fmt.fmt_prepare(dev(a), f))
        B.append(Bs)
    for M, N, K in [(96, 64, 8192), (64, 64, 4096), (40, 50, 64)]:
        a, b = exact_operands(rng, f, M, N, K)
        a, b = (a / 8).astype(np.float32), b         # keep the longer sums below 2^24 units
        a[:, 512:] = 0
        pairs.append((a, b))
        A.append(fmt.fmt_prepare(dev(a), f))
        B.append(fmt.fmt_prepare(dev(b), f))
    out = fmt.fmt_gemm_prepared_batch(A, B)
    torch.cuda.synchronize()
    for i, ((a, b), c) in enumerate(zip(pairs, out)):
        ref = oracle.gemm(a, b, f[0], f[1], f[2], transB=True)
        assert np.array_equal(c.cpu().numpy().view(np.uint32), ref.view(np.uint32)), i


def test_strided_results_keep_their_surroundings(fmt):
    f = (5, 10, True)
    rng = np.random.default_rng(8)
    a, b = exact_operands(rng, f, 100, 60, 96)
    big = torch.full((2, 100, 200), -7.0, device="cuda")
    A = [fmt.fmt_prepare(dev(a), f)] * 2
    B = [fmt.fmt_prepare(dev(b), f)] * 2
    fmt.fmt_gemm_prepared_batch(A, B, out=[big[0, :, 10:70], big[1, :, 100:160]])
    torch.cuda.synchronize()
    ref = oracle.gemm(a, b, f[0], f[1], f[2], transB=True)
    h = big.cpu().numpy()
    assert np.array_equal(h[0, :, 10:70], ref) and np.array_equal(h[1, :, 100:160], ref)
    h[0, :, 10:70] = -7.0
    h[1, :, 100:160] = -7.0
    assert np.all(h == -7.0)


def test_empty_batch_and_argument_errors(fmt):
    f = (6, 9, True)
    assert fmt.fmt_gemm_prepared_batch([], []) == []
    A = fmt.fmt_prepare(torch.randn(64, 96, device="cuda"), f)
    B = fmt.fmt_prepare(torch.randn(32, 96, device="cuda"), f)
    Bk = fmt.fmt_prepare(torch.randn(32, 64, device="cuda"), f)
    Ah = fmt.fmt_prepare(torch.randn(64, 96, device="cuda"), (5, 10, True))
    Bh = fmt.fmt_prepare(torch.randn(32, 96, device="cuda"), (5, 10, True))
    with pytest.raises(fmt.FmtError) as ei:
        fmt.fmt_gemm_prepared_batch([A, A], [B, Bk])                  # k differs in the second product
    assert ei.value.status == -3
    with pytest.raises(fmt.FmtError) as ei:
        fmt.fmt_gemm_prepared_batch([A, Ah], [B, Bh])                 # two formats in one batch
    assert ei.value.status == -1
    c = torch.empty(64, 32, device="cuda")
    with pytest.raises(fmt.FmtError) as ei:
        fmt.fmt_gemm_prepared_batch([A, A], [B, B], out=[c, c])       # two products into one result
    assert ei.value.status == -6
    with pytest.raises(ValueError):
        fmt.fmt_gemm_prepared_batch([A], [B, B])
    with pytest.raises(ValueError):
        fmt.fmt_gemm_prepared_batch([A], [B], out=[torch.empty(64, 33, device="cuda")])
    torch.cuda.synchronize()


def test_config4_layer_twelve_products_one_call_sampled(fmt):
    """The twelve products of configuration 4's layer (forward, dgrad and wgrad of the four projections; 4096
    tokens, d = 1024, FFN 4096) in one call at full size, in the launch shape the benchmark times; one sampled
    element per 128 x 128 tile checked against the oracle's dot product."""
    f = (6, 9, True)
    T, d, ff = 4096, 1024, 4096
    g = torch.Generator(device="cuda").manual_seed(4)
    def rnd(r, c, scale):
        return torch.randn(r, c, device="cuda", generator=g) * scale
    layers = [(d, d), (d, d), (d, ff), (ff, d)]          # (in, out)
    A, B, src = [], [], []
    for fin, fout in layers:
        x, w, dy = rnd(T, fin, 1.0), rnd(fout, fin, 0.03), rnd(T, fout, 1e-3)
        X, Xt = fmt.fmt_prepare_pair(x, f)
        W, Wt = fmt.fmt_prepare_pair(w, f)
        D, Dt = fmt.fmt_prepare_pair(dy, f)
        A += [X, D, Dt]
        B += [W, Wt, Xt]
        src += [(x, w), (dy, w.t()), (dy.t(), x.t())]
    out = fmt.fmt_gemm_prepared_batch(A, B)
    torch.cuda.synchronize()
    rng = np.random.default_rng(12)
    for (a, b), c in zip(src, out):
        M, N = c.shape
        ii = (np.arange(0, M, 128)[:, None] + rng.integers(0, 128, (M // 128, N // 128))).ravel()
        jj = (np.arange(0, N, 128)[None, :] + rng.integers(0, 128, (M // 128, N // 128))).ravel()
        sel = rng.choice(ii.size, 64, replace=False)
        ah = a[torch.from_numpy(ii[sel]).cuda()].cpu().numpy()
        bh = b[torch.from_numpy(jj[sel]).cuda()].cpu().numpy()
        qa = oracle.quantize(ah, f[0], f[1], f[2]).astype(np.float64)
        qb = oracle.quantize(bh, f[0], f[1], f[2]).astype(np.float64)
        ref = np.sum(qa * qb, axis=1)
        got = c.cpu().numpy()[ii[sel], jj[sel]].astype(np.float64)
        scale = np.sqrt(np.sum(qa * qa, axis=1) * np.sum(qb * qb, axis=1))
        assert np.all(np.abs(got - ref) <= 1e-5 * scale)


@pytest.mark.parametrize("tile", [None, "2", "4"])
@pytest.mark.parametrize("f", [(6, 9, True), (5, 10, True), (6, 12, True)])
def test_member_with_k_in_parts(fmt, f, tile, monkeypatch):
    """A product of few tiles and long k beside products that fill the machine: the library runs its k in parts
    inside the shared launch (each part a run of tiles writing a slab of partial sums, summed in part order
    afterwards), or alone -- either way exact data must come out bit for bit, also for a second such member and
    for ragged shapes."""
    if tile is not None:
        monkeypatch.setenv("FMT_GEMM_GROUP_TILE", tile)
    rng = np.random.default_rng(77 + f[1])
    shapes = [(1024, 1024, 512)] * 8 + [(64, 64, 8192), (100, 70, 6000), (256, 256, 96)]
    ab = []
    for M, N, K in shapes:
        a, b = exact_operands(rng, f, M, N, K)
        a[:, 700:] = 0                                   # sums below 2^24 units whatever k
        ab.append((a, b))
    A = [fmt.fmt_prepare(dev(a), f) for a, _ in ab]
    B = [fmt.fmt_prepare(dev(b), f) for _, b in ab]
    out = fmt.fmt_gemm_prepared_batch(A, B)
    torch.cuda.synchronize()
    for (a, b), c, shape in zip(ab, out, shapes):
        ref = oracle.gemm(a, b, f[0], f[1], f[2], transB=True)
        assert np.array_equal(c.cpu().numpy().view(np.uint32), ref.view(np.uint32)), shape


def test_config3_products_one_call_sampled(fmt):
    """Configuration 3's three products (forward, dgrad, wgrad of the 3x3 convolution as im2col products:
    12544 x 256 x 2304 and its permutations) in one call at full size, as the benchmark issues them; one sampled
    element per 128 x 128 tile against the oracle's dot product."""
    f = (6, 9, True)
    M, N, K = 12544, 256, 2304
    g = torch.Generator(device="cuda").manual_seed(3)
    x = torch.randn(M, K, device="cuda", generator=g)
    w = torch.randn(N, K, device="cuda", generator=g) * 0.03
    dy = torch.randn(M, N, device="cuda", generator=g) * 1e-3
    X, Xt = fmt.fmt_prepare_pair(x, f)
    W, Wt = fmt.fmt_prepare_pair(w, f)
    D, Dt = fmt.fmt_prepare_pair(dy, f)
    out = fmt.fmt_gemm_prepared_batch([X, D, Dt], [W, Wt, Xt])
    torch.cuda.synchronize()
    rng = np.random.default_rng(33)
    for (a, b), c in zip([(x, w), (dy, w.t()), (dy.t(), x.t())], out):
        m, n = c.shape
        tm, tn = (m + 127) // 128, (n + 127) // 128
        ii = np.minimum(np.arange(tm)[:, None] * 128 + rng.integers(0, 128, (tm, tn)), m - 1).ravel()
        jj = np.minimum(np.arange(tn)[None, :] * 128 + rng.integers(0, 128, (tm, tn)), n - 1).ravel()
        sel = rng.choice(ii.size, min(96, ii.size), replace=False)
        ah = a[torch.from_numpy(ii[sel]).cuda()].cpu().numpy()
        bh = b[torch.from_numpy(jj[sel]).cuda()].cpu().numpy()
        qa = oracle.quantize(ah, f[0], f[1], f[2]).astype(np.float64)
        qb = oracle.quantize(bh, f[0], f[1], f[2]).astype(np.float64)
        ref = np.sum(qa * qb, axis=1)
        got = c.cpu().numpy()[ii[sel], jj[sel]].astype(np.float64)
        scale = np.sqrt(np.sum(qa * qa, axis=1) * np.sum(qb * qb, axis=1))
        assert np.all(np.abs(got - ref) <= 1e-5 * scale)


def test_config4_layer_twelve_products_every_element(fmt):
    """The same twelve products on the benchmark's own tensors (workloads.config4: N(0,1) activations, N(0, 0.02^2)
    weights, log-normal output gradients that reach into the denormal range and a few binades above plane 0),
    every element of every result against the oracle's product -- 309 GFLOP on the host's cores -- within the
    1e-5 relative Frobenius bound, and element by element within 1e-5 of |a| . |b| (the scale of the sum)."""
    import workloads
    f = (6, 9, True)
    cfg = workloads.config4()
    A, B, src = [], [], []
    for L in cfg["layers"]:
        x, w, dy = L["X"], L["W"], L["dY"]
        X, Xt = fmt.fmt_prepare_pair(dev(x), f)
        W, Wt = fmt.fmt_prepare_pair(dev(w), f)
        D, Dt = fmt.fmt_prepare_pair(dev(dy), f)
        A += [X, D, Dt]
        B += [W, Wt, Xt]
        src += [(x, w, False, True), (dy, w, False, False), (dy, x, True, False)]      # (a, b, transA, transB)
    out = fmt.fmt_gemm_prepared_batch(A, B)
    torch.cuda.synchronize()
    for i, ((a, b, ta, tb), c) in enumerate(zip(src, out)):
        ref = oracle.gemm(a, b, f[0], f[1], f[2], transA=ta, transB=tb)
        got = c.cpu().numpy()
        assert got.shape == ref.shape
        assert rel_err(got, ref) <= TOL, i
        qa = oracle.quantize(a, f[0], f[1], f[2]).astype(np.float64)
        qb = oracle.quantize(b, f[0], f[1], f[2]).astype(np.float64)
        na = np.sqrt((qa * qa).sum(axis=0 if ta else 1))            # norm of every row of op(A)
        nb = np.sqrt((qb * qb).sum(axis=1 if tb else 0))            # ... and of every column of op(B)
        bound = 1e-5 * na[:, None] * nb[None, :]
        assert np.all(np.abs(got.astype(np.float64) - ref.astype(np.float64)) <= bound), i


def test_config3_products_every_element(fmt):
    """Configuration 3 on the benchmark's own tensors (relu activations as the im2col matrix, He-scaled filter,
    log-normal output gradients): forward, dgrad and wgrad in one call -- the weight gradient with its k = 12544
    in parts -- every element against the oracle."""
    import workloads
    f = (6, 9, True)
    cfg = workloads.config3()
    xcol = workloads.im2col_3x3(cfg["X"])
    w, dy = cfg["W"], cfg["dY"]
    X, Xt = fmt.fmt_prepare_pair(dev(xcol), f)
    W, Wt = fmt.fmt_prepare_pair(dev(w), f)
    D, Dt = fmt.fmt_prepare_pair(dev(dy), f)
    out = fmt.fmt_gemm_prepared_batch([X, D, Dt], [W, Wt, Xt])
    torch.cuda.synchronize()
    for i, ((a, b, ta, tb), c) in enumerate(zip([(xcol, w, False, True), (dy, w, False, False), (dy, xcol, True, False)], out)):
        ref = oracle.gemm(a, b, f[0], f[1], f[2], transA=ta, transB=tb)
        got = c.cpu().numpy()
        assert rel_err(got, ref) <= TOL, i
        qa = oracle.quantize(a, f[0], f[1], f[2]).astype(np.float64)
        qb = oracle.quantize(b, f[0], f[1], f[2]).astype(np.float64)
        na = np.sqrt((qa * qa).sum(axis=0 if ta else 1))
        nb = np.sqrt((qb * qb).sum(axis=1 if tb else 0))
        assert np.all(np.abs(got.astype(np.float64) - ref.astype(np.float64)) <= 1e-5 * na[:, None] * nb[None, :]), i
