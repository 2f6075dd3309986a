"""GPU parity of prepared operands: fmt_prepare rounds a tensor once into the matrix cores' 16-bit
layout (caller-owned memory), fmt_gemm_prepared multiplies two of them (Sec. IV-A: the rounded tensor
is used wherever the layer needs it; Sec. III-B: FMACS).  Checked against the CPU oracle -- within the
1e-5 relative Frobenius bound, and bit for bit where every partial sum is exact -- for every piece
scheme (exponent planes for 1/6/9 and 1/6/8, one fp16 piece, one to three bf16 pieces), every
orientation, ragged shapes, all three planes, and one operand shared by several products."""
import numpy as np
import pytest

import oracle
import workloads

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

TOL = 1e-5
FORMATS = [(6, 9, True), (6, 9, False), (6, 8, True), (5, 10, True), (8, 7, False), (8, 7, True), (6, 10, True),
           (7, 16, False), (4, 3, True)]


@pytest.fixture(scope="module")
def fmt():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    import paper_2103_15940_amd as lib
    return lib


@pytest.fixture(autouse=True)
def default_plans(monkeypatch):
    monkeypatch.delenv("FMT_GEMM_PLAN", raising=False)
    monkeypatch.delenv("FMT_GEMM_WINDOW", raising=False)


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def rel_err(got, ref):
    return float(np.linalg.norm(got.astype(np.float64) - ref.astype(np.float64)) /
                 max(np.linalg.norm(ref.astype(np.float64)), 1e-300))


def product(fmt, a_rows_k, b_rows_k, f, ta=False, tb=False):
    """C = a b^T for a [M, K], b [N, K] given as arrays; ta / tb: hand the library the transposed
    storage (K x rows) and let fmt_prepare take the operand transposed."""
    A = fmt.fmt_prepare(dev(a_rows_k.T if ta else a_rows_k), f, trans=ta)
    B = fmt.fmt_prepare(dev(b_rows_k.T if tb else b_rows_k), f, trans=tb)
    C = fmt.fmt_gemm_prepared(A, B)
    torch.cuda.synchronize()
    return C.cpu().numpy()


def want(a_rows_k, b_rows_k, f):
    return oracle.gemm(a_rows_k, b_rows_k, f[0], f[1], f[2], transB=True)


@pytest.mark.parametrize("ta,tb", [(False, False), (False, True), (True, False), (True, True)])
@pytest.mark.parametrize("f", FORMATS)
def test_random_operands_every_scheme_and_orientation(fmt, f, ta, tb):
    rng = np.random.default_rng(7 * f[0] + f[1] + 2 * int(ta) + int(tb))
    M, N, K = 203, 150, 333                      # several units and tiles, ragged in every dimension
    c = oracle.format_constants(f[0], f[1])
    scale = 2.0 ** min(0, c["Emax"] - 4)
    a = (rng.standard_normal((M, K)) * scale).astype(np.float32)
    b = (rng.standard_normal((N, K)) * scale * 0.05).astype(np.float32)
    got, ref = product(fmt, a, b, f, ta, tb), want(a, b, f)
    assert rel_err(got, ref) <= TOL
    # the same operands through fmt_gemm: same kernels, same order of accumulation, same bits
    via_gemm = fmt.fmt_gemm(dev(a), dev(b), f, transB=True)
    torch.cuda.synchronize()
    if 2.0 * M * N * K < 1e9 and f[0] == 6 and f[1] in (8, 9):
        assert rel_err(via_gemm.cpu().numpy(), ref) <= TOL          # small products take two bf16 pieces there
    else:
        assert np.array_equal(via_gemm.cpu().numpy().view(np.uint32), got.view(np.uint32))


@pytest.mark.parametrize("f", [(6, 9, True), (6, 8, False), (5, 10, True), (8, 7, False), (6, 12, True)])
def test_exact_integer_products_are_bit_identical(fmt, f):
    """Small integers times per-row powers of two spread over the format's range: every partial sum is
    exact in fp32 whatever the order, so the result must equal the oracle's bit for bit -- including the
    rows whose scale puts them in the plane above or below the main one."""
    rng = np.random.default_rng(f[1])
    M, N, K = 190, 170, 260
    c = oracle.format_constants(f[0], f[1])
    lo, hi = c["Emin"] + 1, c["Emax"] - 6
    s = rng.integers(lo, hi, M)
    t = rng.integers(lo, hi, N)
    a = (rng.integers(-7, 8, (M, K)) * np.exp2(s.astype(np.float64))[:, None]).astype(np.float32)
    b = (rng.integers(-7, 8, (N, K)) * np.exp2(t.astype(np.float64))[:, None]).astype(np.float32)
    keep = np.abs(s[:, None] + t[None, :]) < 110          # sums (up to 2^14 times 2^(s+t)) inside fp32's normal range
    got, ref = product(fmt, a, b, f), want(a, b, f)
    assert np.array_equal(got.view(np.uint32)[keep], ref.view(np.uint32)[keep])


def test_all_three_planes_in_one_row(fmt):
    """1/6/9: rows that hold values from the smallest denormal (2^-39) to the largest binade (2^31) --
    71 binades, more than two planes of 31 -- so the plane above and the plane below both fill, in A and
    in B, at the same k and at different k.  Integers times powers of two: exact, bit for bit."""
    f = (6, 9, True)
    rng = np.random.default_rng(9)
    M, N, K = 96, 80, 192
    ea = rng.integers(-39, 21, (M, K))
    eb = rng.integers(-39, 21, (N, K))
    ea[:, 5], eb[:, 5] = 20, -39            # above x below at the same k
    ea[:, 6], eb[:, 6] = -39, -39           # below x below
    ea[:, 7], eb[:, 7] = 20, 20             # above x above
    a = (rng.integers(1, 4, (M, K)) * rng.choice([-1, 1], (M, K)) * np.exp2(ea.astype(np.float64))).astype(np.float32)
    b = (rng.integers(1, 4, (N, K)) * rng.choice([-1, 1], (N, K)) * np.exp2(eb.astype(np.float64))).astype(np.float32)
    got, ref = product(fmt, a, b, f), want(a, b, f)
    assert rel_err(got, ref) <= TOL
    # one term dominates each of these columns of k: compare single products exactly
    a1 = np.zeros((M, K), np.float32)
    b1 = np.zeros((N, K), np.float32)
    a1[:, 5:8], b1[:, 5:8] = a[:, 5:8], b[:, 5:8]
    got1, ref1 = product(fmt, a1, b1, f), want(a1, b1, f)
    assert np.array_equal(got1.view(np.uint32), ref1.view(np.uint32))


@pytest.mark.parametrize("f", [(6, 9, True), (6, 9, False), (6, 8, True)])
def test_wide_rows_denormals_and_flush(fmt, f):
    """Gradient-like rows (log-normal, sigma 6 binades around 2^-24) against weights, activations with
    planted huge and tiny values, the format's denormal range with and without flush."""
    rng = np.random.default_rng(40 + f[1] + int(f[2]))
    g = workloads.log2_normal((300, 520), -24.0, 6.0, 0.01, rng)
    w = (rng.standard_normal((200, 520)) * 0.02).astype(np.float32)
    assert rel_err(product(fmt, g, w, f), want(g, w, f)) <= TOL
    x = rng.standard_normal((130, 260)).astype(np.float32)
    for i in range(130):
        x[i, rng.choice(260, 3, replace=False)] = rng.choice([-1, 1]) * (1 + rng.random()) * 2.0 ** rng.choice([20, 25, -33, -36])
    w2 = rng.standard_normal((96, 260)).astype(np.float32)
    assert rel_err(product(fmt, x, w2, f), want(x, w2, f)) <= TOL
    assert rel_err(product(fmt, x, w2, f, ta=True, tb=True), want(x, w2, f)) <= TOL
    d = workloads.log2_normal((90, 200), -33.0, 3.0, 0.1, rng)          # mostly in the denormal range
    bi = rng.integers(-3, 4, (60, 200)).astype(np.float32)
    got, ref = product(fmt, d, bi, f), want(d, bi, f)
    assert rel_err(got, ref) <= TOL


def test_one_operand_feeds_several_products(fmt):
    """Config 2's first layer, call by call as a training step uses the rounded tensors (Sec. IV-A):
    R(X) in the forward product and the weight gradient, R(W) in forward and input gradient, R(dY) in
    both gradients -- six preparations, three products, each against the oracle."""
    f = (6, 9, True)
    cfg = workloads.config2()
    X, W = cfg["X"], cfg["W"][0]                                   # [256, 784], [1024, 784]
    rng = np.random.default_rng(2)
    dY = workloads.log2_normal((256, 1024), -20.0, 5.0, 0.0, rng)
    Xd, Wd, dYd = dev(X), dev(W), dev(dY)
    Xa, Xt = fmt.fmt_prepare(Xd, f), fmt.fmt_prepare(Xd, f, trans=True)        # rows = batch / rows = in
    Wa, Wt = fmt.fmt_prepare(Wd, f), fmt.fmt_prepare(Wd, f, trans=True)        # rows = out / rows = in
    Ga, Gt = fmt.fmt_prepare(dYd, f), fmt.fmt_prepare(dYd, f, trans=True)      # rows = batch / rows = out
    Y = fmt.fmt_gemm_prepared(Xa, Wa)          # X W^T
    dX = fmt.fmt_gemm_prepared(Ga, Wt)         # dY W
    dW = fmt.fmt_gemm_prepared(Gt, Xt)         # dY^T X
    again = fmt.fmt_gemm_prepared(Xa, Wa)      # the operands are not consumed
    torch.cuda.synchronize()
    assert rel_err(Y.cpu().numpy(), oracle.gemm(X, W, *f, transB=True)) <= TOL
    assert rel_err(dX.cpu().numpy(), oracle.gemm(dY, W, *f)) <= TOL
    assert rel_err(dW.cpu().numpy(), oracle.gemm(dY, X, *f, transA=True)) <= TOL
    assert torch.equal(again, Y)


@pytest.mark.parametrize("shape", [(1, 1, 1), (3, 5, 7), (64, 64, 32), (65, 257, 33), (256, 10, 1024), (10, 1024, 256),
                                   (300, 300, 2000)])
def test_shapes(fmt, shape):
    M, N, K = shape
    f = (6, 9, True)
    rng = np.random.default_rng(M + 3 * N + 5 * K)
    a = rng.standard_normal((M, K)).astype(np.float32)
    b = (rng.standard_normal((N, K)) * 0.1).astype(np.float32)
    assert rel_err(product(fmt, a, b, f), want(a, b, f)) <= TOL


@pytest.mark.parametrize("plan", ["2,2,3,0", "1,1,2,1", "4,4,2,1", "4,2,1,1", "2,4,1,0"])
def test_every_tile_and_split_with_planes(fmt, plan, monkeypatch):
    """Forced tiles and k splits with elements in all planes: same bits on every run, within tolerance."""
    monkeypatch.setenv("FMT_GEMM_PLAN", plan)
    f = (6, 9, True)
    rng = np.random.default_rng(70)
    a = rng.standard_normal((260, 1100)).astype(np.float32)
    b = (rng.standard_normal((200, 1100)) * 2.0 ** -8).astype(np.float32)
    for i in range(260):
        a[i, rng.choice(1100, 2, replace=False)] = np.float32(2.0 ** 22)
    for j in range(200):
        b[j, rng.choice(1100, 2, replace=False)] = np.float32(2.0 ** -38)
    ref = want(a, b, f)
    first = product(fmt, a, b, f)
    assert rel_err(first, ref) <= TOL
    assert np.array_equal(product(fmt, a, b, f).view(np.uint32), first.view(np.uint32))


def test_config4_layer_full_size_one_sample_per_tile(fmt):
    """The attention-output layer of config 4 at full size (4096 x 1024 x 1024) forward, dgrad and wgrad
    on prepared operands: one sampled output in every 128 x 128 block of the result (no larger tile
    aligned to 128 can be missed; smaller tiles are covered by the oracle-sized tests) plus the corners."""
    f = (6, 9, True)
    L = workloads.config4()["layers"][1]
    X, W, dY = L["X"], L["W"], L["dY"]
    Xd, Wd, Gd = dev(X), dev(W), dev(dY)
    prods = [("fwd", fmt.fmt_prepare(Xd, f), fmt.fmt_prepare(Wd, f), (X, W, False, True)),
             ("dgrad", fmt.fmt_prepare(Gd, f), fmt.fmt_prepare(Wd, f, trans=True), (dY, W, False, False)),
             ("wgrad", fmt.fmt_prepare(Gd, f, trans=True), fmt.fmt_prepare(Xd, f, trans=True), (dY, X, True, False))]
    rng = np.random.default_rng(4)
    for name, A, B, (a_host, b_host, tA, tB) in prods:
        C = fmt.fmt_gemm_prepared(A, B)
        torch.cuda.synchronize()
        M, N = A.rows, B.rows
        bi, bj = np.meshgrid(np.arange(0, M, 128), np.arange(0, N, 128), indexing="ij")
        rows = (bi + rng.integers(0, 128, bi.shape)).ravel().clip(0, M - 1)
        cols = (bj + rng.integers(0, 128, bj.shape)).ravel().clip(0, N - 1)
        rows = np.concatenate([rows, [0, 0, M - 1, M - 1]])
        cols = np.concatenate([cols, [0, N - 1, 0, N - 1]])
        ref = oracle.gemm_sampled(a_host, b_host, rows, cols, *f, transA=tA, transB=tB)
        got = C.cpu().numpy()[rows, cols]
        assert rel_err(got, ref) <= TOL, name
        # and every sample on its own, against the size of the terms it sums (fp32 accumulation of K exact
        # products errs by a few sqrt(K) 2^-24 of sum |a||b|): a wrong tile cannot hide behind large neighbours
        terms = oracle.gemm_sampled(np.abs(a_host), np.abs(b_host), rows, cols, *f, transA=tA, transB=tB).astype(np.float64)
        K = a_host.shape[0] if tA else a_host.shape[1]
        err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
        assert np.all(err <= 16 * np.sqrt(K) * 2.0 ** -24 * terms + 1e-45), (name, int(np.argmax(err / (terms + 1e-300))))


def test_argument_errors(fmt):
    f = (6, 9, True)
    x = torch.randn(64, 96, device="cuda")
    A = fmt.fmt_prepare(x, f)
    B = fmt.fmt_prepare(torch.randn(32, 64, device="cuda"), f)          # K differs
    with pytest.raises(fmt.FmtError) as ei:
        fmt.fmt_gemm_prepared(A, B)
    assert ei.value.status == -3
    Bh = fmt.fmt_prepare(torch.randn(32, 96, device="cuda"), (5, 10, True))
    with pytest.raises(fmt.FmtError) as ei:
        fmt.fmt_gemm_prepared(A, Bh)
    assert ei.value.status == -1
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(fmt.FmtError) as ei:
        fmt.fmt_prepare(x, f, out=small)
    assert ei.value.status == -3


@pytest.mark.parametrize("f", [(6, 9, True), (6, 8, False), (5, 10, True), (8, 7, False)])
def test_prepare_pair_equals_two_prepares(fmt, f):
    """fmt_prepare_pair gives the two operands that fmt_prepare gives with trans=False and trans=True (ragged
    shape, a row stride larger than the row, gradient-like rows that use all three planes): products on them
    have the same bits, and match the oracle."""
    rng = np.random.default_rng(77)
    rows, cols = 203, 150
    base = workloads.log2_normal((rows, cols + 6), -20.0, 7.0, 0.05, rng)
    X = dev(base)[:, :cols]                                        # ld = cols + 6
    need0, need1 = fmt.fmt_operand_bytes(rows, cols, f), fmt.fmt_operand_bytes(cols, rows, f)
    fill = lambda n: torch.full((n,), 0xAB, dtype=torch.uint8, device="cuda")
    a0, a1, b0, b1 = fill(need0), fill(need1), fill(need0), fill(need1)
    p0, p1 = fmt.fmt_prepare_pair(X, f, out=a0, out_t=a1)
    q0, q1 = fmt.fmt_prepare(X, f, trans=False, out=b0), fmt.fmt_prepare(X, f, trans=True, out=b1)
    B = dev(rng.standard_normal((64, cols)).astype(np.float32))
    Bt = dev(rng.standard_normal((48, rows)).astype(np.float32))
    Bp, Btp = fmt.fmt_prepare(B, f), fmt.fmt_prepare(Bt, f)
    C0, D0 = fmt.fmt_gemm_prepared(p0, Bp), fmt.fmt_gemm_prepared(q0, Bp)
    C1, D1 = fmt.fmt_gemm_prepared(p1, Btp), fmt.fmt_gemm_prepared(q1, Btp)
    torch.cuda.synchronize()
    assert (p0.rows, p0.k, p1.rows, p1.k) == (rows, cols, cols, rows)
    assert torch.equal(C0.view(torch.int32), D0.view(torch.int32)) and torch.equal(C1.view(torch.int32), D1.view(torch.int32))
    ref = oracle.gemm(np.ascontiguousarray(base[:, :cols]), B.cpu().numpy(), f[0], f[1], f[2], transB=True)
    assert rel_err(C0.cpu().numpy(), ref) <= TOL


@pytest.mark.parametrize("cols", ["256", "512", "1024"])
def test_tail_blocks_of_every_width(fmt, cols, monkeypatch):
    """The kernel that adds the products of the elements outside plane 0 owns blocks of 32 rows x 256, 512 or
    1024 columns of C (the library picks the width per launch; the variable forces it).  N = 2100 gives several
    blocks per row and a ragged last one at every width; both operands hold elements of all three planes, at
    equal and at different k.  Integers times powers of two: exact in any order, bit for bit."""
    monkeypatch.setenv("FMT_GEMM_TAIL_COLS", cols)
    f = (6, 9, True)
    rng = np.random.default_rng(int(cols))
    M, N, K = 70, 2100, 160
    ea = np.zeros((M, K), np.int64)
    eb = np.zeros((N, K), np.int64)
    for e, n in ((ea, M), (eb, N)):
        hit = rng.random((n, K)) < 0.03
        e[hit] = rng.choice([-38, -36, 18, 20], size=int(hit.sum()))
    ea[:, 3], eb[:, 3] = 20, -38
    ea[:, 4], eb[:, 4] = -38, -38
    a = (rng.integers(1, 4, (M, K)) * rng.choice([-1, 1], (M, K)) * np.exp2(ea.astype(np.float64))).astype(np.float32)
    b = (rng.integers(1, 4, (N, K)) * rng.choice([-1, 1], (N, K)) * np.exp2(eb.astype(np.float64))).astype(np.float32)
    got, ref = product(fmt, a, b, f), want(a, b, f)
    assert rel_err(got, ref) <= TOL
    # columns of k that hold one plane pair each: single products, exact
    for ks in ([3], [4], [9]):
        a1 = np.zeros_like(a)
        b1 = np.zeros_like(b)
        a1[:, ks], b1[:, ks] = a[:, ks], b[:, ks]
        got1, ref1 = product(fmt, a1, b1, f), want(a1, b1, f)
        assert np.array_equal(got1.view(np.uint32), ref1.view(np.uint32)), ks


@pytest.mark.parametrize("plan", ["4,4,1,1", "2,2,1,1", "1,1,1,1", "2,4,1,1", "2,2,3,1"])
@pytest.mark.parametrize("f", [(6, 9, True), (5, 10, True), (6, 12, True)])
def test_results_at_any_alignment(fmt, f, plan, monkeypatch):
    """The product kernel stores 16 bytes per lane wherever four columns of a row are in range; nothing may
    depend on C being 16-byte aligned.  C is a window of a larger tensor with an odd leading dimension and
    every column offset 0..3 (addresses 4, 8 and 12 bytes off a 16-byte boundary); the rest of the tensor
    must stay untouched.  Exact data, bit for bit."""
    monkeypatch.setenv("FMT_GEMM_PLAN", plan)
    rng = np.random.default_rng(7)
    M, N, K = 300, 270, 96
    a = rng.integers(-7, 8, (M, K)).astype(np.float32)
    b = rng.integers(-7, 8, (N, K)).astype(np.float32)
    A, B = fmt.fmt_prepare(dev(a), f), fmt.fmt_prepare(dev(b), f)
    ref = want(a, b, f)
    for off in range(4):
        big = torch.full((M + 2, 277), -5.0, device="cuda")
        out = big[1:M + 1, off:off + N]
        fmt.fmt_gemm_prepared(A, B, out=out)
        torch.cuda.synchronize()
        h = big.cpu().numpy()
        assert np.array_equal(h[1:M + 1, off:off + N], ref), off
        h[1:M + 1, off:off + N] = -5.0
        assert np.all(h == -5.0), off


@pytest.mark.parametrize("count", [1, 2, 63, 64, 65, 200])
def test_record_lists_at_their_capacity(fmt, count):
    """A prepared plane operand lists up to 64 elements outside plane 0 per 32 rows; a row block with more has
    only its count and is walked through its mask bytes instead.  `count` such elements in ONE block of 32 rows
    of A (and as many in one block of rows of B), at distinct (row, k), some sharing a row, some sharing a k
    with an element of the other operand; every other block has none.  Integers times powers of two: every
    partial sum is exact, so the result must equal the oracle's bit for bit on either path."""
    f = (6, 9, True)
    rng = np.random.default_rng(1000 + count)
    M, N, K = 96, 300, 224
    a = rng.integers(-3, 4, (M, K)).astype(np.float32)
    b = rng.integers(-3, 4, (N, K)).astype(np.float32)
    pos_a = rng.choice(32 * K, count, replace=False)
    pos_b = rng.choice(32 * K, count, replace=False)
    for p in pos_a:                                         # rows 32..63 of A: the plane above and the plane below
        a[32 + p // K, p % K] = float(rng.choice([-3, -1, 1, 2])) * 2.0 ** float(rng.choice([18, 19, -36, -37]))
    for p in pos_b:                                         # rows 64..95 of B
        b[64 + p // K, p % K] = float(rng.choice([-3, -1, 1, 2])) * 2.0 ** float(rng.choice([18, 19, -36, -37]))
    if count >= 2:                                          # an element of A and one of B at the same k
        a[33, 7] = 2.0 ** 19
        b[65, 7] = -(2.0 ** -36)
    got, ref = product(fmt, a, b, f), want(a, b, f)
    assert rel_err(got, ref) <= TOL
    # rows and columns whose sums stay exact: one scale per sum (no mixing of 2^18 and 2^-36 terms in one element)
    clean_rows = np.setdiff1d(np.arange(M), np.arange(32, 64))
    clean_cols = np.setdiff1d(np.arange(N), np.arange(64, 96))
    assert np.array_equal(got[np.ix_(clean_rows, clean_cols)].view(np.uint32), ref[np.ix_(clean_rows, clean_cols)].view(np.uint32))
    # and one element at a time, exactly, through both paths
    for (r, k) in [(32 + pos_a[0] // K, pos_a[0] % K)]:
        a1 = np.zeros_like(a)
        a1[r, k] = a[r, k]
        got1, ref1 = product(fmt, a1, b, f), want(a1, b, f)
        keep = np.ones(N, bool)
        keep[64:96] = np.abs(b[64:96, k]) < 8                # products of two elements outside plane 0 included where exact
        assert np.array_equal(got1[:, keep].view(np.uint32), ref1[:, keep].view(np.uint32))
