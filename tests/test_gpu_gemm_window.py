"""GPU parity of fmt_gemm for 1/6/8 and 1/6/9 through exponent planes (every row of an operand gets an
exact power-of-two scale that moves the binades where it lives into binary16's range -- plane 0, one
fp16 MFMA product per multiply; an element that does not fit there sits, exactly, in the plane above or
the plane below, and a small kernel after the product adds its products one by one).
FMT_GEMM_WINDOW=1 forces the scheme at every size; the cases are built so that a missing scale or a lost
product of an element outside plane 0 shows as a gross error.  (1/6/10 is in the list as a format that
does NOT take this route: it runs on two bf16 pieces.)"""
import os

import numpy as np
import pytest

import oracle
import workloads

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

TOL = 1e-5
FORMATS = [(6, 9, True), (6, 9, False), (6, 10, True), (6, 8, False)]
LAYOUTS = [(False, False), (False, True), (True, False), (True, True)]


@pytest.fixture(scope="module")
def fmt():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    import paper_2103_15940_amd as lib
    return lib


@pytest.fixture(autouse=True)
def forced_window(monkeypatch):
    monkeypatch.setenv("FMT_GEMM_WINDOW", "1")
    monkeypatch.delenv("FMT_GEMM_PLAN", raising=False)


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def rel_err(got, ref):
    return float(np.linalg.norm(got.astype(np.float64) - ref.astype(np.float64)) /
                 max(np.linalg.norm(ref.astype(np.float64)), 1e-300))


def gpu(fmt, A, B, f, tA=False, tB=False):
    Ain = np.ascontiguousarray(A.T) if tA else A
    Bin = np.ascontiguousarray(B.T) if tB else B
    C = fmt.fmt_gemm(dev(Ain), dev(Bin), f, transA=tA, transB=tB)
    torch.cuda.synchronize()
    return C.cpu().numpy()


def ref(A, B, f):
    return oracle.gemm(A, B, f[0], f[1], f[2])


@pytest.mark.parametrize("tA,tB", LAYOUTS)
@pytest.mark.parametrize("f", FORMATS)
def test_row_and_column_scales_bit_exact(fmt, f, tA, tB):
    """Row i of A is small integers times 2^s_i, column j of B small integers times 2^t_j, with s and t
    spread over the format's range: no row needs more than one binade-window, every sum is an integer
    times 2^(s_i + t_j) with few bits, so the result must equal the oracle bit for bit whatever the
    scales (from the extreme ones down to none)."""
    rng = np.random.default_rng(f[1] + 2 * int(tA) + int(tB))
    M, N, K = 150, 140, 200
    s = rng.integers(-29, 26, M)
    t = rng.integers(-29, 26, N)
    s[:4] = [-29, 25, 0, -15]
    A = (rng.integers(-7, 8, (M, K)) * np.exp2(s.astype(np.float64))[:, None]).astype(np.float32)
    B = (rng.integers(-7, 8, (K, N)) * np.exp2(t.astype(np.float64))[None, :]).astype(np.float32)
    got, want = gpu(fmt, A, B, f, tA, tB), ref(A, B, f)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def planted(rng, M, K, base_exp, out_exp, per_row):
    """Rows of values around 2^base_exp with `per_row` elements around 2^out_exp planted in each."""
    X = (rng.standard_normal((M, K)) * 2.0 ** base_exp).astype(np.float32)
    for i in range(M):
        for k in rng.choice(K, per_row, replace=False):
            X[i, k] = np.float32(rng.choice([-1.0, 1.0]) * (1.0 + rng.random()) * 2.0 ** out_exp)
    return X


@pytest.mark.parametrize("per_row", [1, 3, 8])
@pytest.mark.parametrize("tA,tB", LAYOUTS)
def test_large_outliers_in_A(fmt, per_row, tA, tB):
    """Every row of A holds many small normal values (2^-27) and a few huge ones (2^20): 47 binades, plane 0
    keeps the small ones, the huge ones sit in the plane above and carry almost the whole result."""
    f = (6, 9, True)
    rng = np.random.default_rng(100 + per_row)
    A = planted(rng, 130, 260, -27, 20, per_row)
    B = rng.standard_normal((260, 96)).astype(np.float32)
    got, want = gpu(fmt, A, B, f, tA, tB), ref(A, B, f)
    assert rel_err(got, want) <= TOL


@pytest.mark.parametrize("per_col", [1, 8])
@pytest.mark.parametrize("tA,tB", LAYOUTS)
def test_large_outliers_in_B_and_in_both(fmt, per_col, tA, tB):
    f = (6, 9, False)
    rng = np.random.default_rng(200 + per_col)
    A = rng.standard_normal((70, 300)).astype(np.float32)
    Bt = planted(rng, 150, 300, -26, 18, per_col)            # columns of B
    got, want = gpu(fmt, A, Bt.T.copy(), f, tA, tB), ref(A, Bt.T.copy(), f)
    assert rel_err(got, want) <= TOL
    # outliers in both operands, some at the same k: every product must be added exactly once
    A2 = planted(rng, 70, 300, -27, 19, 2)
    A2[:, 7] = np.float32(2.0 ** 19)
    Bt[:, 7] = np.float32(-(2.0 ** 18))
    got, want = gpu(fmt, A2, Bt.T.copy(), f, tA, tB), ref(A2, Bt.T.copy(), f)
    assert rel_err(got, want) <= TOL


def test_many_elements_outside_plane_0(fmt):
    """Rows with many elements in the plane above (there is no limit on how many a row may have), and
    rows whose values spread evenly over 60 binades: about half of every row lives outside plane 0, in
    the plane above and the plane below at once."""
    f = (6, 9, True)
    rng = np.random.default_rng(300)
    A = planted(rng, 64, 256, -27, 20, 9)
    B = rng.standard_normal((256, 80)).astype(np.float32)
    assert rel_err(gpu(fmt, A, B, f), ref(A, B, f)) <= TOL
    A = (rng.choice([-1.0, 1.0], (96, 512)) * np.exp2(rng.uniform(-29.0, 29.0, (96, 512)))).astype(np.float32)
    assert rel_err(gpu(fmt, A, B.repeat(2, axis=0), f), ref(A, B.repeat(2, axis=0), f)) <= TOL


def test_gradient_like_rows(fmt):
    """log2|g| ~ N(-24, 6^2) as in config 4: plane 0 of such a row reaches from the format's smallest
    denormal up to 2; the few values above that sit in the plane above."""
    f = (6, 9, True)
    rng = np.random.default_rng(400)
    G = workloads.log2_normal((300, 520), -24.0, 6.0, 0.01, rng)
    W = (rng.standard_normal((520, 200)) * 0.02).astype(np.float32)
    assert rel_err(gpu(fmt, G, W, f), ref(G, W, f)) <= TOL
    X = rng.standard_normal((300, 330)).astype(np.float32)
    assert rel_err(gpu(fmt, G.T.copy(), X, f, tA=True), ref(G.T.copy(), X, f)) <= TOL      # wgrad layout: G is stored as is


def test_denormals_zeros_and_extremes(fmt):
    """The format's denormal range (multiples of 2^-39), its largest values, all-zero rows and columns,
    rows that only hold denormals."""
    f = (6, 9, True)
    rng = np.random.default_rng(500)
    A = workloads.log2_normal((90, 200), -33.0, 3.0, 0.1, rng)          # mostly denormal in 1/6/9
    A[5] = 0.0
    A[6] = np.float32(2.0 ** -39)
    A[7, :] = (rng.integers(1, 1024, 200) * 2.0 ** 22).astype(np.float32)   # up to 2^32 - 2^22 = maxN
    B = (rng.integers(-3, 4, (200, 60))).astype(np.float32)
    B[:, 3] = 0.0
    got, want = gpu(fmt, A, B, f), ref(A, B, f)
    assert rel_err(got, want) <= TOL
    assert np.array_equal(got[5], np.zeros(60, dtype=np.float32)) and np.array_equal(got[:, 3], np.zeros(90, dtype=np.float32))
    assert np.array_equal(got[6].view(np.uint32), want[6].view(np.uint32))   # integers times 2^-39: exact


@pytest.mark.parametrize("window", ["0", "1"])
def test_nonfinite_operands(fmt, window, monkeypatch):
    """Infinite and NaN operands, and a finite one that overflows the format, through the exponent planes (1)
    and through the two bf16 pieces (0).  What is pinned: an output is non-finite exactly where the oracle's
    is; where the oracle has NaN (a NaN operand, infinity times zero, infinities of both signs) so has the
    library; where the oracle has an infinity the library has that infinity or NaN (splitting an infinite
    value into pieces leaves inf - inf = NaN in the lower piece: the documented latitude); everything else
    is finite and within the tolerance."""
    monkeypatch.setenv("FMT_GEMM_WINDOW", window)
    f = (6, 9, True)
    rng = np.random.default_rng(600)
    A = rng.standard_normal((40, 64)).astype(np.float32)
    B = rng.standard_normal((64, 50)).astype(np.float32)
    A[3, 10] = np.inf
    A[9, 0] = np.nan
    A[20, 5] = 1e30                                   # overflows the format: rounds to infinity
    A[25, 7] = -np.inf
    B[7, 11] = 0.0                                    # -inf * 0 in C[25][11]
    A[30, 1], A[30, 2] = np.inf, np.inf
    B[1, 4], B[2, 4] = 1.0, -1.0                      # inf - inf in C[30][4]
    got, want = gpu(fmt, A, B, f), ref(A, B, f)
    bad = ~np.isfinite(want)
    assert np.array_equal(~np.isfinite(got), bad)
    assert np.isnan(want[25, 11]) and np.isnan(want[30, 4]) and np.isinf(want[3, 0])
    assert np.all(np.isnan(got[np.isnan(want)]))
    inf_at = np.isinf(want)
    assert np.all(np.isnan(got[inf_at]) | (got[inf_at] == want[inf_at]))
    assert rel_err(np.where(bad, 0, got), np.where(bad, 0, want)) <= TOL


@pytest.mark.parametrize("plan", ["2,2,3,0", "1,1,2,0", "4,4,2,1"])
def test_with_split_k_and_reproducible(fmt, plan, monkeypatch):
    monkeypatch.setenv("FMT_GEMM_PLAN", plan)
    f = (6, 9, True)
    rng = np.random.default_rng(700)
    A = planted(rng, 200, 1100, -20, 15, 2)
    B = planted(rng, 180, 1100, -5, -29, 1).T.copy()
    want = ref(A, B, f)
    first = gpu(fmt, A, B, f)
    assert rel_err(first, want) <= TOL
    for _ in range(3):
        assert np.array_equal(gpu(fmt, A, B, f).view(np.uint32), first.view(np.uint32))


def test_agrees_with_two_piece_scheme(fmt, monkeypatch):
    rng = np.random.default_rng(800)
    A = rng.standard_normal((257, 300)).astype(np.float32)
    B = (rng.standard_normal((300, 129)) * 0.02).astype(np.float32)
    f = (6, 9, True)
    one = gpu(fmt, A, B, f)
    monkeypatch.setenv("FMT_GEMM_WINDOW", "0")
    two = gpu(fmt, A, B, f)
    assert rel_err(one, two) <= 1e-6
    assert rel_err(one, ref(A, B, f)) <= TOL


def test_linear_layer_through_the_window(fmt):
    e, m, d = 6, 9, True
    rng = np.random.default_rng(900)
    X = rng.integers(-7, 8, (100, 96)).astype(np.float32)
    s = rng.integers(-28, 20, 130)
    W = (rng.integers(-7, 8, (130, 96)) * np.exp2(s.astype(np.float64))[:, None]).astype(np.float32)
    b = workloads.log2_normal(130, 0.0, 12.0, 0.05, rng)
    Yo, To = oracle.linear(X, W, b, e, m, d)
    h = fmt.new_hist(torch.device("cuda"))
    Y = fmt.fmt_linear(dev(X), dev(W), dev(b), (e, m, d), hist=h).cpu().numpy()
    nan = np.isnan(Yo)
    assert np.array_equal(np.isnan(Y), nan)
    assert np.array_equal(np.where(nan, 0, Y).view(np.uint32), np.where(nan, 0, Yo).astype(np.float32).view(np.uint32))
    ho = oracle.histogram(To, e, m)
    hg = fmt.hist_to_dict(h)
    assert all(int(hg[k]) == int(ho[k]) for k in ("total", "zero", "denormal", "normal", "overflow", "inf", "nan"))
