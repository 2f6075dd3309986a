"""GPU parity of fmt_prepare_pair_batch: the tensors of a step rounded into prepared operands, both orientations
each, in one call (Sec. IV-A: every tensor is rounded once and used in several products).  The operands are
checked through the products they give: bit for bit against the CPU oracle where every partial sum is exact,
within the 1e-5 relative Frobenius bound on random data, and bit for bit against the products of fmt_prepare_pair's
operands -- for the formats that share launches (1/6/m) and those prepared matrix by matrix, ragged and strided
inputs, more matrices than one launch holds, the benchmark's own tensors, and the argument errors."""
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


FORMATS = [(6, 9, True), (6, 8, False), (6, 9, False), (5, 10, True), (8, 7, False), (6, 12, True)]
SHAPES = [(190, 260), (1, 1), (128, 32), (129, 33), (300, 1000), (64, 96), (512, 384), (5, 70), (33, 1), (1, 257)]


def exact_matrix(rng, f, r, c):
    """Small integers times one power of two per matrix: X X^T and X^T X are exact in fp32 in any order."""
    k = oracle.format_constants(f[0], f[1])
    s = int(rng.integers(max(k["Emin"] + 1, -20), min(k["Emax"] - 6, 20)))
    return (rng.integers(-7, 8, (r, c)) * 2.0 ** s).astype(np.float32)


def wide_matrix(rng, f, r, c):
    """Random values over many binades, into the format's denormal range and beyond plane 0 of a 1/6/m operand
    (rows and columns of mixed magnitude: elements in the planes above and below, record lists in use)."""
    k = oracle.format_constants(f[0], f[1])
    lo = max(k["Emin"] - f[1] - 2, -60)
    e = rng.integers(lo, lo + 40, (r, c))
    e[rng.random((r, c)) < 0.9] = lo + 30
    return (rng.standard_normal((r, c)) * np.exp2(e.astype(np.float64))).astype(np.float32)


def gram_products(fmt, ops):
    """X X^T and X^T X from each (operand, transposed operand) pair."""
    out = []
    for op, op_t in ops:
        out.append(fmt.fmt_gemm_prepared(op, op))
        out.append(fmt.fmt_gemm_prepared(op_t, op_t))
    return out


@pytest.mark.parametrize("f", FORMATS)
def test_exact_matrices_bit_identical_to_the_oracle(fmt, f):
    rng = np.random.default_rng(300 + f[1])
    xs = [exact_matrix(rng, f, r, c) for r, c in SHAPES]
    ops = fmt.fmt_prepare_pair_batch([dev(x) for x in xs], f)
    got = gram_products(fmt, ops)
    torch.cuda.synchronize()
    for i, x in enumerate(xs):
        ref = oracle.gemm(x, x, f[0], f[1], f[2], transB=True)
        ref_t = oracle.gemm(x, x, f[0], f[1], f[2], transA=True)
        assert np.array_equal(got[2 * i].cpu().numpy(), ref), (i, x.shape)
        assert np.array_equal(got[2 * i + 1].cpu().numpy(), ref_t), (i, x.shape)


@pytest.mark.parametrize("f", FORMATS)
def test_wide_range_matrices_within_tolerance_and_equal_to_single_calls(fmt, f):
    rng = np.random.default_rng(400 + f[1])
    xs = [wide_matrix(rng, f, r, c) for r, c in SHAPES]
    dx = [dev(x) for x in xs]
    ops = fmt.fmt_prepare_pair_batch(dx, f)
    single = [fmt.fmt_prepare_pair(x, f) for x in dx]
    got, ref_gpu = gram_products(fmt, ops), gram_products(fmt, single)
    torch.cuda.synchronize()
    for i, (g, r) in enumerate(zip(got, ref_gpu)):
        assert torch.equal(g, r), i
    for i, x in enumerate(xs):
        ref = oracle.gemm(x, x, f[0], f[1], f[2], transB=True)
        ref_t = oracle.gemm(x, x, f[0], f[1], f[2], transA=True)
        assert rel_err(got[2 * i].cpu().numpy(), ref) <= TOL, (i, x.shape)
        assert rel_err(got[2 * i + 1].cpu().numpy(), ref_t) <= TOL, (i, x.shape)


@pytest.mark.parametrize("f", [(6, 9, True), (5, 10, True)])
def test_more_matrices_than_one_launch_holds_strided_and_unaligned(fmt, f):
    """40 matrices (a shared launch holds 16): views with a leading dimension beyond the columns and a base that
    is not 16-byte aligned among them; into caller-provided buffers."""
    rng = np.random.default_rng(77)
    xs, dx = [], []
    for i in range(40):
        r, c = int(rng.integers(1, 200)), int(rng.integers(1, 300))
        x = wide_matrix(rng, f, r, c)
        xs.append(x)
        if i % 3 == 1:
            pad = torch.zeros(r, c + 5, device="cuda")
            pad[:, 1:c + 1] = dev(x)
            dx.append(pad[:, 1:c + 1])
        else:
            dx.append(dev(x))
    outs = [torch.empty(fmt.fmt_operand_bytes(x.shape[0], x.shape[1], f) + 64, dtype=torch.uint8, device="cuda") for x in xs]
    outs_t = [torch.empty(fmt.fmt_operand_bytes(x.shape[1], x.shape[0], f), dtype=torch.uint8, device="cuda") for x in xs]
    ops = fmt.fmt_prepare_pair_batch(dx, f, outs=outs, outs_t=outs_t)
    assert all(op.buf is o and op_t.buf is ot for (op, op_t), o, ot in zip(ops, outs, outs_t))
    single = [fmt.fmt_prepare_pair(x, f) for x in dx]
    got, ref_gpu = gram_products(fmt, ops), gram_products(fmt, single)
    torch.cuda.synchronize()
    for i, (g, r) in enumerate(zip(got, ref_gpu)):
        assert torch.equal(g, r), i
    for i in (0, 1, 17, 39):
        x = xs[i]
        assert rel_err(got[2 * i].cpu().numpy(), oracle.gemm(x, x, f[0], f[1], f[2], transB=True)) <= TOL
        assert rel_err(got[2 * i + 1].cpu().numpy(), oracle.gemm(x, x, f[0], f[1], f[2], transA=True)) <= TOL


def test_second_call_into_the_same_buffers(fmt):
    """Operand buffers are reused from step to step: what an earlier call left in them (masks, record counts)
    must not show in the next one's operands."""
    f = (6, 9, True)
    rng = np.random.default_rng(5)
    xs1 = [wide_matrix(rng, f, 200, 300), wide_matrix(rng, f, 96, 512)]
    xs2 = [exact_matrix(rng, f, 200, 300), exact_matrix(rng, f, 96, 512)]
    ops = fmt.fmt_prepare_pair_batch([dev(x) for x in xs1], f)
    outs, outs_t = [o.buf for o, _ in ops], [t.buf for _, t in ops]
    ops2 = fmt.fmt_prepare_pair_batch([dev(x) for x in xs2], f, outs=outs, outs_t=outs_t)
    got = gram_products(fmt, ops2)
    torch.cuda.synchronize()
    for i, x in enumerate(xs2):
        assert np.array_equal(got[2 * i].cpu().numpy(), oracle.gemm(x, x, f[0], f[1], f[2], transB=True))
        assert np.array_equal(got[2 * i + 1].cpu().numpy(), oracle.gemm(x, x, f[0], f[1], f[2], transA=True))


def test_config4_tensors_one_call_same_products_as_single_calls(fmt):
    """The twelve tensors of configuration 4's layer (the benchmark's own: workloads.config4) prepared in one call;
    the twelve products on them equal, bit for bit, those on fmt_prepare_pair's operands (which the every-element
    test of fmt_gemm_prepared_batch checks against the oracle), and sampled elements are checked against the
    oracle's dot products directly."""
    import workloads
    f = (6, 9, True)
    cfg = workloads.config4()
    host = [t for L in cfg["layers"] for t in (L["X"], L["W"], L["dY"])]
    tens = [dev(t) for t in host]
    ops = fmt.fmt_prepare_pair_batch(tens, f)
    single = [fmt.fmt_prepare_pair(t, f) for t in tens]

    def products(o):
        A, B = [], []
        for i in range(0, len(o), 3):
            (X, Xt), (W, Wt), (D, Dt) = o[i], o[i + 1], o[i + 2]
            A += [X, D, Dt]
            B += [W, Wt, Xt]
        return fmt.fmt_gemm_prepared_batch(A, B)

    got, ref = products(ops), products(single)
    torch.cuda.synchronize()
    for i, (g, r) in enumerate(zip(got, ref)):
        assert torch.equal(g, r), i
    rng = np.random.default_rng(9)
    for li in range(len(cfg["layers"])):
        x, w, dy = host[3 * li], host[3 * li + 1], host[3 * li + 2]
        for (a, b), c in zip(((x, w), (dy, w.T), (dy.T, x.T)), got[3 * li:3 * li + 3]):
            M, N = c.shape
            ii, jj = rng.integers(0, M, 48), rng.integers(0, N, 48)
            qa = oracle.quantize(np.ascontiguousarray(a[ii]), f[0], f[1], f[2]).astype(np.float64)
            qb = oracle.quantize(np.ascontiguousarray(b[jj]), f[0], f[1], f[2]).astype(np.float64)
            want = np.sum(qa * qb, axis=1)
            have = c[torch.from_numpy(ii).cuda(), torch.from_numpy(jj).cuda()].cpu().numpy().astype(np.float64)
            scale = np.sqrt(np.sum(qa * qa, axis=1) * np.sum(qb * qb, axis=1))
            assert np.all(np.abs(have - want) <= 1e-5 * scale), li


def test_empty_and_argument_errors(fmt):
    f = (6, 9, True)
    assert fmt.fmt_prepare_pair_batch([], f) == []
    x = torch.randn(64, 96, device="cuda")
    y = torch.randn(32, 48, device="cuda")
    with pytest.raises(ValueError):
        fmt.fmt_prepare_pair_batch([x, y], f, outs=[None])
    big = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    with pytest.raises(fmt.FmtError) as e:                      # two matrices into one buffer
        fmt.fmt_prepare_pair_batch([x, y], f, outs=[big, big])
    assert e.value.status == -6
    with pytest.raises(fmt.FmtError) as e:                      # a buffer too small
        fmt.fmt_prepare_pair_batch([x, y], f, outs=[big, big[:256]])
    assert e.value.status == -3
    inside = big[4096:4096 + 32 * 48 * 4].view(torch.float32).view(32, 48)
    with pytest.raises(fmt.FmtError) as e:                      # an operand buffer over another matrix's input
        fmt.fmt_prepare_pair_batch([x, inside], f, outs=[big, None])
    assert e.value.status == -6
    torch.cuda.synchronize()
