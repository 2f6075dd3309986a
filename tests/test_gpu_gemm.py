"""GPU parity of fmt_gemm (through the C ABI) against the CPU oracle.

Tolerance: relative Frobenius error <= 1e-5 against the fp64-accumulated oracle; where every
partial sum is exactly representable in fp32 the results must be identical."""
import numpy as np
import pytest

import oracle
import workloads

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

TOL = 1e-5
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


def rel_fro(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref)
    return np.linalg.norm(got - ref) / den if den > 0 else np.linalg.norm(got)


def run(fmt, A, B, f, tA=False, tB=False):
    """A is M x K and B is K x N on the host; they are stored transposed when asked."""
    Ain = np.ascontiguousarray(A.T) if tA else A
    Bin = np.ascontiguousarray(B.T) if tB else B
    C = fmt.fmt_gemm(dev(Ain), dev(Bin), f, transA=tA, transB=tB)
    torch.cuda.synchronize()
    ref = oracle.gemm(Ain, Bin, f[0], f[1], f[2], transA=tA, transB=tB)
    return C.cpu().numpy(), ref


@pytest.mark.parametrize("tA,tB", LAYOUTS)
@pytest.mark.parametrize("e,m", [(5, 10), (6, 9), (8, 7), (7, 20), (4, 3)])
def test_exact_integer_case(fmt, e, m, tA, tB):
    """Small integers times powers of two: every partial sum is exact in fp32, so the GPU must equal
    the oracle bit for bit whatever its accumulation order.  Ragged in M, N and K."""
    rng = np.random.default_rng(3)
    M, N, K = 131, 67, 93
    Ai = rng.integers(-7, 8, (M, K))
    Bi = rng.integers(-7, 8, (K, N))
    lim = 2 if e == 4 else 6
    A = (Ai * np.exp2(rng.integers(-lim, lim + 1, (M, 1)))).astype(np.float32)
    B = (Bi * np.exp2(rng.integers(-lim, lim + 1, (1, N)))).astype(np.float32)
    got, ref = run(fmt, A, B, (e, m, True), tA, tB)
    assert np.array_equal(got, ref)


@pytest.mark.parametrize("tA,tB", LAYOUTS)
@pytest.mark.parametrize("e,m,d", VARIANTS)
def test_random_operands_all_layouts(fmt, e, m, d, tA, tB):
    rng = np.random.default_rng(100 * e + m)
    M, N, K = 200, 136, 300                  # two tiles each way with ragged edges, 10 k-blocks (last partial)
    A = (rng.standard_normal((M, K)) * 2.0 ** -10).astype(np.float32)
    B = (rng.standard_normal((K, N)) * 2.0 ** -10).astype(np.float32)
    got, ref = run(fmt, A, B, (e, m, d), tA, tB)
    assert rel_fro(got, ref) <= TOL
    # the operands really were rounded: an unrounded product is further away than the tolerance
    raw = A.astype(np.float64) @ B.astype(np.float64)
    assert rel_fro(raw, ref) > 10 * TOL or (e, m) == (8, 23)


@pytest.mark.parametrize("e,m,d", [(6, 9, True), (5, 10, False), (8, 7, True), (7, 16, True), (8, 23, True),
                                     (3, 12, False)])
def test_wide_range_operands(fmt, e, m, d):
    """Log-normal magnitudes straddling the format's denormal, underflow and normal ranges."""
    rng = np.random.default_rng(7 * e + m)
    c = oracle.format_constants(e, m)
    M, N, K = 96, 80, 160
    centre = max(c["Emin"], -40) + 2
    A = workloads.log2_normal((M, K), centre, min(5.0, (c["Emax"] - centre) / 6.0), 0.05, rng)
    B = workloads.log2_normal((K, N), -2, min(3.0, (c["Emax"] + 2) / 6.0), 0.05, rng)
    got, ref = run(fmt, A, B, (e, m, d), False, True)
    assert np.all(np.isfinite(ref))
    assert rel_fro(got, ref) <= TOL


@pytest.mark.parametrize("m", [9, 23])
def test_fp32_exponent_range_formats_wider_than_bfloat16(fmt, m):
    """1/8/m with m >= 8 (none of the paper's formats): bf16 pieces hold no bit below 2^-133, so an operand
    value is split exactly iff its lowest set bit is at 2^-133 or above.  Pinned: operands with all bits at or
    above 2^-133 give the oracle's product bit for bit (integer data, exact sums); operands that reach below
    lose less than 2^-133 each, so every output is within sum_k |b_k| * 2^-133 of the oracle's."""
    rng = np.random.default_rng(800 + m)
    M, N, K = 40, 24, 64
    bits = min(m + 1, 12)
    ints = rng.integers(-(1 << bits) + 1, 1 << bits, (M, K)).astype(np.float64)
    B = rng.integers(-3, 4, (K, N)).astype(np.float32)
    A = (ints * 2.0 ** -133).astype(np.float32)                  # every set bit at 2^-133 or above
    got, ref = run(fmt, A, B, (8, m, True), False, False)
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))
    A2 = (ints * 2.0 ** -(133 + bits - 2)).astype(np.float32)     # low bits below 2^-133 (fp32 denormals: exact inputs)
    got2, ref2 = run(fmt, A2, B, (8, m, True), False, False)
    bound = np.abs(B).sum(axis=0, dtype=np.float64)[None, :] * 2.0 ** -133
    assert np.all(np.abs(got2.astype(np.float64) - ref2.astype(np.float64)) <= bound)


@pytest.mark.parametrize("shape", [(1, 1, 1), (1, 7, 3), (5, 1, 40), (33, 31, 1), (128, 128, 32), (129, 127, 33),
                                   (256, 10, 1024), (10, 1024, 256), (64, 300, 17)])
def test_shapes(fmt, shape):
    M, N, K = shape
    rng = np.random.default_rng(M * 7 + N * 3 + K)
    A = rng.standard_normal((M, K)).astype(np.float32)
    B = rng.standard_normal((K, N)).astype(np.float32)
    for (tA, tB) in [(False, True), (False, False), (True, False)]:
        got, ref = run(fmt, A, B, (6, 9, True), tA, tB)
        assert rel_fro(got, ref) <= TOL, (shape, tA, tB)


def test_identity_and_outer_product_are_exact(fmt):
    rng = np.random.default_rng(11)
    A = workloads.log2_normal((70, 50), -14, 6, 0.05, rng)
    for (e, m, d) in [(5, 10, True), (6, 9, False), (8, 7, False)]:
        qa = oracle.quantize(A, e, m, d)
        Ain = np.where(np.isfinite(qa), A, 0).astype(np.float32)        # keep inf*0 out of this case
        got, ref = run(fmt, Ain, np.eye(50, dtype=np.float32), (e, m, d))
        assert np.array_equal(got, ref)
        assert np.array_equal(got, oracle.quantize(Ain, e, m, d))
    # K = 1: exact, unrounded products of two 10-bit significands
    a = workloads.log2_normal((40, 1), -3, 2, 0, rng)
    b = workloads.log2_normal((1, 45), -3, 2, 0, rng)
    got, ref = run(fmt, a, b, (6, 9, True))
    assert np.array_equal(got, ref)


def test_leading_dimensions_and_output_view(fmt):
    """Row strides larger than the row length on A, B and C; untouched padding in C."""
    rng = np.random.default_rng(12)
    M, N, K = 70, 45, 90
    Abig = rng.standard_normal((M, K + 11)).astype(np.float32)
    Bbig = rng.standard_normal((N, K + 5)).astype(np.float32)       # stored N x K (transB)
    Ad, Bd = dev(Abig), dev(Bbig)
    Cbig = torch.full((M, N + 9), -7.0, dtype=torch.float32, device="cuda")
    fmt.fmt_gemm(Ad[:, :K], Bd[:, :K], (6, 9, True), transB=True, out=Cbig[:, :N])
    torch.cuda.synchronize()
    ref = oracle.gemm(Abig[:, :K], Bbig[:, :K], 6, 9, True, transB=True)
    out = Cbig.cpu().numpy()
    assert rel_fro(out[:, :N], ref) <= TOL
    assert np.all(out[:, N:] == -7.0)


def test_k_zero_fills_zero_and_empty_succeeds(fmt):
    A = torch.empty((6, 0), dtype=torch.float32, device="cuda")
    B = torch.empty((0, 9), dtype=torch.float32, device="cuda")
    C = torch.full((6, 9), 3.0, dtype=torch.float32, device="cuda")
    fmt.fmt_gemm(A, B, (6, 9, True), out=C)
    torch.cuda.synchronize()
    assert float(C.abs().sum()) == 0.0
    C0 = fmt.fmt_gemm(torch.empty((0, 4), dtype=torch.float32, device="cuda"),
                      torch.empty((4, 5), dtype=torch.float32, device="cuda"), (6, 9, True))
    assert tuple(C0.shape) == (0, 5)


def test_nonfinite_operands_give_nonfinite_outputs_in_the_same_places(fmt):
    rng = np.random.default_rng(13)
    A = rng.standard_normal((40, 64)).astype(np.float32)
    B = rng.standard_normal((64, 40)).astype(np.float32)
    A[3, 5] = np.inf
    A[17, 60] = np.nan
    A[30, 2] = 1e30          # finite, but overflows binary16
    B[9, 21] = -np.inf
    got, ref = run(fmt, A, B, (5, 10, True))
    assert np.array_equal(np.isfinite(got), np.isfinite(ref))
    fin = np.isfinite(ref)
    assert rel_fro(got[fin], ref[fin]) <= TOL


def test_bf16_denormal_operands(fmt):
    """1/8/7/d keeps values below 2^-126 (bf16 denormals); their products with large values are
    ordinary numbers and must not be lost."""
    rng = np.random.default_rng(14)
    A = (rng.integers(1, 128, (64, 64)) * 2.0 ** -133).astype(np.float32)     # every bf16 denormal magnitude
    B = (rng.standard_normal((64, 64)) * 2.0 ** 100).astype(np.float32)
    got, ref = run(fmt, A, B, (8, 7, True))
    assert np.linalg.norm(ref) > 0
    assert rel_fro(got, ref) <= TOL
    got_n, ref_n = run(fmt, A, B, (8, 7, False))
    assert np.all(ref_n == 0) and np.all(got_n == 0)


def test_config1_gemm(fmt):
    cfg = workloads.config1()
    got, ref = run(fmt, cfg["A"], cfg["B"], (6, 9, True))
    assert rel_fro(got, ref) <= TOL


def test_config2_mlp_shapes(fmt):
    """All eight GEMMs of one forward+backward step of the 784-1024-1024-10 MLP at batch 256, on the
    tensors such a step produces (call-by-call parity on identical inputs)."""
    cfg = workloads.config2()
    f = (6, 9, True)
    X, W = cfg["X"], cfg["W"]
    acts = [X]
    for l in range(3):                                     # forward, NT
        A, B = acts[-1], W[l]
        C = fmt.fmt_gemm(dev(A), dev(B), f, transB=True)
        torch.cuda.synchronize()
        out = C.cpu().numpy()
        assert rel_fro(out, oracle.gemm(A, B, *f, transB=True)) <= TOL, ("fwd", l)
        acts.append(np.maximum(out, 0) if l < 2 else out)
    z = acts[-1].astype(np.float64)
    p = np.exp(z - z.max(1, keepdims=True))
    p /= p.sum(1, keepdims=True)
    p[np.arange(z.shape[0]), cfg["labels"]] -= 1.0
    dY = (p / z.shape[0] * cfg["loss_scale"]).astype(np.float32)
    for l in (2, 1, 0):
        Xl = acts[l]
        dW = fmt.fmt_gemm(dev(dY), dev(Xl), f, transA=True)           # wgrad, TN
        torch.cuda.synchronize()
        assert rel_fro(dW.cpu().numpy(), oracle.gemm(dY, Xl, *f, transA=True)) <= TOL, ("wgrad", l)
        if l > 0:
            dX = fmt.fmt_gemm(dev(dY), dev(W[l]), f)                   # dgrad, NN
            torch.cuda.synchronize()
            out = dX.cpu().numpy()
            assert rel_fro(out, oracle.gemm(dY, W[l], *f)) <= TOL, ("dgrad", l)
            dY = (out * (acts[l] > 0)).astype(np.float32)


def _block_samples(M, N, seed, block=64):
    """One output position in every block x block square of an M x N result (64 is the smallest
    workgroup tile, and every k part of a split feeds every output of its tile: no tile of any plan and
    no k part can be skipped), plus the corners."""
    rng = np.random.default_rng(seed)
    bi, bj = np.meshgrid(np.arange(0, M, block), np.arange(0, N, block), indexing="ij")
    rows = np.minimum(bi + rng.integers(0, block, bi.shape), M - 1).ravel()
    cols = np.minimum(bj + rng.integers(0, block, bj.shape), N - 1).ravel()
    return np.concatenate([rows, [0, 0, M - 1, M - 1]]), np.concatenate([cols, [0, N - 1, 0, N - 1]])


def _sampled_check(fmt, A, B, f, tA, tB, nsamp, seed):
    """Full-size product on the GPU; the oracle computes sampled outputs one by one: one in every
    64 x 64 block of the result.  Besides the relative Frobenius error over the samples, every sample is
    held against the size of the terms it sums (fp32 accumulation of K exact products errs by a few
    sqrt(K) 2^-24 of sum |a||b|), so a wrong tile cannot hide behind large neighbours."""
    Ad, Bd = dev(A), dev(B)
    C = fmt.fmt_gemm(Ad, Bd, f, transA=tA, transB=tB)
    torch.cuda.synchronize()
    M, N = C.shape
    rows, cols = _block_samples(M, N, seed)
    got = C[torch.from_numpy(rows).cuda(), torch.from_numpy(cols).cuda()].cpu().numpy()
    ref = oracle.gemm_sampled(A, B, rows, cols, f[0], f[1], f[2], transA=tA, transB=tB)
    terms = oracle.gemm_sampled(np.abs(A), np.abs(B), rows, cols, f[0], f[1], f[2], transA=tA, transB=tB).astype(np.float64)
    K = A.shape[0] if tA else A.shape[1]
    ok = np.isfinite(ref)
    err = np.abs(got.astype(np.float64)[ok] - ref.astype(np.float64)[ok])
    assert np.all(err <= 16 * np.sqrt(K) * 2.0 ** -24 * terms[ok] + 1e-45), (f, tA, tB, int(np.argmax(err / (terms[ok] + 1e-300))))
    assert np.array_equal(np.isfinite(got), ok)
    return rel_fro(got[ok], ref[ok]), C


def test_config3_conv_im2col_full_size(fmt):
    """ResNet-style 3x3 conv as im2col GEMM at batch 64: fwd (NT), dgrad (NN), wgrad (TN) in all six
    variants at full size (M=12544, N=256, K=2304 and permutations); sampled outputs vs the oracle."""
    cfg = workloads.config3()
    Xcol = workloads.im2col_3x3(cfg["X"])                  # 12544 x 2304
    W, dY = cfg["W"], cfg["dY"]
    assert Xcol.shape == (12544, 2304) and W.shape == (256, 2304) and dY.shape == (12544, 256)
    for f in VARIANTS:
        e1, _ = _sampled_check(fmt, Xcol, W, f, False, True, 1500, 1)       # Y = Xcol W^T
        e2, _ = _sampled_check(fmt, dY, W, f, False, False, 1500, 2)        # dXcol = dY W
        e3, _ = _sampled_check(fmt, dY, Xcol, f, True, False, 1500, 3)      # dW = dY^T Xcol
        assert e1 <= TOL and e2 <= TOL and e3 <= TOL, (f, e1, e2, e3)


def test_config4_bert_layer_full_size(fmt):
    """BERT-Large-shaped encoder GEMMs at 4096 tokens, 1/6/9: fwd, dgrad, wgrad of the four linear
    layers; sampled outputs vs the oracle."""
    cfg = workloads.config4()
    f = (6, 9, True)
    for layer in cfg["layers"]:
        X, W, dY = layer["X"], layer["W"], layer["dY"]
        e1, _ = _sampled_check(fmt, X, W, f, False, True, 1000, 4)
        e2, _ = _sampled_check(fmt, dY, W, f, False, False, 1000, 5)
        e3, _ = _sampled_check(fmt, dY, X, f, True, False, 1000, 6)
        assert e1 <= TOL and e2 <= TOL and e3 <= TOL, (layer["name"], e1, e2, e3)


@pytest.mark.parametrize("plan", ["1,1,1", "1,1,3", "2,2,1,0", "2,2,1,1", "2,2,4", "2,4,1", "2,4,2", "4,2,1", "4,2,3",
                                  "4,4,1,0", "4,4,1,1", "4,4,2"])
def test_every_tile_shape_and_split(fmt, plan, monkeypatch):
    """The product kernel's tile shapes, issue-order variants and k splits, forced through the tuning
    override, on a shape with ragged tiles in M, N and K (K spans several splits)."""
    monkeypatch.setenv("FMT_GEMM_PLAN", plan)
    rng = np.random.default_rng(21)
    M, N, K = 300, 270, 1100
    A = (rng.standard_normal((M, K)) * 2.0 ** -6).astype(np.float32)
    B = (rng.standard_normal((K, N)) * 2.0 ** -6).astype(np.float32)
    for f in [(6, 9, True), (8, 7, False), (7, 18, True)]:
        for (tA, tB) in [(False, True), (True, False)]:
            got, ref = run(fmt, A, B, f, tA, tB)
            assert rel_fro(got, ref) <= TOL, (plan, f, tA, tB)
    # exact case: bit-identical whatever the tile or the split
    Ai = rng.integers(-7, 8, (M, K)).astype(np.float32)
    Bi = rng.integers(-7, 8, (K, N)).astype(np.float32)
    got, ref = run(fmt, Ai, Bi, (6, 9, True))
    assert np.array_equal(got, ref)


@pytest.mark.parametrize("plan", ["1,1,1", "2,2,1", "4,4,1", "4,2,1", "2,2,2"])
@pytest.mark.parametrize("f", [(5, 10, True), (6, 9, True), (7, 18, True)])
def test_every_depth_of_the_stage_ring(fmt, plan, f, monkeypatch):
    """k from 1 to 21 blocks of 16: the product kernel's ring of stage buffers runs through every
    number of whole turns and left-over trips, for one, two and three pieces per operand.  Integer
    operands: the result is exact, so it must equal the oracle's bit for bit."""
    monkeypatch.setenv("FMT_GEMM_PLAN", plan)
    monkeypatch.setenv("FMT_GEMM_WINDOW", "0")
    rng = np.random.default_rng(77)
    M, N = 150, 140
    for kb in range(1, 22):
        K = 16 * kb - (3 if kb % 4 == 0 else 0)                      # some depths with a ragged last block
        A = rng.integers(-7, 8, (M, K)).astype(np.float32)
        B = rng.integers(-7, 8, (K, N)).astype(np.float32)
        got, ref = run(fmt, A, B, f, False, kb % 2 == 1)
        assert np.array_equal(got, ref), (plan, f, K)


def test_every_depth_of_the_stage_ring_scaled_piece(fmt, monkeypatch):
    """The same through the single scaled fp16 piece of the 1/6/m formats."""
    monkeypatch.setenv("FMT_GEMM_WINDOW", "1")
    rng = np.random.default_rng(78)
    M, N = 150, 140
    for plan in ["2,2,1", "4,4,1", "1,1,2"]:
        monkeypatch.setenv("FMT_GEMM_PLAN", plan)
        for kb in range(1, 22):
            K = 16 * kb - (5 if kb % 3 == 0 else 0)
            A = (rng.integers(-7, 8, (M, K)) * 2.0 ** -12).astype(np.float32)
            B = rng.integers(-7, 8, (K, N)).astype(np.float32)
            got, ref = run(fmt, A, B, (6, 9, True), kb % 2 == 0, False)
            assert np.array_equal(got, ref), (plan, K)


def test_binary16_denormal_operands(fmt):
    """1/5/10/d operands below 2^-14 (binary16 denormals) times large values: nothing may be
    flushed on the way through the fp16 matrix path; products are small integers times powers of
    two, so the result is exact."""
    rng = np.random.default_rng(15)
    A = (rng.integers(-1023, 1024, (70, 64)) * 2.0 ** -24).astype(np.float32)     # all binary16 denormals
    B = (rng.integers(-3, 4, (64, 50)) * 2.0 ** 13).astype(np.float32)
    got, ref = run(fmt, A, B, (5, 10, True))
    assert np.linalg.norm(ref) > 0
    assert np.array_equal(got, ref)
    got_n, ref_n = run(fmt, A, B, (5, 10, False))
    assert np.all(ref_n == 0) and np.all(got_n == 0)
    # every binary16 value once, against the identity: the fp16 piece conversion is exact
    from fmtdef import decode_codes
    v = decode_codes(5, 10)
    v = v[np.isfinite(v)].reshape(-1, 64)[:960]
    got, ref = run(fmt, v, np.eye(64, dtype=np.float32), (5, 10, True))
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))


def _device_operand(rows, cols, seed, scale=1.0):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    return torch.randn((rows, cols), device="cuda", generator=g) * scale


@pytest.mark.parametrize("f", [(6, 9, True), (8, 7, True)])
@pytest.mark.parametrize("tA", [False, True])
def test_operand_of_more_than_2_to_the_32_elements(fmt, f, tA):
    """op(A) is (2^22 + 70) x 1024 (16 GiB, element offsets beyond 32 bits) in both storage orders, B is
    1024 x 16; operands are drawn on the device and the oracle computes sampled rows of the result from
    the same values (first and last rows, rows around the 2^31- and 2^32-element offsets, random rows)."""
    M, K, N = (1 << 22) + 70, 1024, 16
    A = _device_operand(K, M, 21) if tA else _device_operand(M, K, 21)
    B = _device_operand(K, N, 22, 0.05)
    C = fmt.fmt_gemm(A, B, f, transA=tA)
    torch.cuda.synchronize()
    rng = np.random.default_rng(5)
    edge = [(1 << 31) // K, (1 << 32) // K]
    rows = np.unique(np.concatenate([np.arange(40), np.arange(M - 80, M), rng.integers(0, M, 300)] +
                                    [np.arange(r - 20, r + 20) for r in edge]))
    rows_d = torch.from_numpy(rows).cuda()
    A_rows = (A[:, rows_d].T if tA else A[rows_d]).contiguous().cpu().numpy()
    ref = oracle.gemm(A_rows, B.cpu().numpy(), *f)
    got = C[rows_d].cpu().numpy()
    assert rel_fro(got, ref) <= TOL
    # per sampled row as well: a misplaced row would hide in the norm of 500 good ones
    err = np.linalg.norm(got.astype(np.float64) - ref, axis=1) / np.linalg.norm(ref.astype(np.float64), axis=1)
    assert err.max() <= 1e-4, (rows[err.argmax()], err.max())
    assert bool(torch.isfinite(C).all())


def test_result_of_more_than_2_to_the_32_elements(fmt):
    """C is 65600 x 65600 (16 GiB) with K = 64: output offsets beyond 32 bits.  Sampled outputs against the
    oracle, around the rows where the offset passes 2^31 and 2^32 elements and at the far corner."""
    M = N = 65600
    K = 64
    f = (6, 9, True)
    A = _device_operand(M, K, 31)
    B = _device_operand(N, K, 32, 0.05)
    C = fmt.fmt_gemm(A, B, f, transB=True)
    torch.cuda.synchronize()
    rng = np.random.default_rng(6)
    edge = [(1 << 31) // N, (1 << 32) // N]
    rows = np.unique(np.concatenate([np.arange(8), np.arange(M - 8, M), rng.integers(0, M, 40)] +
                                    [np.arange(r - 2, r + 3) for r in edge]))
    cols = np.unique(np.concatenate([np.arange(8), np.arange(N - 8, N), rng.integers(0, N, 100)]))
    rows_d, cols_d = torch.from_numpy(rows).cuda(), torch.from_numpy(cols).cuda()
    ref = oracle.gemm(A[rows_d].cpu().numpy(), B[cols_d].cpu().numpy(), *f, transB=True)
    got = C[rows_d][:, cols_d].cpu().numpy()
    assert rel_fro(got, ref) <= TOL
    err = np.abs(got.astype(np.float64) - ref) / (np.abs(ref) + 1e-3 * np.abs(ref).mean())
    assert err.max() <= 1e-3, err.max()


@pytest.mark.parametrize("seed", range(48))
def test_seeded_random_cases(fmt, seed, monkeypatch):
    """Shapes, storage orders, leading dimensions, formats (any 2 <= e <= 8, 1 <= m <= 23, d or n), value
    scales and the piece scheme drawn from a seeded generator: each case against the oracle.  The value
    scale keeps the results finite in the format's range; cases with an even seed use small integers times
    row / column powers of two and must match bit for bit."""
    rng = np.random.default_rng(1000 + seed)
    e, m, d = int(rng.integers(2, 9)), int(rng.integers(1, 24)), bool(rng.integers(0, 2))
    M, N, K = (int(v) for v in rng.integers(1, 321, 3))
    tA, tB = bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
    if e == 6 and 8 <= m <= 10:
        monkeypatch.setenv("FMT_GEMM_WINDOW", str(int(rng.integers(0, 2))))
    c = oracle.format_constants(e, m)
    span = int(min(c["Emax"], 20))
    if seed % 2 == 0:
        lim = max(span - 4, 0) // 2
        A = (rng.integers(-3, 4, (M, K)) * np.exp2(rng.integers(-lim, lim + 1, (M, 1)))).astype(np.float32)
        B = (rng.integers(-3, 4, (K, N)) * np.exp2(rng.integers(-lim, lim + 1, (1, N)))).astype(np.float32)
    else:
        A = (rng.standard_normal((M, K)) * 2.0 ** float(rng.uniform(-span / 2, 0))).astype(np.float32)
        B = (rng.standard_normal((K, N)) * 2.0 ** float(rng.uniform(-span / 2, 0))).astype(np.float32)
    As, Bs = (A.T if tA else A), (B.T if tB else B)
    pa, pb, pc = (int(v) for v in rng.integers(0, 6, 3))                # extra leading-dimension padding
    Ad = torch.full((As.shape[0], As.shape[1] + pa), 7.0, device="cuda")
    Bd = torch.full((Bs.shape[0], Bs.shape[1] + pb), 7.0, device="cuda")
    Cd = torch.full((M, N + pc), -3.0, device="cuda")
    Ad[:, :As.shape[1]] = dev(As)
    Bd[:, :Bs.shape[1]] = dev(Bs)
    fmt.fmt_gemm(Ad[:, :As.shape[1]], Bd[:, :Bs.shape[1]], (e, m, d), transA=tA, transB=tB, out=Cd[:, :N])
    torch.cuda.synchronize()
    ref = oracle.gemm(np.ascontiguousarray(As), np.ascontiguousarray(Bs), e, m, d, transA=tA, transB=tB)
    got = Cd.cpu().numpy()
    what = "seed %d: 1/%d/%d/%s %dx%dx%d tA=%s tB=%s" % (seed, e, m, "d" if d else "n", M, N, K, tA, tB)
    assert np.all(got[:, N:] == -3.0), what + ": wrote outside the result"
    assert np.all(np.isfinite(ref)), what
    if seed % 2 == 0:
        assert np.array_equal(got[:, :N], ref), what
    else:
        assert rel_fro(got[:, :N], ref) <= TOL, what
