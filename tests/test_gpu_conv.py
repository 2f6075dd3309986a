"""GPU parity of fmt_conv2d_fwd / _dgrad / _wgrad (convolutions of Sec. IV-A on rounded operands,
patches gathered on the fly) against the CPU oracle's plain definitions: bit for bit where every
partial sum is exact in fp32, within the GEMM tolerance (1e-5 relative Frobenius) otherwise."""
import numpy as np
import pytest

import oracle
import workloads

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

TOL = 1e-5
VARIANTS = [(5, 10, True), (5, 10, False), (6, 9, True), (6, 9, False), (8, 7, True), (8, 7, False)]
GEOMS = [  # N, C, H, W, K, R, S, pad, stride
    (2, 3, 7, 6, 4, 3, 3, (1, 1), (1, 1)),
    (1, 2, 9, 8, 3, 3, 3, (1, 1), (2, 2)),
    (2, 4, 6, 6, 5, 1, 1, (0, 0), (1, 1)),
    (1, 3, 8, 9, 2, 5, 3, (2, 1), (1, 2)),
    (3, 2, 5, 5, 3, 2, 2, (0, 0), (1, 1)),
    (1, 1, 10, 7, 2, 3, 3, (0, 2), (3, 1)),
    (2, 40, 14, 14, 70, 3, 3, (1, 1), (1, 1)),       # several tiles and k-blocks, ragged everywhere
    (3, 33, 15, 13, 65, 3, 3, (1, 1), (2, 2)),
    # channel counts that are multiples of 32: forward and (stride 1) dgrad gather inside the product kernel
    (2, 32, 9, 8, 64, 3, 3, (1, 1), (1, 1)),
    (1, 64, 7, 7, 32, 3, 3, (1, 1), (2, 2)),          # forward in-kernel, dgrad through the gathered operand
    (2, 96, 6, 5, 32, 1, 1, (0, 0), (1, 1)),
    (1, 32, 8, 9, 96, 5, 3, (2, 1), (1, 1)),
    (3, 64, 5, 11, 160, 2, 4, (0, 3), (1, 1)),        # even taps, pad wider than the filter reaches on one side
    (5, 32, 12, 12, 40, 3, 3, (2, 2), (1, 2)),        # only forward qualifies (40 filters)
]


@pytest.fixture(scope="module")
def fmt():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    import paper_2103_15940_amd as lib
    return lib


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def rel_err(got, ref):
    return float(np.linalg.norm(got.astype(np.float64) - ref.astype(np.float64)) /
                 max(np.linalg.norm(ref.astype(np.float64)), 1e-300))


def run_all(fmt, X, W, dY, f, pad, stride):
    Y = fmt.fmt_conv2d_fwd(dev(X), dev(W), f, pad=pad, stride=stride)
    dX = fmt.fmt_conv2d_dgrad(dev(dY), dev(W), X.shape, f, pad=pad, stride=stride)
    dW = fmt.fmt_conv2d_wgrad(dev(dY), dev(X), W.shape, f, pad=pad, stride=stride)
    torch.cuda.synchronize()
    return Y.cpu().numpy(), dX.cpu().numpy(), dW.cpu().numpy()


def oracle_all(X, W, dY, f, pad, stride):
    e, m, d = f
    return (oracle.conv2d_fwd(X, W, e, m, d, pad, stride), oracle.conv2d_dgrad(dY, W, X.shape, e, m, d, pad, stride),
            oracle.conv2d_wgrad(dY, X, W.shape, e, m, d, pad, stride))


@pytest.mark.parametrize("geom", GEOMS)
@pytest.mark.parametrize("f", [(6, 9, True), (5, 10, False), (8, 7, True)])
def test_bit_exact_integer_data(fmt, geom, f):
    """Small integers times powers of two: every partial sum is exact in fp32 in any order."""
    n, c, h, w, k, r, s, pad, stride = geom
    rng = np.random.default_rng(n + 10 * c + 100 * h)
    X = (rng.integers(-4, 5, (n, c, h, w)) * 0.5).astype(np.float32)
    W = (rng.integers(-4, 5, (k, c, r, s)) * 0.25).astype(np.float32)
    P, Q = oracle.conv_out_size(h, w, r, s, pad, stride)
    dY = (rng.integers(-4, 5, (n, k, P, Q)) * 2.0 ** -6).astype(np.float32)
    got = run_all(fmt, X, W, dY, f, pad, stride)
    want = oracle_all(X, W, dY, f, pad, stride)
    for name, g_, w_ in zip(("Y", "dX", "dW"), got, want):
        assert g_.shape == w_.shape
        assert np.array_equal(g_.view(np.uint32), w_.view(np.uint32)), "%s differs for %r" % (name, geom)


@pytest.mark.parametrize("geom", GEOMS)
@pytest.mark.parametrize("f", VARIANTS)
def test_real_data_within_tolerance(fmt, geom, f):
    n, c, h, w, k, r, s, pad, stride = geom
    rng = np.random.default_rng(7 * n + c + f[0])
    X = np.maximum(rng.standard_normal((n, c, h, w)), 0).astype(np.float32)         # ReLU activations
    W = (rng.standard_normal((k, c, r, s)) * np.sqrt(2.0 / (c * r * s))).astype(np.float32)
    P, Q = oracle.conv_out_size(h, w, r, s, pad, stride)
    dY = workloads.log2_normal((n, k, P, Q), -12.0, 3.0, 0.0, rng)
    got = run_all(fmt, X, W, dY, f, pad, stride)
    want = oracle_all(X, W, dY, f, pad, stride)
    for name, g_, w_ in zip(("Y", "dX", "dW"), got, want):
        assert rel_err(g_, w_) <= TOL, "%s: %.3g for %r" % (name, rel_err(g_, w_), geom)


def test_operands_are_rounded(fmt):
    """The convolution of unrounded operands differs; the convolution of pre-rounded operands agrees."""
    rng = np.random.default_rng(8)
    X = rng.standard_normal((2, 8, 10, 10)).astype(np.float32)
    W = rng.standard_normal((6, 8, 3, 3)).astype(np.float32)
    f = (5, 10, True)
    Y = fmt.fmt_conv2d_fwd(dev(X), dev(W), f).cpu().numpy()
    Yq = fmt.fmt_conv2d_fwd(dev(oracle.quantize(X, *f)), dev(oracle.quantize(W, *f)), f).cpu().numpy()
    Y32 = torch.nn.functional.conv2d(torch.from_numpy(X).double(), torch.from_numpy(W).double(), padding=1).numpy()
    assert np.array_equal(Y, Yq)
    assert rel_err(Y, Y32) > 1e-4


def test_empty_and_degenerate(fmt):
    f = (6, 9, True)
    cuda = torch.device("cuda")
    # no images / no filters: empty outputs
    Y = fmt.fmt_conv2d_fwd(torch.empty((0, 3, 5, 5), device=cuda), torch.empty((4, 3, 3, 3), device=cuda), f)
    assert tuple(Y.shape) == (0, 4, 5, 5)
    Y = fmt.fmt_conv2d_fwd(torch.empty((2, 3, 5, 5), device=cuda), torch.empty((0, 3, 3, 3), device=cuda), f)
    assert tuple(Y.shape) == (2, 0, 5, 5)
    # no input channels: an empty sum, zeros
    Y = fmt.fmt_conv2d_fwd(torch.empty((2, 0, 5, 5), device=cuda), torch.empty((4, 0, 3, 3), device=cuda), f,
                           out=torch.full((2, 4, 5, 5), 7.0, device=cuda))
    torch.cuda.synchronize()
    assert float(Y.abs().sum()) == 0.0
    # wgrad over an empty batch: zeros
    dW = fmt.fmt_conv2d_wgrad(torch.empty((0, 4, 5, 5), device=cuda), torch.empty((0, 3, 5, 5), device=cuda), (4, 3, 3, 3), f,
                              out=torch.full((4, 3, 3, 3), 7.0, device=cuda))
    torch.cuda.synchronize()
    assert float(dW.abs().sum()) == 0.0
    # a filter as large as the padded image: one output position
    rng = np.random.default_rng(0)
    X = rng.integers(-3, 4, (1, 2, 3, 3)).astype(np.float32)
    W = rng.integers(-3, 4, (2, 2, 5, 5)).astype(np.float32)
    Y = fmt.fmt_conv2d_fwd(dev(X), dev(W), f, pad=1).cpu().numpy()
    assert Y.shape == (1, 2, 1, 1)
    assert np.array_equal(Y, oracle.conv2d_fwd(X, W, 6, 9, True, (1, 1), (1, 1)))


@pytest.mark.parametrize("f", [(6, 9, True), (5, 10, True), (8, 7, False)])
def test_config3_full_size_sampled(fmt, f):
    """ResNet-style 3x3 convolution of config 3 (batch 64, 256 -> 256 channels, 14 x 14), forward,
    dgrad and wgrad at full size: sampled outputs against the oracle -- one in every 64 x 64 block of
    the underlying product (rows: filters or channels; columns: positions or taps), the smallest tile
    the product kernel has, so that no tile and no k part can be skipped, plus 2000 random ones --
    error measured against the norm of the sampled reference values."""
    cfg = workloads.config3()
    X, W2, dY2 = cfg["X"], cfg["W"], cfg["dY"]
    n, c, h, w = X.shape
    k = W2.shape[0]
    W = W2.reshape(k, c, 3, 3)
    dY = np.ascontiguousarray(dY2.reshape(n, h, w, k).transpose(0, 3, 1, 2))        # the same values as NCHW
    Y, dX, dW = run_all(fmt, X, W, dY, f, (1, 1), (1, 1))
    e, m, d = f
    rng = np.random.default_rng(33)
    def blocks(rows, cols, to_flat):
        bi, bj = np.meshgrid(np.arange(0, rows, 64), np.arange(0, cols, 64), indexing="ij")
        r = np.minimum(bi + rng.integers(0, 64, bi.shape), rows - 1).ravel()
        q = np.minimum(bj + rng.integers(0, 64, bj.shape), cols - 1).ravel()
        return to_flat(r, q)
    hw = h * w
    nchw = lambda chans: (lambda r, q: ((q // hw) * chans + r) * hw + q % hw)       # row = channel, column = (image, position)
    for name, got, ref_fn, pinned in (
            ("Y", Y, lambda s: oracle.conv2d_fwd(X, W, e, m, d, sample=s), blocks(k, n * hw, nchw(k))),
            ("dX", dX, lambda s: oracle.conv2d_dgrad(dY, W, X.shape, e, m, d, sample=s), blocks(c, n * hw, nchw(c))),
            ("dW", dW, lambda s: oracle.conv2d_wgrad(dY, X, W.shape, e, m, d, sample=s), blocks(k, c * 9, lambda r, q: r * c * 9 + q))):
        idx = np.concatenate([pinned, rng.integers(0, got.size, 2000)])
        ref = ref_fn(idx)
        assert np.all(np.isfinite(got))
        assert rel_err(got.ravel()[idx], ref) <= TOL, "%s: %.3g" % (name, rel_err(got.ravel()[idx], ref))


def test_equals_im2col_product_config3_shape(fmt):
    """Forward (patches gathered inside the product kernel, k running tap-major) against fmt_gemm on the
    materialised patch matrix (k running channel-major): the same rounded operands and exact products,
    summed in fp32 in two different orders of the K = 576 terms.  Each order is within about
    sqrt(K) * 2^-24 = 1.4e-6 of the exact sum relative to the Frobenius norm, typically a tenth of that."""
    rng = np.random.default_rng(12)
    X = np.maximum(rng.standard_normal((4, 64, 14, 14)), 0).astype(np.float32)
    W = (rng.standard_normal((96, 64, 3, 3)) * 0.05).astype(np.float32)
    f = (6, 9, True)
    Y = fmt.fmt_conv2d_fwd(dev(X), dev(W), f).cpu().numpy()
    Xcol = workloads.im2col_3x3(X)
    Y2 = fmt.fmt_gemm(dev(Xcol), dev(W.reshape(96, -1)), f, transB=True).cpu().numpy()    # [n*h*w, k]
    Y2 = Y2.reshape(4, 14, 14, 96).transpose(0, 3, 1, 2)
    assert rel_err(Y, Y2) <= 1e-6


@pytest.mark.parametrize("seed", range(36))
def test_seeded_random_geometries(fmt, seed):
    """Batch, channels, image and filter size (filters up to 7 x 6: more than 32 taps included), padding
    (also wider than the filter), stride and format drawn from a seeded generator; exact data, so
    forward, dgrad and wgrad must match the oracle bit for bit."""
    rng = np.random.default_rng(9000 + seed)
    n, c, k = int(rng.integers(1, 4)), int(rng.integers(1, 41)), int(rng.integers(1, 41))
    h, w = int(rng.integers(1, 18)), int(rng.integers(1, 18))
    pad = (int(rng.integers(0, 4)), int(rng.integers(0, 4)))
    r = int(rng.integers(1, min(7, h + 2 * pad[0]) + 1))
    s = int(rng.integers(1, min(6, w + 2 * pad[1]) + 1))
    stride = (int(rng.integers(1, 4)), int(rng.integers(1, 4)))
    f = [(6, 9, True), (5, 10, False), (8, 7, True), (6, 9, False), (7, 12, True), (4, 3, True)][seed % 6]
    X = (rng.integers(-3, 4, (n, c, h, w)) * 0.5).astype(np.float32)
    W = (rng.integers(-3, 4, (k, c, r, s)) * 0.25).astype(np.float32)
    P, Q = oracle.conv_out_size(h, w, r, s, pad, stride)
    dY = (rng.integers(-3, 4, (n, k, P, Q)) * 2.0 ** -3).astype(np.float32)
    got = run_all(fmt, X, W, dY, f, pad, stride)
    want = oracle_all(X, W, dY, f, pad, stride)
    what = "seed %d: n=%d c=%d k=%d %dx%d filter %dx%d pad %r stride %r 1/%d/%d" % (seed, n, c, k, h, w, r, s, pad, stride, f[0], f[1])
    for name, g_, w_ in zip(("Y", "dX", "dW"), got, want):
        assert g_.shape == w_.shape, what
        assert np.all(np.isfinite(w_)), what
        assert np.array_equal(g_.view(np.uint32), w_.view(np.uint32)), "%s differs, %s" % (name, what)


@pytest.mark.parametrize("seed", range(30))
def test_seeded_random_geometries_with_channel_multiples_of_32(fmt, seed):
    """The same draw with channel and filter counts from {32, 64, 96, 128} and at most 32 taps, so that forward
    (any stride) and dgrad (stride 1, every third seed at least) gather their patches inside the product kernel:
    images of several sizes incl. one pixel, padding wider than the filter, strides, six formats (one, two and
    three 16-bit pieces); exact data, bit for bit against the oracle."""
    rng = np.random.default_rng(9500 + seed)
    n = int(rng.integers(1, 4))
    c, k = int(rng.choice([32, 64, 96, 128])), int(rng.choice([32, 64, 96, 128]))
    h, w = int(rng.integers(1, 16)), int(rng.integers(1, 16))
    pad = (int(rng.integers(0, 4)), int(rng.integers(0, 4)))
    r = int(rng.integers(1, min(5, h + 2 * pad[0]) + 1))
    s = int(rng.integers(1, min(6, w + 2 * pad[1]) + 1))
    stride = (1, 1) if seed % 3 == 0 else (int(rng.integers(1, 4)), int(rng.integers(1, 4)))
    f = [(6, 9, True), (5, 10, False), (8, 7, True), (6, 9, False), (7, 20, True), (4, 3, True)][seed % 6]
    X = (rng.integers(-3, 4, (n, c, h, w)) * 0.5).astype(np.float32)
    W = (rng.integers(-3, 4, (k, c, r, s)) * 0.25).astype(np.float32)
    P, Q = oracle.conv_out_size(h, w, r, s, pad, stride)
    dY = (rng.integers(-3, 4, (n, k, P, Q)) * 2.0 ** -3).astype(np.float32)
    got = run_all(fmt, X, W, dY, f, pad, stride)
    want = oracle_all(X, W, dY, f, pad, stride)
    what = "seed %d: n=%d c=%d k=%d %dx%d filter %dx%d pad %r stride %r 1/%d/%d" % (seed, n, c, k, h, w, r, s, pad, stride, f[0], f[1])
    for name, g_, w_ in zip(("Y", "dX", "dW"), got, want):
        assert g_.shape == w_.shape, what
        assert np.all(np.isfinite(w_)), what
        assert np.array_equal(g_.view(np.uint32), w_.view(np.uint32)), "%s differs, %s" % (name, what)


def test_in_kernel_gather_equals_gathered_operand(fmt, monkeypatch):
    """Forward and dgrad with the patches gathered inside the product kernel give, on data whose partial sums
    are exact, the same bits as the route through a gathered operand (FMT_CONV_IMPLICIT=0), and within the
    tolerance on real data; both routes are held to the oracle by the tests above."""
    n, c, h, w, k, r, s, pad, stride = 2, 64, 10, 9, 96, 3, 3, (1, 1), (1, 1)
    rng = np.random.default_rng(11)
    f = (6, 9, True)
    for exact in (True, False):
        if exact:
            X = (rng.integers(-4, 5, (n, c, h, w)) * 0.5).astype(np.float32)
            W = (rng.integers(-4, 5, (k, c, r, s)) * 0.25).astype(np.float32)
            dY = (rng.integers(-4, 5, (n, k, h, w)) * 2.0 ** -6).astype(np.float32)
        else:
            X = rng.standard_normal((n, c, h, w)).astype(np.float32)
            W = (rng.standard_normal((k, c, r, s)) * 0.05).astype(np.float32)
            dY = (rng.standard_normal((n, k, h, w)) * 1e-3).astype(np.float32)
        monkeypatch.delenv("FMT_CONV_IMPLICIT", raising=False)
        a = run_all(fmt, X, W, dY, f, pad, stride)
        monkeypatch.setenv("FMT_CONV_IMPLICIT", "0")
        b = run_all(fmt, X, W, dY, f, pad, stride)
        monkeypatch.delenv("FMT_CONV_IMPLICIT", raising=False)
        for name, g_, w_ in zip(("Y", "dX", "dW"), a, b):
            if exact:
                assert np.array_equal(g_.view(np.uint32), w_.view(np.uint32)), name
            else:
                assert rel_err(g_, w_) <= TOL, name


def test_scratch_of_forward_and_dgrad_is_of_the_size_of_the_tensor(fmt):
    """With the patches gathered inside the product kernel, forward and dgrad hold the rounded tensor (two
    bytes per element and 16-bit piece: 4 B for 1/6/9), the prepared filter and, when k is split, partial sums
    in scratch -- nothing of the size of the patch matrix (R*S times the tensor).  wgrad still prepares a
    patch-sized operand, which the last assertion records."""
    n, c, h, w, k, r, s = 8, 64, 28, 28, 64, 3, 3
    rng = np.random.default_rng(5)
    X = dev(rng.standard_normal((n, c, h, w)).astype(np.float32))
    W = dev((rng.standard_normal((k, c, r, s)) * 0.05).astype(np.float32))
    dY = dev((rng.standard_normal((n, k, h, w)) * 1e-3).astype(np.float32))
    f = (6, 9, True)
    tensor = n * c * h * w
    patch_operand = tensor * r * s * 4                      # what a gathered operand of two 16-bit pieces takes
    filt = 256 * c * r * s * 4                              # the filter operand, rows padded to 256
    slabs = 8 * k * n * h * w * 4                           # generous room for split-k partial sums
    torch.cuda.synchronize()
    fmt.fmt_release_scratch()
    fmt.fmt_conv2d_fwd(X, W, f, pad=(1, 1))
    torch.cuda.synchronize()
    fwd = fmt.fmt_scratch_bytes()["products"]
    assert 4 * tensor <= fwd <= 4 * tensor + filt + slabs + 65536
    assert fwd < patch_operand / 2
    fmt.fmt_release_scratch()
    fmt.fmt_conv2d_dgrad(dY, W, (n, c, h, w), f, pad=(1, 1))
    torch.cuda.synchronize()
    dgrad = fmt.fmt_scratch_bytes()["products"]
    assert 4 * tensor <= dgrad <= 4 * tensor + filt + slabs + 65536
    assert dgrad < patch_operand / 2
    fmt.fmt_release_scratch()
    fmt.fmt_conv2d_wgrad(dY, X, (k, c, r, s), f, pad=(1, 1))
    torch.cuda.synchronize()
    assert fmt.fmt_scratch_bytes()["products"] >= patch_operand
    fmt.fmt_release_scratch()


def test_config3_full_size_every_element(fmt):
    """Config 3 at full size, 1/6/9/d: every element of forward, dgrad and wgrad against the oracle's full
    convolutions (3 x 14.8 GFLOP on the host's cores), within the 1e-5 relative Frobenius bound."""
    f = (6, 9, True)
    cfg = workloads.config3()
    X, W2, dY2 = cfg["X"], cfg["W"], cfg["dY"]
    n, c, h, w = X.shape
    k = W2.shape[0]
    W = W2.reshape(k, c, 3, 3)
    dY = np.ascontiguousarray(dY2.reshape(n, h, w, k).transpose(0, 3, 1, 2))
    Y, dX, dW = run_all(fmt, X, W, dY, f, (1, 1), (1, 1))
    e, m, d = f
    for name, got, ref in (("Y", Y, oracle.conv2d_fwd(X, W, e, m, d)),
                           ("dX", dX, oracle.conv2d_dgrad(dY, W, X.shape, e, m, d)),
                           ("dW", dW, oracle.conv2d_wgrad(dY, X, W.shape, e, m, d))):
        assert got.shape == ref.shape and np.all(np.isfinite(got)), name
        assert rel_err(got, ref) <= TOL, "%s: %.3g" % (name, rel_err(got, ref))
