"""Pins for the oracle's convolution layers (Sec. IV-A: convolutions of the forward and backward
pass run on operands rounded to the format, with unrounded products): a library convolution and
its own autograd gradients in fp64, the im2col + matrix-product route, hand-worked cases and the
adjoint identity that ties forward, dgrad and wgrad together."""
import numpy as np
import pytest

import oracle
import workloads

torch = pytest.importorskip("torch")

GEOMS = [  # N, C, H, W, K, R, S, pad, stride
    (2, 3, 7, 6, 4, 3, 3, (1, 1), (1, 1)),
    (1, 2, 9, 8, 3, 3, 3, (1, 1), (2, 2)),
    (2, 4, 6, 6, 5, 1, 1, (0, 0), (1, 1)),
    (1, 3, 8, 9, 2, 5, 3, (2, 1), (1, 2)),
    (3, 2, 5, 5, 3, 2, 2, (0, 0), (1, 1)),
    (1, 1, 10, 7, 2, 3, 3, (0, 2), (3, 1)),
]


def int_data(rng, shape, lo=-4, hi=5, scale=1.0):
    return (rng.integers(lo, hi, shape) * scale).astype(np.float32)


def torch_conv(Xq, Wq, dYq, pad, stride):
    """fp64 library convolution and the gradients autograd derives for it."""
    x = torch.tensor(Xq.astype(np.float64), requires_grad=True)
    w = torch.tensor(Wq.astype(np.float64), requires_grad=True)
    y = torch.nn.functional.conv2d(x, w, padding=pad, stride=stride)
    gx, gw = torch.autograd.grad(y, (x, w), torch.tensor(dYq.astype(np.float64)))
    return y.detach().numpy(), gx.numpy(), gw.numpy()


@pytest.mark.parametrize("geom", GEOMS)
@pytest.mark.parametrize("fmt", [(6, 9, True), (5, 10, False), (8, 7, True)])
def test_matches_library_convolution_exact_integers(geom, fmt):
    """Small integers times a power of two: every sum is exact in fp64 whatever the order, so the
    oracle must equal the library's convolution and gradients bit for bit."""
    n, c, h, w, k, r, s, pad, stride = geom
    e, m, d = fmt
    rng = np.random.default_rng(n + 10 * c + 100 * h)
    X = int_data(rng, (n, c, h, w), scale=0.5)
    W = int_data(rng, (k, c, r, s), scale=0.25)
    P, Q = oracle.conv_out_size(h, w, r, s, pad, stride)
    dY = int_data(rng, (n, k, P, Q), scale=2.0 ** -6)
    y, gx, gw = torch_conv(X, W, dY, pad, stride)
    assert np.array_equal(oracle.conv2d_fwd(X, W, e, m, d, pad, stride), y.astype(np.float32))
    assert np.array_equal(oracle.conv2d_dgrad(dY, W, X.shape, e, m, d, pad, stride), gx.astype(np.float32))
    assert np.array_equal(oracle.conv2d_wgrad(dY, X, W.shape, e, m, d, pad, stride), gw.astype(np.float32))


@pytest.mark.parametrize("geom", GEOMS)
def test_matches_library_convolution_real_values(geom):
    """Real-valued tensors: operands are rounded to the format first (the library gets the rounded
    values), sums differ from the library's only by fp64 rounding order."""
    n, c, h, w, k, r, s, pad, stride = geom
    e, m, d = 6, 9, True
    rng = np.random.default_rng(7 * n + c)
    X = rng.standard_normal((n, c, h, w)).astype(np.float32)
    W = (rng.standard_normal((k, c, r, s)) * 0.2).astype(np.float32)
    P, Q = oracle.conv_out_size(h, w, r, s, pad, stride)
    dY = workloads.log2_normal((n, k, P, Q), -12.0, 4.0, 0.0, rng)
    Xq, Wq, dYq = (oracle.quantize(t, e, m, d) for t in (X, W, dY))
    assert not np.array_equal(Xq, X)                       # the rounding does something
    y, gx, gw = torch_conv(Xq, Wq, dYq, pad, stride)
    for got, want in ((oracle.conv2d_fwd(X, W, e, m, d, pad, stride), y),
                      (oracle.conv2d_dgrad(dY, W, X.shape, e, m, d, pad, stride), gx),
                      (oracle.conv2d_wgrad(dY, X, W.shape, e, m, d, pad, stride), gw)):
        scale = np.max(np.abs(want)) + 1e-300
        assert np.max(np.abs(got.astype(np.float64) - want)) <= 2.0 ** -23 * scale


def test_im2col_route_3x3():
    """3x3, pad 1, stride 1 through the materialised patch matrix and the matrix-product oracle:
    forward and wgrad visit the same terms in the same order (plus exact zeros), so they agree
    bit for bit; dgrad through col2im associates differently and agrees to fp32 rounding."""
    e, m, d = 6, 9, True
    rng = np.random.default_rng(1)
    n, c, h, w, k = 2, 5, 6, 7, 4
    X = rng.standard_normal((n, c, h, w)).astype(np.float32)
    W = (rng.standard_normal((k, c, 3, 3)) * 0.3).astype(np.float32)
    dY = workloads.log2_normal((n, k, h, w), -10.0, 3.0, 0.0, rng)
    Xcol = workloads.im2col_3x3(X)                              # [n*h*w, c*9]
    W2 = W.reshape(k, c * 9)
    dY2 = np.ascontiguousarray(dY.transpose(0, 2, 3, 1).reshape(n * h * w, k))
    Y2 = oracle.gemm(Xcol, W2, e, m, d, transB=True)            # [n*h*w, k]
    Y = oracle.conv2d_fwd(X, W, e, m, d)
    assert np.array_equal(Y, Y2.reshape(n, h, w, k).transpose(0, 3, 1, 2))
    dW2 = oracle.gemm(dY2, Xcol, e, m, d, transA=True)          # [k, c*9]
    assert np.array_equal(oracle.conv2d_wgrad(dY, X, W.shape, e, m, d), dW2.reshape(k, c, 3, 3))
    dXcol = oracle.gemm(dY2, W2, e, m, d).astype(np.float64).reshape(n, h, w, c, 3, 3)
    dX = np.zeros((n, c, h + 2, w + 2))
    for ky in range(3):
        for kx in range(3):
            dX[:, :, ky:ky + h, kx:kx + w] += dXcol[:, :, :, :, ky, kx].transpose(0, 3, 1, 2)
    got = oracle.conv2d_dgrad(dY, W, X.shape, e, m, d)
    assert np.max(np.abs(got - dX[:, :, 1:-1, 1:-1])) <= 2.0 ** -21 * np.max(np.abs(dX))


def test_hand_worked():
    e, m, d = 5, 10, True
    # 3x3 image, 2x2 filter, no padding, stride 1
    X = np.array([[[[1, 2, 3], [4, 5, 6], [7, 8, 9]]]], dtype=np.float32)
    W = np.array([[[[1, 0], [0, -1]]], [[[0.5, 0.5], [0.5, 0.5]]]], dtype=np.float32)
    Y = oracle.conv2d_fwd(X, W, e, m, d, pad=(0, 0))
    assert Y.tolist() == [[[[-4, -4], [-4, -4]], [[6, 8], [12, 14]]]]
    dY = np.array([[[[1, 0], [0, 0]], [[0, 0], [0, 2]]]], dtype=np.float32)
    # dX = dY[0,0,0,0] * W[0] placed at (0,0)  +  dY[0,1,1,1] * W[1] placed at (1,1)
    dX = oracle.conv2d_dgrad(dY, W, X.shape, e, m, d, pad=(0, 0))
    assert dX.tolist() == [[[[1, 0, 0], [0, 0, 1], [0, 1, 1]]]]
    # dW[k] = sum over positions of dY[k] * patch: k=0 sees the patch at (0,0), k=1 twice the patch at (1,1)
    dW = oracle.conv2d_wgrad(dY, X, W.shape, e, m, d, pad=(0, 0))
    assert dW.tolist() == [[[[1, 2], [4, 5]]], [[[10, 12], [16, 18]]]]
    # stride 2, pad 1, 3x3 filter of ones on a 4x4 image of ones: output 2x2 counts the taps inside
    ones = np.ones((1, 1, 4, 4), dtype=np.float32)
    Y = oracle.conv2d_fwd(ones, np.ones((1, 1, 3, 3), dtype=np.float32), e, m, d, pad=(1, 1), stride=(2, 2))
    assert Y.tolist() == [[[[4, 6], [6, 9]]]]
    # operands are rounded: 2049 is not a binary16 value (rounds to 2048), 0.1 rounds to 0.0999755859375
    Y = oracle.conv2d_fwd(np.full((1, 1, 1, 1), 2049, dtype=np.float32), np.full((1, 1, 1, 1), 0.1, dtype=np.float32),
                          e, m, d, pad=(0, 0))
    assert float(Y[0, 0, 0, 0]) == 2048 * 0.0999755859375


@pytest.mark.parametrize("geom", GEOMS)
def test_adjoint_identity(geom):
    """<conv(X, W), dY> = <X, dgrad(dY, W)> = <W, wgrad(dY, X)>, exactly, for integer data."""
    n, c, h, w, k, r, s, pad, stride = geom
    e, m, d = 6, 9, True
    rng = np.random.default_rng(99 + h)
    X, W = int_data(rng, (n, c, h, w)), int_data(rng, (k, c, r, s))
    P, Q = oracle.conv_out_size(h, w, r, s, pad, stride)
    dY = int_data(rng, (n, k, P, Q))
    a = np.sum(oracle.conv2d_fwd(X, W, e, m, d, pad, stride).astype(np.float64) * dY)
    b = np.sum(oracle.conv2d_dgrad(dY, W, X.shape, e, m, d, pad, stride).astype(np.float64) * X)
    c_ = np.sum(oracle.conv2d_wgrad(dY, X, W.shape, e, m, d, pad, stride).astype(np.float64) * W)
    assert a == b == c_ and a != 0


def test_sampled_outputs_equal_full():
    rng = np.random.default_rng(4)
    X = rng.standard_normal((2, 3, 6, 5)).astype(np.float32)
    W = rng.standard_normal((4, 3, 3, 3)).astype(np.float32)
    dY = rng.standard_normal((2, 4, 6, 5)).astype(np.float32)
    for full, fn in ((oracle.conv2d_fwd(X, W, 6, 9, True), lambda s: oracle.conv2d_fwd(X, W, 6, 9, True, sample=s)),
                     (oracle.conv2d_dgrad(dY, W, X.shape, 6, 9, True), lambda s: oracle.conv2d_dgrad(dY, W, X.shape, 6, 9, True, sample=s)),
                     (oracle.conv2d_wgrad(dY, X, W.shape, 6, 9, True), lambda s: oracle.conv2d_wgrad(dY, X, W.shape, 6, 9, True, sample=s))):
        idx = rng.integers(0, full.size, 50)
        assert np.array_equal(fn(idx), full.ravel()[idx])
