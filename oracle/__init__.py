"""CPU oracle for the emulated 1/e/m floating-point arithmetic -- TEST INFRASTRUCTURE ONLY.

A thin ctypes loader around ``fmt_oracle.c`` (plain C, fp64, written from the paper's
definitions: Sec. III Def. III.1/III.2, Table I, Sec. III-B FMACS, Sec. IV-A roundfp,
Sec. V denormal fraction).  It shares nothing with the GPU library and must not be
imported by it: only ``tests/``, the smoke check and the benchmark's ``cpu_baseline``
leg may use it.  Arrays in, arrays out; no GPU, no torch.

``oracle.fmac_exact`` (pure Python, exact rationals) is the plain definition of FMAC and of
Algorithm 1; the C routines ``fmac`` / ``fmac8_dot`` / ``gemm_fmac8`` here are the fast checker for
sizes it cannot reach and are pinned to it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fmt_oracle.c")
_LIB = os.path.join(_HERE, "libfmt_oracle.so")
_lock = threading.Lock()
_lib = None

NBINS = 64
CLASS_NAMES = ("total", "zero", "underflow", "denormal", "normal", "overflow", "inf", "nan")


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no contraction, no fast-math) and return the .so path."""
    with _lock:
        stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
        if force or stale:
            tmp = _LIB + ".tmp.%d" % os.getpid()
            cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
                   "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra",
                   "-o", tmp, _SRC, "-lm"]
            subprocess.run(cmd, check=True)
            os.replace(tmp, _LIB)
    return _LIB


class DlsState(ctypes.Structure):
    """State of the loss-scale controller (see oracle_dls_step in fmt_oracle.c)."""
    _fields_ = [("loss_scale", ctypes.c_float), ("good_steps", ctypes.c_int32), ("skip", ctypes.c_int32),
                ("steps", ctypes.c_int32), ("nonfinite", ctypes.c_uint64), ("worst_tensor", ctypes.c_int64),
                ("worst_denormal", ctypes.c_uint64), ("worst_total", ctypes.c_uint64),
                ("peak_tensor", ctypes.c_int64), ("peak_step", ctypes.c_int64),
                ("peak_denormal", ctypes.c_uint64), ("peak_total", ctypes.c_uint64)]

    def as_dict(self) -> dict:
        return {name: getattr(self, name) for name, _ in self._fields_}


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        f32p = ctypes.POINTER(ctypes.c_float)
        i64p = ctypes.POINTER(ctypes.c_int64)
        lib.oracle_format_constants.argtypes = [ctypes.c_int, ctypes.c_int] + \
            [ctypes.POINTER(ctypes.c_double)] * 3 + [ctypes.POINTER(ctypes.c_int)] * 2
        lib.oracle_format_constants.restype = ctypes.c_int
        lib.oracle_quantize_one.argtypes = [ctypes.c_float, ctypes.c_int, ctypes.c_int, ctypes.c_int]
        lib.oracle_quantize_one.restype = ctypes.c_float
        lib.oracle_quantize.argtypes = [f32p, f32p, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, ctypes.c_int]
        lib.oracle_quantize.restype = ctypes.c_int
        lib.oracle_histogram.argtypes = [f32p, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                         ctypes.POINTER(ctypes.c_uint64)]
        lib.oracle_histogram.restype = ctypes.c_int
        lib.oracle_gemm.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                    f32p, ctypes.c_int64, f32p, ctypes.c_int64, f32p, ctypes.c_int64,
                                    ctypes.c_int, ctypes.c_int, ctypes.c_int]
        lib.oracle_gemm.restype = ctypes.c_int
        lib.oracle_gemm_sampled.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int64, ctypes.c_int64,
                                            ctypes.c_int64, f32p, ctypes.c_int64, f32p, ctypes.c_int64,
                                            i64p, i64p, ctypes.c_int64, f32p,
                                            ctypes.c_int, ctypes.c_int, ctypes.c_int]
        lib.oracle_gemm_sampled.restype = ctypes.c_int
        lib.oracle_linear_epilogue.argtypes = [f32p, ctypes.c_int64, f32p, ctypes.c_int64, ctypes.c_int64,
                                               f32p, ctypes.c_int64, f32p, ctypes.c_int64] + [ctypes.c_int] * 3
        lib.oracle_linear_epilogue.restype = ctypes.c_int
        lib.oracle_fmac.argtypes = [ctypes.c_float] * 3 + [ctypes.c_int] * 3
        lib.oracle_fmac.restype = ctypes.c_float
        lib.oracle_fmac8_dot.argtypes = [f32p, ctypes.c_int64, f32p, ctypes.c_int64, ctypes.c_int64] + [ctypes.c_int] * 3
        lib.oracle_fmac8_dot.restype = ctypes.c_float
        lib.oracle_gemm_fmac8.argtypes = lib.oracle_gemm.argtypes
        lib.oracle_gemm_fmac8.restype = ctypes.c_int
        lib.oracle_encode.argtypes = [ctypes.c_float, ctypes.c_int, ctypes.c_int]
        lib.oracle_encode.restype = ctypes.c_uint32
        u16p = ctypes.POINTER(ctypes.c_uint16)
        lib.oracle_decode.argtypes = [ctypes.c_uint32, ctypes.c_int, ctypes.c_int]
        lib.oracle_decode.restype = ctypes.c_float
        lib.oracle_pack16.argtypes = [f32p, u16p, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, ctypes.c_int]
        lib.oracle_pack16.restype = ctypes.c_int
        lib.oracle_unpack16.argtypes = [u16p, f32p, ctypes.c_size_t, ctypes.c_int, ctypes.c_int]
        lib.oracle_unpack16.restype = ctypes.c_int
        lib.oracle_conv2d.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_int32), f32p, f32p, i64p, ctypes.c_int64, f32p,
                                      ctypes.c_int, ctypes.c_int, ctypes.c_int]
        lib.oracle_conv2d.restype = ctypes.c_int
        lib.oracle_dls_step.argtypes = [ctypes.POINTER(ctypes.c_uint64), ctypes.c_int64, ctypes.c_float, ctypes.c_float,
                                        ctypes.c_int32, ctypes.c_float, ctypes.c_float, ctypes.POINTER(DlsState)]
        lib.oracle_dls_step.restype = ctypes.c_int
        _lib = lib
    return _lib


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def format_constants(e: int, m: int) -> dict:
    """maxN, minN, minD, Emin, Emax of the 1/e/m format (Sec. III; Table I)."""
    lib = _load()
    mx, mn, md = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
    lo, hi = ctypes.c_int(), ctypes.c_int()
    rc = lib.oracle_format_constants(e, m, mx, mn, md, lo, hi)
    if rc:
        raise ValueError("unsupported format 1/%d/%d" % (e, m))
    return {"maxN": mx.value, "minN": mn.value, "minD": md.value, "Emin": lo.value, "Emax": hi.value}


def quantize(x, e: int, m: int, d: bool) -> np.ndarray:
    """roundfp(X, e, m, d) of Sec. IV-A on a float32 array; returns a float32 array of the same shape."""
    lib = _load()
    xa = _f32(x)
    y = np.empty_like(xa)
    rc = lib.oracle_quantize(_ptr(xa), _ptr(y), xa.size, e, m, int(bool(d)))
    if rc:
        raise ValueError("unsupported format 1/%d/%d" % (e, m))
    return y


def quantize_one(x: float, e: int, m: int, d: bool) -> np.float32:
    return np.float32(_load().oracle_quantize_one(np.float32(x), e, m, int(bool(d))))


def histogram(x, e: int, m: int, exp_lo: int = -48) -> dict:
    """Class counts and 64 binade bins of a float32 tensor (Sec. V); integer counts."""
    lib = _load()
    xa = _f32(x)
    out = np.zeros(8 + NBINS, dtype=np.uint64)
    rc = lib.oracle_histogram(_ptr(xa), xa.size, e, m, exp_lo,
                              out.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64)))
    if rc:
        raise ValueError("unsupported format 1/%d/%d" % (e, m))
    res = {name: int(out[i]) for i, name in enumerate(CLASS_NAMES)}
    res["bins"] = out[8:].copy()
    return res


def _lead(a: np.ndarray) -> int:
    return a.shape[1] if a.ndim == 2 else 1


def gemm(A, B, e: int, m: int, d: bool, transA: bool = False, transB: bool = False) -> np.ndarray:
    """C = Q(op(A)) Q(op(B)), exact products, fp64 sum rounded once to fp32 (FMACS reference)."""
    lib = _load()
    Aa, Ba = _f32(A), _f32(B)
    M, K = (Aa.shape[1], Aa.shape[0]) if transA else Aa.shape
    K2, N = (Ba.shape[1], Ba.shape[0]) if transB else Ba.shape
    if K != K2:
        raise ValueError("inner dimensions differ: %d vs %d" % (K, K2))
    C = np.zeros((M, N), dtype=np.float32)
    rc = lib.oracle_gemm(int(transA), int(transB), M, N, K, _ptr(Aa), max(_lead(Aa), 1),
                         _ptr(Ba), max(_lead(Ba), 1), _ptr(C), max(N, 1), e, m, int(bool(d)))
    if rc:
        raise ValueError("oracle_gemm failed: %d" % rc)
    return C


def gemm_sampled(A, B, rows, cols, e: int, m: int, d: bool,
                 transA: bool = False, transB: bool = False) -> np.ndarray:
    """The same sum as :func:`gemm` for the listed output positions only."""
    lib = _load()
    Aa, Ba = _f32(A), _f32(B)
    M, K = (Aa.shape[1], Aa.shape[0]) if transA else Aa.shape
    K2, N = (Ba.shape[1], Ba.shape[0]) if transB else Ba.shape
    if K != K2:
        raise ValueError("inner dimensions differ: %d vs %d" % (K, K2))
    r = np.ascontiguousarray(rows, dtype=np.int64)
    c = np.ascontiguousarray(cols, dtype=np.int64)
    out = np.zeros(r.size, dtype=np.float32)
    i64p = ctypes.POINTER(ctypes.c_int64)
    rc = lib.oracle_gemm_sampled(int(transA), int(transB), M, N, K, _ptr(Aa), _lead(Aa), _ptr(Ba), _lead(Ba),
                                 r.ctypes.data_as(i64p), c.ctypes.data_as(i64p), r.size, _ptr(out),
                                 e, m, int(bool(d)))
    if rc:
        raise ValueError("oracle_gemm_sampled failed: %d" % rc)
    return out


def linear_epilogue(acc, bias, e: int, m: int, d: bool):
    """(Y, T) with T = R(acc) + R(bias) (fp32 addition, bias per column, may be None) and Y = R(T):
    the output roundings of the quantized Linear layer of Sec. IV-A."""
    lib = _load()
    a = _f32(acc)
    if a.ndim != 2:
        raise ValueError("acc must be 2-D")
    M, N = a.shape
    b = None if bias is None else _f32(bias).ravel()
    if b is not None and b.size != N:
        raise ValueError("bias must have one value per column")
    Y, T = np.empty_like(a), np.empty_like(a)
    bp = None if b is None else _ptr(b)
    rc = lib.oracle_linear_epilogue(_ptr(a), max(N, 1), bp, M, N, _ptr(Y), max(N, 1), _ptr(T), max(N, 1),
                                    e, m, int(bool(d)))
    if rc:
        raise ValueError("oracle_linear_epilogue failed: %d" % rc)
    return Y, T


def linear(X, W, bias, e: int, m: int, d: bool):
    """Quantized Linear forward of Sec. IV-A: Y = R(R(R(X) R(W)^T) + R(b)) with X [batch, in],
    W [out, in]; the inner product is the FMACS reference of :func:`gemm`.  Returns (Y, T)."""
    return linear_epilogue(gemm(X, W, e, m, d, transB=True), bias, e, m, d)


def fmac(a: float, w: float, x: float, e: int, m: int, d: bool) -> np.float32:
    """FMAC of Sec. III-B: the exact a + w*x rounded once to the format (a, w, x values of the format)."""
    return np.float32(_load().oracle_fmac(np.float32(a), np.float32(w), np.float32(x), e, m, int(bool(d))))


def fmac8_dot(w, x, e: int, m: int, d: bool) -> np.float32:
    """Algorithm 1 (FMAC-8) on two vectors of values of the format."""
    wa, xa = _f32(w).ravel(), _f32(x).ravel()
    if wa.size != xa.size:
        raise ValueError("length mismatch")
    return np.float32(_load().oracle_fmac8_dot(_ptr(wa), 1, _ptr(xa), 1, wa.size, e, m, int(bool(d))))


def gemm_fmac8(A, B, e: int, m: int, d: bool, transA: bool = False, transB: bool = False) -> np.ndarray:
    """C[i][j] = FMAC-8 dot product (Algorithm 1) of row i of Q(op(A)) and column j of Q(op(B))."""
    lib = _load()
    Aa, Ba = _f32(A), _f32(B)
    M, K = (Aa.shape[1], Aa.shape[0]) if transA else Aa.shape
    K2, N = (Ba.shape[1], Ba.shape[0]) if transB else Ba.shape
    if K != K2:
        raise ValueError("inner dimensions differ: %d vs %d" % (K, K2))
    C = np.zeros((M, N), dtype=np.float32)
    rc = lib.oracle_gemm_fmac8(int(transA), int(transB), M, N, K, _ptr(Aa), max(_lead(Aa), 1),
                               _ptr(Ba), max(_lead(Ba), 1), _ptr(C), max(N, 1), e, m, int(bool(d)))
    if rc:
        raise ValueError("oracle_gemm_fmac8 failed: %d" % rc)
    return C


def encode(v, e: int, m: int) -> np.ndarray:
    """(1+e+m)-bit codes of values that already belong to the format (Sec. III encoding)."""
    lib = _load()
    va = _f32(v).ravel()
    return np.array([lib.oracle_encode(float(t), e, m) for t in va], dtype=np.uint32).reshape(np.shape(v))


def pack16(x, e: int, m: int, d: bool) -> np.ndarray:
    """Codes (uint16, 1+e+m <= 16 bits used) of roundfp(x, e, m, d): Sec. IV-A rounding, Sec. III encoding."""
    lib = _load()
    xa = _f32(x)
    codes = np.empty(xa.shape, dtype=np.uint16)
    rc = lib.oracle_pack16(_ptr(xa), codes.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)), xa.size, e, m, int(bool(d)))
    if rc:
        raise ValueError("format 1/%d/%d has no 16-bit code" % (e, m))
    return codes


def unpack16(codes, e: int, m: int) -> np.ndarray:
    """float32 values of (1+e+m)-bit codes (Sec. III); NaN codes give the canonical quiet NaN."""
    lib = _load()
    ca = np.ascontiguousarray(codes, dtype=np.uint16)
    y = np.empty(ca.shape, dtype=np.float32)
    rc = lib.oracle_unpack16(ca.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)), _ptr(y), ca.size, e, m)
    if rc:
        raise ValueError("format 1/%d/%d has no 16-bit code" % (e, m))
    return y


def dls_init(loss_scale: float) -> DlsState:
    """Fresh controller state: scale S, no steps seen, no peak yet."""
    st = DlsState()
    st.loss_scale = loss_scale
    st.worst_tensor = -1
    st.peak_tensor = -1
    st.peak_step = -1
    return st


def dls_step(hists, state: DlsState, growth: float = 2.0, backoff: float = 0.5, interval: int = 2000,
             min_scale: float = 1.0, max_scale: float = 2.0 ** 24) -> DlsState:
    """One step of the loss-scale controller on the statistics of the step's gradient tensors
    (array of shape [count, 72], uint64); updates and returns ``state``."""
    h = np.ascontiguousarray(np.asarray(hists, dtype=np.uint64).reshape(-1, 8 + NBINS))
    rc = _load().oracle_dls_step(h.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64)), h.shape[0], growth, backoff,
                                 interval, min_scale, max_scale, ctypes.byref(state))
    if rc:
        raise ValueError("oracle_dls_step failed: %d" % rc)
    return state


def conv_out_size(h: int, w: int, r: int, s: int, pad, stride):
    """Output height and width of a convolution with zero padding and no dilation."""
    return (h + 2 * pad[0] - r) // stride[0] + 1, (w + 2 * pad[1] - s) // stride[1] + 1


def _conv(which: int, a, b, geom, out_shape, e, m, d, sample):
    lib = _load()
    g = (ctypes.c_int32 * 11)(*[int(v) for v in geom])
    aa, ba = _f32(a), _f32(b)
    i64p = ctypes.POINTER(ctypes.c_int64)
    if sample is None:
        out = np.empty(out_shape, dtype=np.float32)
        rc = lib.oracle_conv2d(which, g, _ptr(aa), _ptr(ba), None, out.size, _ptr(out), e, m, int(bool(d)))
    else:
        idx = np.ascontiguousarray(sample, dtype=np.int64).ravel()
        out = np.empty(idx.size, dtype=np.float32)
        rc = lib.oracle_conv2d(which, g, _ptr(aa), _ptr(ba), idx.ctypes.data_as(i64p), idx.size, _ptr(out),
                               e, m, int(bool(d)))
    if rc:
        raise ValueError("oracle_conv2d failed: %d" % rc)
    return out


def _geom(xshape, wshape, pad, stride):
    n, c, h, w = xshape
    k, c2, r, s = wshape
    if c != c2:
        raise ValueError("channel mismatch")
    return (n, c, h, w, k, r, s, pad[0], pad[1], stride[0], stride[1])


def conv2d_fwd(X, W, e, m, d, pad=(1, 1), stride=(1, 1), sample=None) -> np.ndarray:
    """Y[n,k,p,q] = sum_{c,r,s} Q(X)[n,c,p*sh-ph+r,q*sw-pw+s] * Q(W)[k,c,r,s] (Sec. IV-A, FMACS reference:
    exact products, fp64 sum, one rounding to fp32).  ``sample``: flat output indices to compute only those."""
    X, W = _f32(X), _f32(W)
    g = _geom(X.shape, W.shape, pad, stride)
    P, Q = conv_out_size(g[2], g[3], g[5], g[6], pad, stride)
    return _conv(0, X, W, g, (g[0], g[4], P, Q), e, m, d, sample)


def conv2d_dgrad(dY, W, xshape, e, m, d, pad=(1, 1), stride=(1, 1), sample=None) -> np.ndarray:
    """dX[n,c,h,w] = sum_{k,r,s} Q(dY)[n,k,p,q] * Q(W)[k,c,r,s] over the (p, q) that read (h, w) through tap (r, s)."""
    dY, W = _f32(dY), _f32(W)
    g = _geom(xshape, W.shape, pad, stride)
    return _conv(1, dY, W, g, tuple(xshape), e, m, d, sample)


def conv2d_wgrad(dY, X, wshape, e, m, d, pad=(1, 1), stride=(1, 1), sample=None) -> np.ndarray:
    """dW[k,c,r,s] = sum_{n,p,q} Q(dY)[n,k,p,q] * Q(X)[n,c,p*sh-ph+r,q*sw-pw+s]."""
    dY, X = _f32(dY), _f32(X)
    g = _geom(X.shape, wshape, pad, stride)
    return _conv(2, dY, X, g, tuple(wshape), e, m, d, sample)
