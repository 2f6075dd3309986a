"""Thin Python binding of libfmt (C ABI declared in ``include/fmt.h``).

Argument marshalling only: every step of the path -- the rounding kernel of Sec. IV-A, the
per-tensor statistics of Sec. V and the FMACS matrix product of Sec. III-B -- runs in the
hand-written HIP kernels behind the C ABI.  PyTorch is used for device memory and streams.
There is no CPU fallback: if ``libfmt.so`` has not been built, importing this package raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import NamedTuple, Optional

# torch is imported before libfmt.so is loaded on purpose: torch ships its own copy of the HIP
# runtime, and the tensors whose pointers are handed to libfmt live in that runtime's context.
# Loading torch first makes libfmt bind to the same runtime (same SONAME) instead of bringing a
# second one into the process, which would not see torch's device.
import torch  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
# FMT_LIB_PATH selects another build of the same library (tuning builds); default: the in-tree one
LIB_PATH = os.environ.get("FMT_LIB_PATH") or os.path.join(_HERE, "libfmt.so")

FMT_NBINS = 64
EXP_LO_DEFAULT = -48
CLASS_NAMES = ("total", "zero", "underflow", "denormal", "normal", "overflow", "inf", "nan")
EXPORTS = ("fmt_quantize", "fmt_quantize_static", "fmt_histogram", "fmt_gemm", "fmt_operand_bytes", "fmt_prepare", "fmt_prepare_pair", "fmt_prepare_pair_batch", "fmt_quantize_prepare_pair_batch", "fmt_gemm_prepared", "fmt_gemm_prepared_batch", "fmt_linear_prepared", "fmt_gemm_fmac8", "fmt_linear", "fmt_pack16", "fmt_unpack16", "fmt_linear_pack16", "fmt_conv2d_fwd", "fmt_conv2d_dgrad", "fmt_conv2d_wgrad", "fmt_dls_init", "fmt_dls_step", "fmt_format_info", "fmt_format_thresholds",
           "fmt_scratch_bytes", "fmt_release_scratch", "fmt_status_string")


class Format(NamedTuple):
    """The triple of Def. III.2: e exponent bits, m stored mantissa bits, denormals kept or flushed."""
    e: int
    m: int
    denorm: bool = True

    @property
    def name(self) -> str:
        return "1/%d/%d/%s" % (self.e, self.m, "d" if self.denorm else "n")


BINARY16 = Format(5, 10, True)
BFLOAT16 = Format(8, 7, False)
FP169 = Format(6, 9, True)


class _CFormat(ctypes.Structure):
    _fields_ = [("e", ctypes.c_int32), ("m", ctypes.c_int32), ("denorm", ctypes.c_int32)]


class _CConv2d(ctypes.Structure):
    _fields_ = [(name, ctypes.c_int32) for name in ("n", "c", "h", "w", "k", "r", "s", "pad_h", "pad_w",
                                                     "stride_h", "stride_w")]


class _CDlsParams(ctypes.Structure):
    _fields_ = [("growth", ctypes.c_float), ("backoff", ctypes.c_float), ("interval", ctypes.c_int32),
                ("min_scale", ctypes.c_float), ("max_scale", ctypes.c_float)]


class _CDlsState(ctypes.Structure):
    _fields_ = [("loss_scale", ctypes.c_float), ("good_steps", ctypes.c_int32), ("skip", ctypes.c_int32),
                ("steps", ctypes.c_int32), ("nonfinite", ctypes.c_uint64), ("worst_tensor", ctypes.c_int64),
                ("worst_denormal", ctypes.c_uint64), ("worst_total", ctypes.c_uint64),
                ("peak_tensor", ctypes.c_int64), ("peak_step", ctypes.c_int64),
                ("peak_denormal", ctypes.c_uint64), ("peak_total", ctypes.c_uint64)]


class _COperand(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("bytes", ctypes.c_size_t), ("rows", ctypes.c_int64), ("k", ctypes.c_int64),
                ("format", _CFormat), ("scheme", ctypes.c_int32)]


class FmtError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s (status %d)" % (where, status_string(status), status))


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            "libfmt.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
            "(or `python paper_2103_15940_amd/build.py`) first; there is no fallback path")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    lib.fmt_quantize.argtypes = [vp, vp, sz, _CFormat, vp, i32, vp]
    lib.fmt_quantize.restype = ctypes.c_int
    lib.fmt_quantize_static.argtypes = lib.fmt_quantize.argtypes
    lib.fmt_quantize_static.restype = ctypes.c_int
    lib.fmt_histogram.argtypes = [vp, sz, _CFormat, vp, i32, vp]
    lib.fmt_histogram.restype = ctypes.c_int
    lib.fmt_gemm.argtypes = [ctypes.c_int, ctypes.c_int, i64, i64, i64, vp, i64, vp, i64, vp, i64, _CFormat, vp]
    lib.fmt_gemm.restype = ctypes.c_int
    lib.fmt_operand_bytes.argtypes = [i64, i64, _CFormat, ctypes.POINTER(sz)]
    lib.fmt_operand_bytes.restype = ctypes.c_int
    lib.fmt_prepare.argtypes = [vp, i64, ctypes.c_int, i64, i64, _CFormat, vp, sz, ctypes.POINTER(_COperand), vp]
    lib.fmt_prepare.restype = ctypes.c_int
    lib.fmt_prepare_pair.argtypes = [vp, i64, i64, i64, _CFormat, vp, sz, ctypes.POINTER(_COperand), vp, sz,
                                     ctypes.POINTER(_COperand), vp]
    lib.fmt_prepare_pair.restype = ctypes.c_int
    lib.fmt_prepare_pair_batch.argtypes = [i64, ctypes.POINTER(vp), ctypes.POINTER(i64), ctypes.POINTER(i64), ctypes.POINTER(i64),
                                           _CFormat, ctypes.POINTER(vp), ctypes.POINTER(sz), ctypes.POINTER(_COperand),
                                           ctypes.POINTER(vp), ctypes.POINTER(sz), ctypes.POINTER(_COperand), vp]
    lib.fmt_prepare_pair_batch.restype = ctypes.c_int
    lib.fmt_quantize_prepare_pair_batch.argtypes = [i64, ctypes.POINTER(vp), ctypes.POINTER(i64), ctypes.POINTER(i64),
                                                    ctypes.POINTER(i64), _CFormat, ctypes.POINTER(vp), ctypes.POINTER(i64),
                                                    ctypes.POINTER(vp), i32, ctypes.POINTER(vp), ctypes.POINTER(sz),
                                                    ctypes.POINTER(_COperand), ctypes.POINTER(vp), ctypes.POINTER(sz),
                                                    ctypes.POINTER(_COperand), vp]
    lib.fmt_quantize_prepare_pair_batch.restype = ctypes.c_int
    lib.fmt_gemm_prepared.argtypes = [ctypes.POINTER(_COperand), ctypes.POINTER(_COperand), vp, i64, vp]
    lib.fmt_gemm_prepared.restype = ctypes.c_int
    lib.fmt_gemm_prepared_batch.argtypes = [i64, ctypes.POINTER(ctypes.POINTER(_COperand)),
                                            ctypes.POINTER(ctypes.POINTER(_COperand)), ctypes.POINTER(vp),
                                            ctypes.POINTER(i64), vp]
    lib.fmt_gemm_prepared_batch.restype = ctypes.c_int
    lib.fmt_linear_prepared.argtypes = [ctypes.POINTER(_COperand), ctypes.POINTER(_COperand), vp, vp, i64, vp, i32, vp]
    lib.fmt_linear_prepared.restype = ctypes.c_int
    lib.fmt_gemm_fmac8.argtypes = lib.fmt_gemm.argtypes
    lib.fmt_gemm_fmac8.restype = ctypes.c_int
    lib.fmt_linear.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp, vp, i64, _CFormat, vp, i32, vp]
    lib.fmt_linear.restype = ctypes.c_int
    lib.fmt_pack16.argtypes = [vp, vp, sz, _CFormat, vp, i32, vp]
    lib.fmt_pack16.restype = ctypes.c_int
    lib.fmt_unpack16.argtypes = [vp, vp, sz, _CFormat, vp]
    lib.fmt_unpack16.restype = ctypes.c_int
    lib.fmt_linear_pack16.argtypes = lib.fmt_linear.argtypes
    lib.fmt_linear_pack16.restype = ctypes.c_int
    for fn in (lib.fmt_conv2d_fwd, lib.fmt_conv2d_dgrad, lib.fmt_conv2d_wgrad):
        fn.argtypes = [_CConv2d, vp, vp, vp, _CFormat, vp]
        fn.restype = ctypes.c_int
    lib.fmt_dls_init.argtypes = [vp, ctypes.c_float, vp]
    lib.fmt_dls_init.restype = ctypes.c_int
    lib.fmt_dls_step.argtypes = [vp, i64, _CDlsParams, vp, vp]
    lib.fmt_dls_step.restype = ctypes.c_int
    dp, ip = ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int32)
    lib.fmt_format_info.argtypes = [_CFormat, dp, dp, dp, ip, ip]
    lib.fmt_format_info.restype = ctypes.c_int
    lib.fmt_format_thresholds.argtypes = [_CFormat, ctypes.POINTER(ctypes.c_uint32)]
    lib.fmt_format_thresholds.restype = ctypes.c_int
    lib.fmt_scratch_bytes.argtypes = [vp, ctypes.POINTER(ctypes.c_size_t)]
    lib.fmt_scratch_bytes.restype = ctypes.c_int
    lib.fmt_release_scratch.argtypes = []
    lib.fmt_release_scratch.restype = ctypes.c_int
    lib.fmt_status_string.argtypes = [ctypes.c_int]
    lib.fmt_status_string.restype = ctypes.c_char_p
    return lib


_lib = _load()


def _cfmt(f) -> _CFormat:
    e, m, d = f
    return _CFormat(int(e), int(m), 1 if d else 0)


def status_string(status: int) -> str:
    return _lib.fmt_status_string(int(status)).decode()


def _check(rc: int, where: str) -> None:
    if rc != 0:
        raise FmtError(rc, where)


def _stream_ptr(stream) -> int:
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


def _dev_f32(t, name: str):
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda or t.dtype != torch.float32:
        raise TypeError("%s must be a float32 tensor on the GPU" % name)
    return t


def new_hist(device="cuda"):
    """Device buffer for one fmt_hist_t (72 x int64)."""
    import torch
    return torch.empty(8 + FMT_NBINS, dtype=torch.int64, device=device)


def hist_to_dict(hist) -> dict:
    """Copies a device fmt_hist_t to the host: class counts as ints, bins as a numpy uint64 array."""
    import numpy as np
    h = hist.cpu().numpy().astype(np.uint64)
    out = {name: int(h[i]) for i, name in enumerate(CLASS_NAMES)}
    out["bins"] = h[8:].copy()
    return out


def fmt_quantize(x, fmt, out=None, hist=None, exp_lo: int = EXP_LO_DEFAULT, stream=None, static: bool = False):
    """y = Q_{e,m,d|n}(x) elementwise (Sec. IV-A roundfp); ``out`` may be ``x`` itself.  When a
    ``hist`` buffer (see :func:`new_hist`) is given, the statistics of :func:`fmt_histogram` are
    produced in the same pass.  Asynchronous on ``stream`` (default: torch's current stream).
    ``static=True`` calls ``fmt_quantize_static``, the entry point that allocates nothing (pass ``out``,
    or this wrapper's own ``torch.empty_like`` allocates the result)."""
    import torch
    _dev_f32(x, "x")
    if not x.is_contiguous():
        raise ValueError("x must be contiguous")
    if out is None:
        out = torch.empty_like(x)
    _dev_f32(out, "out")
    if not out.is_contiguous() or out.numel() != x.numel():
        raise ValueError("out must be contiguous and as large as x")
    hp = None
    if hist is not None:
        if hist.dtype != torch.int64 or hist.numel() != 8 + FMT_NBINS or not hist.is_cuda:
            raise TypeError("hist must be a GPU int64 tensor of 72 elements")
        hp = hist.data_ptr()
    entry = _lib.fmt_quantize_static if static else _lib.fmt_quantize
    rc = entry(x.data_ptr(), out.data_ptr(), x.numel(), _cfmt(fmt), hp, int(exp_lo), _stream_ptr(stream))
    _check(rc, "fmt_quantize_static" if static else "fmt_quantize")
    return out


def fmt_histogram(x, fmt, hist=None, exp_lo: int = EXP_LO_DEFAULT, stream=None):
    """Per-tensor class counts and 64 binade bins (Sec. V) into a device fmt_hist_t; returns it."""
    import torch
    _dev_f32(x, "x")
    if not x.is_contiguous():
        raise ValueError("x must be contiguous")
    if hist is None:
        hist = new_hist(x.device)
    if hist.dtype != torch.int64 or hist.numel() != 8 + FMT_NBINS or not hist.is_cuda:
        raise TypeError("hist must be a GPU int64 tensor of 72 elements")
    rc = _lib.fmt_histogram(x.data_ptr(), x.numel(), _cfmt(fmt), hist.data_ptr(), int(exp_lo), _stream_ptr(stream))
    _check(rc, "fmt_histogram")
    return hist


def _gemm_call(entry, where, A, B, fmt, transA, transB, out, stream):
    for t, name in ((A, "A"), (B, "B")):
        _dev_f32(t, name)
        if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
            raise ValueError("%s must be 2-D with unit column stride" % name)
    M, K = (A.shape[1], A.shape[0]) if transA else (A.shape[0], A.shape[1])
    K2, N = (B.shape[1], B.shape[0]) if transB else (B.shape[0], B.shape[1])
    if K != K2:
        raise ValueError("inner dimensions differ: %d vs %d" % (K, K2))
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=A.device)
    _dev_f32(out, "out")
    if out.dim() != 2 or tuple(out.shape) != (M, N) or (N > 1 and out.stride(1) != 1):
        raise ValueError("out must be an M x N tensor with unit column stride")
    lda = A.stride(0) if A.shape[0] > 1 else max(A.shape[1], 1)
    ldb = B.stride(0) if B.shape[0] > 1 else max(B.shape[1], 1)
    ldc = out.stride(0) if M > 1 else max(N, 1)
    rc = entry(int(transA), int(transB), M, N, K, A.data_ptr(), lda, B.data_ptr(), ldb,
               out.data_ptr(), ldc, _cfmt(fmt), _stream_ptr(stream))
    _check(rc, where)
    return out


def fmt_gemm(A, B, fmt, transA: bool = False, transB: bool = False, out=None, stream=None):
    """C = Q(op(A)) Q(op(B)) with exact products and fp32 accumulation (FMACS, Sec. III-B).
    A, B are 2-D row-major float32 GPU tensors (a row stride larger than the row length is
    passed on as the leading dimension)."""
    return _gemm_call(_lib.fmt_gemm, "fmt_gemm", A, B, fmt, transA, transB, out, stream)


class PreparedOperand:
    """A rounded operand in the matrix cores' 16-bit layout (see ``fmt_prepare`` in fmt.h): the device
    buffer (a uint8 tensor that keeps the memory alive) and the descriptor the C calls take."""

    def __init__(self, buf, desc):
        self.buf = buf
        self.desc = desc

    @property
    def rows(self) -> int:
        return int(self.desc.rows)

    @property
    def k(self) -> int:
        return int(self.desc.k)


def fmt_operand_bytes(rows: int, k: int, fmt) -> int:
    n = ctypes.c_size_t()
    _check(_lib.fmt_operand_bytes(int(rows), int(k), _cfmt(fmt), ctypes.byref(n)), "fmt_operand_bytes")
    return int(n.value)


def fmt_prepare(X, fmt, trans: bool = False, out=None, stream=None) -> PreparedOperand:
    """Rounds the 2-D float32 GPU tensor X to the format once and stores it as a prepared operand of
    X.shape[0] rows (``trans=False``) or, transposed, of X.shape[1] rows (``trans=True``).  ``out`` may be
    a uint8 GPU tensor (256-byte aligned, at least :func:`fmt_operand_bytes` long) to prepare into."""
    import torch
    _dev_f32(X, "X")
    if X.dim() != 2 or (X.shape[1] > 1 and X.stride(1) != 1):
        raise ValueError("X must be 2-D with unit column stride")
    rows, k = (X.shape[1], X.shape[0]) if trans else (X.shape[0], X.shape[1])
    need = fmt_operand_bytes(rows, k, fmt)
    if out is None:
        out = torch.empty(need, dtype=torch.uint8, device=X.device)
    if not isinstance(out, torch.Tensor) or out.dtype != torch.uint8 or not out.is_cuda or not out.is_contiguous():
        raise TypeError("out must be a contiguous GPU uint8 tensor")
    desc = _COperand()
    ld = X.stride(0) if X.shape[0] > 1 else max(X.shape[1], 1)
    rc = _lib.fmt_prepare(X.data_ptr(), ld, int(bool(trans)), rows, k, _cfmt(fmt), out.data_ptr(), out.numel(),
                          ctypes.byref(desc), _stream_ptr(stream))
    _check(rc, "fmt_prepare")
    return PreparedOperand(out, desc)


def fmt_prepare_pair(X, fmt, out=None, out_t=None, stream=None):
    """Both orientations of the 2-D float32 GPU tensor X as prepared operands in one call: returns
    (X as stored, X transposed), the operands :func:`fmt_prepare` gives with ``trans=False`` and ``trans=True``."""
    import torch
    _dev_f32(X, "X")
    if X.dim() != 2 or (X.shape[1] > 1 and X.stride(1) != 1):
        raise ValueError("X must be 2-D with unit column stride")
    rows, cols = X.shape
    bufs = []
    for buf, (r, k) in ((out, (rows, cols)), (out_t, (cols, rows))):
        if buf is None:
            buf = torch.empty(fmt_operand_bytes(r, k, fmt), dtype=torch.uint8, device=X.device)
        if not isinstance(buf, torch.Tensor) or buf.dtype != torch.uint8 or not buf.is_cuda or not buf.is_contiguous():
            raise TypeError("out and out_t must be contiguous GPU uint8 tensors")
        bufs.append(buf)
    d0, d1 = _COperand(), _COperand()
    ld = X.stride(0) if rows > 1 else max(cols, 1)
    rc = _lib.fmt_prepare_pair(X.data_ptr(), ld, rows, cols, _cfmt(fmt), bufs[0].data_ptr(), bufs[0].numel(), ctypes.byref(d0),
                               bufs[1].data_ptr(), bufs[1].numel(), ctypes.byref(d1), _stream_ptr(stream))
    _check(rc, "fmt_prepare_pair")
    return PreparedOperand(bufs[0], d0), PreparedOperand(bufs[1], d1)


def _pair_batch_args(Xs, fmt, outs, outs_t):
    """Checks and marshals what the two batch prepare calls share: the matrices and the operand buffers."""
    import torch
    n = len(Xs)
    outs = [None] * n if outs is None else list(outs)
    outs_t = [None] * n if outs_t is None else list(outs_t)
    if len(outs) != n or len(outs_t) != n:
        raise ValueError("outs and outs_t must be as long as Xs")
    bufs, bufs_t = [], []
    for X, o, ot in zip(Xs, outs, outs_t):
        _dev_f32(X, "X")
        if X.dim() != 2 or (X.shape[1] > 1 and X.stride(1) != 1):
            raise ValueError("every X must be 2-D with unit column stride")
        rows, cols = X.shape
        pair = []
        for buf, (r, k) in ((o, (rows, cols)), (ot, (cols, rows))):
            if buf is None:
                buf = torch.empty(fmt_operand_bytes(r, k, fmt), dtype=torch.uint8, device=X.device)
            if not isinstance(buf, torch.Tensor) or buf.dtype != torch.uint8 or not buf.is_cuda or not buf.is_contiguous():
                raise TypeError("outs and outs_t must hold contiguous GPU uint8 tensors")
            pair.append(buf)
        bufs.append(pair[0])
        bufs_t.append(pair[1])
    m = max(n, 1)
    c = {
        "X": (ctypes.c_void_p * m)(*[X.data_ptr() for X in Xs]),
        "ld": (ctypes.c_int64 * m)(*[X.stride(0) if X.shape[0] > 1 else max(X.shape[1], 1) for X in Xs]),
        "rows": (ctypes.c_int64 * m)(*[X.shape[0] for X in Xs]),
        "cols": (ctypes.c_int64 * m)(*[X.shape[1] for X in Xs]),
        "data": (ctypes.c_void_p * m)(*[b.data_ptr() for b in bufs]),
        "bytes": (ctypes.c_size_t * m)(*[b.numel() for b in bufs]),
        "data_t": (ctypes.c_void_p * m)(*[b.data_ptr() for b in bufs_t]),
        "bytes_t": (ctypes.c_size_t * m)(*[b.numel() for b in bufs_t]),
        "op": (_COperand * m)(), "op_t": (_COperand * m)(),
    }
    return bufs, bufs_t, c


def _pair_batch_result(n, bufs, bufs_t, c):
    result = []
    for i in range(n):
        a, b = _COperand(), _COperand()
        ctypes.memmove(ctypes.byref(a), ctypes.byref(c["op"][i]), ctypes.sizeof(_COperand))
        ctypes.memmove(ctypes.byref(b), ctypes.byref(c["op_t"][i]), ctypes.sizeof(_COperand))
        result.append((PreparedOperand(bufs[i], a), PreparedOperand(bufs_t[i], b)))
    return result


def fmt_prepare_pair_batch(Xs, fmt, outs=None, outs_t=None, stream=None):
    """:func:`fmt_prepare_pair` for a sequence of 2-D float32 GPU tensors in one call (shared launches for the
    1/6/m formats).  ``outs`` / ``outs_t``: optional sequences of uint8 GPU tensors to prepare into.  Returns a
    list of (X as stored, X transposed) operand pairs."""
    Xs = list(Xs)
    bufs, bufs_t, c = _pair_batch_args(Xs, fmt, outs, outs_t)
    rc = _lib.fmt_prepare_pair_batch(len(Xs), c["X"], c["ld"], c["rows"], c["cols"], _cfmt(fmt), c["data"], c["bytes"], c["op"],
                                     c["data_t"], c["bytes_t"], c["op_t"], _stream_ptr(stream))
    _check(rc, "fmt_prepare_pair_batch")
    return _pair_batch_result(len(Xs), bufs, bufs_t, c)


def fmt_quantize_prepare_pair_batch(Xs, fmt, Ys, hists, exp_lo: int = EXP_LO_DEFAULT, outs=None, outs_t=None, stream=None):
    """The rounding pass over a sequence of 2-D float32 GPU tensors in one call (1/6/m formats): ``Ys[i]`` receives
    ``Xs[i]`` rounded to the format (as :func:`fmt_quantize` gives it; may be ``Xs[i]`` itself), ``hists[i]`` (from
    :func:`new_hist`) its statistics, and the result is the list of (X as stored, X transposed) operand pairs of
    :func:`fmt_prepare_pair_batch` -- every tensor is read once."""
    Xs, Ys, hists = list(Xs), list(Ys), list(hists)
    n = len(Xs)
    if len(Ys) != n or len(hists) != n:
        raise ValueError("Ys and hists must be as long as Xs")
    for X, Y in zip(Xs, Ys):
        _dev_f32(Y, "Y")
        if Y.dim() != 2 or tuple(Y.shape) != tuple(X.shape) or (Y.shape[1] > 1 and Y.stride(1) != 1):
            raise ValueError("every Y must have the shape of its X and unit column stride")
    import torch
    for h in hists:
        if not isinstance(h, torch.Tensor) or h.dtype != torch.int64 or h.numel() != 8 + FMT_NBINS or not h.is_cuda:
            raise TypeError("every hist must be a GPU int64 tensor of 72 elements")
    bufs, bufs_t, c = _pair_batch_args(Xs, fmt, outs, outs_t)
    m = max(n, 1)
    yp = (ctypes.c_void_p * m)(*[Y.data_ptr() for Y in Ys])
    ldy = (ctypes.c_int64 * m)(*[Y.stride(0) if Y.shape[0] > 1 else max(Y.shape[1], 1) for Y in Ys])
    hp = (ctypes.c_void_p * m)(*[h.data_ptr() for h in hists])
    rc = _lib.fmt_quantize_prepare_pair_batch(n, c["X"], c["ld"], c["rows"], c["cols"], _cfmt(fmt), yp, ldy, hp, int(exp_lo),
                                              c["data"], c["bytes"], c["op"], c["data_t"], c["bytes_t"], c["op_t"],
                                              _stream_ptr(stream))
    _check(rc, "fmt_quantize_prepare_pair_batch")
    return _pair_batch_result(n, bufs, bufs_t, c)


def fmt_gemm_prepared(A: PreparedOperand, B: PreparedOperand, out=None, stream=None):
    """C[i][j] = sum_k Q(a)[i][k] Q(b)[j][k] on two prepared operands (FMACS, Sec. III-B): one launch."""
    import torch
    M, N = A.rows, B.rows
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=A.buf.device)
    _dev_f32(out, "out")
    if out.dim() != 2 or tuple(out.shape) != (M, N) or (N > 1 and out.stride(1) != 1):
        raise ValueError("out must be an M x N tensor with unit column stride")
    ldc = out.stride(0) if M > 1 else max(N, 1)
    rc = _lib.fmt_gemm_prepared(ctypes.byref(A.desc), ctypes.byref(B.desc), out.data_ptr(), ldc, _stream_ptr(stream))
    _check(rc, "fmt_gemm_prepared")
    return out


def fmt_gemm_prepared_batch(A, B, out=None, stream=None):
    """The products C[i] = A[i] B[i]^T of two equally long sequences of prepared operands in one call; the small
    ones share kernel launches (Sec. IV-A: the three products of every layer are known once the step's tensors
    are rounded).  Returns the list of results."""
    import torch
    A, B = list(A), list(B)
    n = len(A)
    if len(B) != n:
        raise ValueError("A and B must hold the same number of operands")
    if out is None:
        out = [torch.empty((a.rows, b.rows), dtype=torch.float32, device=a.buf.device) for a, b in zip(A, B)]
    out = list(out)
    if len(out) != n:
        raise ValueError("out must hold one tensor per product")
    ldc = []
    for a, b, c in zip(A, B, out):
        _dev_f32(c, "out")
        if c.dim() != 2 or tuple(c.shape) != (a.rows, b.rows) or (b.rows > 1 and c.stride(1) != 1):
            raise ValueError("every out must be an M x N tensor with unit column stride")
        ldc.append(c.stride(0) if a.rows > 1 else max(b.rows, 1))
    PA = (ctypes.POINTER(_COperand) * max(n, 1))(*[ctypes.pointer(a.desc) for a in A])
    PB = (ctypes.POINTER(_COperand) * max(n, 1))(*[ctypes.pointer(b.desc) for b in B])
    PC = (ctypes.c_void_p * max(n, 1))(*[c.data_ptr() for c in out])
    LD = (ctypes.c_int64 * max(n, 1))(*ldc)
    rc = _lib.fmt_gemm_prepared_batch(n, PA, PB, PC, LD, _stream_ptr(stream))
    _check(rc, "fmt_gemm_prepared_batch")
    return out


def fmt_linear_prepared(X: PreparedOperand, W: PreparedOperand, bias, out=None, hist=None,
                        exp_lo: int = EXP_LO_DEFAULT, stream=None):
    """:func:`fmt_linear` on operands prepared with :func:`fmt_prepare` (X: the batch rows, W: the rows of the
    weight matrix): product, bias, output roundings and the statistics of the output, with no rounding or
    layout pass over X and W in the call (Sec. IV-A)."""
    import torch
    M, N = X.rows, W.rows
    bp = None
    if bias is not None:
        _dev_f32(bias, "bias")
        if bias.dim() != 1 or bias.numel() != N or not bias.is_contiguous():
            raise ValueError("bias must be a contiguous vector with one value per output column")
        bp = bias.data_ptr()
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=X.buf.device)
    _dev_f32(out, "out")
    if out.dim() != 2 or tuple(out.shape) != (M, N) or (N > 1 and out.stride(1) != 1):
        raise ValueError("out must be an M x N tensor with unit column stride")
    hp = None
    if hist is not None:
        if hist.dtype != torch.int64 or hist.numel() != 8 + FMT_NBINS or not hist.is_cuda:
            raise TypeError("hist must be a GPU int64 tensor of 72 elements")
        hp = hist.data_ptr()
    ldy = out.stride(0) if M > 1 else max(N, 1)
    rc = _lib.fmt_linear_prepared(ctypes.byref(X.desc), ctypes.byref(W.desc), bp, out.data_ptr(), ldy, hp, int(exp_lo),
                                  _stream_ptr(stream))
    _check(rc, "fmt_linear_prepared")
    return out


def fmt_gemm_fmac8(A, B, fmt, transA: bool = False, transB: bool = False, out=None, stream=None):
    """The same product with the FMAC-8 accumulation of Sec. IV-A, Algorithm 1; the result is a
    tensor of values of the format."""
    return _gemm_call(_lib.fmt_gemm_fmac8, "fmt_gemm_fmac8", A, B, fmt, transA, transB, out, stream)


def fmt_linear(X, W, bias, fmt, out=None, hist=None, exp_lo: int = EXP_LO_DEFAULT, stream=None):
    """Quantized fully connected layer of Sec. IV-A: Y = R(R(R(X) R(W)^T) + R(b)) with X [batch, in],
    W [out, in], bias [out] or None.  With a ``hist`` buffer the statistics of t = R(acc) + R(b),
    the values entering the last rounding, are produced in the same pass."""
    import torch
    for t, name in ((X, "X"), (W, "W")):
        _dev_f32(t, name)
        if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
            raise ValueError("%s must be 2-D with unit column stride" % name)
    M, K = X.shape
    N, K2 = W.shape
    if K != K2:
        raise ValueError("inner dimensions differ: %d vs %d" % (K, K2))
    bp = None
    if bias is not None:
        _dev_f32(bias, "bias")
        if bias.dim() != 1 or bias.numel() != N or not bias.is_contiguous():
            raise ValueError("bias must be a contiguous vector with one value per output column")
        bp = bias.data_ptr()
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=X.device)
    _dev_f32(out, "out")
    if out.dim() != 2 or tuple(out.shape) != (M, N) or (N > 1 and out.stride(1) != 1):
        raise ValueError("out must be an M x N tensor with unit column stride")
    hp = None
    if hist is not None:
        if hist.dtype != torch.int64 or hist.numel() != 8 + FMT_NBINS or not hist.is_cuda:
            raise TypeError("hist must be a GPU int64 tensor of 72 elements")
        hp = hist.data_ptr()
    ldx = X.stride(0) if M > 1 else max(K, 1)
    ldw = W.stride(0) if N > 1 else max(K, 1)
    ldy = out.stride(0) if M > 1 else max(N, 1)
    rc = _lib.fmt_linear(M, N, K, X.data_ptr(), ldx, W.data_ptr(), ldw, bp, out.data_ptr(), ldy, _cfmt(fmt),
                         hp, int(exp_lo), _stream_ptr(stream))
    _check(rc, "fmt_linear")
    return out


def _dev_codes(t, name: str):
    import torch
    if not isinstance(t, torch.Tensor) or t.dtype not in (torch.int16, torch.uint16) or not t.is_cuda:
        raise TypeError("%s must be a GPU int16 (or uint16) tensor holding the 16-bit codes" % name)
    return t


def _hist_ptr(hist):
    import torch
    if hist is None:
        return None
    if hist.dtype != torch.int64 or hist.numel() != 8 + FMT_NBINS or not hist.is_cuda:
        raise TypeError("hist must be a GPU int64 tensor of 72 elements")
    return hist.data_ptr()


def fmt_pack16(x, fmt, out=None, hist=None, exp_lo: int = EXP_LO_DEFAULT, stream=None):
    """:func:`fmt_quantize` with the result stored as the format's own 16-bit codes (Sec. III;
    needs 1 + e + m <= 16): returns an int16 tensor of x's shape holding the code bit patterns."""
    import torch
    _dev_f32(x, "x")
    if not x.is_contiguous():
        raise ValueError("x must be contiguous")
    if out is None:
        out = torch.empty(x.shape, dtype=torch.int16, device=x.device)
    _dev_codes(out, "out")
    if not out.is_contiguous() or out.numel() != x.numel():
        raise ValueError("out must be contiguous and as large as x")
    rc = _lib.fmt_pack16(x.data_ptr(), out.data_ptr(), x.numel(), _cfmt(fmt), _hist_ptr(hist), int(exp_lo),
                         _stream_ptr(stream))
    _check(rc, "fmt_pack16")
    return out


def fmt_unpack16(codes, fmt, out=None, stream=None):
    """fp32 values of 16-bit codes (the inverse of :func:`fmt_pack16` on its results)."""
    import torch
    _dev_codes(codes, "codes")
    if not codes.is_contiguous():
        raise ValueError("codes must be contiguous")
    if out is None:
        out = torch.empty(codes.shape, dtype=torch.float32, device=codes.device)
    _dev_f32(out, "out")
    if not out.is_contiguous() or out.numel() != codes.numel():
        raise ValueError("out must be contiguous and as large as codes")
    rc = _lib.fmt_unpack16(codes.data_ptr(), out.data_ptr(), codes.numel(), _cfmt(fmt), _stream_ptr(stream))
    _check(rc, "fmt_unpack16")
    return out


def fmt_linear_pack16(X, W, bias, fmt, out=None, hist=None, exp_lo: int = EXP_LO_DEFAULT, stream=None):
    """:func:`fmt_linear` with the output stored as 16-bit codes (int16 tensor [batch, out])."""
    import torch
    for t, name in ((X, "X"), (W, "W")):
        _dev_f32(t, name)
        if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
            raise ValueError("%s must be 2-D with unit column stride" % name)
    M, K = X.shape
    N, K2 = W.shape
    if K != K2:
        raise ValueError("inner dimensions differ: %d vs %d" % (K, K2))
    bp = None
    if bias is not None:
        _dev_f32(bias, "bias")
        if bias.dim() != 1 or bias.numel() != N or not bias.is_contiguous():
            raise ValueError("bias must be a contiguous vector with one value per output column")
        bp = bias.data_ptr()
    if out is None:
        out = torch.empty((M, N), dtype=torch.int16, device=X.device)
    _dev_codes(out, "out")
    if out.dim() != 2 or tuple(out.shape) != (M, N) or (N > 1 and out.stride(1) != 1):
        raise ValueError("out must be an M x N tensor with unit column stride")
    ldx = X.stride(0) if M > 1 else max(K, 1)
    ldw = W.stride(0) if N > 1 else max(K, 1)
    ldy = out.stride(0) if M > 1 else max(N, 1)
    rc = _lib.fmt_linear_pack16(M, N, K, X.data_ptr(), ldx, W.data_ptr(), ldw, bp, out.data_ptr(), ldy, _cfmt(fmt),
                                _hist_ptr(hist), int(exp_lo), _stream_ptr(stream))
    _check(rc, "fmt_linear_pack16")
    return out


def _pair(v):
    return (int(v), int(v)) if isinstance(v, int) else (int(v[0]), int(v[1]))


def _conv_geom(xshape, wshape, pad, stride):
    n, c, h, w = (int(v) for v in xshape)
    k, c2, r, s = (int(v) for v in wshape)
    if c != c2:
        raise ValueError("channel mismatch: input has %d, filter has %d" % (c, c2))
    (ph, pw), (sh, sw) = _pair(pad), _pair(stride)
    if sh < 1 or sw < 1 or h + 2 * ph < r or w + 2 * pw < s:
        raise ValueError("bad convolution geometry")
    P, Q = (h + 2 * ph - r) // sh + 1, (w + 2 * pw - s) // sw + 1
    return _CConv2d(n, c, h, w, k, r, s, ph, pw, sh, sw), (n, k, P, Q)


def _dense4(t, name, shape=None):
    _dev_f32(t, name)
    if t.dim() != 4 or not t.is_contiguous():
        raise ValueError("%s must be a contiguous 4-D tensor" % name)
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError("%s must have shape %r" % (name, tuple(shape)))


def fmt_conv2d_fwd(X, W, fmt, pad=1, stride=1, out=None, stream=None):
    """Y = conv(Q(X), Q(W)) with exact products and fp32 accumulation (Sec. IV-A); X [n,c,h,w], W [k,c,r,s],
    Y [n,k,P,Q].  No fp32 patch matrix is formed: the library gathers the patches from the rounded tensor
    straight into its 16-bit operand layout."""
    import torch
    _dense4(X, "X")
    _dense4(W, "W")
    g, yshape = _conv_geom(X.shape, W.shape, pad, stride)
    if out is None:
        out = torch.empty(yshape, dtype=torch.float32, device=X.device)
    _dense4(out, "out", yshape)
    _check(_lib.fmt_conv2d_fwd(g, X.data_ptr(), W.data_ptr(), out.data_ptr(), _cfmt(fmt), _stream_ptr(stream)),
           "fmt_conv2d_fwd")
    return out


def fmt_conv2d_dgrad(dY, W, xshape, fmt, pad=1, stride=1, out=None, stream=None):
    """dX of the same convolution from dY [n,k,P,Q] and W [k,c,r,s]; ``xshape`` = (n, c, h, w)."""
    import torch
    _dense4(W, "W")
    g, yshape = _conv_geom(xshape, W.shape, pad, stride)
    _dense4(dY, "dY", yshape)
    if out is None:
        out = torch.empty(tuple(int(v) for v in xshape), dtype=torch.float32, device=dY.device)
    _dense4(out, "out", xshape)
    _check(_lib.fmt_conv2d_dgrad(g, dY.data_ptr(), W.data_ptr(), out.data_ptr(), _cfmt(fmt), _stream_ptr(stream)),
           "fmt_conv2d_dgrad")
    return out


def fmt_conv2d_wgrad(dY, X, wshape, fmt, pad=1, stride=1, out=None, stream=None):
    """dW of the same convolution from dY [n,k,P,Q] and X [n,c,h,w]; ``wshape`` = (k, c, r, s)."""
    import torch
    _dense4(X, "X")
    g, yshape = _conv_geom(X.shape, wshape, pad, stride)
    _dense4(dY, "dY", yshape)
    if out is None:
        out = torch.empty(tuple(int(v) for v in wshape), dtype=torch.float32, device=dY.device)
    _dense4(out, "out", wshape)
    _check(_lib.fmt_conv2d_wgrad(g, dY.data_ptr(), X.data_ptr(), out.data_ptr(), _cfmt(fmt), _stream_ptr(stream)),
           "fmt_conv2d_wgrad")
    return out


DLS_STATE_BYTES = ctypes.sizeof(_CDlsState)


def fmt_dls_init(loss_scale: float, device=None, state=None, stream=None):
    """A fresh loss-scale controller state in device memory (a uint8 tensor of DLS_STATE_BYTES)."""
    import torch
    if state is None:
        state = torch.empty(DLS_STATE_BYTES, dtype=torch.uint8, device=device if device is not None else "cuda")
    if state.dtype != torch.uint8 or state.numel() != DLS_STATE_BYTES or not state.is_cuda:
        raise TypeError("state must be a GPU uint8 tensor of %d bytes" % DLS_STATE_BYTES)
    _check(_lib.fmt_dls_init(state.data_ptr(), float(loss_scale), _stream_ptr(stream)), "fmt_dls_init")
    return state


def fmt_dls_step(hists, state, growth: float = 2.0, backoff: float = 0.5, interval: int = 2000,
                 min_scale: float = 1.0, max_scale: float = 2.0 ** 24, stream=None):
    """One step of the loss-scale controller / denormal-fraction monitor (Sec. II, Sec. V) on the
    statistics of the step's gradient tensors: ``hists`` is a GPU int64 tensor [count, 72] (rows as
    :func:`new_hist`), or None for a step without tensors.  Updates ``state`` on the device."""
    import torch
    count, hp = 0, None
    if hists is not None:
        if hists.dtype != torch.int64 or not hists.is_cuda or not hists.is_contiguous() or \
                hists.numel() % (8 + FMT_NBINS):
            raise TypeError("hists must be a contiguous GPU int64 tensor of [count, 72]")
        count = hists.numel() // (8 + FMT_NBINS)
        hp = hists.data_ptr() if count else None
    prm = _CDlsParams(growth, backoff, interval, min_scale, max_scale)
    _check(_lib.fmt_dls_step(hp, count, prm, state.data_ptr(), _stream_ptr(stream)), "fmt_dls_step")
    return state


def dls_state_to_dict(state) -> dict:
    """Copies a device fmt_dls_state_t to the host."""
    raw = bytes(state.cpu().numpy().tobytes())
    st = _CDlsState.from_buffer_copy(raw)
    return {name: getattr(st, name) for name, _ in _CDlsState._fields_}


def fmt_format_info(fmt) -> dict:
    """Closed-form constants of a format (Sec. III; Table I)."""
    mx, mn, md = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
    lo, hi = ctypes.c_int32(), ctypes.c_int32()
    _check(_lib.fmt_format_info(_cfmt(fmt), mx, mn, md, lo, hi), "fmt_format_info")
    return {"maxN": mx.value, "minN": mn.value, "minD": md.value, "Emin": lo.value, "Emax": hi.value}


def fmt_format_thresholds(fmt) -> dict:
    """Bit-pattern thresholds of the underflow, flush and overflow rules (host computation)."""
    out = (ctypes.c_uint32 * 3)()
    _check(_lib.fmt_format_thresholds(_cfmt(fmt), out), "fmt_format_thresholds")
    return {"t_zero": int(out[0]), "t_den": int(out[1]), "t_ovf": int(out[2])}


def fmt_scratch_bytes(stream=None) -> dict:
    """Bytes of library-owned scratch held for `stream` on the current device."""
    out = (ctypes.c_size_t * 3)()
    _check(_lib.fmt_scratch_bytes(_stream_ptr(stream), out), "fmt_scratch_bytes")
    return {"statistics": int(out[0]), "products": int(out[1]), "accumulators": int(out[2])}


def fmt_release_scratch() -> None:
    _check(_lib.fmt_release_scratch(), "fmt_release_scratch")


def raw_library() -> ctypes.CDLL:
    """The loaded C library (for tests of the C ABI itself)."""
    return _lib
