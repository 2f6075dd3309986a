"""C-ABI checks that need no GPU: the library loads, exports every symbol the header declares,
validates arguments before touching the device, and its host-side format logic (closed-form
constants, bit-pattern thresholds) agrees with the oracle for every supported (e, m)."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2103_15940_amd as fmt

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_header_symbols_are_exported():
    text = open(os.path.join(ROOT, "include", "fmt.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(fmt_[a-z0-9_]+)\s*\(", text))
    assert declared == set(fmt.EXPORTS)
    lib = ctypes.CDLL(fmt.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


def test_struct_layout():
    text = open(os.path.join(ROOT, "include", "fmt.h")).read()
    assert "uint64_t total, zero, underflow, denormal, normal, overflow, inf, nan;" in text
    assert ctypes.sizeof(fmt._CFormat) == 12
    assert 8 * (8 + fmt.FMT_NBINS) == 576
    assert ctypes.sizeof(fmt._CDlsState) == 80 and ctypes.sizeof(fmt._CDlsParams) == 20


def test_status_strings():
    for code in range(0, -9, -1):
        s = fmt.status_string(code)
        assert isinstance(s, str) and s and (code == 0 or s != "ok") and s != "unknown status"
    assert fmt.status_string(-99) == "unknown status"
    # the status a call returns instead of growing its scratch under stream capture is declared and named
    text = open(os.path.join(ROOT, "include", "fmt.h")).read()
    assert re.search(r"FMT_ERR_CAPTURE\s*=\s*-8", text)
    assert "captured" in fmt.status_string(-8)


@pytest.mark.parametrize("e,m", [(5, 10), (6, 9), (8, 7), (2, 1), (8, 23), (7, 16)])
def test_format_info_matches_oracle_closed_forms(e, m):
    assert fmt.fmt_format_info((e, m, True)) == oracle.format_constants(e, m)


def test_unsupported_formats_rejected():
    lib = fmt.raw_library()
    for e, m in [(1, 5), (9, 7), (5, 0), (5, 24), (-1, 3)]:
        with pytest.raises(fmt.FmtError) as ei:
            fmt.fmt_format_info((e, m, True))
        assert ei.value.status == -1
        # the compute entry points refuse the format before looking at any pointer
        assert lib.fmt_quantize(None, None, 0, fmt._CFormat(e, m, 1), None, -48, None) == -1
        assert lib.fmt_histogram(None, 0, fmt._CFormat(e, m, 1), None, -48, None) == -1
        assert lib.fmt_gemm(0, 0, 1, 1, 1, None, 1, None, 1, None, 1, fmt._CFormat(e, m, 1), None) == -1


def test_argument_validation_without_gpu():
    """All of these return before any HIP call, so they run on a host without a GPU."""
    lib = fmt.raw_library()
    f = fmt._CFormat(6, 9, 1)
    buf = (ctypes.c_float * 1024)()
    base = ctypes.addressof(buf)
    # null pointers
    assert lib.fmt_quantize(None, base, 4, f, None, -48, None) == -2
    assert lib.fmt_quantize(base, None, 4, f, None, -48, None) == -2
    assert lib.fmt_histogram(base, 4, f, None, -48, None) == -2
    assert lib.fmt_gemm(0, 0, 2, 2, 2, None, 2, base, 2, base + 64, 2, f, None) == -2
    # misaligned
    assert lib.fmt_quantize(base + 2, base, 4, f, None, -48, None) == -4
    assert lib.fmt_histogram(base, 4, f, base + 4, -48, None) == -4
    assert lib.fmt_gemm(0, 0, 2, 2, 2, base + 1, 2, base + 64, 2, base + 128, 2, f, None) == -4
    # exp_lo window
    assert lib.fmt_histogram(base, 4, f, base + 64, -193, None) == -5
    assert lib.fmt_histogram(base, 4, f, base + 64, 129, None) == -5
    # sizes
    assert lib.fmt_quantize(base, base, 1 << 40, f, None, -48, None) == -3
    assert lib.fmt_gemm(0, 0, -1, 2, 2, base, 2, base, 2, base, 2, f, None) == -3
    assert lib.fmt_gemm(0, 0, 2, 2, 4, base, 3, base + 64, 2, base + 128, 2, f, None) == -3     # lda < K
    assert lib.fmt_gemm(1, 0, 4, 2, 2, base, 3, base + 64, 2, base + 128, 2, f, None) == -3     # lda < M (A^T)
    assert lib.fmt_gemm(0, 1, 2, 2, 4, base, 4, base + 64, 3, base + 128, 2, f, None) == -3     # ldb < K (B^T)
    assert lib.fmt_gemm(0, 0, 2, 4, 2, base, 2, base + 64, 4, base + 128, 3, f, None) == -3     # ldc < N
    # aliasing
    assert lib.fmt_quantize(base, base + 8, 4, f, None, -48, None) == -6                          # partial overlap
    assert lib.fmt_gemm(0, 0, 2, 2, 2, base, 2, base + 64, 2, base + 8, 2, f, None) == -6
    # empty problems succeed without a launch
    assert lib.fmt_quantize(None, None, 0, f, None, -48, None) == 0
    assert lib.fmt_gemm(0, 0, 0, 5, 3, None, 3, None, 5, None, 5, f, None) == 0
    assert lib.fmt_gemm(0, 0, 5, 0, 3, None, 3, None, 1, None, 1, f, None) == 0
    # fmt_linear: X is M x K, W is N x K; same checks, plus the bias and the statistics record
    bad = fmt._CFormat(9, 7, 1)
    assert lib.fmt_linear(2, 2, 2, None, 2, None, 2, None, None, 2, bad, None, -48, None) == -1
    assert lib.fmt_linear(2, 2, 2, None, 2, base + 64, 2, None, base + 128, 2, f, None, -48, None) == -2
    assert lib.fmt_linear(2, 2, 2, base, 2, base + 64, 2, None, None, 2, f, None, -48, None) == -2
    assert lib.fmt_linear(2, 2, 4, base, 3, base + 64, 4, None, base + 128, 2, f, None, -48, None) == -3   # ldx < K
    assert lib.fmt_linear(2, 2, 4, base, 4, base + 64, 3, None, base + 128, 2, f, None, -48, None) == -3   # ldw < K
    assert lib.fmt_linear(2, 4, 2, base, 2, base + 64, 2, None, base + 128, 3, f, None, -48, None) == -3   # ldy < N
    assert lib.fmt_linear(2, 2, 2, base, 2, base + 64, 2, base + 33, base + 128, 2, f, None, -48, None) == -4
    assert lib.fmt_linear(2, 2, 2, base, 2, base + 64, 2, None, base + 128, 2, f, base + 196, -48, None) == -4
    assert lib.fmt_linear(2, 2, 2, base, 2, base + 64, 2, None, base + 128, 2, f, base + 192, 129, None) == -5
    assert lib.fmt_linear(2, 2, 2, base, 2, base + 64, 2, None, base + 8, 2, f, None, -48, None) == -6     # Y over X
    assert lib.fmt_linear(2, 2, 2, base, 2, base + 64, 2, base + 132, base + 128, 2, f, None, -48, None) == -6  # Y over b
    assert lib.fmt_linear(0, 2, 2, None, 2, None, 2, None, None, 2, f, None, -48, None) == 0
    # packed 16-bit codes: only formats with 1 + e + m <= 16 have them
    wide = fmt._CFormat(8, 8, 1)
    assert lib.fmt_pack16(base, base + 64, 4, wide, None, -48, None) == -1
    assert lib.fmt_unpack16(base, base + 64, 4, wide, None) == -1
    assert lib.fmt_linear_pack16(2, 2, 2, base, 2, base + 64, 2, None, base + 128, 2, wide, None, -48, None) == -1
    assert lib.fmt_pack16(base, None, 4, f, None, -48, None) == -2
    assert lib.fmt_pack16(base, base + 65, 4, f, None, -48, None) == -4            # codes need 2-byte alignment
    assert lib.fmt_pack16(base, base + 8, 4, f, None, -48, None) == -6             # codes over x
    assert lib.fmt_pack16(None, None, 0, f, None, -48, None) == 0
    assert lib.fmt_unpack16(None, base, 4, f, None) == -2
    assert lib.fmt_unpack16(base + 1, base + 64, 4, f, None) == -4
    assert lib.fmt_unpack16(base + 4, base, 4, f, None) == -6
    assert lib.fmt_unpack16(None, None, 0, f, None) == 0
    assert lib.fmt_linear_pack16(2, 2, 2, base, 2, base + 64, 2, None, None, 2, f, None, -48, None) == -2
    assert lib.fmt_linear_pack16(2, 4, 2, base, 2, base + 64, 2, None, base + 128, 3, f, None, -48, None) == -3   # ldy < N
    assert lib.fmt_linear_pack16(2, 2, 2, base, 2, base + 64, 2, None, base + 129, 2, f, None, -48, None) == -4
    assert lib.fmt_linear_pack16(2, 2, 2, base, 2, base + 64, 2, None, base + 4, 2, f, None, -48, None) == -6     # Y16 over X
    assert lib.fmt_linear_pack16(0, 2, 2, None, 2, None, 2, None, None, 2, f, None, -48, None) == 0
    # convolutions: geometry first, then pointers
    G = fmt._CConv2d
    ok = G(2, 3, 5, 5, 4, 3, 3, 1, 1, 1, 1)            # X 2x3x5x5 (150), W 4x3x3x3 (108), Y 2x4x5x5 (200)
    big = (ctypes.c_float * 4096)()
    b0 = ctypes.addressof(big)
    for fn in (lib.fmt_conv2d_fwd, lib.fmt_conv2d_dgrad, lib.fmt_conv2d_wgrad):
        assert fn(ok, b0, b0 + 4096, b0 + 8192, bad, None) == -1
        assert fn(G(2, 3, 5, 5, 4, 0, 3, 1, 1, 1, 1), b0, b0 + 4096, b0 + 8192, f, None) == -3   # r < 1
        assert fn(G(2, 3, 5, 5, 4, 3, 3, 1, 1, 0, 1), b0, b0 + 4096, b0 + 8192, f, None) == -3   # stride < 1
        assert fn(G(2, 3, 5, 5, 4, 3, 3, -1, 1, 1, 1), b0, b0 + 4096, b0 + 8192, f, None) == -3  # pad < 0
        assert fn(G(2, 3, 2, 5, 4, 7, 3, 1, 1, 1, 1), b0, b0 + 4096, b0 + 8192, f, None) == -3   # filter beyond the padded image
        assert fn(G(-1, 3, 5, 5, 4, 3, 3, 1, 1, 1, 1), b0, b0 + 4096, b0 + 8192, f, None) == -3
        assert fn(G(1 << 20, 1 << 10, 5, 5, 4, 3, 3, 1, 1, 1, 1), b0, b0 + 4096, b0 + 8192, f, None) == -3   # too large
        assert fn(ok, None, b0 + 4096, b0 + 8192, f, None) == -2
        assert fn(ok, b0, None, b0 + 8192, f, None) == -2
        assert fn(ok, b0, b0 + 4096, None, f, None) == -2
        assert fn(ok, b0 + 2, b0 + 4096, b0 + 8192, f, None) == -4
        assert fn(ok, b0, b0 + 4096, b0 + 16, f, None) == -6                                     # output over the first input
        assert fn(ok, b0, b0 + 4096, b0 + 4096 + 64, f, None) == -6                              # output over the second input
    assert lib.fmt_conv2d_fwd(G(0, 3, 5, 5, 4, 3, 3, 1, 1, 1, 1), None, None, None, f, None) == 0
    assert lib.fmt_conv2d_wgrad(G(2, 3, 5, 5, 0, 3, 3, 1, 1, 1, 1), None, None, None, f, None) == 0
    # loss-scale controller
    P = fmt._CDlsParams
    good = P(2.0, 0.5, 2000, 1.0, 65536.0)
    assert lib.fmt_dls_init(None, 1024.0, None) == -2
    assert lib.fmt_dls_init(base + 4, 1024.0, None) == -4
    for bad_scale in (0.0, -1.0, float("inf"), float("nan")):
        assert lib.fmt_dls_init(base, bad_scale, None) == -5
    assert lib.fmt_dls_step(base, 1, good, None, None) == -2
    assert lib.fmt_dls_step(None, 1, good, base, None) == -2
    assert lib.fmt_dls_step(base, -1, good, base + 1024, None) == -3
    assert lib.fmt_dls_step(base + 4, 1, good, base + 1024, None) == -4
    for bad_prm in (P(0.5, 0.5, 10, 1.0, 2.0), P(2.0, 0.0, 10, 1.0, 2.0), P(2.0, 1.5, 10, 1.0, 2.0), P(2.0, 0.5, 0, 1.0, 2.0),
                    P(2.0, 0.5, 10, 0.0, 2.0), P(2.0, 0.5, 10, 4.0, 2.0), P(float("nan"), 0.5, 10, 1.0, 2.0),
                    P(2.0, 0.5, 10, 1.0, float("inf"))):
        assert lib.fmt_dls_step(base, 1, bad_prm, base + 1024, None) == -5


def _f32(bits):
    return np.array(bits, dtype=np.uint32).view(np.float32)


def test_thresholds_match_oracle_for_every_format():
    """For all 7 x 23 supported (e, m): the three bit-pattern thresholds the kernels compare
    against sit exactly where the oracle's rounding changes class."""
    for e in range(2, 9):
        for m in range(1, 24):
            t = fmt.fmt_format_thresholds((e, m, True))
            c = oracle.format_constants(e, m)
            tz, td, to = t["t_zero"], t["t_den"], t["t_ovf"]
            probe = _f32([tz, tz + 1, td - 1, td, to - 1, to, max(tz, 1) - 1])
            q = oracle.quantize(probe, e, m, True).astype(np.float64)
            assert q[0] == 0.0, (e, m)
            assert q[1] > 0.0, (e, m)
            if td - 1 > 0:
                assert q[2] < c["minN"], (e, m)
            assert q[3] >= c["minN"], (e, m)
            assert np.isfinite(q[4]) and q[4] == c["maxN"], (e, m)
            assert np.isinf(q[5]), (e, m)
            assert tz < td < to <= 0x7F800000


def test_prepared_operand_calls_validate_without_gpu():
    """fmt_operand_bytes is a host computation; fmt_prepare and fmt_gemm_prepared check their arguments
    before any HIP call."""
    lib = fmt.raw_library()
    f = fmt._CFormat(6, 9, 1)
    n = ctypes.c_size_t()
    assert lib.fmt_operand_bytes(100, 200, f, ctypes.byref(n)) == 0
    # 100 rows pad to 256, 200 k to 224: at least 2 bytes per padded element, at most 6 plus the row scales and masks
    assert 256 * 224 * 2 <= n.value <= 256 * 224 * 6 + 16384 and n.value % 256 == 0
    bigger = ctypes.c_size_t()
    assert lib.fmt_operand_bytes(1000, 200, f, ctypes.byref(bigger)) == 0 and bigger.value > n.value
    assert lib.fmt_operand_bytes(0, 200, f, ctypes.byref(n)) == -3
    assert lib.fmt_operand_bytes(100, 1 << 31, f, ctypes.byref(n)) == -3
    assert lib.fmt_operand_bytes(100, 200, fmt._CFormat(9, 9, 1), ctypes.byref(n)) == -1
    assert lib.fmt_operand_bytes(100, 200, f, None) == -2
    buf = (ctypes.c_char * 1024)()
    base = (ctypes.addressof(buf) + 255) // 256 * 256
    op = fmt._COperand()
    x = ctypes.c_void_p(base)
    assert lib.fmt_prepare(None, 200, 0, 100, 200, f, base, 1 << 30, ctypes.byref(op), None) == -2
    assert lib.fmt_prepare(x, 100, 0, 100, 200, f, base + 512, 1 << 30, ctypes.byref(op), None) == -3      # ld < k
    assert lib.fmt_prepare(x, 200, 0, 100, 200, f, base + 512 + 4, 1 << 30, ctypes.byref(op), None) == -4  # data not 256-byte aligned
    assert lib.fmt_prepare(x, 200, 0, 100, 200, f, base + 512, 64, ctypes.byref(op), None) == -3           # buffer too small
    assert lib.fmt_prepare(x, 200, 0, 100, 200, f, base, 1 << 30, ctypes.byref(op), None) == -6            # buffer overlaps X
    need = ctypes.c_size_t()
    lib.fmt_operand_bytes(64, 96, f, ctypes.byref(need))
    a = fmt._COperand(base, need.value, 64, 96, f, 16)
    b = fmt._COperand(base + (1 << 20), need.value, 64, 64, f, 16)
    c = ctypes.c_void_p(base + (1 << 21))
    assert lib.fmt_gemm_prepared(ctypes.byref(a), ctypes.byref(b), c, 64, None) == -3        # k differs
    b.k = 96
    assert lib.fmt_gemm_prepared(ctypes.byref(a), None, c, 64, None) == -2
    assert lib.fmt_gemm_prepared(ctypes.byref(a), ctypes.byref(b), c, 32, None) == -3        # ldc < N
    b.format = fmt._CFormat(5, 10, 1)
    assert lib.fmt_gemm_prepared(ctypes.byref(a), ctypes.byref(b), c, 64, None) == -1        # formats differ
    b.format = f
    b.scheme = 2
    assert lib.fmt_gemm_prepared(ctypes.byref(a), ctypes.byref(b), c, 64, None) == -1        # schemes differ
    b.scheme = 16
    a.bytes = 128
    assert lib.fmt_gemm_prepared(ctypes.byref(a), ctypes.byref(b), c, 64, None) == -3        # operand buffer too small
    a.bytes = need.value
    assert lib.fmt_gemm_prepared(ctypes.byref(a), ctypes.byref(b), ctypes.c_void_p(base + 256), 64, None) == -6   # C overlaps A


def test_scratch_query_rejects_null():
    """fmt_scratch_bytes validates its output pointer before any GPU call."""
    lib = fmt.raw_library()
    assert lib.fmt_scratch_bytes(None, None) == -2          # FMT_ERR_NULL


def test_linear_prepared_validates_before_any_gpu_call():
    """fmt_linear_prepared: NULL operands and a mismatch of the two operands are refused on a host without a GPU."""
    import ctypes
    lib = fmt.raw_library()
    assert lib.fmt_linear_prepared(None, None, None, None, 0, None, -48, None) == -2     # FMT_ERR_NULL
    a = fmt._COperand(ctypes.c_void_p(256), 1 << 20, 32, 64, fmt._CFormat(6, 9, 1), 16)
    b = fmt._COperand(ctypes.c_void_p(1 << 30), 1 << 20, 32, 64, fmt._CFormat(5, 10, 1), 0)
    y = ctypes.c_void_p(1 << 40)
    assert lib.fmt_linear_prepared(ctypes.byref(a), ctypes.byref(b), None, y, 32, None, -48, None) == -1   # formats differ


def test_gemm_prepared_batch_validates_before_any_gpu_call():
    """fmt_gemm_prepared_batch: count, NULL arrays, mixed formats and overlapping results are refused on a host
    without a GPU; an empty batch succeeds."""
    import ctypes
    lib = fmt.raw_library()
    assert lib.fmt_gemm_prepared_batch(0, None, None, None, None, None) == 0
    assert lib.fmt_gemm_prepared_batch(-1, None, None, None, None, None) == -3
    assert lib.fmt_gemm_prepared_batch(2, None, None, None, None, None) == -2
    P = ctypes.POINTER(fmt._COperand)
    a = fmt._COperand(ctypes.c_void_p(256), 1 << 20, 32, 64, fmt._CFormat(6, 9, 1), 16)
    b = fmt._COperand(ctypes.c_void_p(1 << 30), 1 << 20, 32, 64, fmt._CFormat(6, 9, 1), 16)
    ah = fmt._COperand(ctypes.c_void_p(1 << 31), 1 << 20, 32, 64, fmt._CFormat(5, 10, 1), 0)
    bh = fmt._COperand(ctypes.c_void_p(1 << 32), 1 << 20, 32, 64, fmt._CFormat(5, 10, 1), 0)
    ld = (ctypes.c_int64 * 2)(32, 32)
    C = (ctypes.c_void_p * 2)(1 << 40, 1 << 41)
    A2, B2 = (P * 2)(ctypes.pointer(a), ctypes.pointer(ah)), (P * 2)(ctypes.pointer(b), ctypes.pointer(bh))
    assert lib.fmt_gemm_prepared_batch(2, A2, B2, C, ld, None) == -1          # two formats in one batch
    A1, B1 = (P * 2)(ctypes.pointer(a), ctypes.pointer(a)), (P * 2)(ctypes.pointer(b), ctypes.pointer(b))
    Csame = (ctypes.c_void_p * 2)(1 << 40, (1 << 40) + 64)
    assert lib.fmt_gemm_prepared_batch(2, A1, B1, Csame, ld, None) == -6      # results overlap
    Cop = (ctypes.c_void_p * 2)(1 << 40, 256)
    assert lib.fmt_gemm_prepared_batch(2, A1, B1, Cop, ld, None) == -6        # a result overlaps an operand
    A0 = (P * 2)(ctypes.pointer(a), None)
    assert lib.fmt_gemm_prepared_batch(2, A0, B1, C, ld, None) == -2


def test_prepare_pair_batch_validates_before_any_gpu_call():
    """fmt_prepare_pair_batch: count, NULL arrays and entries, small buffers and overlaps across matrices are
    refused on a host without a GPU; an empty batch succeeds."""
    import ctypes
    lib = fmt.raw_library()
    f = fmt._CFormat(6, 9, 1)
    none = [None] * 4
    assert lib.fmt_prepare_pair_batch(0, *none, f, None, None, None, None, None, None, None) == 0
    assert lib.fmt_prepare_pair_batch(-1, *none, f, None, None, None, None, None, None, None) == -3
    assert lib.fmt_prepare_pair_batch(5000, *none, f, None, None, None, None, None, None, None) == -3
    assert lib.fmt_prepare_pair_batch(2, *none, f, None, None, None, None, None, None, None) == -2
    n0, n1 = ctypes.c_size_t(), ctypes.c_size_t()
    assert lib.fmt_operand_bytes(64, 96, f, ctypes.byref(n0)) == 0 and lib.fmt_operand_bytes(96, 64, f, ctypes.byref(n1)) == 0
    vp2, i2, s2 = ctypes.c_void_p * 2, ctypes.c_int64 * 2, ctypes.c_size_t * 2
    X = vp2(1 << 30, 1 << 31)
    ld, rows, cols = i2(96, 96), i2(64, 64), i2(96, 96)
    data, data_t = vp2(1 << 40, 1 << 41), vp2(1 << 42, 1 << 43)
    by, by_t = s2(n0.value, n0.value), s2(n1.value, n1.value)
    op, op_t = (fmt._COperand * 2)(), (fmt._COperand * 2)()

    def call(**kw):
        a = dict(X=X, ld=ld, rows=rows, cols=cols, data=data, by=by, data_t=data_t, by_t=by_t)
        a.update(kw)
        return lib.fmt_prepare_pair_batch(2, a["X"], a["ld"], a["rows"], a["cols"], f, a["data"], a["by"], op, a["data_t"],
                                          a["by_t"], op_t, None)

    assert call(X=vp2(1 << 30, None)) == -2                                   # an entry without a matrix
    assert call(by=s2(n0.value, n0.value - 1)) == -3                          # second matrix: buffer too small
    assert call(ld=i2(96, 95)) == -3                                          # leading dimension below the columns
    assert call(data=vp2(1 << 40, (1 << 40) + 256)) == -6                     # two matrices' operands overlap
    assert call(data_t=vp2(1 << 42, (1 << 30) + 256)) == -6                   # an operand over the other matrix's input
    assert call(data=vp2(1 << 40, (1 << 41) + 1)) == -4                       # alignment
    assert lib.fmt_prepare_pair_batch(2, X, ld, rows, cols, fmt._CFormat(9, 9, 1), data, by, op, data_t, by_t, op_t, None) == -1


def test_quantize_prepare_pair_batch_validates_before_any_gpu_call():
    """fmt_quantize_prepare_pair_batch: count, NULL arrays and entries, formats without exponent planes are refused
    by the library itself only at launch, so here: the argument checks that need no GPU."""
    import ctypes
    lib = fmt.raw_library()
    f = fmt._CFormat(6, 9, 1)
    z = [None] * 4
    assert lib.fmt_quantize_prepare_pair_batch(0, *z, f, None, None, None, -48, None, None, None, None, None, None, None) == 0
    assert lib.fmt_quantize_prepare_pair_batch(-1, *z, f, None, None, None, -48, None, None, None, None, None, None, None) == -3
    assert lib.fmt_quantize_prepare_pair_batch(2, *z, f, None, None, None, -48, None, None, None, None, None, None, None) == -2
    n0, n1 = ctypes.c_size_t(), ctypes.c_size_t()
    assert lib.fmt_operand_bytes(64, 96, f, ctypes.byref(n0)) == 0 and lib.fmt_operand_bytes(96, 64, f, ctypes.byref(n1)) == 0
    vp2, i2, s2 = ctypes.c_void_p * 2, ctypes.c_int64 * 2, ctypes.c_size_t * 2
    base = dict(X=vp2(1 << 30, 1 << 31), ld=i2(96, 96), rows=i2(64, 64), cols=i2(96, 96), Y=vp2(1 << 33, 1 << 34),
                ldy=i2(96, 96), hist=vp2(1 << 35, 1 << 36), data=vp2(1 << 40, 1 << 41), by=s2(n0.value, n0.value),
                data_t=vp2(1 << 42, 1 << 43), by_t=s2(n1.value, n1.value))
    op, op_t = (fmt._COperand * 2)(), (fmt._COperand * 2)()

    def call(exp_lo=-48, **kw):
        a = dict(base)
        a.update(kw)
        return lib.fmt_quantize_prepare_pair_batch(2, a["X"], a["ld"], a["rows"], a["cols"], f, a["Y"], a["ldy"], a["hist"], exp_lo,
                                                   a["data"], a["by"], op, a["data_t"], a["by_t"], op_t, None)

    assert call(Y=vp2(1 << 33, None)) == -2                                   # an entry without a rounded copy
    assert call(hist=vp2(1 << 35, None)) == -2
    assert call(ldy=i2(96, 95)) == -3                                         # leading dimension below the columns
    assert call(hist=vp2(1 << 35, (1 << 36) + 4)) == -4                       # statistics record not 8-byte aligned
    assert call(Y=vp2(1 << 33, (1 << 31) + 64)) == -6                         # a rounded copy shifted over its input
    assert call(hist=vp2(1 << 35, 1 << 35)) == -6                             # two matrices, one record
    assert call(Y=vp2(1 << 33, (1 << 40) + 256)) == -6                        # a rounded copy over another operand
    assert call(exp_lo=10 ** 6) == -5                                         # window out of range

