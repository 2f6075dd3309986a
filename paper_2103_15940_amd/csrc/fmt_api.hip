// C-ABI entry points of libfmt: argument validation, format constants, scratch management.
// The arithmetic lives in fmt_stream.hip (quantize / histogram) and fmt_gemm.hip.
#include <vector>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <utility>

#include "fmt_internal.h"

namespace fmt {

void report_hip_error(const char *expr, const char *file, int line, hipError_t err)
{
    if (std::getenv("FMT_VERBOSE"))
        std::fprintf(stderr, "libfmt: %s failed at %s:%d: %s\n", expr, file, line, hipGetErrorString(err));
}

static bool format_ok(fmt_format_t f) { return f.e >= 2 && f.e <= 8 && f.m >= 1 && f.m <= 23; }

// Thresholds of the format on the fp32 bit pattern of |x| (Sec. III: Emax = bias,
// Emin = 1 - bias, minD = 2^(Emin-m); rounding is to nearest, ties to even).
int make_quant_params(fmt_format_t f, int32_t exp_lo, QuantParams *p)
{
    if (!format_ok(f)) return FMT_ERR_FORMAT;
    if (exp_lo < FMT_EXP_LO_MIN || exp_lo > FMT_EXP_LO_MAX) return FMT_ERR_RANGE;
    const int e = f.e, m = f.m;
    const int bias = (1 << (e - 1)) - 1;
    const int emin = 1 - bias, emax = bias;
    const uint32_t shift = 23u - (uint32_t)m;
    const uint32_t minn_bits = (uint32_t)(emin + 127) << 23;

    p->shift = shift;
    p->lsb_width = shift ? 1u : 0u;
    p->rbias = shift ? ((1u << (shift - 1)) - 1u) : 0u;
    p->nmask = ~((1u << shift) - 1u);
    p->mode = (e == 8) ? 1 : (m <= 22 ? 0 : 2);
    p->minn_bits = minn_bits;
    p->shift23 = shift << 23;
    const uint32_t cbits = (uint32_t)(emin + 23 - m + 127) << 23;  // 2^(Emin+23-m), a normal fp32 for every e, m
    std::memcpy(&p->cmagic, &cbits, sizeof(float));

    if (e < 8) {
        // minD/2 = 2^(Emin-m-1) is a normal fp32; below minN the fp32 spacing is 2^(Emin-24)
        p->t_zero = (uint32_t)(emin - m - 1 + 127) << 23;
        p->t_den = minn_bits - (1u << shift);
    } else {
        // Emin = -126 is fp32's own: inputs below minN are fp32 denormals, spacing 2^-149
        p->t_zero = (m <= 22) ? (1u << (22 - m)) : 0u;
        p->t_den = (m <= 22) ? minn_bits - (1u << (22 - m)) : minn_bits;
    }
    const uint32_t maxn_bits = ((uint32_t)(emax + 127) << 23) | (((1u << m) - 1u) << shift);
    p->t_ovf = (m <= 22) ? maxn_bits + (1u << (shift - 1)) : (uint32_t)(emax + 128) << 23;
    p->exp_lo = exp_lo;
    p->sign_pos = (uint32_t)(e + m);
    p->top_code = ((1u << e) - 1u) << m;
    return FMT_OK;
}

// ------------------------------------------------------------------ scratch
static std::mutex g_mu;
static std::map<std::pair<int, hipStream_t>, Scratch> g_scratch;

// Scratch only ever grows outside stream capture: a graph being recorded would keep the addresses of
// the buffer that is freed here, and hipMalloc / hipFree / hipMemset are not capturable anyway.
static int grow(hipStream_t stream, void **buf, size_t *have, size_t want)
{
    if (want <= *have) return FMT_OK;
    hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
    FMT_HIP_CHECK(hipStreamIsCapturing(stream, &capturing));
    if (capturing != hipStreamCaptureStatusNone) return FMT_ERR_CAPTURE;
    if (*buf) {
        FMT_HIP_CHECK(hipFree(*buf));  // synchronises the device: no kernel still uses it
        *buf = nullptr;
        *have = 0;
    }
    size_t cap = (want + 4095) & ~(size_t)4095;
    FMT_HIP_CHECK(hipMalloc(buf, cap));
    FMT_HIP_CHECK(hipMemset(*buf, 0, cap));   // the partial histogram records must start at zero
    FMT_HIP_CHECK(hipDeviceSynchronize());    // ... before a kernel on any stream adds to them
    *have = cap;
    return FMT_OK;
}

int get_scratch(hipStream_t stream, size_t hist_bytes, size_t gemm_bytes, Scratch *out)
{
    int dev = 0;
    FMT_HIP_CHECK(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lk(g_mu);
    Scratch &s = g_scratch[std::make_pair(dev, stream)];
    int rc = grow(stream, &s.hist_partials, &s.hist_bytes, hist_bytes);
    if (rc != FMT_OK) return rc;
    rc = grow(stream, &s.gemm_ws, &s.gemm_bytes, gemm_bytes);
    if (rc != FMT_OK) return rc;
    *out = s;
    return FMT_OK;
}

int get_acc_scratch(hipStream_t stream, size_t bytes, float **out)
{
    int dev = 0;
    FMT_HIP_CHECK(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lk(g_mu);
    Scratch &s = g_scratch[std::make_pair(dev, stream)];
    int rc = grow(stream, &s.acc_ws, &s.acc_bytes, bytes);
    if (rc != FMT_OK) return rc;
    *out = static_cast<float *>(s.acc_ws);
    return FMT_OK;
}

int device_cu_count(int *cus)
{
    static std::mutex mu;
    static std::map<int, int> cache;
    int dev = 0;
    FMT_HIP_CHECK(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lk(mu);
    auto it = cache.find(dev);
    if (it == cache.end()) {
        int n = 0;
        FMT_HIP_CHECK(hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev));
        it = cache.emplace(dev, n > 0 ? n : 256).first;
    }
    *cus = it->second;
    return FMT_OK;
}

static bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

static bool overlap(const void *a, size_t abytes, const void *b, size_t bbytes)
{
    uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
    return a0 < b0 + bbytes && b0 < a0 + abytes;
}

}  // namespace fmt

using namespace fmt;

extern "C" {

int fmt_quantize(const float *x, float *y, size_t n, fmt_format_t f,
                 fmt_hist_t *hist, int32_t exp_lo, void *stream)
{
    QuantParams p;
    int rc = make_quant_params(f, hist ? exp_lo : FMT_EXP_LO_DEFAULT, &p);
    if (rc != FMT_OK) return rc;
    if (n >= ((size_t)1 << 40)) return FMT_ERR_SHAPE;
    if (n > 0 && (!x || !y)) return FMT_ERR_NULL;
    if (!aligned(x, 4) || !aligned(y, 4) || !aligned(hist, 8)) return FMT_ERR_ALIGN;
    if (n > 0 && x != y && overlap(x, n * 4, y, n * 4)) return FMT_ERR_ALIAS;
    if (n == 0 && !hist) return FMT_OK;
    return launch_stream(x, y, n, p, f.denorm == 0, hist, static_cast<hipStream_t>(stream));
}

int fmt_quantize_static(const float *x, float *y, size_t n, fmt_format_t f,
                        fmt_hist_t *hist, int32_t exp_lo, void *stream)
{
    QuantParams p;
    int rc = make_quant_params(f, hist ? exp_lo : FMT_EXP_LO_DEFAULT, &p);
    if (rc != FMT_OK) return rc;
    if (n > FMT_STATIC_MAX_ELEMENTS) return FMT_ERR_SHAPE;
    if (n > 0 && (!x || !y)) return FMT_ERR_NULL;
    if (!aligned(x, 4) || !aligned(y, 4) || !aligned(hist, 8)) return FMT_ERR_ALIGN;
    if (n > 0 && x != y && overlap(x, n * 4, y, n * 4)) return FMT_ERR_ALIAS;
    if (n == 0 && !hist) return FMT_OK;
    return launch_stream_static(x, y, n, p, f.denorm == 0, hist, static_cast<hipStream_t>(stream));
}

int fmt_histogram(const float *x, size_t n, fmt_format_t f,
                  fmt_hist_t *hist, int32_t exp_lo, void *stream)
{
    QuantParams p;
    int rc = make_quant_params(f, exp_lo, &p);
    if (rc != FMT_OK) return rc;
    if (n >= ((size_t)1 << 40)) return FMT_ERR_SHAPE;
    if (!hist || (n > 0 && !x)) return FMT_ERR_NULL;
    if (!aligned(x, 4) || !aligned(hist, 8)) return FMT_ERR_ALIGN;
    return launch_stream(x, nullptr, n, p, false, hist, static_cast<hipStream_t>(stream));
}

// Shared argument checks of the two matrix products; *launch is set when a kernel must run.
static int check_gemm_args(int transA, int transB, int64_t M, int64_t N, int64_t K, const float *A, int64_t lda,
                           const float *B, int64_t ldb, float *C, int64_t ldc, bool *launch)
{
    *launch = false;
    const int64_t lim = (int64_t)1 << 31;
    if (M < 0 || N < 0 || K < 0 || M >= lim || N >= lim || K >= lim) return FMT_ERR_SHAPE;
    if (M == 0 || N == 0) return FMT_OK;
    if (!C) return FMT_ERR_NULL;
    if (K > 0 && (!A || !B)) return FMT_ERR_NULL;
    if (ldc < N) return FMT_ERR_SHAPE;
    if (K > 0) {
        if (lda < (transA ? M : K) || ldb < (transB ? K : N)) return FMT_ERR_SHAPE;
        if (lda >= lim || ldb >= lim) return FMT_ERR_SHAPE;
    }
    if (ldc >= lim) return FMT_ERR_SHAPE;
    if (!aligned(A, 4) || !aligned(B, 4) || !aligned(C, 4)) return FMT_ERR_ALIGN;
    if (K > 0) {
        const size_t abytes = 4 * (size_t)(((transA ? K : M) - 1) * lda + (transA ? M : K));
        const size_t bbytes = 4 * (size_t)(((transB ? N : K) - 1) * ldb + (transB ? K : N));
        const size_t cbytes = 4 * (size_t)((M - 1) * ldc + N);
        if (overlap(C, cbytes, A, abytes) || overlap(C, cbytes, B, bbytes)) return FMT_ERR_ALIAS;
    }
    *launch = true;
    return FMT_OK;
}

int fmt_gemm(int transA, int transB, int64_t M, int64_t N, int64_t K,
             const float *A, int64_t lda, const float *B, int64_t ldb,
             float *C, int64_t ldc, fmt_format_t f, void *stream)
{
    QuantParams p;
    int rc = make_quant_params(f, FMT_EXP_LO_DEFAULT, &p);
    if (rc != FMT_OK) return rc;
    bool launch = false;
    rc = check_gemm_args(transA, transB, M, N, K, A, lda, B, ldb, C, ldc, &launch);
    if (rc != FMT_OK || !launch) return rc;
    return launch_gemm(transA != 0, transB != 0, M, N, K, A, lda, B, ldb, C, ldc, f, p,
                       static_cast<hipStream_t>(stream));
}

int fmt_operand_bytes(int64_t rows, int64_t k, fmt_format_t f, size_t *bytes)
{
    if (!format_ok(f)) return FMT_ERR_FORMAT;
    if (!bytes) return FMT_ERR_NULL;
    const int64_t lim = (int64_t)1 << 31;
    if (rows < 1 || k < 1 || rows >= lim || k >= lim) return FMT_ERR_SHAPE;
    int scheme = 0;
    return prepared_operand_bytes(rows, k, f, bytes, &scheme);
}

int fmt_prepare(const float *X, int64_t ld, int trans, int64_t rows, int64_t k, fmt_format_t f,
                void *data, size_t bytes, fmt_operand_t *op, void *stream)
{
    QuantParams p;
    int rc = make_quant_params(f, FMT_EXP_LO_DEFAULT, &p);
    if (rc != FMT_OK) return rc;
    const int64_t lim = (int64_t)1 << 31;
    if (rows < 1 || k < 1 || rows >= lim || k >= lim) return FMT_ERR_SHAPE;
    if (!X || !data || !op) return FMT_ERR_NULL;
    if (ld < (trans ? rows : k) || ld >= lim) return FMT_ERR_SHAPE;
    if (!aligned(X, 4) || !aligned(data, 256)) return FMT_ERR_ALIGN;
    size_t need = 0;
    int scheme = 0;
    rc = prepared_operand_bytes(rows, k, f, &need, &scheme);
    if (rc != FMT_OK) return rc;
    if (bytes < need) return FMT_ERR_SHAPE;
    const size_t xbytes = 4 * (size_t)(((trans ? k : rows) - 1) * ld + (trans ? rows : k));
    if (overlap(data, need, X, xbytes)) return FMT_ERR_ALIAS;
    rc = launch_prepare_operand(X, ld, trans, rows, k, f, p, data, static_cast<hipStream_t>(stream));
    if (rc != FMT_OK) return rc;
    op->data = data;
    op->bytes = bytes;
    op->rows = rows;
    op->k = k;
    op->format = f;
    op->scheme = scheme;
    return FMT_OK;
}

// Everything fmt_prepare_pair checks before it launches; the bytes and schemes of the two operands come back.
static int check_pair(const float *X, int64_t ld, int64_t rows, int64_t cols, fmt_format_t f, const void *data, size_t bytes,
                      const void *data_t, size_t bytes_t, size_t *need, int *scheme, size_t *need_t, int *scheme_t)
{
    const int64_t lim = (int64_t)1 << 31;
    if (rows < 1 || cols < 1 || rows >= lim || cols >= lim) return FMT_ERR_SHAPE;
    if (!X || !data || !data_t) return FMT_ERR_NULL;
    if (ld < cols || ld >= lim) return FMT_ERR_SHAPE;
    if (!aligned(X, 4) || !aligned(data, 256) || !aligned(data_t, 256)) return FMT_ERR_ALIGN;
    int rc = prepared_operand_bytes(rows, cols, f, need, scheme);
    if (rc != FMT_OK) return rc;
    rc = prepared_operand_bytes(cols, rows, f, need_t, scheme_t);
    if (rc != FMT_OK) return rc;
    if (bytes < *need || bytes_t < *need_t) return FMT_ERR_SHAPE;
    const size_t xbytes = 4 * (size_t)((rows - 1) * ld + cols);
    if (overlap(data, *need, X, xbytes) || overlap(data_t, *need_t, X, xbytes) || overlap(data, *need, data_t, *need_t))
        return FMT_ERR_ALIAS;
    return FMT_OK;
}

int fmt_prepare_pair(const float *X, int64_t ld, int64_t rows, int64_t cols, fmt_format_t f,
                     void *data, size_t bytes, fmt_operand_t *op,
                     void *data_t, size_t bytes_t, fmt_operand_t *op_t, void *stream)
{
    QuantParams p;
    int rc = make_quant_params(f, FMT_EXP_LO_DEFAULT, &p);
    if (rc != FMT_OK) return rc;
    if (!op || !op_t) return FMT_ERR_NULL;
    size_t need = 0, need_t = 0;
    int scheme = 0, scheme_t = 0;
    rc = check_pair(X, ld, rows, cols, f, data, bytes, data_t, bytes_t, &need, &scheme, &need_t, &scheme_t);
    if (rc != FMT_OK) return rc;
    rc = launch_prepare_pair(X, ld, rows, cols, f, p, data, data_t, static_cast<hipStream_t>(stream));
    if (rc != FMT_OK) return rc;
    *op = fmt_operand_t{data, bytes, rows, cols, f, scheme};
    *op_t = fmt_operand_t{data_t, bytes_t, cols, rows, f, scheme_t};
    return FMT_OK;
}

int fmt_prepare_pair_batch(int64_t count, const float *const *X, const int64_t *ld, const int64_t *rows, const int64_t *cols,
                           fmt_format_t f, void *const *data, const size_t *bytes, fmt_operand_t *op,
                           void *const *data_t, const size_t *bytes_t, fmt_operand_t *op_t, void *stream)
{
    QuantParams p;
    int rc = make_quant_params(f, FMT_EXP_LO_DEFAULT, &p);
    if (rc != FMT_OK) return rc;
    if (count < 0 || count > 4096) return FMT_ERR_SHAPE;
    if (count == 0) return FMT_OK;
    if (!X || !ld || !rows || !cols || !data || !bytes || !op || !data_t || !bytes_t || !op_t) return FMT_ERR_NULL;
    std::vector<PrepPairItem> items((size_t)count);
    std::vector<size_t> need((size_t)count), need_t((size_t)count);
    std::vector<int> scheme((size_t)count), scheme_t((size_t)count);
    for (int64_t i = 0; i < count; ++i) {
        rc = check_pair(X[i], ld[i], rows[i], cols[i], f, data[i], bytes[i], data_t[i], bytes_t[i], &need[i], &scheme[i],
                        &need_t[i], &scheme_t[i]);
        if (rc != FMT_OK) return rc;
        items[i] = PrepPairItem{X[i], ld[i], rows[i], cols[i], data[i], data_t[i]};
    }
    // no operand may lie over another tensor's operands or over any of the inputs (the launches are shared)
    for (int64_t i = 0; i < count; ++i)
        for (int64_t j = 0; j < count; ++j) {
            if (j == i) continue;
            const size_t xbytes = 4 * (size_t)((rows[j] - 1) * ld[j] + cols[j]);
            if (overlap(data[i], need[i], X[j], xbytes) || overlap(data_t[i], need_t[i], X[j], xbytes) ||
                overlap(data[i], need[i], data[j], need[j]) || overlap(data[i], need[i], data_t[j], need_t[j]) ||
                overlap(data_t[i], need_t[i], data_t[j], need_t[j]))
                return FMT_ERR_ALIAS;
        }
    rc = launch_prepare_pair_batch(count, items.data(), f, p, static_cast<hipStream_t>(stream), nullptr);
    if (rc != FMT_OK) return rc;
    for (int64_t i = 0; i < count; ++i) {
        op[i] = fmt_operand_t{data[i], bytes[i], rows[i], cols[i], f, scheme[i]};
        op_t[i] = fmt_operand_t{data_t[i], bytes_t[i], cols[i], rows[i], f, scheme_t[i]};
    }
    return FMT_OK;
}

int fmt_quantize_prepare_pair_batch(int64_t count, const float *const *X, const int64_t *ld, const int64_t *rows,
                                    const int64_t *cols, fmt_format_t f, float *const *Y, const int64_t *ldy,
                                    fmt_hist_t *const *hist, int32_t exp_lo, void *const *data, const size_t *bytes,
                                    fmt_operand_t *op, void *const *data_t, const size_t *bytes_t, fmt_operand_t *op_t,
                                    void *stream)
{
    QuantParams p;
    int rc = make_quant_params(f, exp_lo, &p);
    if (rc != FMT_OK) return rc;
    if (count < 0 || count > 4096) return FMT_ERR_SHAPE;
    if (count == 0) return FMT_OK;
    if (!X || !ld || !rows || !cols || !Y || !ldy || !hist || !data || !bytes || !op || !data_t || !bytes_t || !op_t)
        return FMT_ERR_NULL;
    std::vector<PrepPairItem> items((size_t)count);
    std::vector<RoundItem> round((size_t)count);
    std::vector<size_t> need((size_t)count), need_t((size_t)count), xbytes((size_t)count), ybytes((size_t)count);
    std::vector<int> scheme((size_t)count), scheme_t((size_t)count);
    const int64_t lim = (int64_t)1 << 31;
    for (int64_t i = 0; i < count; ++i) {
        rc = check_pair(X[i], ld[i], rows[i], cols[i], f, data[i], bytes[i], data_t[i], bytes_t[i], &need[i], &scheme[i],
                        &need_t[i], &scheme_t[i]);
        if (rc != FMT_OK) return rc;
        if (!Y[i] || !hist[i]) return FMT_ERR_NULL;
        if (ldy[i] < cols[i] || ldy[i] >= lim) return FMT_ERR_SHAPE;
        if (!aligned(Y[i], 4) || !aligned(hist[i], 8)) return FMT_ERR_ALIGN;
        xbytes[i] = 4 * (size_t)((rows[i] - 1) * ld[i] + cols[i]);
        ybytes[i] = 4 * (size_t)((rows[i] - 1) * ldy[i] + cols[i]);
        // in place (same address, same leading dimension) is fine: an element is read and written by one thread
        if (!(Y[i] == X[i] && ldy[i] == ld[i]) && overlap(Y[i], ybytes[i], X[i], xbytes[i])) return FMT_ERR_ALIAS;
        if (overlap(Y[i], ybytes[i], data[i], need[i]) || overlap(Y[i], ybytes[i], data_t[i], need_t[i]) ||
            overlap(hist[i], sizeof(fmt_hist_t), Y[i], ybytes[i]) || overlap(hist[i], sizeof(fmt_hist_t), data[i], need[i]) ||
            overlap(hist[i], sizeof(fmt_hist_t), data_t[i], need_t[i]))
            return FMT_ERR_ALIAS;
        items[i] = PrepPairItem{X[i], ld[i], rows[i], cols[i], data[i], data_t[i]};
        round[i] = RoundItem{Y[i], ldy[i], hist[i]};
    }
    // nothing written for one matrix may lie over anything of another
    for (int64_t i = 0; i < count; ++i)
        for (int64_t j = 0; j < count; ++j) {
            if (j == i) continue;
            const void *out[4] = {data[i], data_t[i], Y[i], hist[i]};
            const size_t outb[4] = {need[i], need_t[i], ybytes[i], sizeof(fmt_hist_t)};
            const void *other[5] = {X[j], data[j], data_t[j], Y[j], hist[j]};
            const size_t otherb[5] = {xbytes[j], need[j], need_t[j], ybytes[j], sizeof(fmt_hist_t)};
            for (int a = 0; a < 4; ++a)
                for (int b = 0; b < 5; ++b)
                    if (overlap(out[a], outb[a], other[b], otherb[b])) return FMT_ERR_ALIAS;
        }
    rc = launch_prepare_pair_batch(count, items.data(), f, p, static_cast<hipStream_t>(stream), round.data());
    if (rc != FMT_OK) return rc;
    for (int64_t i = 0; i < count; ++i) {
        op[i] = fmt_operand_t{data[i], bytes[i], rows[i], cols[i], f, scheme[i]};
        op_t[i] = fmt_operand_t{data_t[i], bytes_t[i], cols[i], rows[i], f, scheme_t[i]};
    }
    return FMT_OK;
}

// Everything fmt_gemm_prepared checks before it launches.
static int check_prepared(const fmt_operand_t *A, const fmt_operand_t *B, const float *C, int64_t ldc)
{
    if (!A || !B) return FMT_ERR_NULL;
    if (!format_ok(A->format)) return FMT_ERR_FORMAT;
    if (A->format.e != B->format.e || A->format.m != B->format.m || (A->format.denorm != 0) != (B->format.denorm != 0) ||
        A->scheme != B->scheme)
        return FMT_ERR_FORMAT;
    const int64_t lim = (int64_t)1 << 31;
    if (A->rows < 1 || B->rows < 1 || A->k < 1 || A->rows >= lim || B->rows >= lim || A->k >= lim) return FMT_ERR_SHAPE;
    if (A->k != B->k || ldc < B->rows || ldc >= lim) return FMT_ERR_SHAPE;
    if (!A->data || !B->data || !C) return FMT_ERR_NULL;
    if (!aligned(A->data, 256) || !aligned(B->data, 256) || !aligned(C, 4)) return FMT_ERR_ALIGN;
    size_t na = 0, nb = 0;
    int sa = 0, sb = 0;
    int rc = prepared_operand_bytes(A->rows, A->k, A->format, &na, &sa);
    if (rc != FMT_OK) return rc;
    rc = prepared_operand_bytes(B->rows, B->k, B->format, &nb, &sb);
    if (rc != FMT_OK) return rc;
    if (sa != A->scheme || sb != B->scheme) return FMT_ERR_FORMAT;     // prepared under another scheme selection
    if (A->bytes < na || B->bytes < nb) return FMT_ERR_SHAPE;
    const size_t cbytes = 4 * (size_t)((A->rows - 1) * ldc + B->rows);
    if (overlap(C, cbytes, A->data, na) || overlap(C, cbytes, B->data, nb)) return FMT_ERR_ALIAS;
    return FMT_OK;
}

int fmt_gemm_prepared(const fmt_operand_t *A, const fmt_operand_t *B, float *C, int64_t ldc, void *stream)
{
    const int rc = check_prepared(A, B, C, ldc);
    if (rc != FMT_OK) return rc;
    return launch_gemm_prepared(A->data, B->data, A->rows, B->rows, A->k, A->scheme, A->format, C, ldc,
                                static_cast<hipStream_t>(stream));
}

int fmt_gemm_prepared_batch(int64_t count, const fmt_operand_t *const *A, const fmt_operand_t *const *B, float *const *C,
                            const int64_t *ldc, void *stream)
{
    if (count < 0 || count > 4096) return FMT_ERR_SHAPE;
    if (count == 0) return FMT_OK;
    if (!A || !B || !C || !ldc) return FMT_ERR_NULL;
    std::vector<BatchItem> items((size_t)count);
    for (int64_t i = 0; i < count; ++i) {
        const int rc = check_prepared(A[i], B[i], C[i], ldc[i]);
        if (rc != FMT_OK) return rc;
        const fmt_operand_t &a = *A[i], &a0 = *A[0];
        if (a.format.e != a0.format.e || a.format.m != a0.format.m || (a.format.denorm != 0) != (a0.format.denorm != 0) ||
            a.scheme != a0.scheme)
            return FMT_ERR_FORMAT;
        items[(size_t)i] = BatchItem{a.data, B[i]->data, a.rows, B[i]->rows, a.k, C[i], ldc[i]};
    }
    // no result may overlap another result or any operand of the batch (the products run concurrently)
    auto cbytes = [&](int64_t i) { return 4 * (size_t)((A[i]->rows - 1) * ldc[i] + B[i]->rows); };
    for (int64_t i = 0; i < count; ++i)
        for (int64_t j = 0; j < count; ++j) {
            if (j > i && overlap(C[i], cbytes(i), C[j], cbytes(j))) return FMT_ERR_ALIAS;
            if (j != i && (overlap(C[i], cbytes(i), A[j]->data, A[j]->bytes) || overlap(C[i], cbytes(i), B[j]->data, B[j]->bytes)))
                return FMT_ERR_ALIAS;
        }
    return launch_gemm_prepared_batch((int)count, items.data(), A[0]->scheme, A[0]->format, static_cast<hipStream_t>(stream));
}

int fmt_linear_prepared(const fmt_operand_t *X, const fmt_operand_t *W, const float *b, float *Y, int64_t ldy,
                        fmt_hist_t *hist, int32_t exp_lo, void *stream)
{
    int rc = check_prepared(X, W, Y, ldy);
    if (rc != FMT_OK) return rc;
    QuantParams p;
    rc = make_quant_params(X->format, hist ? exp_lo : FMT_EXP_LO_DEFAULT, &p);
    if (rc != FMT_OK) return rc;
    if (hist && !aligned(hist, 8)) return FMT_ERR_ALIGN;
    if (b) {
        if (!aligned(b, 4)) return FMT_ERR_ALIGN;
        if (overlap(Y, 4 * (size_t)((X->rows - 1) * ldy + W->rows), b, 4 * (size_t)W->rows)) return FMT_ERR_ALIAS;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    rc = launch_gemm_prepared(X->data, W->data, X->rows, W->rows, X->k, X->scheme, X->format, Y, ldy, s);
    if (rc != FMT_OK) return rc;
    return launch_linear_epilogue(Y, ldy, X->rows, W->rows, b, p, X->format.denorm == 0, hist, s);
}

int fmt_gemm_fmac8(int transA, int transB, int64_t M, int64_t N, int64_t K,
                   const float *A, int64_t lda, const float *B, int64_t ldb,
                   float *C, int64_t ldc, fmt_format_t f, void *stream)
{
    QuantParams p;
    int rc = make_quant_params(f, FMT_EXP_LO_DEFAULT, &p);
    if (rc != FMT_OK) return rc;
    bool launch = false;
    rc = check_gemm_args(transA, transB, M, N, K, A, lda, B, ldb, C, ldc, &launch);
    if (rc != FMT_OK || !launch) return rc;
    return launch_gemm_fmac8(transA != 0, transB != 0, M, N, K, A, lda, B, ldb, C, ldc, f, p,
                             static_cast<hipStream_t>(stream));
}

int fmt_linear(int64_t M, int64_t N, int64_t K,
               const float *X, int64_t ldx, const float *W, int64_t ldw, const float *b,
               float *Y, int64_t ldy, fmt_format_t f,
               fmt_hist_t *hist, int32_t exp_lo, void *stream)
{
    QuantParams p;
    int rc = make_quant_params(f, hist ? exp_lo : FMT_EXP_LO_DEFAULT, &p);
    if (rc != FMT_OK) return rc;
    if (hist && !aligned(hist, 8)) return FMT_ERR_ALIGN;
    bool launch = false;
    rc = check_gemm_args(0, 1, M, N, K, X, ldx, W, ldw, Y, ldy, &launch);
    if (rc != FMT_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (!launch) return launch_linear_epilogue(Y, ldy, 0, 0, nullptr, p, f.denorm == 0, hist, s);
    if (b) {
        if (!aligned(b, 4)) return FMT_ERR_ALIGN;
        if (overlap(Y, 4 * (size_t)((M - 1) * ldy + N), b, 4 * (size_t)N)) return FMT_ERR_ALIAS;
    }
    rc = launch_gemm(0, 1, M, N, K, X, ldx, W, ldw, Y, ldy, f, p, s);
    if (rc != FMT_OK) return rc;
    return launch_linear_epilogue(Y, ldy, M, N, b, p, f.denorm == 0, hist, s);
}

static bool has_code16(fmt_format_t f) { return 1 + f.e + f.m <= 16; }

int fmt_pack16(const float *x, uint16_t *codes, size_t n, fmt_format_t f,
               fmt_hist_t *hist, int32_t exp_lo, void *stream)
{
    QuantParams p;
    int rc = make_quant_params(f, hist ? exp_lo : FMT_EXP_LO_DEFAULT, &p);
    if (rc != FMT_OK) return rc;
    if (!has_code16(f)) return FMT_ERR_FORMAT;
    if (n >= ((size_t)1 << 40)) return FMT_ERR_SHAPE;
    if (n > 0 && (!x || !codes)) return FMT_ERR_NULL;
    if (!aligned(x, 4) || !aligned(codes, 2) || !aligned(hist, 8)) return FMT_ERR_ALIGN;
    if (n > 0 && overlap(x, n * 4, codes, n * 2)) return FMT_ERR_ALIAS;
    if (n == 0 && !hist) return FMT_OK;
    return launch_stream(x, codes, n, p, f.denorm == 0, hist, static_cast<hipStream_t>(stream), true);
}

int fmt_unpack16(const uint16_t *codes, float *y, size_t n, fmt_format_t f, void *stream)
{
    QuantParams p;
    int rc = make_quant_params(f, FMT_EXP_LO_DEFAULT, &p);
    if (rc != FMT_OK) return rc;
    if (!has_code16(f)) return FMT_ERR_FORMAT;
    if (n >= ((size_t)1 << 40)) return FMT_ERR_SHAPE;
    if (n > 0 && (!codes || !y)) return FMT_ERR_NULL;
    if (!aligned(codes, 2) || !aligned(y, 4)) return FMT_ERR_ALIGN;
    if (n > 0 && overlap(codes, n * 2, y, n * 4)) return FMT_ERR_ALIAS;
    return launch_unpack16(codes, y, n, p, static_cast<hipStream_t>(stream));
}

int fmt_linear_pack16(int64_t M, int64_t N, int64_t K,
                      const float *X, int64_t ldx, const float *W, int64_t ldw, const float *b,
                      uint16_t *Y16, int64_t ldy, fmt_format_t f,
                      fmt_hist_t *hist, int32_t exp_lo, void *stream)
{
    QuantParams p;
    int rc = make_quant_params(f, hist ? exp_lo : FMT_EXP_LO_DEFAULT, &p);
    if (rc != FMT_OK) return rc;
    if (!has_code16(f)) return FMT_ERR_FORMAT;
    if (hist && !aligned(hist, 8)) return FMT_ERR_ALIGN;
    const int64_t lim = (int64_t)1 << 31;
    if (M < 0 || N < 0 || K < 0 || M >= lim || N >= lim || K >= lim) return FMT_ERR_SHAPE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (M == 0 || N == 0) return launch_linear_epilogue_pack16(nullptr, 0, Y16, ldy, 0, 0, nullptr, p, f.denorm == 0, hist, s);
    if (!Y16 || (K > 0 && (!X || !W))) return FMT_ERR_NULL;
    if (ldy < N || ldy >= lim) return FMT_ERR_SHAPE;
    if (K > 0 && (ldx < K || ldw < K || ldx >= lim || ldw >= lim)) return FMT_ERR_SHAPE;
    if (!aligned(X, 4) || !aligned(W, 4) || !aligned(Y16, 2) || !aligned(b, 4)) return FMT_ERR_ALIGN;
    const size_t ybytes = 2 * (size_t)((M - 1) * ldy + N);
    if (K > 0 && (overlap(Y16, ybytes, X, 4 * (size_t)((M - 1) * ldx + K)) ||
                  overlap(Y16, ybytes, W, 4 * (size_t)((N - 1) * ldw + K))))
        return FMT_ERR_ALIAS;
    if (b && overlap(Y16, ybytes, b, 4 * (size_t)N)) return FMT_ERR_ALIAS;
    float *acc = nullptr;
    rc = get_acc_scratch(s, (size_t)M * (size_t)N * sizeof(float), &acc);
    if (rc != FMT_OK) return rc;
    rc = launch_gemm(0, 1, M, N, K, X, ldx, W, ldw, acc, N, f, p, s);
    if (rc != FMT_OK) return rc;
    return launch_linear_epilogue_pack16(acc, N, Y16, ldy, M, N, b, p, f.denorm == 0, hist, s);
}

// Validates a convolution call; *launch is false when the output is empty.  which: 0 forward
// (a = X, b = W, out = Y), 1 dgrad (dY, W, dX), 2 wgrad (dY, X, dW).
static int check_conv_args(int which, const fmt_conv2d_t &g, const float *a, const float *b, float *out, bool *launch)
{
    *launch = false;
    const int64_t lim = (int64_t)1 << 31;
    if (g.n < 0 || g.c < 0 || g.k < 0 || g.h < 1 || g.w < 1 || g.r < 1 || g.s < 1) return FMT_ERR_SHAPE;
    if (g.pad_h < 0 || g.pad_w < 0 || g.stride_h < 1 || g.stride_w < 1) return FMT_ERR_SHAPE;
    if ((int64_t)g.h + 2 * (int64_t)g.pad_h < g.r || (int64_t)g.w + 2 * (int64_t)g.pad_w < g.s) return FMT_ERR_SHAPE;
    if (g.pad_h >= (1 << 20) || g.pad_w >= (1 << 20)) return FMT_ERR_SHAPE;
    const int64_t P = (g.h + 2 * g.pad_h - g.r) / g.stride_h + 1, Q = (g.w + 2 * g.pad_w - g.s) / g.stride_w + 1;
    const int64_t hw = (int64_t)g.h * g.w, pq = P * Q, rs = (int64_t)g.r * g.s;
    if (hw >= lim || pq >= lim || rs >= lim) return FMT_ERR_SHAPE;
    const int64_t x_elems = (int64_t)g.n * g.c, y_elems = (int64_t)g.n * g.k, w_elems = (int64_t)g.k * g.c;
    if (x_elems >= lim || y_elems >= lim || w_elems >= lim) return FMT_ERR_SHAPE;
    if (x_elems * hw >= lim || y_elems * pq >= lim || w_elems * rs >= lim) return FMT_ERR_SHAPE;
    if ((int64_t)g.n * pq >= lim || (int64_t)g.n * hw >= lim || g.c * rs >= lim || g.k * rs >= lim) return FMT_ERR_SHAPE;
    const size_t xb = 4 * (size_t)(x_elems * hw), yb = 4 * (size_t)(y_elems * pq), wb = 4 * (size_t)(w_elems * rs);
    const size_t ab = which == 0 ? xb : yb, bb = which == 2 ? xb : wb, ob = which == 0 ? yb : (which == 1 ? xb : wb);
    if (ob == 0) return FMT_OK;
    if (!out || (ab > 0 && !a) || (bb > 0 && !b)) return FMT_ERR_NULL;
    if (!aligned(a, 4) || !aligned(b, 4) || !aligned(out, 4)) return FMT_ERR_ALIGN;
    if ((ab > 0 && overlap(out, ob, a, ab)) || (bb > 0 && overlap(out, ob, b, bb))) return FMT_ERR_ALIAS;
    *launch = true;
    return FMT_OK;
}

static int conv_entry(int which, const fmt_conv2d_t &g, const float *a, const float *b, float *out, fmt_format_t f,
                      void *stream)
{
    QuantParams p;
    int rc = make_quant_params(f, FMT_EXP_LO_DEFAULT, &p);
    if (rc != FMT_OK) return rc;
    bool launch = false;
    rc = check_conv_args(which, g, a, b, out, &launch);
    if (rc != FMT_OK || !launch) return rc;
    return launch_conv2d(which, g, a, b, out, f, p, static_cast<hipStream_t>(stream));
}

int fmt_conv2d_fwd(fmt_conv2d_t g, const float *X, const float *W, float *Y, fmt_format_t f, void *stream)
{
    return conv_entry(0, g, X, W, Y, f, stream);
}

int fmt_conv2d_dgrad(fmt_conv2d_t g, const float *dY, const float *W, float *dX, fmt_format_t f, void *stream)
{
    return conv_entry(1, g, dY, W, dX, f, stream);
}

int fmt_conv2d_wgrad(fmt_conv2d_t g, const float *dY, const float *X, float *dW, fmt_format_t f, void *stream)
{
    return conv_entry(2, g, dY, X, dW, f, stream);
}

int fmt_dls_init(fmt_dls_state_t *state, float loss_scale, void *stream)
{
    if (!state) return FMT_ERR_NULL;
    if (!aligned(state, 8)) return FMT_ERR_ALIGN;
    if (!(loss_scale > 0.0f) || !std::isfinite(loss_scale)) return FMT_ERR_RANGE;
    return launch_dls_init(state, loss_scale, static_cast<hipStream_t>(stream));
}

int fmt_dls_step(const fmt_hist_t *hists, int64_t count, fmt_dls_params_t prm,
                 fmt_dls_state_t *state, void *stream)
{
    if (count < 0 || count >= ((int64_t)1 << 40)) return FMT_ERR_SHAPE;
    if (!state || (count > 0 && !hists)) return FMT_ERR_NULL;
    if (!aligned(state, 8) || !aligned(hists, 8)) return FMT_ERR_ALIGN;
    const bool ok = std::isfinite(prm.growth) && std::isfinite(prm.backoff) && std::isfinite(prm.min_scale) &&
                    std::isfinite(prm.max_scale) && prm.growth >= 1.0f && prm.backoff > 0.0f && prm.backoff <= 1.0f &&
                    prm.interval >= 1 && prm.min_scale > 0.0f && prm.min_scale <= prm.max_scale;
    if (!ok) return FMT_ERR_RANGE;
    return launch_dls_step(hists, count, prm, state, static_cast<hipStream_t>(stream));
}

int fmt_format_info(fmt_format_t f, double *maxN, double *minN, double *minD,
                    int32_t *Emin, int32_t *Emax)
{
    if (!format_ok(f)) return FMT_ERR_FORMAT;
    const int bias = (1 << (f.e - 1)) - 1;
    const int emin = 1 - bias, emax = bias;
    if (Emin) *Emin = emin;
    if (Emax) *Emax = emax;
    if (minN) *minN = std::ldexp(1.0, emin);
    if (minD) *minD = std::ldexp(1.0, emin - f.m);
    if (maxN) *maxN = std::ldexp(2.0 - std::ldexp(1.0, -f.m), emax);
    return FMT_OK;
}

int fmt_format_thresholds(fmt_format_t f, uint32_t *out)
{
    QuantParams p;
    int rc = make_quant_params(f, FMT_EXP_LO_DEFAULT, &p);
    if (rc != FMT_OK) return rc;
    if (!out) return FMT_ERR_NULL;
    out[0] = p.t_zero;
    out[1] = p.t_den;
    out[2] = p.t_ovf;
    return FMT_OK;
}

int fmt_scratch_bytes(void *stream, size_t *out)
{
    if (out == nullptr) return FMT_ERR_NULL;
    int dev = 0;
    FMT_HIP_CHECK(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lk(g_mu);
    out[0] = out[1] = out[2] = 0;
    auto it = g_scratch.find(std::make_pair(dev, static_cast<hipStream_t>(stream)));
    if (it != g_scratch.end()) {
        out[0] = it->second.hist_bytes;
        out[1] = it->second.gemm_bytes;
        out[2] = it->second.acc_bytes;
    }
    return FMT_OK;
}

int fmt_release_scratch(void)
{
    int dev = 0;
    FMT_HIP_CHECK(hipGetDevice(&dev));
    FMT_HIP_CHECK(hipDeviceSynchronize());
    std::lock_guard<std::mutex> lk(g_mu);
    for (auto it = g_scratch.begin(); it != g_scratch.end();) {
        if (it->first.first == dev) {
            if (it->second.hist_partials) (void)hipFree(it->second.hist_partials);
            if (it->second.acc_ws) (void)hipFree(it->second.acc_ws);
            if (it->second.gemm_ws) (void)hipFree(it->second.gemm_ws);
            it = g_scratch.erase(it);
        } else {
            ++it;
        }
    }
    return FMT_OK;
}

const char *fmt_status_string(int status)
{
    switch (status) {
        case FMT_OK: return "ok";
        case FMT_ERR_FORMAT: return "unsupported format: need 2 <= e <= 8 and 1 <= m <= 23";
        case FMT_ERR_NULL: return "a required pointer is NULL";
        case FMT_ERR_SHAPE: return "bad shape: negative or too large dimension, or leading dimension too small";
        case FMT_ERR_ALIGN: return "a data pointer is not aligned to its element size";
        case FMT_ERR_RANGE: return "a scalar parameter is out of range (exp_lo window, loss-scale parameters)";
        case FMT_ERR_ALIAS: return "output overlaps an input";
        case FMT_ERR_HIP: return "a HIP runtime call failed";
        case FMT_ERR_CAPTURE: return "library scratch would have to grow while the stream is being captured into a graph";
        default: return "unknown status";
    }
}

}  // extern "C"
