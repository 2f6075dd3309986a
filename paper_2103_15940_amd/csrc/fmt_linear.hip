// Output roundings of the quantized Linear layer (Sec. IV-A): Y = R( R(acc) + R(b) ), where acc
// is the fp32-accumulated product of the rounded operands (what fmt_gemm leaves in Y), b the bias
// (one value per output column), "+" a single-precision addition and R the rounding to the
// format.  The statistics of Sec. V are taken of t = R(acc) + R(b), the tensor that enters the
// last rounding, in the same pass.
//
// With PACK the accumulators come from a buffer of their own and the result is stored as the
// format's 16-bit codes (Sec. III): 6 bytes per element instead of 8.
//
// HBM-bound: one read and one write of the M x N output (8 bytes per element), the bias row is
// rounded once per thread and kept in registers.  A workgroup owns a strip of 1024 columns
// (256 lanes x 4) and a range of rows; rows are walked four at a time so that four 128-bit loads
// are in flight per lane.
#include "fmt_hist.h"
#include "fmt_internal.h"
#include "fmt_quant.h"

namespace fmt {

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
constexpr int kLBlock = 256;
constexpr int kLCopies = 32;
constexpr int kLRows = 4;                 // rows per trip (independent loads in flight)

// A: accumulators (leading dimension lda); Y: output, fp32 patterns (== A, in place) or, with PACK,
// uint16_t codes.  VEC: 128-bit loads and full-width stores are possible for whole lanes.
template <int MODE, bool FTZ, bool HIST, bool DEEP, bool VEC, bool PACK>
__global__ __launch_bounds__(kLBlock) void linear_epilogue_kernel(const uint32_t *A, int64_t lda, void *Yv, int64_t ldy,
                                                                  int M, int N, const uint32_t *__restrict__ bias,
                                                                  int rows_per_wg, QuantParams p,
                                                                  unsigned long long *__restrict__ partials)
{
    constexpr int EM = MODE == kModeInteger ? kModeInteger : kModeMagic;
    uint32_t *Y = static_cast<uint32_t *>(Yv);
    uint16_t *Y16 = static_cast<uint16_t *>(Yv);
    __shared__ __attribute__((aligned(16))) uint32_t tbl[HIST ? kHistRows * kLCopies : 4];
    __shared__ uint32_t s_bins[FMT_NBINS];
    __shared__ uint32_t s_cls[8];
    const uint32_t tid = threadIdx.x;
    const uint32_t copy = tid & (kLCopies - 1);
    Counts w;
    if (HIST) hist_begin<kLCopies, kLBlock>(tbl, s_bins, s_cls, tid);

    const int64_t c0 = ((int64_t)blockIdx.x * kLBlock + (int64_t)tid) * 4;
    const int ncol = N - c0 < 4 ? (N - c0 < 0 ? 0 : (int)(N - c0)) : 4;      // valid columns of this lane
    float rb[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
        rb[j] = (bias != nullptr && j < ncol) ? __uint_as_float(quantize_bits<MODE, FTZ>(bias[c0 + j], p)) : 0.0f;
    const bool has_bias = bias != nullptr;

    const int r_begin = blockIdx.y * rows_per_wg;
    const int r_end = min(M, r_begin + rows_per_wg);
    const bool full = VEC && ncol == 4;       // 128-bit accesses for this lane
    for (int r = r_begin; r < r_end; r += kLRows) {
        u32x4 v[kLRows];
#pragma unroll
        for (int i = 0; i < kLRows; ++i) {
            v[i] = u32x4{0u, 0u, 0u, 0u};
            if (r + i < r_end) {
                const uint32_t *row = A + (size_t)(r + i) * lda + c0;
                if (full) {
                    v[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(row));
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (j < ncol) v[i][j] = row[j];
                }
            }
        }
#pragma unroll
        for (int i = 0; i < kLRows; ++i) {
            const bool rv = r + i < r_end;
            u32x4 o;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                uint32_t t = quantize_bits<MODE, FTZ>(v[i][j], p);
                // single-precision addition of two values of the format; without a bias t = R(acc)
                if (has_bias) t = __float_as_uint(__fadd_rn(__uint_as_float(t), rb[j]));
                if (HIST) account<DEEP, kLCopies>(t & 0x7FFFFFFFu, rv && j < ncol, p, tbl, copy, w);
                o[j] = quantize_bits<MODE, FTZ>(t, p);
            }
            if (rv && PACK) {
                uint16_t *row = Y16 + (size_t)(r + i) * ldy + c0;
                uint32_t c[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) c[j] = encode_bits<EM>(o[j], p);
                if (full) {
                    __builtin_nontemporal_store(u32x2{c[0] | (c[1] << 16), c[2] | (c[3] << 16)}, reinterpret_cast<u32x2 *>(row));
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (j < ncol) row[j] = (uint16_t)c[j];
                }
            } else if (rv) {
                uint32_t *row = Y + (size_t)(r + i) * ldy + c0;
                if (full) {
                    __builtin_nontemporal_store(o, reinterpret_cast<u32x4 *>(row));
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (j < ncol) row[j] = o[j];
                }
            }
        }
    }
    if (HIST)
        hist_end<kLCopies, kLBlock>(tbl, s_bins, s_cls, w, p, partials,
                                    (blockIdx.y * gridDim.x + blockIdx.x) % kShards, tid);
}

template <int MODE, bool FTZ, bool HIST, bool DEEP, bool PACK>
int launch_v(const float *A, int64_t lda, void *Y, int64_t ldy, int M, int N, const float *bias, const QuantParams &p,
             fmt_hist_t *hist, hipStream_t stream)
{
    int cus = 0;
    int rc = device_cu_count(&cus);
    if (rc != FMT_OK) return rc;
    const int strips = (N + kLBlock * 4 - 1) / (kLBlock * 4);
    // about 16 workgroups per compute unit (fewer leave the memory system idle: a lane has only four
    // loads in flight); with statistics at least 8 rows each so that clearing and folding the LDS
    // table stays a small part of a workgroup's work
    const int64_t want = (int64_t)cus * 16;
    int64_t row_groups = (want + strips - 1) / strips;
    const int min_rows = HIST ? 8 : kLRows;
    int64_t rows_per_wg = (M + row_groups - 1) / row_groups;
    if (rows_per_wg < min_rows) rows_per_wg = min_rows;
    rows_per_wg = (rows_per_wg + kLRows - 1) / kLRows * kLRows;
    row_groups = (M + rows_per_wg - 1) / rows_per_wg;
    if (row_groups > 65535) {                  // grid.y limit: make the row ranges longer instead
        rows_per_wg = ((M + 65534) / 65535 + kLRows - 1) / kLRows * kLRows;
        row_groups = (M + rows_per_wg - 1) / rows_per_wg;
    }
    unsigned long long *partials = nullptr;
    if (HIST) {
        Scratch s;
        rc = get_scratch(stream, kHistScratchBytes, 0, &s);
        if (rc != FMT_OK) return rc;
        partials = static_cast<unsigned long long *>(s.hist_partials);
    }
    const bool vec = (reinterpret_cast<uintptr_t>(A) % 16 == 0) && (lda % 4 == 0) &&
                     (reinterpret_cast<uintptr_t>(Y) % (PACK ? 8 : 16) == 0) && (ldy % 4 == 0);
    const dim3 grid((unsigned)strips, (unsigned)row_groups);
    const uint32_t *a = reinterpret_cast<const uint32_t *>(A);
    const uint32_t *b = reinterpret_cast<const uint32_t *>(bias);
    if (vec)
        hipLaunchKernelGGL((linear_epilogue_kernel<MODE, FTZ, HIST, DEEP, true, PACK>), grid, dim3(kLBlock), 0, stream, a,
                           lda, Y, ldy, M, N, b, (int)rows_per_wg, p, partials);
    else
        hipLaunchKernelGGL((linear_epilogue_kernel<MODE, FTZ, HIST, DEEP, false, PACK>), grid, dim3(kLBlock), 0, stream, a,
                           lda, Y, ldy, M, N, b, (int)rows_per_wg, p, partials);
    FMT_HIP_CHECK(hipGetLastError());
    if (HIST) return launch_hist_finalize(partials, (size_t)M * (size_t)N, hist, stream);
    return FMT_OK;
}

template <int MODE, bool FTZ, bool PACK>
int launch_h(const float *A, int64_t lda, void *Y, int64_t ldy, int M, int N, const float *bias, const QuantParams &p,
             fmt_hist_t *hist, hipStream_t stream)
{
    if (!hist) return launch_v<MODE, FTZ, false, false, PACK>(A, lda, Y, ldy, M, N, bias, p, hist, stream);
    if (p.exp_lo < -126) return launch_v<MODE, FTZ, true, true, PACK>(A, lda, Y, ldy, M, N, bias, p, hist, stream);
    return launch_v<MODE, FTZ, true, false, PACK>(A, lda, Y, ldy, M, N, bias, p, hist, stream);
}

}  // namespace

int launch_linear_epilogue(float *Y, int64_t ldy, int64_t M, int64_t N, const float *bias, const QuantParams &p,
                           bool ftz, fmt_hist_t *hist, hipStream_t stream)
{
    if (M == 0 || N == 0) {
        if (hist) return launch_hist_finalize(nullptr, 0, hist, stream);
        return FMT_OK;
    }
#define FMT_RUN(MD)                                                                                                   \
    (ftz ? launch_h<MD, true, false>(Y, ldy, Y, ldy, (int)M, (int)N, bias, p, hist, stream)                          \
         : launch_h<MD, false, false>(Y, ldy, Y, ldy, (int)M, (int)N, bias, p, hist, stream))
    if (p.mode == kModeMagic) return FMT_RUN(kModeMagic);
    if (p.mode == kModeInteger) return FMT_RUN(kModeInteger);
    return FMT_RUN(kModeMixed);
#undef FMT_RUN
}

int launch_linear_epilogue_pack16(const float *acc, int64_t lda, uint16_t *Y16, int64_t ldy, int64_t M, int64_t N,
                                  const float *bias, const QuantParams &p, bool ftz, fmt_hist_t *hist,
                                  hipStream_t stream)
{
    if (p.mode == kModeMixed) return FMT_ERR_FORMAT;     // m == 23 has no 16-bit code
    if (M == 0 || N == 0) {
        if (hist) return launch_hist_finalize(nullptr, 0, hist, stream);
        return FMT_OK;
    }
#define FMT_RUN(MD)                                                                                                   \
    (ftz ? launch_h<MD, true, true>(acc, lda, Y16, ldy, (int)M, (int)N, bias, p, hist, stream)                       \
         : launch_h<MD, false, true>(acc, lda, Y16, ldy, (int)M, (int)N, bias, p, hist, stream))
    if (p.mode == kModeInteger) return FMT_RUN(kModeInteger);
    return FMT_RUN(kModeMagic);
#undef FMT_RUN
}

}  // namespace fmt
