// Internal declarations shared by the translation units of libfmt (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "fmt.h"

namespace fmt {

// Bit-level description of one format, derived on the host from (e, m) (Sec. III).
// All thresholds are on a = |x| taken as an unsigned integer (the fp32 bit pattern with
// the sign cleared), which is monotone in |x| over zeros, denormals, normals and infinity.
struct QuantParams {
    uint32_t shift;       // 23 - m: low fp32 mantissa bits that the format drops
    uint32_t lsb_width;   // 1 when shift > 0, else 0 (width of the "last kept bit" field)
    uint32_t rbias;       // 2^(shift-1) - 1 (0 when shift == 0): RNE = add rbias + last kept bit, truncate
    uint32_t nmask;       // ~(2^shift - 1)
    int32_t mode;         // how the rounding is carried out (see fmt_stream.hip)
    uint32_t minn_bits;   // pattern of minN = 2^Emin
    uint32_t shift23;     // shift << 23: added to an exponent field it gives the pattern of 2^(E+23-m)
    float cmagic;         // 2^(Emin + 23 - m): adding and subtracting it rounds to a multiple of minD
    uint32_t t_zero;      // result is zero        <=>  a <= t_zero   (minD/2, the tie goes to zero)
    uint32_t t_den;       // result is below minN  <=>  a <  t_den    (minN - minD/2, the tie goes to minN)
    uint32_t t_ovf;       // result is infinite    <=>  a >= t_ovf    (maxN + ulp/2, the tie goes to infinity)
    int32_t exp_lo;       // lowest binade of the histogram window
    uint32_t sign_pos;    // e + m: position of the sign in the format's (1+e+m)-bit code
    uint32_t top_code;    // (2^e - 1) << m: code of +infinity
};

// Fills p from the format; returns FMT_OK or FMT_ERR_FORMAT / FMT_ERR_RANGE.
int make_quant_params(fmt_format_t f, int32_t exp_lo, QuantParams *p);

// Library-owned scratch of one (device, stream) pair.
struct Scratch {
    void *hist_partials = nullptr;  // per-workgroup partial counts of the stream kernels
    size_t hist_bytes = 0;
    void *gemm_ws = nullptr;        // pre-split GEMM operands
    size_t gemm_bytes = 0;
    void *acc_ws = nullptr;         // fp32 accumulators of fmt_linear_pack16
    size_t acc_bytes = 0;
};

// Returns the scratch record for (current device, stream), growing the requested buffers.
int get_scratch(hipStream_t stream, size_t hist_bytes, size_t gemm_bytes, Scratch *out);

int device_cu_count(int *cus);

// Stream kernels (fmt_stream.hip).  y: n floats, or with pack16 n uint16_t codes, or nullptr (statistics only).
// fixed_partials: partial statistics records to use instead of the (device, stream) scratch, or nullptr.
int launch_stream(const float *x, void *y, size_t n, const QuantParams &p, bool ftz,
                  fmt_hist_t *hist, hipStream_t stream, bool pack16 = false,
                  unsigned long long *fixed_partials = nullptr);
// The same pass with the partial records in the library's file-scope device array: allocates nothing.
int launch_stream_static(const float *x, float *y, size_t n, const QuantParams &p, bool ftz,
                         fmt_hist_t *hist, hipStream_t stream);
int launch_unpack16(const uint16_t *codes, float *y, size_t n, const QuantParams &p, hipStream_t stream);

// GEMM (fmt_gemm.hip)
int launch_gemm(int transA, int transB, int64_t M, int64_t N, int64_t K,
                const float *A, int64_t lda, const float *B, int64_t ldb,
                float *C, int64_t ldc, fmt_format_t f, const QuantParams &p, hipStream_t stream);

// Prepared operands in caller-owned memory (fmt_gemm.hip).  scheme: opaque tag of the representation.
int prepared_operand_bytes(int64_t rows, int64_t K, fmt_format_t f, size_t *bytes, int *scheme);
int launch_prepare_operand(const float *X, int64_t ld, int trans, int64_t rows, int64_t K, fmt_format_t f,
                           const QuantParams &p, void *buf, hipStream_t stream);
int launch_prepare_pair(const float *X, int64_t ld, int64_t rows, int64_t cols, fmt_format_t f, const QuantParams &p, void *buf0,
                        void *buf1, hipStream_t stream);
struct PrepPairItem {
    const float *X;
    int64_t ld, rows, cols;
    void *buf0, *buf1;
};
struct RoundItem {              // with the operands: the matrix rounded to fp32 (Y, leading dimension ldy) and its statistics
    float *Y;
    int64_t ldy;
    fmt_hist_t *hist;
};
int launch_prepare_pair_batch(int64_t count, const PrepPairItem *items, fmt_format_t f, const QuantParams &p, hipStream_t stream,
                              const RoundItem *round);
int launch_gemm_prepared(const void *A, const void *B, int64_t M, int64_t N, int64_t K, int scheme, fmt_format_t f,
                         float *C, int64_t ldc, hipStream_t stream);
// One product of a batch on prepared operands: C (M x N, leading dimension ldc) = A (M rows) B^T (N rows), both of k = K.
struct BatchItem {
    const void *A, *B;
    int64_t M, N, K;
    float *C;
    int64_t ldc;
};
int launch_gemm_prepared_batch(int count, const BatchItem *items, int scheme, fmt_format_t f, hipStream_t stream);

// Convolutions as products of gathered operands (fmt_gemm.hip); which: 0 forward, 1 dgrad, 2 wgrad
int launch_conv2d(int which, const fmt_conv2d_t &g, const float *a, const float *b, float *out, fmt_format_t f,
                  const QuantParams &p, hipStream_t stream);

// FMAC-8 GEMM (fmt_fmac8.hip)
int launch_gemm_fmac8(int transA, int transB, int64_t M, int64_t N, int64_t K,
                      const float *A, int64_t lda, const float *B, int64_t ldb,
                      float *C, int64_t ldc, fmt_format_t f, const QuantParams &p, hipStream_t stream);

// Output roundings of the Linear layer (fmt_linear.hip): in place on Y, or from the accumulators
// acc (leading dimension lda) into 16-bit codes Y16.
int launch_linear_epilogue(float *Y, int64_t ldy, int64_t M, int64_t N, const float *bias, const QuantParams &p,
                           bool ftz, fmt_hist_t *hist, hipStream_t stream);
int launch_linear_epilogue_pack16(const float *acc, int64_t lda, uint16_t *Y16, int64_t ldy, int64_t M, int64_t N,
                                  const float *bias, const QuantParams &p, bool ftz, fmt_hist_t *hist,
                                  hipStream_t stream);
// Library scratch for the accumulators of fmt_linear_pack16 (per device and stream, grown on demand).
int get_acc_scratch(hipStream_t stream, size_t bytes, float **out);

// Loss-scale controller (fmt_dls.hip)
int launch_dls_init(fmt_dls_state_t *state, float loss_scale, hipStream_t stream);
int launch_dls_step(const fmt_hist_t *hists, int64_t count, fmt_dls_params_t prm, fmt_dls_state_t *state,
                    hipStream_t stream);

// Reports a failed HIP call on stderr when the environment variable FMT_VERBOSE is set.
void report_hip_error(const char *expr, const char *file, int line, hipError_t err);

#define FMT_HIP_CHECK(expr)                                          \
    do {                                                             \
        hipError_t err__ = (expr);                                   \
        if (err__ != hipSuccess) {                                   \
            ::fmt::report_hip_error(#expr, __FILE__, __LINE__, err__); \
            (void)hipGetLastError();                                 \
            return FMT_ERR_HIP;                                      \
        }                                                            \
    } while (0)

}  // namespace fmt
