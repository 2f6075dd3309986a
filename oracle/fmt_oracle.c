/*
 * CPU oracle for emulated 1/e/m floating-point arithmetic.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the GPU
 * library is checked against.  It shares no code, header, table or helper with
 * the GPU path and must never be called from it.  Only tests, the smoke check and
 * the benchmark's cpu_baseline leg load it.
 *
 * Everything is written from the paper's definitions:
 *   - a floating-point number x = M * 2^(E-p+1)                      (Sec. III, Def. III.1)
 *   - normal / denormal split and the hidden-bit convention          (Sec. III)
 *   - the system quadruple s/e/p/d                                    (Sec. III, Def. III.2)
 *   - the constants of the three 16-bit formats                      (Table I)
 *   - roundfp: round each fp32 element to the nearest representable
 *     value with e exponent bits and p stored mantissa bits, denormal
 *     range allowed (d) or flushed (n)                                (Sec. IV-A)
 *   - FMACS matmul: operands in the format, exact products,
 *     accumulation in a wider type                                    (Sec. III-B, Sec. IV-A)
 *   - the quantized Linear layer Y = R(R(R(W^T) R(X)) + R(B))          (Sec. IV-A)
 *   - FMAC and the FMAC-8 dot product                                 (Sec. III-B, Sec. IV-A, Algorithm 1)
 *   - denormal fraction of a tensor                                   (Sec. V)
 *   - the (1+e+m)-bit codes of the format's values                    (Sec. III)
 *
 * Notation used below: e = exponent bits, m = stored mantissa bits (the "p" of
 * Def. III.2 and Table I), bias = 2^(e-1)-1 ("vanilla" bias), Emax = bias,
 * Emin = 1-bias, minN = 2^Emin, minD = 2^(Emin-m), maxN = (2-2^-m) * 2^Emax.
 *
 * All floating-point work is done in fp64 with frexp / ldexp / nearbyint: an fp32
 * input has at most 24 significant bits and every scale used is a power of two
 * >= 2^-149, so each intermediate quantity is exact in fp64.  No bit tricks.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_NBINS 64
/* layout of the 72-entry count vector written by oracle_histogram */
enum { O_TOTAL = 0, O_ZERO, O_UNDERFLOW, O_DENORMAL, O_NORMAL, O_OVERFLOW, O_INF, O_NAN, O_BINS };

static int fmt_ok(int e, int m) { return e >= 2 && e <= 8 && m >= 1 && m <= 23; }

/* Closed-form constants of the format (Sec. III; Table I lists three instances). */
int oracle_format_constants(int e, int m, double *maxN, double *minN, double *minD,
                            int *Emin, int *Emax)
{
    if (!fmt_ok(e, m)) return -1;
    int bias = (1 << (e - 1)) - 1;
    int emax = bias, emin = 1 - bias;
    if (Emin) *Emin = emin;
    if (Emax) *Emax = emax;
    if (minN) *minN = ldexp(1.0, emin);
    if (minD) *minD = ldexp(1.0, emin - m);
    if (maxN) *maxN = ldexp(2.0 - ldexp(1.0, -m), emax);
    return 0;
}

static float canonical_nan(void)
{
    uint32_t u = 0x7FC00000u;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/*
 * Magnitude of Q_{e,m,d}(x) for finite non-zero x, as an fp64 (may be +inf).
 * Round-to-nearest, ties to even, onto the grid of spacing 2^(max(E,Emin)-m),
 * where E = floor(log2|x|); anything that rounds to 2^(Emax+1) or more is
 * overflow and becomes infinity (Sec. IV-A: "nearest representable"; the tie
 * rule, the overflow rule are the IEEE-754 ones the paper defers to in Sec. III).
 */
static double round_magnitude_d(double a, int e, int m)
{
    int bias = (1 << (e - 1)) - 1;
    int emax = bias, emin = 1 - bias;
    int ex;
    (void)frexp(a, &ex);          /* a = f * 2^ex with f in [0.5, 1)  =>  E = ex - 1 */
    int E = ex - 1;
    int q = (E > emin ? E : emin) - m;
    double k = nearbyint(ldexp(a, -q));   /* default rounding mode: nearest, ties to even */
    double r = ldexp(k, q);
    if (r >= ldexp(1.0, emax + 1)) return INFINITY;
    return r;
}

/* roundfp(x, e, m, d) for one element (Sec. IV-A). d != 0: denormal range allowed. */
float oracle_quantize_one(float x, int e, int m, int d)
{
    if (isnan(x)) return canonical_nan();
    if (isinf(x) || x == 0.0f) return x;                 /* signed zero / infinity kept */
    double r = round_magnitude_d(fabs((double)x), e, m);
    if (!d) {                                            /* "n": denormals are flushed to 0 (Sec. V-C) */
        int emin = 2 - (1 << (e - 1));
        if (r < ldexp(1.0, emin)) r = 0.0;
    }
    return (float)copysign(r, (double)x);                /* exact: r is an fp32 value */
}

int oracle_quantize(const float *x, float *y, size_t n, int e, int m, int d)
{
    if (!fmt_ok(e, m)) return -1;
    for (size_t i = 0; i < n; ++i) y[i] = oracle_quantize_one(x[i], e, m, d);
    return 0;
}

/*
 * Per-tensor statistics (Sec. V: the denormal fraction of a tensor; the bins are the
 * distribution of element magnitudes by binade).  out[0..7] = total, zero, underflow,
 * denormal, normal, overflow, inf, nan; out[8..71] = bins.  Classes are judged on
 * the value the element has after rounding with denormals allowed; the bin is the
 * binade floor(log2|x|) of the input, shifted by exp_lo and clamped into [0, 63].
 * NaN and zero are not binned; infinities go to the top bin.
 */
int oracle_histogram(const float *x, size_t n, int e, int m, int exp_lo, uint64_t *out)
{
    if (!fmt_ok(e, m)) return -1;
    int emin = 2 - (1 << (e - 1));
    double minN = ldexp(1.0, emin);
    for (int i = 0; i < O_BINS + ORACLE_NBINS; ++i) out[i] = 0;
    for (size_t i = 0; i < n; ++i) {
        float v = x[i];
        out[O_TOTAL]++;
        if (isnan(v)) { out[O_NAN]++; continue; }
        if (v == 0.0f) { out[O_ZERO]++; continue; }
        if (isinf(v)) { out[O_INF]++; out[O_BINS + ORACLE_NBINS - 1]++; continue; }
        double a = fabs((double)v);
        double r = round_magnitude_d(a, e, m);
        if (r == 0.0) out[O_UNDERFLOW]++;
        else if (isinf(r)) out[O_OVERFLOW]++;
        else if (r < minN) out[O_DENORMAL]++;
        else out[O_NORMAL]++;
        int ex;
        (void)frexp(a, &ex);
        long b = (long)(ex - 1) - (long)exp_lo;
        if (b < 0) b = 0;
        if (b > ORACLE_NBINS - 1) b = ORACLE_NBINS - 1;
        out[O_BINS + b]++;
    }
    return 0;
}

/* element (i,k) of op(A), op(A) being M x K: A is M x K row-major, or K x M when transposed */
static inline float op_at(const float *A, int64_t ld, int trans, int64_t i, int64_t k)
{
    return trans ? A[k * ld + i] : A[i * ld + k];
}

/*
 * FMACS matrix product (Sec. III-B, Sec. IV-A): C = Q(op(A)) * Q(op(B)), products not
 * rounded, sum taken in fp64 in plain k order and rounded once to fp32.  The
 * quantized operands have <= 24-bit significands, so each product is exact in fp64;
 * the fp64 sum is the reference that an fp32-accumulating FMACS chain approximates.
 * op(A) is M x K, op(B) is K x N, row-major with leading dimensions in elements.
 */
int oracle_gemm(int transA, int transB, int64_t M, int64_t N, int64_t K,
                const float *A, int64_t lda, const float *B, int64_t ldb,
                float *C, int64_t ldc, int e, int m, int d)
{
    if (!fmt_ok(e, m) || M < 0 || N < 0 || K < 0) return -1;
    if (M == 0 || N == 0) return 0;
    /* quantized operands, held as fp64; qb is stored N x K so the k loop is contiguous */
    double *qa = (double *)malloc(sizeof(double) * (size_t)(M * (K ? K : 1)));
    double *qb = (double *)malloc(sizeof(double) * (size_t)(N * (K ? K : 1)));
    if (!qa || !qb) { free(qa); free(qb); return -2; }
    for (int64_t i = 0; i < M; ++i)
        for (int64_t k = 0; k < K; ++k)
            qa[i * K + k] = (double)oracle_quantize_one(op_at(A, lda, transA, i, k), e, m, d);
    for (int64_t j = 0; j < N; ++j)
        for (int64_t k = 0; k < K; ++k)
            qb[j * K + k] = (double)oracle_quantize_one(op_at(B, ldb, !transB, j, k), e, m, d);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t j = 0; j < N; ++j) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k) acc += qa[i * K + k] * qb[j * K + k];
            C[i * ldc + j] = (float)acc;
        }
    }
    free(qa);
    free(qb);
    return 0;
}

/* The same sum for a list of output positions only: out[s] = C[rows[s], cols[s]]. */
int oracle_gemm_sampled(int transA, int transB, int64_t M, int64_t N, int64_t K,
                        const float *A, int64_t lda, const float *B, int64_t ldb,
                        const int64_t *rows, const int64_t *cols, int64_t nsamples,
                        float *out, int e, int m, int d)
{
    if (!fmt_ok(e, m) || M < 0 || N < 0 || K < 0) return -1;
    for (int64_t s = 0; s < nsamples; ++s) {
        int64_t i = rows[s], j = cols[s];
        if (i < 0 || i >= M || j < 0 || j >= N) return -3;
        double acc = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            double a = (double)oracle_quantize_one(op_at(A, lda, transA, i, k), e, m, d);
            double b = (double)oracle_quantize_one(op_at(B, ldb, !transB, j, k), e, m, d);
            acc += a * b;
        }
        out[s] = (float)acc;
    }
    return 0;
}

/*
 * Layer epilogue of the quantized Linear layer (Sec. IV-A): Y = R( R(acc) + R(b) ), where acc is
 * the matrix product R(W^T) . R(X) before any output rounding, b the bias (one value per output
 * column) and "+" a single-precision addition.  t = R(acc) + R(b) (the value that enters the last
 * rounding) is returned too, since that is the tensor whose statistics are logged.
 * bias may be NULL (then t = R(acc)).
 */
int oracle_linear_epilogue(const float *acc, int64_t ldacc, const float *bias, int64_t M, int64_t N,
                           float *Y, int64_t ldy, float *T, int64_t ldt, int e, int m, int d)
{
    if (!fmt_ok(e, m) || M < 0 || N < 0) return -1;
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j) {
            float t = oracle_quantize_one(acc[i * ldacc + j], e, m, d);
            if (bias) t = t + oracle_quantize_one(bias[j], e, m, d);      /* fp32 addition */
            if (T) T[i * ldt + j] = t;
            Y[i * ldy + j] = oracle_quantize_one(t, e, m, d);
        }
    return 0;
}

/*
 * FMAC (Sec. III-B): a16 = o(a16 + x16 * y16), one rounding of the exact sum to the format.
 * a, w, x are values of the format.  The product of two <= 24-bit significands is exact in fp64.
 * The sum a + w*x is in general NOT exact in fp64 (the exponents may be far apart), and rounding
 * it to fp64 first and to the format second could round twice.  The sum is therefore taken with
 * "round to odd": TwoSum gives the fp64 sum s and its exact error err; when err != 0 the exact sum
 * lies strictly between two fp64 neighbours, and the one whose last bit is odd is kept.  A value
 * rounded to odd at 53 bits rounds to any format of <= 51 bits exactly as the exact sum would
 * (the classic double-rounding remedy).  The format rounding is then the same as in roundfp.
 *
 * This routine is the FAST checker (used where the matrices are too large for rational arithmetic).
 * The definition of FMAC and of Algorithm 1 is oracle/fmac_exact.py -- the exact sum as a rational,
 * rounded by a search over the enumerated value set -- and tests/test_oracle_fmac_exact.py holds this
 * routine to it, bit for bit, for every format family (including the e >= 7 formats).
 */
static double sum_round_to_odd(double a, double p)
{
    double s = a + p;
    if (isnan(s) || isinf(s)) return s;
    double bb = s - a;                        /* TwoSum (Knuth): err = (a - (s - bb)) + (p - bb), exact */
    double err = (a - (s - bb)) + (p - bb);
    if (err != 0.0) {
        uint64_t u;
        memcpy(&u, &s, sizeof u);
        if ((u & 1u) == 0)                    /* s is the even neighbour: the odd one lies on err's side */
            s = nextafter(s, err > 0.0 ? INFINITY : -INFINITY);
    }
    return s;
}

static float round_double_to_format(double s, int e, int m, int d)
{
    if (isnan(s)) return canonical_nan();
    if (isinf(s) || s == 0.0) return (float)s;
    double r = round_magnitude_d(fabs(s), e, m);
    if (!d) {
        int emin = 2 - (1 << (e - 1));
        if (r < ldexp(1.0, emin)) r = 0.0;
    }
    return (float)copysign(r, s);
}

float oracle_fmac(float a, float w, float x, int e, int m, int d)
{
    double p = (double)w * (double)x;         /* exact */
    return round_double_to_format(sum_round_to_odd((double)a, p), e, m, d);
}

/*
 * FMAC-8 dot product (Sec. IV-A, Algorithm 1), in the listing's own order: a 16-bit accumulator
 * a takes 8 consecutive FMACs; at every i that is a multiple of 8 it is first added into the
 * fp32 master accumulator A with an fp32 addition and reset; after the loop A takes the last a
 * and the result is R(A).  w and x hold values of the format.
 */
float oracle_fmac8_dot(const float *w, int64_t sw, const float *x, int64_t sx, int64_t n, int e, int m, int d)
{
    float A = 0.0f;
    float a = 0.0f;
    for (int64_t i = 0; i < n; ++i) {
        if (i % 8 == 0) {
            A = A + a;                        /* single-precision addition */
            a = 0.0f;
        }
        a = oracle_fmac(a, w[i * sw], x[i * sx], e, m, d);
    }
    A = A + a;
    return oracle_quantize_one(A, e, m, d);
}

/* C[i][j] = FMAC-8 dot product of row i of Q(op(A)) and column j of Q(op(B)). */
int oracle_gemm_fmac8(int transA, int transB, int64_t M, int64_t N, int64_t K,
                      const float *A, int64_t lda, const float *B, int64_t ldb,
                      float *C, int64_t ldc, int e, int m, int d)
{
    if (!fmt_ok(e, m) || M < 0 || N < 0 || K < 0) return -1;
    if (M == 0 || N == 0) return 0;
    float *qa = (float *)malloc(sizeof(float) * (size_t)(M * (K ? K : 1)));
    float *qb = (float *)malloc(sizeof(float) * (size_t)(N * (K ? K : 1)));
    if (!qa || !qb) { free(qa); free(qb); return -2; }
    for (int64_t i = 0; i < M; ++i)
        for (int64_t k = 0; k < K; ++k)
            qa[i * K + k] = oracle_quantize_one(op_at(A, lda, transA, i, k), e, m, d);
    for (int64_t j = 0; j < N; ++j)
        for (int64_t k = 0; k < K; ++k)
            qb[j * K + k] = oracle_quantize_one(op_at(B, ldb, !transB, j, k), e, m, d);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j)
            C[i * ldc + j] = oracle_fmac8_dot(qa + i * K, 1, qb + j * K, 1, K, e, m, d);
    free(qa);
    free(qb);
    return 0;
}

/*
 * 16-bit (1+e+m-bit) code of a value of the format (Sec. III: stored exponent field 0 for
 * zero/denormal, all ones for infinity/NaN, hidden bit not stored).  v must already be a
 * value of the format (the output of oracle_quantize_one).
 */
uint32_t oracle_encode(float v, int e, int m)
{
    int bias = (1 << (e - 1)) - 1;
    int emin = 1 - bias;
    uint32_t sign = signbit(v) ? 1u : 0u;
    uint32_t top = ((1u << e) - 1u);
    if (isnan(v)) return (top << m) | (1u << (m - 1));
    uint32_t field, mant;
    double a = fabs((double)v);
    if (isinf(v)) { field = top; mant = 0; }
    else if (a == 0.0) { field = 0; mant = 0; }
    else if (a < ldexp(1.0, emin)) { field = 0; mant = (uint32_t)ldexp(a, m - emin); }
    else {
        int ex;
        double f = frexp(a, &ex);             /* a = f*2^ex, f in [0.5,1) */
        int E = ex - 1;
        field = (uint32_t)(E + bias);
        mant = (uint32_t)(ldexp(f, m + 1)) - (1u << m);
    }
    return (sign << (e + m)) | (field << m) | mant;
}

/*
 * Value of a (1+e+m)-bit code (Sec. III, Def. III.1 with the hidden-bit convention and the special
 * encodings): sign s, stored exponent field f, mantissa field t;
 *   f == 0:         (-1)^s * t * 2^(Emin-m)                 zero and the denormal range
 *   0 < f < 2^e-1:  (-1)^s * (2^m + t) * 2^(f-bias-m)       normal numbers, E = f - bias
 *   f == 2^e-1:     t == 0: (-1)^s * infinity, else NaN (returned as the canonical quiet NaN)
 * Bits of `code` above bit e+m are ignored.  Every such value is an fp32 value (e <= 8, m <= 23).
 */
float oracle_decode(uint32_t code, int e, int m)
{
    int bias = (1 << (e - 1)) - 1;
    int emin = 1 - bias;
    uint32_t top = (1u << e) - 1u;
    uint32_t sign = (code >> (e + m)) & 1u;
    uint32_t field = (code >> m) & top;
    uint32_t mant = code & ((1u << m) - 1u);
    double v;
    if (field == top) {
        if (mant != 0) return canonical_nan();
        v = INFINITY;
    } else if (field == 0) {
        v = ldexp((double)mant, emin - m);
    } else {
        v = ldexp((double)((1u << m) + mant), (int)field - bias - m);
    }
    return (float)(sign ? -v : v);
}

/*
 * Packed storage of a tensor in the format: codes[i] = code of roundfp(x[i]) (Sec. IV-A rounding,
 * Sec. III encoding), and back.  Needs 1 + e + m <= 16.
 */
int oracle_pack16(const float *x, uint16_t *codes, size_t n, int e, int m, int d)
{
    if (!fmt_ok(e, m) || 1 + e + m > 16) return -1;
    for (size_t i = 0; i < n; ++i) codes[i] = (uint16_t)oracle_encode(oracle_quantize_one(x[i], e, m, d), e, m);
    return 0;
}

int oracle_unpack16(const uint16_t *codes, float *y, size_t n, int e, int m)
{
    if (!fmt_ok(e, m) || 1 + e + m > 16) return -1;
    for (size_t i = 0; i < n; ++i) y[i] = oracle_decode(codes[i], e, m);
    return 0;
}

/*
 * Loss-scale controller and denormal-fraction monitor, one call per training step.
 *
 * Sec. II describes loss scaling (the loss is multiplied by a factor S before backpropagation so
 * that small gradients do not underflow; weight gradients are divided by S again) and names
 * dynamic loss scaling as the automated choice of S from the gradient distribution; Sec. V logs
 * the denormal fraction of every tensor and reports the highest one observed.  The paper gives
 * no update rule or parameters; this is the usual controller, written out:
 *   - the step's records are the fmt_hist-style statistics (72 uint64 each: total, zero,
 *     underflow, denormal, normal, overflow, inf, nan, 64 bins) of the scaled gradient tensors;
 *   - nonfinite = sum over the records of overflow + inf + nan;
 *   - nonfinite > 0: the step is skipped, S <- max(S * backoff, min_scale), the run of good
 *     steps restarts;
 *   - otherwise the run grows by one, and when it reaches `interval`,
 *     S <- min(S * growth, max_scale) and the run restarts;
 *   - worst tensor of the step = largest denormal / total (fp64 quotient, records with
 *     total == 0 ignored, ties to the lowest index); the running peak over all steps is replaced
 *     when the step's worst fraction is strictly larger.
 * The products S * backoff and S * growth are single-precision multiplications.
 */
typedef struct {
    float loss_scale;
    int32_t good_steps;
    int32_t skip;
    int32_t steps;
    uint64_t nonfinite;
    int64_t worst_tensor;
    uint64_t worst_denormal, worst_total;
    int64_t peak_tensor;
    int64_t peak_step;
    uint64_t peak_denormal, peak_total;
} oracle_dls_state;

int oracle_dls_step(const uint64_t *hists, int64_t count, float growth, float backoff, int32_t interval,
                    float min_scale, float max_scale, oracle_dls_state *st)
{
    if (count < 0 || !st || interval < 1) return -1;
    uint64_t nonfinite = 0;
    int64_t worst = -1;
    double worst_frac = -1.0;
    for (int64_t i = 0; i < count; ++i) {
        const uint64_t *h = hists + 72 * i;
        nonfinite += h[5] + h[6] + h[7];
        if (h[0] > 0) {
            double frac = (double)h[3] / (double)h[0];
            if (frac > worst_frac) { worst_frac = frac; worst = i; }
        }
    }
    st->nonfinite = nonfinite;
    st->worst_tensor = worst;
    st->worst_denormal = worst >= 0 ? hists[72 * worst + 3] : 0;
    st->worst_total = worst >= 0 ? hists[72 * worst + 0] : 0;
    if (nonfinite > 0) {
        st->skip = 1;
        float s = st->loss_scale * backoff;
        st->loss_scale = s < min_scale ? min_scale : s;
        st->good_steps = 0;
    } else {
        st->skip = 0;
        st->good_steps += 1;
        if (st->good_steps >= interval) {
            float s = st->loss_scale * growth;
            st->loss_scale = s > max_scale ? max_scale : s;
            st->good_steps = 0;
        }
    }
    if (worst >= 0) {
        double peak_frac = st->peak_total > 0 ? (double)st->peak_denormal / (double)st->peak_total : -1.0;
        if (worst_frac > peak_frac) {
            st->peak_tensor = worst;
            st->peak_step = st->steps;
            st->peak_denormal = st->worst_denormal;
            st->peak_total = st->worst_total;
        }
    }
    st->steps += 1;
    return 0;
}

/*
 * Convolution layers (Sec. IV-A: the inner matrix multiplies "or convolutions" of the forward and
 * backward pass use FMACS: operands rounded to the format, products not rounded, fp32 result).
 * Plain definitions, NCHW tensors, filter [K][C][R][S], zero padding, no dilation, no groups.
 * Every sum is taken in fp64 in the order written (exact products of <= 24-bit significands) and
 * rounded once to fp32, as in oracle_gemm.
 *   geometry g[11] = { N, C, H, W, K, R, S, pad_h, pad_w, stride_h, stride_w };
 *   P = (H + 2 pad_h - R) / stride_h + 1,  Q = (W + 2 pad_w - S) / stride_w + 1.
 *   forward  Y[n][k][p][q]  = sum_{c,r,s} Q(X[n][c][p*sh - ph + r][q*sw - pw + s]) * Q(Wt[k][c][r][s])
 *   dgrad    dX[n][c][h][w] = sum_{k,r,s} Q(dY[n][k][p][q]) * Q(Wt[k][c][r][s]),  p*sh - ph + r = h, q*sw - pw + s = w
 *   wgrad    dW[k][c][r][s] = sum_{n,p,q} Q(dY[n][k][p][q]) * Q(X[n][c][p*sh - ph + r][q*sw - pw + s])
 * (out-of-range input positions contribute zero).  Each has a variant that computes only a list
 * of output elements given by their flat indices.
 */
typedef struct { int64_t N, C, H, W, K, R, S, ph, pw, sh, sw, P, Q; } conv_geom;

static int conv_geom_from(const int32_t *g, conv_geom *o)
{
    o->N = g[0]; o->C = g[1]; o->H = g[2]; o->W = g[3]; o->K = g[4]; o->R = g[5]; o->S = g[6];
    o->ph = g[7]; o->pw = g[8]; o->sh = g[9]; o->sw = g[10];
    if (o->N < 0 || o->C < 0 || o->H < 1 || o->W < 1 || o->K < 0 || o->R < 1 || o->S < 1) return -1;
    if (o->ph < 0 || o->pw < 0 || o->sh < 1 || o->sw < 1) return -1;
    if (o->H + 2 * o->ph < o->R || o->W + 2 * o->pw < o->S) return -1;
    o->P = (o->H + 2 * o->ph - o->R) / o->sh + 1;
    o->Q = (o->W + 2 * o->pw - o->S) / o->sw + 1;
    return 0;
}

static float conv_fwd_one(const conv_geom *g, const float *X, const float *Wt, int64_t idx, int e, int m, int d)
{
    int64_t q = idx % g->Q, p = (idx / g->Q) % g->P, k = (idx / (g->Q * g->P)) % g->K, n = idx / (g->Q * g->P * g->K);
    double acc = 0.0;
    for (int64_t c = 0; c < g->C; ++c)
        for (int64_t r = 0; r < g->R; ++r)
            for (int64_t s = 0; s < g->S; ++s) {
                int64_t h = p * g->sh - g->ph + r, w = q * g->sw - g->pw + s;
                if (h < 0 || h >= g->H || w < 0 || w >= g->W) continue;
                double x = (double)oracle_quantize_one(X[((n * g->C + c) * g->H + h) * g->W + w], e, m, d);
                double f = (double)oracle_quantize_one(Wt[((k * g->C + c) * g->R + r) * g->S + s], e, m, d);
                acc += x * f;
            }
    return (float)acc;
}

static float conv_dgrad_one(const conv_geom *g, const float *dY, const float *Wt, int64_t idx, int e, int m, int d)
{
    int64_t w = idx % g->W, h = (idx / g->W) % g->H, c = (idx / (g->W * g->H)) % g->C, n = idx / (g->W * g->H * g->C);
    double acc = 0.0;
    for (int64_t k = 0; k < g->K; ++k)
        for (int64_t r = 0; r < g->R; ++r)
            for (int64_t s = 0; s < g->S; ++s) {
                int64_t ph = h + g->ph - r, pw = w + g->pw - s;
                if (ph < 0 || pw < 0 || ph % g->sh || pw % g->sw) continue;
                int64_t p = ph / g->sh, q = pw / g->sw;
                if (p >= g->P || q >= g->Q) continue;
                double y = (double)oracle_quantize_one(dY[((n * g->K + k) * g->P + p) * g->Q + q], e, m, d);
                double f = (double)oracle_quantize_one(Wt[((k * g->C + c) * g->R + r) * g->S + s], e, m, d);
                acc += y * f;
            }
    return (float)acc;
}

static float conv_wgrad_one(const conv_geom *g, const float *dY, const float *X, int64_t idx, int e, int m, int d)
{
    int64_t s = idx % g->S, r = (idx / g->S) % g->R, c = (idx / (g->S * g->R)) % g->C, k = idx / (g->S * g->R * g->C);
    double acc = 0.0;
    for (int64_t n = 0; n < g->N; ++n)
        for (int64_t p = 0; p < g->P; ++p)
            for (int64_t q = 0; q < g->Q; ++q) {
                int64_t h = p * g->sh - g->ph + r, w = q * g->sw - g->pw + s;
                if (h < 0 || h >= g->H || w < 0 || w >= g->W) continue;
                double y = (double)oracle_quantize_one(dY[((n * g->K + k) * g->P + p) * g->Q + q], e, m, d);
                double x = (double)oracle_quantize_one(X[((n * g->C + c) * g->H + h) * g->W + w], e, m, d);
                acc += y * x;
            }
    return (float)acc;
}

/* which: 0 forward (a = X, b = Wt, out = Y), 1 dgrad (a = dY, b = Wt, out = dX), 2 wgrad (a = dY, b = X, out = dW).
 * idx == NULL: all `count` = size-of-output elements in order; else out[i] = element idx[i]. */
int oracle_conv2d(int which, const int32_t *geom, const float *a, const float *b, const int64_t *idx, int64_t count,
                  float *out, int e, int m, int d)
{
    conv_geom g;
    if (!fmt_ok(e, m) || conv_geom_from(geom, &g)) return -1;
    int64_t total = which == 0 ? g.N * g.K * g.P * g.Q : which == 1 ? g.N * g.C * g.H * g.W : g.K * g.C * g.R * g.S;
    if (!idx && count != total) return -2;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < count; ++i) {
        int64_t j = idx ? idx[i] : i;
        if (j < 0 || j >= total) { out[i] = NAN; continue; }
        out[i] = which == 0 ? conv_fwd_one(&g, a, b, j, e, m, d)
               : which == 1 ? conv_dgrad_one(&g, a, b, j, e, m, d)
                            : conv_wgrad_one(&g, a, b, j, e, m, d);
    }
    return 0;
}
