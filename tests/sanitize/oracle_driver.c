/* Host-side sanitizer run of the CPU oracle: calls every entry point of oracle/fmt_oracle.c on
 * exactly sized heap buffers (empty, ragged, strided, special values), so that AddressSanitizer and
 * UndefinedBehaviorSanitizer see every access and every shift the oracle makes.  Built and run by
 * tests/test_sanitizers.py with -fsanitize=address,undefined -fno-sanitize-recover=all: any finding
 * aborts with a non-zero exit code.  Prints a checksum so that the calls cannot be optimised away. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_format_constants(int e, int m, double *maxN, double *minN, double *minD, int *Emin, int *Emax);
float oracle_quantize_one(float x, int e, int m, int d);
int oracle_quantize(const float *x, float *y, size_t n, int e, int m, int d);
int oracle_histogram(const float *x, size_t n, int e, int m, int exp_lo, uint64_t *out);
int oracle_gemm(int transA, int transB, int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B,
                int64_t ldb, float *C, int64_t ldc, int e, int m, int d);
int oracle_gemm_sampled(int transA, int transB, int64_t M, int64_t N, int64_t K, const float *A, int64_t lda,
                        const float *B, int64_t ldb, const int64_t *rows, const int64_t *cols, int64_t count, float *out,
                        int e, int m, int d);
int oracle_linear_epilogue(const float *acc, int64_t ldacc, const float *bias, int64_t M, int64_t N, float *Y, int64_t ldy,
                           float *T, int64_t ldt, int e, int m, int d);
float oracle_fmac(float a, float w, float x, int e, int m, int d);
float oracle_fmac8_dot(const float *w, int64_t sw, const float *x, int64_t sx, int64_t n, int e, int m, int d);
int oracle_gemm_fmac8(int transA, int transB, int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B,
                      int64_t ldb, float *C, int64_t ldc, int e, int m, int d);
uint32_t oracle_encode(float v, int e, int m);
float oracle_decode(uint32_t code, int e, int m);
int oracle_pack16(const float *x, uint16_t *codes, size_t n, int e, int m, int d);
int oracle_unpack16(const uint16_t *codes, float *y, size_t n, int e, int m);
typedef struct {
    float loss_scale;
    int32_t good_steps, skip, steps;
    uint64_t nonfinite;
    int64_t worst_tensor;
    uint64_t worst_denormal, worst_total;
    int64_t peak_tensor, peak_step;
    uint64_t peak_denormal, peak_total;
} dls_state;
int oracle_dls_step(const uint64_t *hists, int64_t count, float growth, float backoff, int32_t interval, float min_scale,
                    float max_scale, dls_state *st);
int oracle_conv2d(int which, const int32_t *geom, const float *a, const float *b, const int64_t *idx, int64_t count,
                  float *out, int e, int m, int d);

static uint64_t lcg = 88172645463325252ull;
static uint32_t next_bits(void)
{
    lcg ^= lcg << 13; lcg ^= lcg >> 7; lcg ^= lcg << 17;
    return (uint32_t)(lcg >> 16);
}

/* n floats on the heap: a mix of random bit patterns (every class: NaN, infinities, fp32 denormals)
 * and moderate values. */
static float *make(size_t n, int wild)
{
    float *p = (float *)malloc(n ? n * sizeof(float) : 1);
    for (size_t i = 0; i < n; ++i) {
        uint32_t u = next_bits();
        if (!wild || (i & 3)) u = (u & 0x807FFFFFu) | ((uint32_t)(110 + (int)(next_bits() % 30)) << 23);
        memcpy(&p[i], &u, 4);
    }
    return p;
}

static double checksum = 0.0;
static void fold(const float *p, size_t n)
{
    for (size_t i = 0; i < n; ++i)
        if (isfinite(p[i])) checksum += (double)p[i] * 1e-3;
}

int main(void)
{
    static const int fmts[][2] = {{5, 10}, {6, 9}, {8, 7}, {2, 1}, {8, 23}, {7, 16}, {4, 3}};
    for (size_t fi = 0; fi < sizeof fmts / sizeof fmts[0]; ++fi) {
        const int e = fmts[fi][0], m = fmts[fi][1];
        double a, b, c;
        int lo, hi;
        if (oracle_format_constants(e, m, &a, &b, &c, &lo, &hi)) return 2;
        if (oracle_format_constants(e, m, NULL, NULL, NULL, NULL, NULL)) return 2;
        for (int d = 0; d < 2; ++d) {
            static const size_t sizes[] = {0, 1, 7, 1000};
            for (size_t si = 0; si < 4; ++si) {
                const size_t n = sizes[si];
                float *x = make(n, 1), *y = (float *)malloc(n ? n * 4 : 1);
                uint64_t *h = (uint64_t *)malloc(72 * 8);
                if (oracle_quantize(x, y, n, e, m, d)) return 3;
                if (oracle_histogram(x, n, e, m, -48, h) || oracle_histogram(x, n, e, m, -192, h) ||
                    oracle_histogram(x, n, e, m, 128, h))
                    return 3;
                fold(y, n);
                checksum += (double)h[0];
                if (1 + e + m <= 16) {
                    uint16_t *codes = (uint16_t *)malloc(n ? n * 2 : 1);
                    if (oracle_pack16(x, codes, n, e, m, d) || oracle_unpack16(codes, y, n, e, m)) return 4;
                    fold(y, n);
                    free(codes);
                }
                free(x); free(y); free(h);
            }
            if (1 + e + m <= 16)
                for (uint32_t code = 0; code < (1u << (1 + e + m)); code += 37) {
                    const float v = oracle_decode(code, e, m);
                    if (!isnan(v) && oracle_encode(v, e, m) != code) return 5;
                }
            /* products: every layout, ragged shapes, leading dimensions larger than the rows, K = 0 */
            static const int shapes[][3] = {{1, 1, 1}, {3, 5, 7}, {9, 4, 0}, {6, 7, 17}};
            for (size_t s = 0; s < 4; ++s) {
                const int M = shapes[s][0], N = shapes[s][1], K = shapes[s][2];
                for (int t = 0; t < 4; ++t) {
                    const int tA = t & 1, tB = t >> 1;
                    const int lda = (tA ? M : K) + 2, ldb = (tB ? K : N) + 1, ldc = N + 3;
                    float *A = make((size_t)((tA ? K : M) - 1 > 0 ? (tA ? K : M) - 1 : 0) * lda + (tA ? M : K), 0);
                    float *B = make((size_t)((tB ? N : K) - 1 > 0 ? (tB ? N : K) - 1 : 0) * ldb + (tB ? K : N), 0);
                    float *C = (float *)calloc((size_t)(M - 1) * ldc + N, 4);
                    if (oracle_gemm(tA, tB, M, N, K, A, lda, B, ldb, C, ldc, e, m, d)) return 6;
                    fold(C, (size_t)(M - 1) * ldc + N);
                    if (oracle_gemm_fmac8(tA, tB, M, N, K, A, lda, B, ldb, C, ldc, e, m, d)) return 6;
                    fold(C, (size_t)(M - 1) * ldc + N);
                    int64_t rows[3] = {0, M - 1, M / 2}, cols[3] = {N - 1, 0, N / 2};
                    float out[3];
                    if (oracle_gemm_sampled(tA, tB, M, N, K, A, lda, B, ldb, rows, cols, 3, out, e, m, d)) return 6;
                    fold(out, 3);
                    float *bias = make((size_t)N, 1), *Y = (float *)malloc((size_t)M * N * 4), *T = (float *)malloc((size_t)M * N * 4);
                    if (oracle_linear_epilogue(C, ldc, bias, M, N, Y, N, T, N, e, m, d)) return 7;
                    if (oracle_linear_epilogue(C, ldc, NULL, M, N, Y, N, NULL, 0, e, m, d)) return 7;
                    fold(Y, (size_t)M * N);
                    free(A); free(B); free(C); free(bias); free(Y); free(T);
                }
            }
            float *w = make(41, 0), *x = make(41, 0);
            for (int n = 0; n <= 20; ++n) checksum += (double)oracle_fmac8_dot(w, 2, x, 2, n, e, m, d);
            checksum += (double)oracle_fmac(oracle_quantize_one(w[0], e, m, d), oracle_quantize_one(w[1], e, m, d),
                                            oracle_quantize_one(x[1], e, m, d), e, m, d);
            free(w); free(x);
            /* convolutions: stride, padding wider than the filter allows, one-pixel images, sampled and full */
            static const int32_t geoms[][11] = {{2, 3, 5, 4, 2, 3, 3, 1, 1, 1, 1}, {1, 2, 6, 7, 3, 2, 4, 2, 3, 2, 3},
                                                {1, 1, 1, 1, 1, 1, 1, 0, 0, 1, 1}};
            for (size_t gi = 0; gi < 3; ++gi) {
                const int32_t *g = geoms[gi];
                const int n = g[0], cc = g[1], hh = g[2], ww = g[3], k = g[4], r = g[5], s = g[6];
                const int P = (hh + 2 * g[7] - r) / g[9] + 1, Q = (ww + 2 * g[8] - s) / g[10] + 1;
                const size_t nx = (size_t)n * cc * hh * ww, nw = (size_t)k * cc * r * s, ny = (size_t)n * k * P * Q;
                float *X = make(nx, 0), *W = make(nw, 0), *dY = make(ny, 0);
                float *Yo = (float *)malloc(ny * 4), *dX = (float *)malloc(nx * 4), *dW = (float *)malloc(nw * 4);
                if (oracle_conv2d(0, g, X, W, NULL, (int64_t)ny, Yo, e, m, d)) return 8;
                if (oracle_conv2d(1, g, dY, W, NULL, (int64_t)nx, dX, e, m, d)) return 8;
                if (oracle_conv2d(2, g, dY, X, NULL, (int64_t)nw, dW, e, m, d)) return 8;
                int64_t idx[2] = {0, (int64_t)ny - 1};
                float two[2];
                if (oracle_conv2d(0, g, X, W, idx, 2, two, e, m, d)) return 8;
                fold(Yo, ny); fold(dX, nx); fold(dW, nw); fold(two, 2);
                free(X); free(W); free(dY); free(Yo); free(dX); free(dW);
            }
        }
    }
    uint64_t *recs = (uint64_t *)calloc(3 * 72, 8);
    recs[0] = 100; recs[3] = 40; recs[72] = 50; recs[72 + 3] = 30; recs[144 + 5] = 1;
    dls_state st;
    memset(&st, 0, sizeof st);
    st.loss_scale = 1024.0f; st.worst_tensor = -1; st.peak_tensor = -1; st.peak_step = -1;
    if (oracle_dls_step(recs, 2, 2.0f, 0.5f, 1, 1.0f, 65536.0f, &st)) return 9;
    if (oracle_dls_step(recs, 3, 2.0f, 0.5f, 1, 1.0f, 65536.0f, &st)) return 9;
    if (oracle_dls_step(NULL, 0, 2.0f, 0.5f, 1, 1.0f, 65536.0f, &st)) return 9;
    checksum += st.loss_scale;
    free(recs);
    printf("oracle sanitizer run ok, checksum %.6g\n", checksum);
    return 0;
}
