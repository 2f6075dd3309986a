/* Host-side sanitizer run of the library's boundary: every entry point of include/fmt.h is called with
 * arguments that its validation must refuse BEFORE any GPU call (NULL, misaligned, overlapping,
 * negative, too large, unsupported formats), and the host helpers are run over every supported format.
 * The argument-checking translation unit (csrc/fmt_api.hip) is compiled with
 * -fsanitize=address,undefined for the host; any finding aborts with a non-zero exit code.  No GPU is
 * touched: every call here returns from the validation code. */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "fmt.h"

#define EXPECT(call, want)                                                              \
    do {                                                                                \
        int got__ = (call);                                                             \
        if (got__ != (want)) {                                                          \
            printf("%s: got %d (%s), want %d\n", #call, got__, fmt_status_string(got__), (want)); \
            return 1;                                                                   \
        }                                                                               \
    } while (0)

int main(void)
{
    /* host helpers over every supported and some unsupported formats */
    for (int e = 0; e <= 10; ++e)
        for (int m = -1; m <= 25; ++m) {
            fmt_format_t f = {e, m, 1};
            double a, b, c;
            int32_t lo, hi;
            uint32_t thr[3];
            size_t bytes = 0;
            const int ok = e >= 2 && e <= 8 && m >= 1 && m <= 23;
            EXPECT(fmt_format_info(f, &a, &b, &c, &lo, &hi), ok ? FMT_OK : FMT_ERR_FORMAT);
            EXPECT(fmt_format_info(f, NULL, NULL, NULL, NULL, NULL), ok ? FMT_OK : FMT_ERR_FORMAT);
            EXPECT(fmt_format_thresholds(f, thr), ok ? FMT_OK : FMT_ERR_FORMAT);
            EXPECT(fmt_operand_bytes(1, 1, f, &bytes), ok ? FMT_OK : FMT_ERR_FORMAT);
            EXPECT(fmt_operand_bytes(2147483647, 2147483647, f, &bytes), ok ? FMT_ERR_SHAPE : FMT_ERR_FORMAT);
        }
    for (int s = 1; s >= -12; --s)
        if (fmt_status_string(s) == NULL) return 1;

    fmt_format_t f = {6, 9, 1}, bad = {9, 9, 1}, wide = {8, 23, 1};
    char *raw = (char *)malloc(8192);
    char *base = (char *)(((size_t)raw + 255) / 256 * 256);
    float *x = (float *)base, *y = (float *)(base + 2048);
    fmt_hist_t *h = (fmt_hist_t *)(base + 4096);
    /* stream calls */
    EXPECT(fmt_quantize(x, y, 4, bad, NULL, -48, NULL), FMT_ERR_FORMAT);
    EXPECT(fmt_quantize(NULL, y, 4, f, NULL, -48, NULL), FMT_ERR_NULL);
    EXPECT(fmt_quantize((float *)(base + 2), y, 4, f, NULL, -48, NULL), FMT_ERR_ALIGN);
    EXPECT(fmt_quantize(x, x + 1, 4, f, NULL, -48, NULL), FMT_ERR_ALIAS);
    EXPECT(fmt_quantize(x, y, 4, f, h, 1000, NULL), FMT_ERR_RANGE);
    EXPECT(fmt_quantize(x, y, (size_t)1 << 40, f, NULL, -48, NULL), FMT_ERR_SHAPE);
    EXPECT(fmt_quantize(NULL, NULL, 0, f, NULL, -48, NULL), FMT_OK);
    EXPECT(fmt_quantize_static(x, y, ((size_t)1 << 36) + 1, f, NULL, -48, NULL), FMT_ERR_SHAPE);
    EXPECT(fmt_quantize_static(x, x + 1, 4, f, NULL, -48, NULL), FMT_ERR_ALIAS);
    EXPECT(fmt_histogram(x, 4, f, NULL, -48, NULL), FMT_ERR_NULL);
    EXPECT(fmt_histogram(x, 4, f, (fmt_hist_t *)(base + 4100), -48, NULL), FMT_ERR_ALIGN);
    EXPECT(fmt_pack16(x, (uint16_t *)y, 4, wide, NULL, -48, NULL), FMT_ERR_FORMAT);
    EXPECT(fmt_pack16(x, (uint16_t *)x, 4, f, NULL, -48, NULL), FMT_ERR_ALIAS);
    EXPECT(fmt_unpack16((const uint16_t *)(base + 1), y, 4, f, NULL), FMT_ERR_ALIGN);
    /* products */
    EXPECT(fmt_gemm(0, 0, -1, 1, 1, x, 1, x, 1, y, 1, f, NULL), FMT_ERR_SHAPE);
    EXPECT(fmt_gemm(0, 0, 2, 2, 2, x, 1, x, 2, y, 2, f, NULL), FMT_ERR_SHAPE);
    EXPECT(fmt_gemm(0, 0, 2, 2, 2, x, 2, x, 2, x + 1, 2, f, NULL), FMT_ERR_ALIAS);
    EXPECT(fmt_gemm(0, 0, 2, 2, 2, NULL, 2, x, 2, y, 2, f, NULL), FMT_ERR_NULL);
    EXPECT(fmt_gemm(0, 0, 0, 5, 5, NULL, 5, NULL, 5, NULL, 5, f, NULL), FMT_OK);
    EXPECT(fmt_gemm_fmac8(1, 1, 2, 2, 2, x, 2, x, 2, (float *)(base + 2050), 2, f, NULL), FMT_ERR_ALIGN);
    EXPECT(fmt_linear(2, 2, 2, x, 2, x, 2, y, y, 2, f, NULL, -48, NULL), FMT_ERR_ALIAS);
    EXPECT(fmt_linear_pack16(2, 2, 2, x, 2, x, 2, NULL, (uint16_t *)y, 1, f, NULL, -48, NULL), FMT_ERR_SHAPE);
    fmt_operand_t op, a, b;
    EXPECT(fmt_prepare(x, 4, 0, 4, 8, f, base + 2048, 4096, &op, NULL), FMT_ERR_SHAPE);
    EXPECT(fmt_prepare(x, 8, 0, 4, 8, f, base + 2048, 64, &op, NULL), FMT_ERR_SHAPE);
    EXPECT(fmt_prepare(x, 8, 0, 4, 8, f, base + 2052, (size_t)1 << 30, &op, NULL), FMT_ERR_ALIGN);
    EXPECT(fmt_prepare(x, 8, 0, 4, 8, f, base, (size_t)1 << 30, &op, NULL), FMT_ERR_ALIAS);
    EXPECT(fmt_prepare(x, 8, 0, 4, 8, f, base + 2048, (size_t)1 << 30, NULL, NULL), FMT_ERR_NULL);
    memset(&a, 0, sizeof a);
    memset(&b, 0, sizeof b);
    a.format = b.format = f;
    a.rows = b.rows = 4; a.k = 8; b.k = 16;
    a.data = base; b.data = base + 256; a.bytes = b.bytes = (size_t)1 << 30;
    EXPECT(fmt_gemm_prepared(&a, &b, y, 4, NULL), FMT_ERR_SHAPE);
    EXPECT(fmt_gemm_prepared(&a, NULL, y, 4, NULL), FMT_ERR_NULL);
    b.k = 8; b.format = bad;
    EXPECT(fmt_gemm_prepared(&a, &b, y, 4, NULL), FMT_ERR_FORMAT);
    EXPECT(fmt_linear_prepared(&a, &b, NULL, y, 4, NULL, -48, NULL), FMT_ERR_FORMAT);
    EXPECT(fmt_linear_prepared(NULL, &b, NULL, y, 4, NULL, -48, NULL), FMT_ERR_NULL);
    b.format = f; b.k = 16;
    EXPECT(fmt_linear_prepared(&a, &b, NULL, y, 4, NULL, -48, NULL), FMT_ERR_SHAPE);
    fmt_operand_t op_t;
    EXPECT(fmt_prepare_pair(x, 4, 4, 8, f, base + 2048, 4096, &op, base + 8192, 4096, &op_t, NULL), FMT_ERR_SHAPE);
    EXPECT(fmt_prepare_pair(x, 8, 4, 8, f, base + 2048, 64, &op, base + 8192, 64, &op_t, NULL), FMT_ERR_SHAPE);
    EXPECT(fmt_prepare_pair(x, 8, 4, 8, f, base + 2048, (size_t)1 << 30, &op, base + 8196, (size_t)1 << 30, &op_t, NULL), FMT_ERR_ALIGN);
    EXPECT(fmt_prepare_pair(x, 8, 4, 8, f, base + 2048, (size_t)1 << 30, &op, base + 2304, (size_t)1 << 30, &op_t, NULL), FMT_ERR_ALIAS);
    EXPECT(fmt_prepare_pair(x, 8, 4, 8, f, base + 2048, (size_t)1 << 30, &op, NULL, (size_t)1 << 30, &op_t, NULL), FMT_ERR_NULL);
    EXPECT(fmt_prepare_pair(x, 8, 0, 8, f, base + 2048, (size_t)1 << 30, &op, base + 8192, (size_t)1 << 30, &op_t, NULL), FMT_ERR_SHAPE);
    EXPECT(fmt_scratch_bytes(NULL, NULL), FMT_ERR_NULL);
    {
        const fmt_operand_t *pa[2] = {&a, &a}, *pb[2] = {&b, NULL};
        float *pc[2] = {y, y};
        int64_t ld[2] = {4, 4};
        EXPECT(fmt_gemm_prepared_batch(0, NULL, NULL, NULL, NULL, NULL), FMT_OK);
        EXPECT(fmt_gemm_prepared_batch(-1, pa, pb, pc, ld, NULL), FMT_ERR_SHAPE);
        EXPECT(fmt_gemm_prepared_batch(2, pa, NULL, pc, ld, NULL), FMT_ERR_NULL);
        EXPECT(fmt_gemm_prepared_batch(2, pa, pb, pc, ld, NULL), FMT_ERR_SHAPE);     /* first product: k differs */
        pb[0] = NULL;
        EXPECT(fmt_gemm_prepared_batch(2, pa, pb, pc, ld, NULL), FMT_ERR_NULL);      /* first product: no B */
    }
    {
        const float *px[2] = {x, x};
        int64_t d2[2] = {4, 4}, r2[2] = {4, 4}, c2[2] = {4, 4};
        void *pd[2] = {(void *)0x10000, (void *)0x20000}, *pt[2] = {(void *)0x30000, (void *)0x40000};
        size_t nb[2] = {0, 0};
        fmt_operand_t o2[2], t2[2];
        EXPECT(fmt_prepare_pair_batch(0, NULL, NULL, NULL, NULL, f, NULL, NULL, NULL, NULL, NULL, NULL, NULL), FMT_OK);
        EXPECT(fmt_prepare_pair_batch(-1, px, d2, r2, c2, f, pd, nb, o2, pt, nb, t2, NULL), FMT_ERR_SHAPE);
        EXPECT(fmt_prepare_pair_batch(2, px, d2, r2, c2, f, pd, nb, NULL, pt, nb, t2, NULL), FMT_ERR_NULL);
        EXPECT(fmt_prepare_pair_batch(2, px, d2, r2, c2, f, pd, nb, o2, pt, nb, t2, NULL), FMT_ERR_SHAPE);  /* buffers of 0 bytes */
        {
            float *py[2] = {y, y + 64};
            int64_t dy2[2] = {4, 4};
            fmt_hist_t *ph[2] = {(fmt_hist_t *)0x50000, (fmt_hist_t *)0x60000};
            EXPECT(fmt_quantize_prepare_pair_batch(0, NULL, NULL, NULL, NULL, f, NULL, NULL, NULL, -48, NULL, NULL, NULL, NULL, NULL, NULL, NULL), FMT_OK);
            EXPECT(fmt_quantize_prepare_pair_batch(2, px, d2, r2, c2, f, NULL, dy2, ph, -48, pd, nb, o2, pt, nb, t2, NULL), FMT_ERR_NULL);
            EXPECT(fmt_quantize_prepare_pair_batch(2, px, d2, r2, c2, f, py, dy2, ph, -48, pd, nb, o2, pt, nb, t2, NULL), FMT_ERR_SHAPE);  /* buffers of 0 bytes */
            EXPECT(fmt_quantize_prepare_pair_batch(2, px, d2, r2, c2, f, py, dy2, ph, 1 << 20, pd, nb, o2, pt, nb, t2, NULL), FMT_ERR_RANGE);
        }
        c2[1] = 5;
        nb[0] = nb[1] = (size_t)1 << 20;
        EXPECT(fmt_prepare_pair_batch(2, px, d2, r2, c2, f, pd, nb, o2, pt, nb, t2, NULL), FMT_ERR_SHAPE);  /* ld < cols */
    }
    /* convolutions */
    fmt_conv2d_t g = {1, 1, 4, 4, 1, 3, 3, 1, 1, 1, 1};
    EXPECT(fmt_conv2d_fwd(g, NULL, x, y, f, NULL), FMT_ERR_NULL);
    g.stride_h = 0;
    EXPECT(fmt_conv2d_dgrad(g, x, x, y, f, NULL), FMT_ERR_SHAPE);
    g.stride_h = 1; g.r = 9;
    EXPECT(fmt_conv2d_wgrad(g, x, x, y, f, NULL), FMT_ERR_SHAPE);
    g.r = 3; g.n = 0;
    EXPECT(fmt_conv2d_fwd(g, NULL, NULL, NULL, f, NULL), FMT_OK);
    /* loss scaling */
    fmt_dls_params_t prm = {2.0f, 0.5f, 0, 1.0f, 65536.0f};
    EXPECT(fmt_dls_step(h, 1, prm, (fmt_dls_state_t *)y, NULL), FMT_ERR_RANGE);
    prm.interval = 1;
    EXPECT(fmt_dls_step(NULL, 1, prm, (fmt_dls_state_t *)y, NULL), FMT_ERR_NULL);
    EXPECT(fmt_dls_init((fmt_dls_state_t *)y, -1.0f, NULL), FMT_ERR_RANGE);
    EXPECT(fmt_dls_init(NULL, 1.0f, NULL), FMT_ERR_NULL);
    free(raw);
    printf("abi sanitizer run ok\n");
    return 0;
}
