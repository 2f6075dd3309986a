/*
 * libfmt -- emulated mixed-precision training arithmetic in parametrised 1/e/m
 * floating-point formats on AMD MI355X (gfx950).
 *
 * The formats are those of the paper "Representation range needs for 16-bit neural
 * network training": one sign bit, e exponent bits with the usual ("vanilla") bias
 * 2^(e-1)-1, m stored mantissa bits with a hidden leading bit, and a flag that says
 * whether the denormal range is kept ("d") or flushed to zero ("n")  (Sec. III,
 * Def. III.1 and Def. III.2; Table I lists 1/5/10/d, 1/6/9/d and 1/8/7/n).  Derived
 * constants: Emax = bias, Emin = 1 - bias, minN = 2^Emin, minD = 2^(Emin-m),
 * maxN = (2 - 2^-m) * 2^Emax.
 *
 * Three operations are exported, each taking the format as the triple the paper's
 * rounding kernel takes (Sec. IV-A, roundfp_cuda(X, e, p, d)):
 *
 *   fmt_quantize   elementwise fp32 -> nearest value of the format (result kept as fp32),
 *                  optionally fused with the statistics of fmt_histogram
 *   fmt_histogram  per-tensor statistics: how many elements are zero / underflow /
 *                  denormal / normal / overflow / inf / nan in the format (the "denormal
 *                  fraction" the paper logs for every tensor, Sec. V) and a 64-bin
 *                  histogram of the elements' binades
 *   fmt_gemm       C = Q(op(A)) * Q(op(B)) with exact products and fp32 accumulation:
 *                  the FMACS instruction of Sec. III-B applied to a matrix product, as
 *                  used for fully connected layers and im2col convolutions in forward,
 *                  dgrad and wgrad (Sec. IV-A)
 * and, beyond these three:
 *   fmt_operand_bytes / fmt_prepare / fmt_prepare_pair / fmt_prepare_pair_batch / fmt_quantize_prepare_pair_batch /
 *   fmt_gemm_prepared / fmt_gemm_prepared_batch / fmt_linear_prepared   fmt_gemm (and fmt_linear) in two steps: a tensor is rounded once
 *                  into a reusable operand in caller-owned memory (Sec. IV-A rounds each tensor once and
 *                  uses it in several products), and products run on two such operands
 *   fmt_gemm_fmac8 the same product with the FMAC-8 accumulation of Algorithm 1 (Sec. IV-A)
 *   fmt_linear     the quantized fully connected layer of Sec. IV-A (product, bias, output roundings, statistics)
 *   fmt_pack16 / fmt_unpack16 / fmt_linear_pack16   the same roundings with the result stored as the
 *                  format's own 16-bit codes (Sec. III) instead of fp32: half the bytes written
 *   fmt_conv2d_*   convolution forward / dgrad / wgrad as the same product on patches gathered on the fly
 *   fmt_dls_step   loss-scale controller and denormal-fraction monitor on the device (Sec. II, Sec. V)
 *   fmt_quantize_static   fmt_quantize for callers that cannot allocate device memory
 *
 * Conventions common to all calls
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library never
 *     frees or keeps caller memory.  `stream` is a hipStream_t passed as void*
 *     (NULL = the default stream).  Calls are asynchronous on that stream: results are
 *     valid once the caller has synchronised with it.
 *   - The library keeps small per-(device, stream) scratch buffers of its own (partial
 *     histogram counts; pre-split GEMM operands).  They are created on first use with
 *     hipMalloc, grow when a larger problem arrives, and live until fmt_release_scratch()
 *     or process exit.  Calls on one stream are serialised by the stream; calls on
 *     different streams use different scratch and may overlap.  Once a call of the same
 *     kind and size has run on a stream, further calls on it neither allocate nor
 *     synchronise (scratch is cleared by kernels, not by memset), so they can be recorded
 *     into a HIP graph on that stream and replayed.  A recorded graph holds the addresses of
 *     the scratch it was recorded with: any later call on that stream that makes the scratch
 *     grow (a larger problem) frees the old buffers and INVALIDATES every graph recorded
 *     before it, as does fmt_release_scratch(); record again after either.  A call that
 *     would have to grow scratch while its stream is being captured allocates nothing,
 *     launches nothing and returns FMT_ERR_CAPTURE: run the same call once outside capture first.
 *   - Arguments are validated before any GPU call, so argument errors are reported
 *     even on a host without a GPU.  No exception or abort crosses this boundary:
 *     every call returns FMT_OK (0) or a negative fmt_status.
 *   - Supported formats: 2 <= e <= 8, 1 <= m <= 23 (the upper limits are the paper's,
 *     Sec. IV-A; the lower limits keep at least one normal binade and one mantissa bit).
 */
#ifndef FMT_H_
#define FMT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum fmt_status {
    FMT_OK = 0,
    FMT_ERR_FORMAT = -1, /* e outside [2,8] or m outside [1,23]                              */
    FMT_ERR_NULL = -2,   /* a required pointer is NULL                                       */
    FMT_ERR_SHAPE = -3,  /* negative dimension, leading dimension too small, size too large  */
    FMT_ERR_ALIGN = -4,  /* a data pointer is not aligned to its element size                */
    FMT_ERR_RANGE = -5,  /* a scalar parameter is out of range (exp_lo window, loss-scale parameters) */
    FMT_ERR_ALIAS = -6,  /* GEMM output overlaps an input                                    */
    FMT_ERR_HIP = -7,    /* a HIP runtime call failed (launch, allocation, no device)        */
    FMT_ERR_CAPTURE = -8 /* library scratch would have to grow while the stream is being captured */
} fmt_status;

/* The format triple of Def. III.2 (sign bits are always 1).
 * denorm: 1 = "d", denormal range allowed; 0 = "n", denormal results flushed to zero. */
typedef struct fmt_format {
    int32_t e;      /* exponent bits,        2..8  */
    int32_t m;      /* stored mantissa bits, 1..23 (the paper's p of Def. III.2 / Table I) */
    int32_t denorm; /* 1 = d, 0 = n */
} fmt_format_t;

#define FMT_NBINS 64
#define FMT_EXP_LO_MIN (-192)
#define FMT_EXP_LO_MAX 128
#define FMT_EXP_LO_DEFAULT (-48)

/*
 * Per-tensor statistics; lives in DEVICE memory (576 bytes, 8-byte aligned).
 * All members are integer counts, so the result does not depend on the order in which
 * the GPU visits the elements.
 *
 * Classes are judged on r = |Q_{e,m,d}(x)|, the magnitude after rounding with the
 * denormal range allowed -- for the "n" variant of a format the `denormal` count is
 * therefore exactly the number of elements the quantizer flushes:
 *   nan        x is NaN                         (not binned)
 *   inf        x is +-infinity                  (counted in the last bin)
 *   zero       x is +-0                         (not binned)
 *   underflow  x finite, non-zero, r == 0
 *   denormal   0 < r < minN
 *   normal     minN <= r <= maxN
 *   overflow   x finite, r == infinity
 * total = number of elements = sum of the seven classes.
 * bins[b] counts the non-zero, non-NaN elements with
 *   b = clamp(floor(log2|x|) - exp_lo, 0, FMT_NBINS-1),
 * i.e. one bin per binade of the INPUT over the window [exp_lo, exp_lo+63]; everything
 * below the window lands in bin 0, everything above it (and infinities) in bin 63.
 * The denormal fraction of Sec. V is denormal / total (or / (total - zero)).
 */
typedef struct fmt_hist {
    uint64_t total, zero, underflow, denormal, normal, overflow, inf, nan;
    uint64_t bins[FMT_NBINS];
} fmt_hist_t;

/*
 * fmt_quantize -- the rounding kernel of Sec. IV-A (roundfp_cuda(X, e, p, d)).
 *
 *   y[i] = Q_{e,m,d|n}(x[i]) for i in [0, n): round to nearest, ties to even, onto the
 *   values of the format; magnitudes that round to 2^(Emax+1) or more become +-infinity;
 *   magnitudes of at most minD/2 become +-0 (the tie at minD/2 goes to zero); with
 *   denorm == 0 any result below minN is replaced by +-0 (the flush acts on the rounded
 *   value, so inputs that round up to minN survive).  The sign of x is kept, also on
 *   zeros.  Any NaN becomes the quiet NaN 0x7FC00000.  fp32-denormal inputs are
 *   handled exactly.  The result is stored as fp32.
 *
 *   x     device, n contiguous floats, 4-byte aligned (16-byte alignment of x and y
 *         enables the fastest path; any 4-byte alignment is accepted)
 *   y     device, n floats; y == x (in place) is allowed, partial overlap is not
 *   hist  device, or NULL.  When given, the statistics of fmt_histogram(x, n, f, hist,
 *         exp_lo) are produced in the same pass over x; *hist is overwritten.
 *   n == 0 succeeds without a launch (*hist, when given, is zeroed).
 *   n must be below 2^40.
 */
int fmt_quantize(const float *x, float *y, size_t n, fmt_format_t f,
                 fmt_hist_t *hist, int32_t exp_lo, void *stream);

/*
 * fmt_quantize_static -- fmt_quantize for callers that cannot allocate device memory: code that runs
 * under HIP graph capture from its first call on, tight serving loops, harnesses that forbid
 * hipMalloc.  Arguments, result and errors are fmt_quantize's, bit for bit; the difference is where
 * the partial statistics records live while the pass runs: not in per-(device, stream) scratch that
 * is created with hipMalloc on first use, but in a fixed array of FMT_STATIC_SCRATCH_BYTES inside the
 * library's device image, of which every GPU holds one copy from the moment the library is loaded
 * there until the process ends.  The call allocates and frees nothing, on the device or through any
 * library, and never synchronises.
 *   - n must not exceed FMT_STATIC_MAX_ELEMENTS (else FMT_ERR_SHAPE, nothing is launched).
 *   - All calls on one GPU share that GPU's array, whatever their stream: calls with statistics that
 *     overlap in time on one GPU race on it and give wrong counts.  Put them on one stream, or order
 *     them with events.  (Calls with hist == NULL do not touch the array.)
 *   - The array keeps the last call's contents; the call clears it on the stream before it counts.
 */
#define FMT_STATIC_SCRATCH_BYTES 36864
#define FMT_STATIC_MAX_ELEMENTS ((size_t)1 << 36)
int fmt_quantize_static(const float *x, float *y, size_t n, fmt_format_t f,
                        fmt_hist_t *hist, int32_t exp_lo, void *stream);

/*
 * fmt_histogram -- per-tensor statistics without writing a quantized copy (the
 * logging of Sec. V: denormal fraction of activations, weights and gradients).
 * *hist (device) is overwritten with the counts described at fmt_hist_t.  The counts
 * do not depend on f.denorm.  n == 0 zeroes *hist.  n must be below 2^40.
 */
int fmt_histogram(const float *x, size_t n, fmt_format_t f,
                  fmt_hist_t *hist, int32_t exp_lo, void *stream);

/*
 * fmt_gemm -- matrix product with FMACS semantics (Sec. III-B: a32 = o(a32 + x16*y16);
 * Sec. IV-A: operands are rounded to the format, products are not rounded).
 *
 *   C[i][j] = sum_k Q(op(A))[i][k] * Q(op(B))[k][j],   i < M, j < N, k < K
 *
 * Each product is exact; the sum is accumulated in fp32 (order unspecified) and C is
 * returned as unrounded fp32 -- the caller applies fmt_quantize to C where the layer
 * formula of Sec. IV-A rounds the output.  Row-major storage, leading dimensions in
 * elements:
 *   transA == 0: A is M x K (lda >= K);   transA != 0: A is K x M (lda >= M)
 *   transB == 0: B is K x N (ldb >= N);   transB != 0: B is N x K (ldb >= K)
 *   C is M x N (ldc >= N).
 * A fully connected layer Y = X W^T is (transA, transB) = (0, 1); its dgrad dX = dY W is
 * (0, 0); its wgrad dW = dY^T X is (1, 0).  A convolution is the same three products on
 * the im2col matrix, which the caller materialises.
 * A, B, C are device pointers, 4-byte aligned; C must not overlap A or B.  M, N or K
 * equal to 0 succeeds (K == 0 with M, N > 0 zero-fills C).  Dimensions must be below 2^31.
 * Infinite or NaN operands (including finite inputs that overflow the format) give
 * non-finite results in exactly the affected outputs: NaN where the sum of Sec. III-B is NaN;
 * where that sum is an infinity, that infinity or NaN (which of the two is not specified).
 * Formats with e == 8 and m >= 8 (fp32's exponent range with more mantissa than bfloat16; none of
 * the paper's): an operand value enters the products without its bits below 2^-133, i.e. values
 * of magnitude below 2^(m-133) may lose up to 2^-133; every other format, 1/8/7 included, is exact.
 * This holds for every product call of this header (prepared operands, fmt_linear, convolutions).
 */
int fmt_gemm(int transA, int transB, int64_t M, int64_t N, int64_t K,
             const float *A, int64_t lda, const float *B, int64_t ldb,
             float *C, int64_t ldc, fmt_format_t f, void *stream);

/*
 * Prepared operands -- the rounded operand of a product, made once and used by every product that
 * needs it.
 *
 * Sec. IV-A rounds a tensor where it enters a layer and then uses the ROUNDED tensor wherever the
 * layer needs it: R(X) feeds the forward product and the weight gradient, R(W) the forward product
 * and the input gradient, R(dY) both gradients.  fmt_gemm is handed fp32 operands and has to round
 * and re-lay them out on every call; fmt_prepare does that work once per tensor and orientation and
 * leaves the result -- the values of Q(op(X)) in the 16-bit operand layout of the matrix cores -- in
 * memory the CALLER owns, and fmt_gemm_prepared multiplies two such operands with one kernel launch:
 *
 *     C[i][j] = sum_k Q(a)[i][k] * Q(b)[j][k]        (exact products, fp32 accumulation: FMACS, Sec. III-B)
 *
 * bit for bit what fmt_gemm returns for the same operands (same kernels, same order of accumulation).
 *
 * fmt_operand_bytes  size in bytes of the device buffer a prepared operand of `rows` x `k` needs.
 * fmt_prepare        op(X) is `rows` x `k`: trans == 0: X is rows x k, row-major, ld >= k;
 *                    trans != 0: X is k x rows, row-major, ld >= rows (the operand is X transposed).
 *                    data: device memory of at least fmt_operand_bytes(rows, k, f) bytes, 256-byte
 *                    aligned, not overlapping X; *op (HOST memory) is filled in and describes the
 *                    operand from then on.  The library keeps no reference to either; the operand is
 *                    valid once the stream has executed the call and until the caller overwrites or
 *                    frees `data`.  fmt_prepare uses no library scratch, allocates nothing, and can be
 *                    recorded into a graph.
 * fmt_gemm_prepared  A->rows = M, B->rows = N, A->k == B->k = K, same format and same scheme (operands
 *                    prepared by the same build with the same environment); C is M x N, ldc >= N, must
 *                    not overlap either operand.  For a fully connected layer with X [batch, in],
 *                    W [out, in], dY [batch, out]:  Y = (X, trans 0)(W, trans 0);  dX = (dY, trans 0)
 *                    (W, trans 1);  dW = (dY, trans 1)(X, trans 1).
 * rows, k >= 1 and below 2^31; non-finite operands as for fmt_gemm.  Errors as for fmt_gemm;
 * FMT_ERR_SHAPE also when `bytes` is too small or the two operands do not fit each other,
 * FMT_ERR_FORMAT when their formats or schemes differ.
 */
typedef struct fmt_operand {
    void *data;            /* device buffer (caller-owned) */
    size_t bytes;          /* its size */
    int64_t rows, k;       /* op(X) is rows x k */
    fmt_format_t format;
    int32_t scheme;        /* how the values are represented for the matrix cores (set by fmt_prepare) */
} fmt_operand_t;

int fmt_operand_bytes(int64_t rows, int64_t k, fmt_format_t f, size_t *bytes);
int fmt_prepare(const float *X, int64_t ld, int trans, int64_t rows, int64_t k, fmt_format_t f,
                void *data, size_t bytes, fmt_operand_t *op, void *stream);

/*
 * fmt_prepare_pair -- both orientations of one matrix X (rows x cols, element (r, c) at X[r*ld + c], ld >= cols) in
 * one call: `op` = X as stored (rows = rows, k = cols), `op_t` = X transposed (rows = cols, k = rows), exactly the
 * operands that fmt_prepare(X, ld, 0, rows, cols, ...) and fmt_prepare(X, ld, 1, cols, rows, ...) produce, in
 * data / data_t (sizes from fmt_operand_bytes(rows, cols, ...) and fmt_operand_bytes(cols, rows, ...); the two
 * buffers must not overlap each other or X).  A training step uses each of X, W and dY in both orientations
 * (Sec. IV-A: Y = X W^T, dX = dY W, dW = dY^T X), and preparing the two together takes half the launches.
 * Errors as for fmt_prepare.
 */
int fmt_prepare_pair(const float *X, int64_t ld, int64_t rows, int64_t cols, fmt_format_t f,
                     void *data, size_t bytes, fmt_operand_t *op,
                     void *data_t, size_t bytes_t, fmt_operand_t *op_t, void *stream);

/*
 * fmt_prepare_pair_batch -- fmt_prepare_pair for `count` matrices in one call: matrix i is X[i] (rows[i] x cols[i],
 * leading dimension ld[i]), its operands go to data[i] (bytes[i]) and data_t[i] (bytes_t[i]) and are described in
 * op[i] and op_t[i].  All arrays are HOST arrays of `count` entries (op and op_t are written); X[i], data[i] and
 * data_t[i] are DEVICE pointers.  One format for all.  The operands equal fmt_prepare_pair's (products on them give
 * the same bits).  The tensors of a layer's step (Sec. IV-A: input, weights and incoming gradient, each rounded
 * once and used in both orientations) are small enough that one launch per tensor leaves the device partly idle;
 * formats whose operands are exponent planes (1/6/m) share one statistics launch and one prepare launch per 16
 * matrices, other formats are prepared matrix by matrix.
 * Errors: count < 0 or > 4096 -> FMT_ERR_SHAPE (0 is a no-op); a NULL array or entry -> FMT_ERR_NULL; per matrix as
 * for fmt_prepare_pair; a prepared buffer that overlaps another matrix's buffers or any input -> FMT_ERR_ALIAS.
 * Everything is checked before the first launch; no device memory is allocated.
 */
int fmt_prepare_pair_batch(int64_t count, const float *const *X, const int64_t *ld, const int64_t *rows, const int64_t *cols,
                           fmt_format_t f, void *const *data, const size_t *bytes, fmt_operand_t *op,
                           void *const *data_t, const size_t *bytes_t, fmt_operand_t *op_t, void *stream);
/*
 * fmt_quantize_prepare_pair_batch -- the whole rounding pass of Sec. IV-A over `count` matrices in one call: for
 * matrix i what fmt_quantize gives (the rounded values as fp32 in Y[i], leading dimension ldy[i] >= cols[i]; the
 * statistics of Sec. V in the DEVICE record hist[i], window exp_lo .. exp_lo + 63) and what fmt_prepare_pair_batch
 * gives (both prepared orientations), from ONE read of X[i].  Formats whose prepared operands are exponent planes
 * only (1/6/m); other formats -> FMT_ERR_FORMAT (use fmt_quantize and fmt_prepare_pair_batch).  Y[i] may be X[i]
 * (same address and leading dimension: in place); otherwise nothing written may overlap anything else of the call
 * (FMT_ERR_ALIAS).  Arrays are HOST arrays of `count` entries; Y[i], hist[i], data[i], data_t[i] DEVICE pointers
 * (hist[i] 8-byte aligned).  Other arguments and errors as for fmt_prepare_pair_batch; FMT_ERR_RANGE for exp_lo as
 * for fmt_quantize.  Uses the stream's library scratch for the partial statistics records (576 KiB against the
 * 36 KiB of fmt_quantize: the first call on a stream makes that scratch grow, which invalidates graphs recorded on
 * the stream before it, and cannot happen inside a capture -- run the call once eagerly first; see the notes on
 * scratch at the top).
 */
int fmt_quantize_prepare_pair_batch(int64_t count, const float *const *X, const int64_t *ld, const int64_t *rows,
                                    const int64_t *cols, fmt_format_t f, float *const *Y, const int64_t *ldy,
                                    fmt_hist_t *const *hist, int32_t exp_lo, void *const *data, const size_t *bytes,
                                    fmt_operand_t *op, void *const *data_t, const size_t *bytes_t, fmt_operand_t *op_t,
                                    void *stream);
int fmt_gemm_prepared(const fmt_operand_t *A, const fmt_operand_t *B, float *C, int64_t ldc, void *stream);

/*
 * fmt_gemm_prepared_batch -- `count` independent products on prepared operands in one call:
 * C[i] = A[i] B[i]^T for i in [0, count), each exactly what fmt_gemm_prepared(A[i], B[i], C[i], ldc[i]) computes
 * (the FMACS sums of Sec. III-B; the order of accumulation is unspecified in both).  A training step of a
 * network holds many products of modest size whose operands are all known when the step's tensors have been
 * rounded (Sec. IV-A: three products per layer); handing them over together lets the library run the small
 * ones in shared kernel launches, so that a launch's start-up and drain are paid once per batch and not once
 * per product.  An operand may serve several products of the batch.
 * A, B, C, ldc: HOST arrays of `count` entries (read before the call returns); the fmt_operand_t they point to
 * are host memory as everywhere.  All operands of the batch share one format and one scheme (FMT_ERR_FORMAT
 * otherwise).  No C[i] may overlap another C[j] or any operand of the batch (FMT_ERR_ALIAS): the products are
 * not ordered among themselves.  count == 0 succeeds; count < 0 or > 4096: FMT_ERR_SHAPE.  Other errors as for
 * fmt_gemm_prepared, found before anything is launched.  Uses the library's per-stream scratch only for the
 * products that fmt_gemm_prepared itself would split over k.
 */
int fmt_gemm_prepared_batch(int64_t count, const fmt_operand_t *const *A, const fmt_operand_t *const *B,
                            float *const *C, const int64_t *ldc, void *stream);

/*
 * fmt_linear_prepared -- fmt_linear (below) on operands prepared with fmt_prepare: the quantized fully connected
 * layer of Sec. IV-A, Y = R( R(acc) + R(b) ) with acc[i][j] = sum_k Q(x)[i][k] Q(w)[j][k], where X holds the
 * M = X->rows rows of the input and W the N = W->rows rows of the weight matrix (both with the same k, format and
 * scheme; the format is the operands').  b (N values, may be NULL: no bias), Y (M x N, ldy >= N), hist
 * (may be NULL) and exp_lo as for fmt_linear; the result and the statistics are those of fmt_linear on the tensors
 * the operands were prepared from whenever the accumulation order does not matter (it is unspecified in both).
 * A weight operand prepared once serves every forward call until the weights change.  Errors as for
 * fmt_gemm_prepared and fmt_linear.
 */
int fmt_linear_prepared(const fmt_operand_t *X, const fmt_operand_t *W, const float *b, float *Y, int64_t ldy,
                        fmt_hist_t *hist, int32_t exp_lo, void *stream);

/*
 * fmt_gemm_fmac8 -- matrix product with the FMAC-8 accumulation of Sec. IV-A, Algorithm 1, for
 * hardware that only offers FMAC (Sec. III-B: a16 = o(a16 + x16*y16), one rounding).
 *
 * C[i][j] is the dot product of row i of Q(op(A)) and column j of Q(op(B)) computed exactly as
 * the algorithm lists it: a 16-bit accumulator a (a value of the format) takes 8 consecutive
 * fused multiply-adds, each rounding the EXACT sum a + w_k*x_k once to the format (with the
 * format's overflow and denormal/flush rules); at every k that is a multiple of 8 it is first
 * added into an fp32 master accumulator with an fp32 addition and reset to zero; after the last
 * k the master takes the last a and the result is Q(master), stored as fp32.  The order of the
 * roundings is fixed by the algorithm, so the result is reproducible bit for bit.
 *
 * Arguments, layouts, limits and errors as for fmt_gemm (K == 0 gives zeros).  This path runs
 * on the vector ALUs (a sequential chain of roundings per output), not on the matrix cores.
 */
int fmt_gemm_fmac8(int transA, int transB, int64_t M, int64_t N, int64_t K,
                   const float *A, int64_t lda, const float *B, int64_t ldb,
                   float *C, int64_t ldc, fmt_format_t f, void *stream);

/*
 * fmt_linear -- forward pass of the quantized fully connected layer of Sec. IV-A:
 *
 *     Y = R( R( R(X) R(W)^T ) + R(b) )
 *
 * X is the M x K input (row-major, leading dimension ldx >= K; M = batch), W the N x K weight
 * ([out, in] as the layer stores it, ldw >= K), b the bias of N values or NULL, Y the M x N
 * output (ldy >= N).  R is fmt_quantize's rounding to format f; the inner product is fmt_gemm's
 * (exact products of the rounded operands, fp32 accumulation, see there for its error bound);
 * its result is rounded to the format, the rounded bias is added with ONE single-precision
 * addition, and the sum t is rounded again.  Given the accumulator values, t and Y are
 * determined bit for bit.
 *
 * If hist is not NULL it receives the statistics (Sec. V, as fmt_histogram defines them, window
 * starting at 2^exp_lo) of t = R(acc) + R(b), the M*N values that enter the last rounding: the
 * classes say what that rounding does to the layer's output (how much underflows, overflows or
 * lands in the denormal range).  hist is a DEVICE pointer; exp_lo is ignored when hist is NULL.
 *
 * All pointers are device pointers, 4-byte aligned; Y must not overlap X, W or b.  M or N equal
 * to 0 succeeds (an all-zero fmt_hist_t is written); K == 0 gives t = R(b).  Dimensions and
 * leading dimensions must be below 2^31.  Errors as for fmt_gemm and fmt_histogram.
 */
int fmt_linear(int64_t M, int64_t N, int64_t K,
               const float *X, int64_t ldx, const float *W, int64_t ldw, const float *b,
               float *Y, int64_t ldy, fmt_format_t f,
               fmt_hist_t *hist, int32_t exp_lo, void *stream);

/*
 * Packed storage.  A value of a 1/e/m format with 1 + e + m <= 16 has a code of that many bits
 * (Sec. III: Def. III.1 with the hidden bit not stored, the "vanilla" bias, and the reserved
 * encodings), kept in the low bits of a uint16_t, upper bits zero:
 *     bit e+m          sign
 *     bits [m, e+m)    stored exponent: 0 = zero / denormal range (value = mantissa * 2^(Emin-m)),
 *                      2^e - 1 = infinity (mantissa 0) or NaN, otherwise E + bias
 *     bits [0, m)      stored mantissa (normal numbers: the bits after the hidden leading 1)
 * 1/5/10 codes are IEEE binary16 patterns, 1/8/7 codes are bfloat16 patterns (the upper half of the
 * fp32 pattern).  Formats with 1 + e + m > 16 have no such code: FMT_ERR_FORMAT.
 *
 * fmt_pack16   codes[i] = code of Q_{e,m,d|n}(x[i]), the rounding of fmt_quantize (any NaN gives the
 *              quiet-NaN code: sign 0, exponent all ones, top mantissa bit).  hist as in fmt_quantize:
 *              statistics of x in the same pass, or NULL.  6 bytes move per element instead of 8.
 *              codes: device, n uint16_t, 2-byte aligned (8-byte alignment, with x 16-byte aligned,
 *              enables the fastest path); must not overlap x.
 * fmt_unpack16 y[i] = value of codes[i] as fp32 (exact; NaN codes give 0x7FC00000; bits of a code
 *              above bit e+m are ignored).  f.denorm is not used: a code of the denormal range is
 *              decoded as what it says.  y must not overlap codes.
 * n == 0 succeeds without a launch (*hist, when given, is zeroed).  n must be below 2^40.
 */
int fmt_pack16(const float *x, uint16_t *codes, size_t n, fmt_format_t f,
               fmt_hist_t *hist, int32_t exp_lo, void *stream);
int fmt_unpack16(const uint16_t *codes, float *y, size_t n, fmt_format_t f, void *stream);

/*
 * fmt_linear_pack16 -- fmt_linear with the layer's output stored as 16-bit codes (see fmt_pack16):
 * Y16[i][j] = code of Y[i][j], the M x N result of fmt_linear (ldy >= N, in uint16_t elements).
 * The fp32 accumulators live in library scratch (M*N floats, grown on first use like the other
 * scratch), so the output stage reads 4 bytes and writes 2 per element.  Everything else --
 * arguments, statistics, limits, errors -- as for fmt_linear; needs 1 + e + m <= 16.
 */
int fmt_linear_pack16(int64_t M, int64_t N, int64_t K,
                      const float *X, int64_t ldx, const float *W, int64_t ldw, const float *b,
                      uint16_t *Y16, int64_t ldy, fmt_format_t f,
                      fmt_hist_t *hist, int32_t exp_lo, void *stream);

/*
 * Convolution layers (Sec. IV-A: the inner matrix multiplies "or convolutions" of the forward and
 * backward pass use FMACS -- operands rounded to the format, products not rounded, fp32
 * accumulation).  2-D convolution with zero padding, no dilation, no groups, on dense tensors:
 *   X, dX   [n][c][h][w]            (NCHW)
 *   W, dW   [k][c][r][s]            (k filters)
 *   Y, dY   [n][k][P][Q],  P = (h + 2 pad_h - r) / stride_h + 1,  Q = (w + 2 pad_w - s) / stride_w + 1
 *
 *   fmt_conv2d_fwd    Y[n][k][p][q]  = sum_{c,r,s} Q(X)[n][c][p*stride_h - pad_h + r][q*stride_w - pad_w + s] * Q(W)[k][c][r][s]
 *   fmt_conv2d_dgrad  dX[n][c][h][w] = sum over (k, r, s) and the (p, q) with p*stride_h - pad_h + r = h,
 *                                      q*stride_w - pad_w + s = w  of  Q(dY)[n][k][p][q] * Q(W)[k][c][r][s]
 *   fmt_conv2d_wgrad  dW[k][c][r][s] = sum_{n,p,q} Q(dY)[n][k][p][q] * Q(X)[n][c][p*stride_h - pad_h + r][q*stride_w - pad_w + s]
 * (positions outside the tensor contribute zero).  These are fmt_gemm's products on the patch
 * matrix of the convolution -- same rounding of the operands, exact products, fp32 accumulation in
 * unspecified order, unrounded fp32 result, same error bound -- but nobody forms the fp32 patch
 * matrix (r*s times the size of the tensor): the tensor is rounded once into 16-bit pieces in library
 * scratch (2 bytes per tensor element and piece of the format; freed by fmt_release_scratch) and the
 * patches are gathered from that.  fmt_conv2d_fwd with c a multiple of 32, and fmt_conv2d_dgrad with k a
 * multiple of 32 and stride 1, both with r*s <= 32, gather inside the product kernel: their scratch is of
 * the size of the tensor.  The other cases and fmt_conv2d_wgrad gather in the operand preparation, into a
 * 16-bit operand of the size of the patch matrix (2 bytes per patch element and piece) in scratch.
 *
 * All pointers are device pointers, 4-byte aligned; the output must not overlap an input.
 * Sizes: n, c, k >= 0; h, w, r, s >= 1; pad >= 0; stride >= 1; h + 2 pad_h >= r, w + 2 pad_w >= s;
 * every tensor and each of n*P*Q, n*h*w, c*r*s, k*r*s must have fewer than 2^31 elements
 * (else FMT_ERR_SHAPE).  An empty output succeeds without a launch; an empty sum gives zeros.
 */
typedef struct fmt_conv2d {
    int32_t n, c, h, w;          /* input: batch, channels, height, width */
    int32_t k, r, s;             /* filters, filter height, filter width  */
    int32_t pad_h, pad_w, stride_h, stride_w;
} fmt_conv2d_t;

int fmt_conv2d_fwd(fmt_conv2d_t g, const float *X, const float *W, float *Y, fmt_format_t f, void *stream);
int fmt_conv2d_dgrad(fmt_conv2d_t g, const float *dY, const float *W, float *dX, fmt_format_t f, void *stream);
int fmt_conv2d_wgrad(fmt_conv2d_t g, const float *dY, const float *X, float *dW, fmt_format_t f, void *stream);

/*
 * Loss scaling (Sec. II) and the per-step monitoring of Sec. V, kept on the device so that a
 * training step never waits for the host.
 *
 * Sec. II: the loss is multiplied by a factor S before backpropagation so that small activation
 * gradients do not fall into the denormal range or underflow; weight gradients are divided by S
 * before the update; dynamic loss scaling chooses S from the gradients themselves.  Sec. V: the
 * denormal fraction of every tensor is logged as it is computed and the highest fraction observed
 * over all tensors is reported.  The paper states no update rule or parameters; the controller
 * here is the customary one, with every parameter supplied by the caller.
 *
 * fmt_dls_state_t lives in DEVICE memory (8-byte aligned).  fmt_dls_init writes a fresh state.
 * fmt_dls_step inspects the statistics of one training step -- `count` fmt_hist_t records,
 * contiguous in device memory, of the step's (scaled) gradient tensors, as produced by
 * fmt_quantize / fmt_histogram / fmt_linear -- and updates *state:
 *   nonfinite     = sum over the records of overflow + inf + nan
 *   nonfinite > 0 : skip = 1 (the caller must drop this step's update),
 *                   loss_scale = max(loss_scale * backoff, min_scale), good_steps = 0
 *   otherwise     : skip = 0, good_steps += 1, and when good_steps reaches `interval`:
 *                   loss_scale = min(loss_scale * growth, max_scale), good_steps = 0
 *   worst_*       = index and counts of the record with the largest denormal / total (fp64
 *                   quotient; records with total == 0 are ignored; ties go to the lowest index;
 *                   worst_tensor = -1 when there is none)
 *   peak_*        = the largest such fraction over all steps so far, with the step (0-based) and
 *                   the record index where it occurred; replaced only by a strictly larger one
 *   steps        += 1
 * The two products are single-precision multiplications, so the sequence of scales is reproducible
 * bit for bit.  count == 0 is a clean step without tensors.
 * Parameter limits (else FMT_ERR_RANGE): growth >= 1, 0 < backoff <= 1, interval >= 1,
 * 0 < min_scale <= max_scale, all finite; fmt_dls_init: loss_scale > 0 and finite.
 */
typedef struct fmt_dls_state {
    float loss_scale;      /* S: multiply the loss by it, divide the weight gradients by it */
    int32_t good_steps;    /* length of the current run of steps without non-finite gradients */
    int32_t skip;          /* 1: the step just inspected must be skipped */
    int32_t steps;         /* steps inspected so far */
    uint64_t nonfinite;    /* overflow + inf + nan over the records of the last step */
    int64_t worst_tensor;  /* last step: record with the largest denormal fraction, or -1 */
    uint64_t worst_denormal, worst_total;
    int64_t peak_tensor;   /* all steps: where the largest denormal fraction occurred, or -1 */
    int64_t peak_step;
    uint64_t peak_denormal, peak_total;
} fmt_dls_state_t;

typedef struct fmt_dls_params {
    float growth;          /* factor applied after `interval` clean steps, e.g. 2   */
    float backoff;         /* factor applied on a non-finite gradient, e.g. 0.5     */
    int32_t interval;      /* clean steps before the scale grows, e.g. 2000         */
    float min_scale;
    float max_scale;
} fmt_dls_params_t;

int fmt_dls_init(fmt_dls_state_t *state, float loss_scale, void *stream);
int fmt_dls_step(const fmt_hist_t *hists, int64_t count, fmt_dls_params_t prm,
                 fmt_dls_state_t *state, void *stream);

/*
 * fmt_format_info -- closed-form constants of a format (Sec. III; Table I), computed on
 * the host.  Any output pointer may be NULL.  Returns FMT_ERR_FORMAT for an unsupported
 * format.
 */
int fmt_format_info(fmt_format_t f, double *maxN, double *minN, double *minD,
                    int32_t *Emin, int32_t *Emax);

/*
 * fmt_format_thresholds -- the three decision thresholds of a format on the fp32 bit pattern
 * of |x| (sign bit cleared; the pattern is monotone in |x|), computed on the host:
 *   out[0] = t_zero: Q(x) is +-0            <=>  pattern <= t_zero   (pattern of minD/2)
 *   out[1] = t_den:  |Q_d(x)| < minN        <=>  pattern <  t_den    (pattern of minN - minD/2)
 *   out[2] = t_ovf:  Q(x) is +-infinity     <=>  pattern >= t_ovf, pattern <= 0x7F800000
 * These are the comparisons the kernels use for the underflow, flush and overflow rules of
 * fmt_quantize and for the classes of fmt_hist_t; exported so that they can be checked on a
 * host without a GPU.  out is a HOST pointer to three uint32_t.
 */
int fmt_format_thresholds(fmt_format_t f, uint32_t *out);

/*
 * fmt_scratch_bytes -- bytes of library-owned scratch that the current device holds for `stream`
 * right now: out[0] partial statistics records, out[1] the product workspace (prepared operands of
 * fmt_gemm / fmt_linear / the convolutions, rounded convolution tensors, split-k partial sums),
 * out[2] the accumulators of fmt_linear_pack16.  out is a HOST pointer to three size_t.  Host-only
 * bookkeeping: no GPU call besides looking up the current device, no synchronisation.
 */
int fmt_scratch_bytes(void *stream, size_t *out);

/* Frees the library-owned scratch buffers of the current device (synchronises it first). */
int fmt_release_scratch(void);

/* Human-readable name of a status code; never NULL. */
const char *fmt_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* FMT_H_ */
