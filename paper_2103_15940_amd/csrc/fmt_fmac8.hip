// fmt_gemm_fmac8: matrix product with the FMAC-8 accumulation of Sec. IV-A, Algorithm 1.
//
// Every output element is a dot product taken in groups of 8 consecutive k: inside a group a 16-bit
// accumulator a (a value of the format, starting at zero) takes 8 fused multiply-adds,
// a = Q(a + w_k * x_k) with ONE rounding of the exact sum to the format (FMAC of Sec. III-B); after
// the group it is added into an fp32 master accumulator with one fp32 addition; the result is
// Q(master).  (Operands are zero-padded to whole groups: a + 0 * 0 = a is a value of the format, so a
// padded step changes nothing.)  The chain of roundings is sequential by definition, so this is plain
// ALU work (no matrix cores), bound by the rate at which the vector units issue instructions: one per
// lane and clock.
//
// Formats with e <= 6 and m <= 11 run the fused step in single precision around the hardware's own
// fused multiply-add, s = fma(w, x, a): the exact sum rounded ONCE to 24 bits.  Rounding s to the
// format afterwards equals rounding the exact sum directly unless s lands exactly on a midpoint of
// the format's grid while the exact sum does not; only a wave that holds such a lane (rare) computes
// the exact error of the sum and puts that lane on the side of the midpoint where the exact sum lies.
// 14 vector instructions per fused step instead of 22.
//
// The fused step is done in fp64: the product of two <= 24-bit significands is exact; the sum
// a + w*x is rounded to odd (TwoSum gives the exact error; if it is non-zero and the fp64 sum is
// the even neighbour, step to the odd one), which makes the following rounding to the format
// (<= 24 significant bits) equal to a single rounding of the exact sum.  That rounding uses
// (|s| + C) - C with C = 2^(max(E,Emin) - m + 52), the fp64 adder's own round-to-nearest-even.
#include <cstdlib>
#include <type_traits>

#include "fmt_internal.h"
#include "fmt_quant.h"

namespace fmt {

struct Fmac8Params {
    double ovf;          // magnitudes >= ovf round to infinity: (2 - 2^-(m+1)) * 2^Emax
    double minn;         // 2^Emin
    int32_t emin_biased; // Emin + 1023 (fp64 exponent field of minN)
    int32_t m;
    int32_t ftz;
};

// Q_{e,m,d|n} of an fp64 value that is either exact or rounded to odd; result as fp64 (a value of the format).
__device__ __forceinline__ double quantize_f64(double s, const Fmac8Params &f)
{
    const double as = fabs(s);
    const uint64_t ebits = (uint64_t)(__double_as_longlong(as) >> 52);
    const uint64_t ce = (ebits > (uint64_t)f.emin_biased ? ebits : (uint64_t)f.emin_biased) + (uint64_t)(52 - f.m);
    const double c = __longlong_as_double((long long)(ce << 52));
    double r = (as + c) - c;                       // RNE on the format's grid; NaN stays NaN
    if (f.ftz && r < f.minn) r = 0.0;
    if (as >= f.ovf) r = __longlong_as_double(0x7FF0000000000000ll);   // overflow and infinities
    return copysign(r, s);
}

// a + p rounded to odd (p = w*x exact).
__device__ __forceinline__ double add_round_to_odd(double a, double p)
{
    double s = a + p;
    const double bb = s - a;
    const double err = (a - (s - bb)) + (p - bb);  // exact error of the fp64 addition (TwoSum)
    long long u = __double_as_longlong(s);
    // err != 0 (and finite): the exact sum lies strictly between s and its neighbour on err's side
    if (err != 0.0 && err == err && (u & 1ll) == 0) {
        const bool away = (err > 0.0) == (s > 0.0);  // neighbour further from zero <=> pattern + 1
        u += away ? 1ll : -1ll;
        s = __longlong_as_double(u);
    }
    return s;
}

// The fused step in single precision, for formats with e <= 6 and m <= 11: the product of two
// (m+1)-bit significands has at most 24 bits and, with Emin >= -30, lies in fp32's normal range, so
// w * x and the error term of TwoSum are exact in fp32.
// The step around the hardware FMA (see the top of the file), in two parts so that the rare exact
// correction costs one branch per 16 steps instead of one per step.
struct FmaConsts {
    float minn, tovf, inf2;     // 2^Emin; the input magnitude from which the result is infinite; 2^(Emax+1)
};

// Common path: returns Q(fma(w, x, a)) and, in `tie`, whether the 24-bit sum sits exactly on a midpoint
// of the format's grid (then fmac_fix decides).  FIRST: the step from a zero accumulator -- the sum is the
// product itself, exact in 24 bits, so its rounding needs no second look (a midpoint there is a true tie).
template <bool FTZ, bool FIRST = false>
__device__ __forceinline__ float fmac_try(float a, float w, float x, const QuantParams &qp, const FmaConsts &k, bool &tie)
{
    const float s = FIRST ? __fmul_rn(w, x) : __fmaf_rn(w, x, a);   // exact product, exact sum, one rounding to 24 bits
    // C = 2^(max(E, Emin) + 23 - m): (|s| + C) - C rounds |s| to the format's grid around it (RNE).  For an
    // infinite or NaN s the pattern of C is a NaN, so r is: the selection below restores the infinity.
    const uint32_t ce = max(__float_as_uint(s) & 0x7F800000u, qp.minn_bits) + qp.shift23;
    const float c = __uint_as_float(ce), fa = fabsf(s);
    float r = __fsub_rn(__fadd_rn(fa, c), c);
    tie = !FIRST && fabsf(__fsub_rn(fa, r)) == __uint_as_float(ce - (24u << 23));   // moved by exactly half a step, C * 2^-24
    if (FTZ) r = r < k.minn ? 0.0f : r;                   // the flush acts on the rounded value
    r = fa >= k.tovf ? __uint_as_float(0x7F800000u) : r;  // false for NaN, which stays NaN
    return copysignf(r, s);
}

// Exact correction for the lanes where fmac_try reported a midpoint: a + w*x = s + err exactly (TwoSum on
// the exact product); a non-zero err puts the exact sum off the midpoint, on err's side, and the result
// is the grid neighbour on that side.
template <bool FTZ>
__device__ __forceinline__ float fmac_fix(float tried, float a, float w, float x, const QuantParams &qp, const FmaConsts &k)
{
    const float p = __fmul_rn(w, x);                       // exact (two (m+1)-bit significands)
    const float s = __fadd_rn(a, p);                       // the same 24-bit sum the FMA gave
    const float bb = __fsub_rn(s, a);
    const float err = __fadd_rn(__fsub_rn(a, __fsub_rn(s, bb)), __fsub_rn(p, bb));
    const uint32_t ce = max(__float_as_uint(s) & 0x7F800000u, qp.minn_bits) + qp.shift23;
    const float c = __uint_as_float(ce), fa = fabsf(s), half = __uint_as_float(ce - (24u << 23));
    const float r0 = __fsub_rn(__fadd_rn(fa, c), c);
    const bool tie = fabsf(__fsub_rn(fa, r0)) == half;
    if (!tie || !(err != 0.0f)) return tried;              // a true tie keeps the even neighbour the adder chose
    float r = ((err > 0.0f) == (s > 0.0f)) ? __fadd_rn(fa, half) : __fsub_rn(fa, half);
    if (FTZ) r = r < k.minn ? 0.0f : r;
    r = r >= k.inf2 ? __uint_as_float(0x7F800000u) : r;
    return copysignf(r, s);
}

constexpr int kFTile = 64;     // outputs per workgroup edge
constexpr int kFK = 32;        // k per LDS stage (a multiple of 8: FMAC-8 groups never straddle stages)

template <int MODE, bool FTZ, bool F32>
__global__ __launch_bounds__(256) void fmac8_kernel(const uint32_t *__restrict__ A, int64_t lda, int transA,
                                                    const uint32_t *__restrict__ B, int64_t ldb, int transB,
                                                    float *__restrict__ C, int64_t ldc, int M, int N, int K,
                                                    int tiles_n, QuantParams qp, Fmac8Params fp)
{
    __shared__ float sa[kFK][kFTile + 4];          // rounded operand values, [k][row]
    __shared__ float sb[kFK][kFTile + 4];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int row0 = (blockIdx.x / tiles_n) * kFTile, col0 = (blockIdx.x % tiles_n) * kFTile;

    typedef typename std::conditional<F32, float, double>::type acc_t;
    float acc32[4][4];                             // the fp32 master accumulators
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc32[i][j] = 0.0f;
    const FmaConsts fk = {__uint_as_float(qp.minn_bits), __uint_as_float(qp.t_ovf),
                          __uint_as_float((qp.t_ovf & 0x7F800000u) + 0x00800000u)};   // t_ovf lies in the top binade

    for (int k0 = 0; k0 < K; k0 += kFK) {
        // stage: 64 x 32 values of each operand, rounded to the format on the way in
#pragma unroll
        for (int it = 0; it < 8; ++it) {
            const int idx = it * 256 + tid;
            // A: consecutive lanes walk k when k is contiguous in memory, rows otherwise
            const int ar = transA ? idx % kFTile : idx / kFK, ak = transA ? idx / kFTile : idx % kFK;
            const int br = transB ? idx / kFK : idx % kFTile, bk = transB ? idx % kFK : idx / kFTile;
            const int gr = row0 + ar, gk = k0 + ak;
            uint32_t va = 0u, vb = 0u;
            if (gr < M && gk < K) va = transA ? A[(size_t)gk * lda + gr] : A[(size_t)gr * lda + gk];
            const int gc = col0 + br, gkb = k0 + bk;
            if (gc < N && gkb < K) vb = transB ? B[(size_t)gc * ldb + gkb] : B[(size_t)gkb * ldb + gc];
            sa[ak][ar] = __uint_as_float(quantize_bits<MODE, FTZ>(va, qp));
            sb[bk][br] = __uint_as_float(quantize_bits<MODE, FTZ>(vb, qp));
        }
        __syncthreads();
        // groups of 8 k (the stage is zero-padded beyond K): 8 fused steps from a = 0, then one fp32 addition
        for (int g = 0; g < kFK / 8; ++g) {
            acc_t a16[4][4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) a16[i][j] = (acc_t)0;
#pragma unroll
            for (int kk = g * 8; kk < g * 8 + 8; ++kk) {
                acc_t w[4], x[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    w[i] = (acc_t)sa[kk][ty * 4 + i];
                    x[i] = (acc_t)sb[kk][tx * 4 + i];
                }
                if constexpr (F32) {
                    // the 16 chains take their step; which lanes met a midpoint is kept as wave masks
                    float nx[4][4];
                    unsigned long long met[4][4], any = 0ull;
                    const bool first = kk == g * 8;        // known at compile time: the loop over kk is unrolled
#pragma unroll
                    for (int i = 0; i < 4; ++i)
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            bool tie;
                            nx[i][j] = first ? fmac_try<FTZ, true>(a16[i][j], w[i], x[j], qp, fk, tie)
                                             : fmac_try<FTZ, false>(a16[i][j], w[i], x[j], qp, fk, tie);
                            met[i][j] = __ballot(tie);
                            any |= met[i][j];
                        }
                    if (any != 0ull) {                     // wave-uniform
#pragma unroll
                        for (int i = 0; i < 4; ++i)
#pragma unroll
                            for (int j = 0; j < 4; ++j)
                                if (met[i][j] != 0ull) nx[i][j] = fmac_fix<FTZ>(nx[i][j], a16[i][j], w[i], x[j], qp, fk);
                    }
#pragma unroll
                    for (int i = 0; i < 4; ++i)
#pragma unroll
                        for (int j = 0; j < 4; ++j) a16[i][j] = nx[i][j];
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
#pragma unroll
                        for (int j = 0; j < 4; ++j) a16[i][j] = quantize_f64(add_round_to_odd(a16[i][j], w[i] * x[j]), fp);
                }
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc32[i][j] = acc32[i][j] + (float)a16[i][j];   // single-precision addition
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = row0 + ty * 4 + i;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = col0 + tx * 4 + j;
            if (r < M && c < N)
                C[(size_t)r * ldc + c] = __uint_as_float(quantize_bits<MODE, FTZ>(__float_as_uint(acc32[i][j]), qp));
        }
    }
}

template <int MODE, bool FTZ, bool F32>
static int launch(int transA, int transB, int M, int N, int K, const float *A, int64_t lda, const float *B, int64_t ldb,
                  float *C, int64_t ldc, const QuantParams &qp, const Fmac8Params &fp, hipStream_t stream)
{
    const int tiles_m = (M + kFTile - 1) / kFTile, tiles_n = (N + kFTile - 1) / kFTile;
    if ((int64_t)tiles_m * tiles_n >= ((int64_t)1 << 31)) return FMT_ERR_SHAPE;
    hipLaunchKernelGGL((fmac8_kernel<MODE, FTZ, F32>), dim3(tiles_m * tiles_n), dim3(256), 0, stream,
                       reinterpret_cast<const uint32_t *>(A), lda, transA, reinterpret_cast<const uint32_t *>(B), ldb,
                       transB, C, ldc, M, N, K, tiles_n, qp, fp);
    FMT_HIP_CHECK(hipGetLastError());
    return FMT_OK;
}

// FMT_FMAC8_F64=1 keeps every format on the double-precision step (tests compare the two).
static bool fmac8_force_f64()
{
    const char *env = getenv("FMT_FMAC8_F64");
    return env != nullptr && env[0] == '1';
}

int launch_gemm_fmac8(int transA, int transB, int64_t M, int64_t N, int64_t K, const float *A, int64_t lda,
                      const float *B, int64_t ldb, float *C, int64_t ldc, fmt_format_t f, const QuantParams &qp,
                      hipStream_t stream)
{
    const int bias = (1 << (f.e - 1)) - 1;
    Fmac8Params fp;
    fp.ovf = ldexp(2.0 - ldexp(1.0, -(f.m + 1)), bias);
    fp.minn = ldexp(1.0, 1 - bias);
    fp.emin_biased = 1 - bias + 1023;
    fp.m = f.m;
    fp.ftz = f.denorm == 0;
    const bool ftz = f.denorm == 0;
#define FMT_RUN(MD, F32)                                                                                              \
    (ftz ? launch<MD, true, F32>(transA, transB, (int)M, (int)N, (int)K, A, lda, B, ldb, C, ldc, qp, fp, stream)      \
         : launch<MD, false, F32>(transA, transB, (int)M, (int)N, (int)K, A, lda, B, ldb, C, ldc, qp, fp, stream))
    // single-precision fused step where it is exact (see fmac_f32): 1/5/10, 1/6/9 and their neighbours
    if (f.e <= 6 && f.m <= 11 && !fmac8_force_f64()) return FMT_RUN(kModeMagic, true);
    if (qp.mode == kModeMagic) return FMT_RUN(kModeMagic, false);
    if (qp.mode == kModeInteger) return FMT_RUN(kModeInteger, false);
    return FMT_RUN(kModeMixed, false);
#undef FMT_RUN
}

}  // namespace fmt
