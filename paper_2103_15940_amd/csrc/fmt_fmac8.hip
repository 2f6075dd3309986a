// fmt_gemm_fmac8: matrix product with the FMAC-8 accumulation of Sec. IV-A, Algorithm 1.
//
// Every output element is one dot product run exactly as the algorithm lists it: a 16-bit
// accumulator a takes 8 consecutive FMACs, a = Q(a + w_i * x_i) with ONE rounding of the exact sum
// to the format (FMAC of Sec. III-B); at every i that is a multiple of 8 it is added into an fp32
// master accumulator with an fp32 addition and reset; the result is Q(master).  The chain of
// roundings is sequential by definition, so this is plain ALU work (no matrix cores): the bound
// is the vector rate (single precision where the fused step is exact in it, else double).
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
// (m+1)-bit significands has at most 24 bits and, with Emin >= -30, lies in fp32's normal range,
// so w * x is exact; TwoSum's error term is exact for the same reason; the sum rounded to odd has
// 24 significant bits, at least two more than the format, so rounding it to the format equals one
// rounding of the exact sum -- with quantize_bits, the rounding every other kernel uses.  Half the
// register file and twice the vector rate of the fp64 step.
template <int MODE, bool FTZ>
__device__ __forceinline__ float fmac_f32(float a, float w, float x, const QuantParams &qp)
{
    const float p = __fmul_rn(w, x);
    const float s = __fadd_rn(a, p);
    const float bb = __fsub_rn(s, a);
    const float err = __fadd_rn(__fsub_rn(a, __fsub_rn(s, bb)), __fsub_rn(p, bb));
    uint32_t u = __float_as_uint(s);
    if (err != 0.0f && err == err && (u & 1u) == 0u) {
        const bool away = (err > 0.0f) == (s > 0.0f);
        u += away ? 1u : 0xFFFFFFFFu;
    }
    return __uint_as_float(quantize_bits<MODE, FTZ>(u, qp));
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
    acc_t acc16[4][4];                             // the 16-bit accumulators (values of the format)
    float acc32[4][4];                             // the fp32 master accumulators
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            acc16[i][j] = (acc_t)0;
            acc32[i][j] = 0.0f;
        }

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
        const int kmax = min(kFK, K - k0);
        for (int kk = 0; kk < kmax; ++kk) {
            if ((kk & 7) == 0) {                   // global index k0 + kk is a multiple of 8 as well
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        acc32[i][j] = acc32[i][j] + (float)acc16[i][j];   // single-precision addition
                        acc16[i][j] = (acc_t)0;
                    }
            }
            acc_t w[4], x[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                w[i] = (acc_t)sa[kk][ty * 4 + i];
                x[i] = (acc_t)sb[kk][tx * 4 + i];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if constexpr (F32)
                        acc16[i][j] = fmac_f32<MODE, FTZ>(acc16[i][j], w[i], x[j], qp);
                    else
                        acc16[i][j] = quantize_f64(add_round_to_odd(acc16[i][j], w[i] * x[j]), fp);
                }
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = row0 + ty * 4 + i;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = col0 + tx * 4 + j;
            if (r < M && c < N) {
                const float master = acc32[i][j] + (float)acc16[i][j];
                C[(size_t)r * ldc + c] = __uint_as_float(quantize_bits<MODE, FTZ>(__float_as_uint(master), qp));
            }
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
