// Device-side rounding to a 1/e/m format on the fp32 bit pattern (Sec. IV-A), shared by the
// stream kernels and the GEMM operand loaders.
#pragma once

#include "fmt_internal.h"

namespace fmt {

// How the rounding is carried out (uniform per launch, chosen on the host from (e, m)):
enum : int {
    kModeMagic = 0,    // e < 8, m <= 22: (|x| + C) - C with C = 2^(max(E, Emin) + 23 - m)
    kModeInteger = 1,  // e == 8: RNE on the integer pattern (fp32's denormal grid is the format's own)
    kModeMixed = 2     // e < 8, m == 23: nothing to round at or above minN, fixed grid below
};

// Q_{e,m,d|n} on one fp32 bit pattern.
template <int MODE, bool FTZ>
__device__ __forceinline__ uint32_t quantize_bits(uint32_t u, const QuantParams &p)
{
    const uint32_t a = u & 0x7FFFFFFFu;
    uint32_t r;
    if (MODE == kModeMagic) {
        // C has ulp 2^(max(E,Emin)-m) and |x| < C, so the hardware's RNE addition lands on the
        // format's grid and the subtraction is exact.  For |x| >= t_ovf the pattern of C may be
        // meaningless; those lanes are overwritten below.
        const uint32_t ce = max(a & 0x7F800000u, p.minn_bits) + p.shift23;
        const float c = __uint_as_float(ce);
        r = __float_as_uint((__uint_as_float(a) + c) - c);
    } else if (MODE == kModeInteger) {
        const uint32_t lsb = __builtin_amdgcn_ubfe(a, p.shift, p.lsb_width);
        r = (a + p.rbias + lsb) & p.nmask;
    } else {
        const float rbf = (__uint_as_float(a) + p.cmagic) - p.cmagic;
        r = (a < p.minn_bits) ? __float_as_uint(rbf) : a;
    }
    if (FTZ) r = (a < p.t_den) ? 0u : r;
    r = (a >= p.t_ovf) ? 0x7F800000u : r;
    r |= (u & 0x80000000u);
    return (a > 0x7F800000u) ? 0x7FC00000u : r;
}

// (1+e+m)-bit code (Sec. III) of r, the pattern of a value of the format (quantize_bits' result);
// needs 1 + e + m <= 16, so MODE is kModeMagic (e < 8) or kModeInteger (e == 8).  At or above minN
// the code is the fp32 pattern rebased to the format's bias and shifted; below minN the stored
// mantissa is |r| / minD, read off the pattern of |r| + minN (exact: |r| is a multiple of minD);
// with e == 8 fp32's own denormal patterns are the format's.
template <int MODE>
__device__ __forceinline__ uint32_t encode_bits(uint32_t r, const QuantParams &p)
{
    const uint32_t a = r & 0x7FFFFFFFu;
    uint32_t ae = a;
    if (MODE != kModeInteger) {
        const float t = __uint_as_float(a) + __uint_as_float(p.minn_bits);
        ae = a < p.minn_bits ? __float_as_uint(t) - 0x00800000u : a;
    }
    uint32_t c = (ae - (p.minn_bits - 0x00800000u)) >> p.shift;
    const uint32_t quiet = 1u << (22u - p.shift);                          // top mantissa bit, 2^(m-1)
    c = a >= 0x7F800000u ? (a > 0x7F800000u ? p.top_code | quiet : p.top_code) : c;
    return c | ((r >> 31) << p.sign_pos);
}

// fp32 pattern of the value of a (1+e+m)-bit code; bits above the sign are ignored, NaN codes
// give the quiet NaN 0x7FC00000.  INTEGER: e == 8.
template <bool INTEGER>
__device__ __forceinline__ uint32_t decode_bits(uint32_t code, const QuantParams &p)
{
    const uint32_t body = code & ((1u << p.sign_pos) - 1u);
    const uint32_t sign = ((code >> p.sign_pos) & 1u) << 31;
    uint32_t a = (body << p.shift) + (p.minn_bits - 0x00800000u);
    if (!INTEGER) {
        // exponent field 0: mantissa * minD = (minN with that mantissa) - minN, exactly
        const float t = __uint_as_float(p.minn_bits | (body << p.shift)) - __uint_as_float(p.minn_bits);
        a = body < (1u << (23u - p.shift)) ? __float_as_uint(t) : a;
    }
    if (body >= p.top_code) return body == p.top_code ? (0x7F800000u | sign) : 0x7FC00000u;
    return a | sign;
}

// The same rounding with the variant chosen at run time (uniform per launch), for kernels that
// round a handful of values and are not worth six instantiations.
__device__ __forceinline__ uint32_t quantize_bits_rt(uint32_t u, const QuantParams &p, bool ftz)
{
    if (p.mode == kModeMagic) return ftz ? quantize_bits<kModeMagic, true>(u, p) : quantize_bits<kModeMagic, false>(u, p);
    if (p.mode == kModeInteger) return ftz ? quantize_bits<kModeInteger, true>(u, p) : quantize_bits<kModeInteger, false>(u, p);
    return ftz ? quantize_bits<kModeMixed, true>(u, p) : quantize_bits<kModeMixed, false>(u, p);
}

}  // namespace fmt
