// fmt_gemm: C = Q(op(A)) * Q(op(B)) with exact products and fp32 accumulation -- the FMACS
// instruction of Sec. III-B applied to the matrix products of Sec. IV-A.
//
// The matrix cores have no 1/6/9 (or general 1/e/m) operand type, so each rounded operand
// value r is split exactly into P bf16 pieces r = p0 + p1 (+ p2): p0 is r truncated to bf16's
// 8 significant bits, p1 the (exactly representable) remainder, and so on.  bf16 has fp32's
// exponent range, so every piece of a format with e <= 8 fits.  A product r*s is then the sum
// of the P*P piece products, each exact inside the bf16 MFMA, accumulated in its fp32
// accumulator: exact products, fp32 accumulation -- FMACS.  P = 1 for m <= 7 (bfloat16),
// P = 2 for m <= 15 (1/6/9), P = 3 up to m = 23.  Formats whose values are all binary16 values
// (e <= 5, m <= 10: binary16 itself) need no split: one fp16 piece on the fp16 MFMA.
//
// Two kernels:
//   prepare  reads one fp32 operand (either layout), rounds it to the format, splits it and
//            writes the pieces into a library-owned workspace, zero-padded and already in the
//            order the product kernel consumes: units of 32 rows x 32 k per piece, each unit
//            stored as [k-chunk of 8][row][8 x bf16] so that a wave's MFMA operand fetch is one
//            contiguous 1 KiB read.
//   product  workgroup tiles of 64x64 up to 256x256, 4 waves of MFMA 32x32x16 tiles each, operand
//            stages loaded from global memory straight into LDS (a ring of stage buffers, 32 k per
//            stage), optional split of the k range with a deterministic reduction.
//
// Formats with a 6-bit exponent and at most 10 significant bits (1/6/9, 1/6/8) take a cheaper exact
// route, "exponent planes": their significands fit binary16, only their exponent range does not.
// Every row of an operand gets a power-of-two scale 2^S that moves the binades where the row lives
// into binary16's exactly representable range (plane 0, the only one the main loop reads: ONE fp16
// MFMA product per multiply).  A value that does not fit there -- too large, or with bits below
// binary16's last denormal bit -- fits exactly under the scale 2^(S-w) (plane "above") or 2^(S+w)
// (plane "below"), w = 40 - m binades being what one plane holds; three planes cover the whole range
// of the format whatever S is.  A per-(32 rows x 32 k) mask says which planes hold anything, and every 32
// rows carry a short list of their elements outside plane 0 (with a count that says when the list did
// not hold them all: then the masks lead to them); a small kernel after the product kernel adds the
// products of those few elements, one fp32 fused multiply-add each, in a fixed order.  Exact products,
// fp32 accumulation, nothing that can overflow into a wrong result, no fallback product: the result is
// reproducible bit for bit.
//
// Several products on prepared operands can share launches (launch_gemm_prepared_batch): the product and the
// tail kernel exist in a form that takes a table of products and finds a workgroup's product from its id.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <type_traits>
#include <vector>

#include "fmt_hist.h"
#include "fmt_internal.h"
#include "fmt_quant.h"

#ifndef FMT_GEMM_KS
#define FMT_GEMM_KS 2      // 16-k steps per LDS stage
#endif
#ifndef FMT_GEMM_KS_MULTI
#define FMT_GEMM_KS_MULTI 1  // ... with two or three pieces per operand (twice / three times the bytes per k)
#endif
#ifndef FMT_GEMM_NST
#define FMT_GEMM_NST 4     // LDS stage buffers (at most; see pipe_nst)
#endif

namespace fmt {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

// Piece scheme PS: 1, 2, 3 = that many bf16 pieces; 0 = one fp16 piece (formats inside binary16).
constexpr int pieces_of(int ps) { return ps == 0 ? 1 : ps; }
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kUnitRows = 32;                 // rows per unit (one MFMA fragment)
constexpr int kUnitK = 32;                    // k per unit (two MFMA steps of 16)
constexpr int kUnitVec = kUnitRows * kUnitK * 2 / 16;   // 16-byte vectors per unit per piece = 128
constexpr int kFastRows = 4;                  // groups of 64 rows per workgroup in the fast patch gather (kRowPad = 64 * kFastRows)
constexpr int kRowPad = 256;                  // prepared operands are padded to a multiple of this many rows

// Rounds one fp32 pattern to the format and splits the result into the 16-bit patterns of its
// pieces: P bf16 pieces, or the single fp16 pattern when the format's values are all binary16
// values (e <= 5, m <= 10).
template <int MODE, bool FTZ, int PS>
__device__ __forceinline__ void round_and_split(uint32_t u, const QuantParams &p, uint32_t (&piece)[pieces_of(PS)])
{
    constexpr int P = pieces_of(PS);
    const uint32_t r = quantize_bits<MODE, FTZ>(u, p);
    if (PS == 0) {
        // exact fp32 -> fp16 of a value known to be representable: normal numbers by moving the
        // fields, denormals as the integer count of 2^-24 steps (an exact fp32 product)
        const uint32_t a = r & 0x7FFFFFFFu;
        uint32_t h = a >= 0x38800000u ? (a - 0x38000000u) >> 13 : (uint32_t)(__uint_as_float(a) * 16777216.0f);
        h = a >= 0x7F800000u ? (a > 0x7F800000u ? 0x7E00u : 0x7C00u) : h;
        piece[0] = h | ((r >> 16) & 0x8000u);
        return;
    }
    const uint32_t hi = r & 0xFFFF0000u;
    piece[0] = hi >> 16;
    if (P >= 2) {
        // infinities and NaN stay in the first piece alone
        const bool finite = (r & 0x7F800000u) != 0x7F800000u;
        const float rem = finite ? __uint_as_float(r) - __uint_as_float(hi) : 0.0f;   // exact
        const uint32_t rb = __float_as_uint(rem);
        piece[P >= 2 ? 1 : 0] = rb >> 16;
        if (P >= 3) {
            const float rem2 = rem - __uint_as_float(rb & 0xFFFF0000u);                // exact
            piece[P >= 3 ? 2 : 0] = __float_as_uint(rem2) >> 16;
        }
    }
}

// Workspace address (in 16-byte vectors) of chunk c (8 consecutive k) of row `row` in unit
// (rb, kb), piece `piece`.
__device__ __forceinline__ size_t unit_vec_index(int rb, int kb, int kblocks, int P, int piece, int c, int row)
{
    return (((size_t)rb * kblocks + kb) * P + piece) * kUnitVec + c * kUnitRows + row;
}

// Exponent planes of one prepared operand (formats with e == 6 and m <= 9; see the top of this file).
//   S      scale exponent per (padded) row: plane 0 holds value * 2^S, the plane above value * 2^(S-w),
//          the plane below value * 2^(S+w), each as a binary16 value
//   mask   one byte per unit (32 rows x 32 k): bit 0 set always, bit 1 / bit 2 set when the unit has
//          an element in the plane above / below; only then has that plane's unit been written
//   plane  16-byte vectors from one plane's pieces to the next (planes 1 and 2 follow plane 0)
//   recs   per row of units (32 rows x all k), the elements outside plane 0 as records (k << 5 | row in the unit,
//          true value as fp32 bits), in no particular order, and rec_cnt how many there are; a row of units
//          with more than kRecCap of them keeps only the count (its elements are then found through the masks)
struct Planes {
    int *S;
    uint8_t *mask;
    size_t plane;
    int w;               // 40 - m: binades one plane holds
    uint32_t *rec_cnt;
    uint32_t *recs;      // pairs of words, kRecCap pairs per row of units
};
constexpr int kRecCap = 64;

constexpr int kWinTmin = 0, kWinTmax = 31;              // range of plane 0's top binade T (S = 15 - T): with
                                                        // three planes every value of a 1/6/m format, m <= 9, fits

// How element (row, k) of an operand is found in memory.
enum {
    kSrcMatrix = 0,     // X[row*ld + k] (kcontig) or X[k*ld + row]
    kSrcPatchRows = 1,  // convolution patches: row = (n, y, x) on a grid gy x gx, k = (ch, r, s)
    kSrcPatchK = 2,     // the same patches transposed: row = (ch, r, s), k = (n, y, x)
    kSrcChannelRows = 3,  // NCHW tensor as a matrix: row = channel, k = (n, position)
    kSrcFilterT = 4,    // filter [K][C][R][S] with row = c, k = (kout, r, s)
    kSrcFilterTap = 5   // filter [K][C][R][S] with k = (tap, channel): element (row, k) sits at
                        // row*th + (k % D)*tw + k / D, D = k0.d channels (th, tw hold the two strides)
};

// Division of a 31-bit dividend by a divisor fixed at launch, as a multiply-high and a shift
// (m = floor(2^(31+l) / d) + 1 with l = ceil(log2 d) gives floor(a / d) for every 0 <= a < 2^31).
struct FastDiv {
    uint32_t m;
    int sh;      // l - 1; d == 1 is handled apart
    int d;
};

static FastDiv make_fastdiv(int d)
{
    FastDiv f{0u, 0, d < 1 ? 1 : d};
    if (f.d > 1) {
        int l = 0;
        while (((int64_t)1 << l) < f.d) ++l;
        f.m = (uint32_t)((((uint64_t)1 << (31 + l)) / (uint64_t)f.d) + 1);
        f.sh = l - 1;
    }
    return f;
}

__device__ __forceinline__ void divmod(const FastDiv &f, int a, int &q, int &r)
{
    q = f.d == 1 ? a : (int)(__umulhi((uint32_t)a, f.m) >> f.sh);
    r = a - q * f.d;
}

// Geometry of a gathered operand.  Patches read T[n][ch][iy][ix] of an NCHW tensor with tc
// channels of th x tw, where iy = (y*mul_y + off_y + tap*r) / den_y must divide exactly and lie in
// [0, th) (else the element is zero), likewise ix.  Forward and wgrad: mul = stride, off = -pad,
// tap = +1, den = 1; dgrad (patches of dY seen from an input position): mul = 1, off = +pad,
// tap = -1, den = stride.
struct Gather {
    int kind;
    int tc, th, tw;
    int gy, gx;
    int R, S;
    int mul_y, mul_x, off_y, off_x, tap, den_y, den_x;
    // pre != 0: the tensor was rounded and split beforehand (round_split_kernel); X then points to
    // the piece patterns, two per 32-bit word, in (P+1)/2 planes of `plane` elements each (a patch
    // element is reused R*S times, so rounding it once pays)
    int pre, plane;
    // fast != 0 (patch rows, den == 1, R*S <= 32, pre): the taps inside the tensor are kept as a
    // per-lane bit mask and the element offset splits into a per-lane and a per-k (scalar) part;
    // element plane-1 of the rounded tensor is a zero that out-of-range taps read
    int fast;
    // fast == 2: the same for the transposed patches (rows = taps, k = positions; see gather_taps)
    // divisors of the index decompositions: rows by (r0 inner, r1 outer), k by (k0 inner, k1 outer)
    FastDiv r0, r1, k0, k1;
};

// One operand of a prepare launch: X is fp32, `rows` x K after op(); for a plain matrix element
// (r, k) sits at X[r*ld + k] (kcontig) or X[k*ld + r]; vec4: base 16-byte aligned and ld a
// multiple of 4.  kcontig also selects the lane mapping (8 lanes along k per row, or lanes
// along rows) for the gathered kinds.
struct PrepOperand {
    const uint32_t *X;
    u32x4 *W;
    int64_t ld;
    int rows;
    int kcontig;
    int vec4;
    unsigned nblocks;   // workgroups of this operand: slabs * row groups
    Gather g;
    Planes pl;          // pl.S != nullptr: scaled fp16 exponent planes (PS == 0, plain matrices only)
};

// Operand B of a convolution product gathered by the product kernel itself: row = position (n, y, x)
// on a grid gy x gx, k = (tap, channel) with the channel running fastest, read from the rounded tensor
// in pixel-major order T[piece][n][iy][ix][channel] (16-bit pieces, 8 channels per 16-byte vector; tc is a
// multiple of 32, so a stage of 16 or 32 k lies inside one tap).  iy = y*mul_y + off_y + tap_sign*r, likewise
// ix; a tap outside the tensor reads the zero vector at index `zero`.  Every index counts 16-byte vectors
// from T and fits 31 bits.
struct Implicit {
    const u32x4 *T;
    int piece_vec;      // vectors per piece
    int zero;           // index of a vector of zeros
    int c8;             // channels / 8
    int th, tw, gy, gx;
    int mul_y, mul_x, off_y, off_x, tap_sign;
    int R, S;
    int rows;
    FastDiv r0, r1;     // row -> (n, y, x): by gx, then by gy
    FastDiv kc;         // stage number -> (tap, channel block): by channels / (k per stage)
    FastDiv ks;         // tap -> (r, s): by S
};

// Offset of tap (r, s) seen from the spatial base (by, bx) = (y*mul + off) inside one h x w plane,
// or -1 when the tap falls outside the tensor (or, for dgrad, between the strides).  All tensors
// have fewer than 2^31 elements, so 32-bit offsets suffice.
template <bool DIV>
__device__ __forceinline__ int tap_offset(const Gather &g, int by, int bx, int r, int s)
{
    int iy = by + g.tap * r, ix = bx + g.tap * s;
    if (DIV) {
        if (iy < 0 || ix < 0) return -1;
        const int qy = iy / g.den_y, qx = ix / g.den_x;
        if (qy * g.den_y != iy || qx * g.den_x != ix) return -1;
        iy = qy;
        ix = qx;
    }
    return ((unsigned)iy < (unsigned)g.th && (unsigned)ix < (unsigned)g.tw) ? iy * g.tw + ix : -1;
}

template <bool DIV>
__device__ __forceinline__ void gather_patches(const PrepOperand &o, int row, int k0, int K, int (&idx)[8])
{
    const Gather &g = o.g;
    const int hw = g.th * g.tw;
    if (g.kind == kSrcPatchRows) {
        // fixed position (n, y, x); k runs over (ch, r, s).  Lanes run along rows in this layout, so
        // k0 is the same in the whole wave and its decomposition and the walk over the taps are
        // scalar work.
        int x, t, y, n;
        divmod(g.r0, row, t, x);
        divmod(g.r1, t, n, y);
        const int by = y * g.mul_y + g.off_y, bx = x * g.mul_x + g.off_x;
        const int ku = __builtin_amdgcn_readfirstlane(k0);
        int s, t2, r, ch;
        divmod(g.k0, ku, t2, s);
        divmod(g.k1, t2, ch, r);
        const int nplane = n * g.tc * hw;
        int cplane = ch * hw;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int off = tap_offset<DIV>(g, by, bx, r, s);
            if (ku + j < K && off >= 0) idx[j] = nplane + cplane + off;
            if (++s == g.S) {
                s = 0;
                if (++r == g.R) {
                    r = 0;
                    cplane += hw;
                }
            }
        }
    } else {
        // fixed tap (ch, r, s); k runs over the positions (n, y, x)
        int s, t, r, ch;
        divmod(g.r0, row, t, s);
        divmod(g.r1, t, ch, r);
        int x, t2, y, n;
        divmod(g.k0, k0, t2, x);
        divmod(g.k1, t2, n, y);
        int plane = (n * g.tc + ch) * hw;
        const int step = g.tc * hw;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int off = tap_offset<DIV>(g, y * g.mul_y + g.off_y, x * g.mul_x + g.off_x, r, s);
            if (k0 + j < K && off >= 0) idx[j] = plane + off;
            if (++x == g.gx) {
                x = 0;
                if (++y == g.gy) {
                    y = 0;
                    plane += step;
                }
            }
        }
    }
}

// Element offsets of (row, k0 .. k0+7) of a gathered operand in its tensor; -1 = a zero (padding,
// a tap between the strides, beyond rows / K).
__device__ __forceinline__ void gather8(const PrepOperand &o, int row, int k0, int K, int (&idx)[8])
{
    const Gather &g = o.g;
#pragma unroll
    for (int j = 0; j < 8; ++j) idx[j] = -1;
    if (row >= o.rows || k0 >= K) return;
    if (g.kind == kSrcPatchRows || g.kind == kSrcPatchK) {
        if (g.den_y == 1 && g.den_x == 1)
            gather_patches<false>(o, row, k0, K, idx);
        else
            gather_patches<true>(o, row, k0, K, idx);
    } else if (g.kind == kSrcFilterTap) {
        int ch, tap;
        divmod(g.k0, k0, tap, ch);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (k0 + j < K) idx[j] = row * g.th + ch * g.tw + tap;
            if (++ch == g.k0.d) {
                ch = 0;
                ++tap;
            }
        }
    } else {
        // kSrcChannelRows: k = (image, position), L = g.k0.d positions; kSrcFilterT: k = (filter, tap),
        // L = R*S taps; element (row, k) sits at ((k / L) * tc + row) * L + k % L in both
        const int L = g.k0.d;
        int pos, q;
        divmod(g.k0, k0, q, pos);
        int base = (q * g.tc + row) * L;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (k0 + j < K) idx[j] = base + pos;
            if (++pos == L) {
                pos = 0;
                base += g.tc * L;
            }
        }
    }
}

// Rounds a tensor to the format and splits it once, elementwise, for operands that are gathered
// many times: word plane w (n + 1 words, the last one zero) holds piece 2w in its low half and
// piece 2w+1 in its high half.
template <int MODE, bool FTZ, int PS>
__global__ __launch_bounds__(256) void round_split_kernel(const uint32_t *__restrict__ x, uint32_t *__restrict__ out,
                                                          int n, QuantParams p)
{
    constexpr int P = pieces_of(PS);
    const size_t plane = (size_t)n + 1;          // one extra element per plane, always zero
    for (int i = blockIdx.x * 256 + threadIdx.x; i < n; i += gridDim.x * 256) {
        uint32_t pc[P];
        round_and_split<MODE, FTZ, PS>(x[i], p, pc);
        out[i] = pc[0] | (P >= 2 ? pc[P >= 2 ? 1 : 0] << 16 : 0u);
        if (P >= 3) out[plane + i] = pc[P >= 3 ? 2 : 0];
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        out[n] = 0u;
        if (P >= 3) out[plane + n] = 0u;
    }
}

// Rounds an NCHW tensor (C a multiple of 32) to the format, splits it, and writes the pieces in
// pixel-major order out[piece][pixel][channel] (16 bits per element) -- the operand the product kernel
// gathers convolution patches from.  A workgroup takes 64 consecutive pixels (of the flattened n*h*w)
// by 32 channels: reads run along pixels, the transposition goes through LDS, and a lane writes 8
// consecutive channels of one pixel as one 16-byte vector.  One vector of zeros follows the last piece.
template <int MODE, bool FTZ, int PS>
__global__ __launch_bounds__(256) void nhwc_split_kernel(const uint32_t *__restrict__ x, u32x4 *__restrict__ out, int C,
                                                         int HW, int npix, QuantParams p)
{
    constexpr int P = pieces_of(PS);
    constexpr int kPitch = 18;                                  // 32-bit words per pixel row (16 + 2: odd multiple of 2)
    __shared__ uint32_t tile[P][64][kPitch];
    const int tid = threadIdx.x;
    const int pix = tid % 64, cg = tid / 64;
    const int gp = blockIdx.x * 64 + pix, cb = blockIdx.y;
    const bool valid = gp < npix;
    const int n = valid ? gp / HW : 0, hw = valid ? gp - n * HW : 0;
    const uint32_t *src = x + ((size_t)n * C + cb * 32 + cg * 8) * HW + hw;
    uint32_t pc[8][P];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const uint32_t u = valid ? src[(size_t)i * HW] : 0u;
        round_and_split<MODE, FTZ, PS>(u, p, pc[i]);
    }
#pragma unroll
    for (int q = 0; q < P; ++q)
#pragma unroll
        for (int i = 0; i < 4; ++i) tile[q][pix][cg * 4 + i] = pc[2 * i][q] | (pc[2 * i + 1][q] << 16);
    __syncthreads();
    const int opix = tid / 4, part = tid % 4;
    const int ogp = blockIdx.x * 64 + opix;
    const size_t piece_vec = (size_t)npix * (C / 8);
    if (ogp < npix) {
#pragma unroll
        for (int q = 0; q < P; ++q) {
            u32x4 w;
#pragma unroll
            for (int i = 0; i < 4; ++i) w[i] = tile[q][opix][part * 4 + i];
            out[q * piece_vec + (size_t)ogp * (C / 8) + cb * 4 + part] = w;
        }
    }
    if (blockIdx.x == 0 && blockIdx.y == 0 && tid == 0) out[P * piece_vec] = u32x4{0u, 0u, 0u, 0u};
}

// Transposed patches (wgrad: rows = taps (ch, r, s), k = positions (n, y, x)), pre-rounded tensor.
// A workgroup takes one unit of 32 taps and 256 positions, one position per lane: which taps fall
// inside the tensor is a per-lane bit mask and the walk over the taps is scalar work, exactly as in
// the forward gather; what differs is the output, which wants 8 consecutive positions of ONE tap in
// a lane.  Each wave therefore passes its 8 taps x 64 positions through a tile of its own in LDS and
// reads them back transposed (rows padded to 72 words against bank conflicts).
template <int P>
__device__ __forceinline__ void gather_taps(const PrepOperand &o, unsigned bid, int K, int kblocks)
{
    constexpr int NW = (P + 1) / 2;                    // 32-bit word planes per element
    __shared__ uint32_t tile[4][NW][8][72];
    const Gather &g = o.g;
    const uint32_t *__restrict__ X = o.X;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ngroups = (kblocks + 7) / 8;
    const int pg = (int)(bid % (unsigned)ngroups), rb = (int)(bid / (unsigned)ngroups);
    const int hw = g.th * g.tw;
    const int pos = pg * 256 + tid;
    int x, t, y, n;
    divmod(g.k0, pos, t, x);
    divmod(g.k1, t, n, y);
    const int by = y * g.mul_y + g.off_y, bx = x * g.mul_x + g.off_x;
    const int lo_r = max(0, -by), hi_r = min(g.R, g.th - by);
    const int lo_s = max(0, -bx), hi_s = min(g.S, g.tw - bx);
    const int ns = hi_s - lo_s;
    const uint32_t mx = ns <= 0 ? 0u : ((ns >= 32 ? 0xFFFFFFFFu : (1u << ns) - 1u) << lo_s);
    uint32_t mask = 0u;
    for (int r = 0; r < g.R; ++r)
        if (r >= lo_r && r < hi_r) mask |= mx << (r * g.S);
    if (pos >= K) mask = 0u;
    const int lane_base = n * g.tc * hw + by * g.tw + bx;
    const int zero = g.plane - 1;
    const int gi = lane >> 3, li = lane & 7;           // after the transpose: positions gi*8 .. gi*8+7 of tap li
    const int pb = pg * 256 + wave * 64 + gi * 8;       // first of this lane's 8 positions
    const int kb = pb / kUnitK, c = (pb % kUnitK) / 8;
    for (int pass = 0; pass < 4; ++pass) {
        const int tap0 = rb * 32 + pass * 8;           // the same in the whole workgroup
        int s, t2, r, ch;
        divmod(g.r0, tap0, t2, s);
        divmod(g.r1, t2, ch, r);
        int rs = r * g.S + s;
        int delta = ch * hw + r * g.tw + s;
        uint32_t w[NW][8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const bool ok = tap0 + j < o.rows && ((mask >> rs) & 1u);
            const uint32_t idx = (uint32_t)(ok ? lane_base + delta : zero);
#pragma unroll
            for (int q = 0; q < NW; ++q) w[q][j] = X[(size_t)q * g.plane + idx];
            ++rs;
            ++delta;
            if (++s == g.S) {
                s = 0;
                delta += g.tw - g.S;
                if (++r == g.R) {
                    r = 0;
                    rs = 0;
                    delta += hw - g.R * g.tw;
                }
            }
        }
        __syncthreads();                               // the previous pass's tile has been read
#pragma unroll
        for (int q = 0; q < NW; ++q)
#pragma unroll
            for (int j = 0; j < 8; ++j) tile[wave][q][j][lane] = w[q][j];
        __syncthreads();
        uint32_t v[NW][8];
#pragma unroll
        for (int q = 0; q < NW; ++q)
#pragma unroll
            for (int m = 0; m < 8; ++m) v[q][m] = tile[wave][q][li][gi * 8 + m];
        if (kb < kblocks) {
            const int rr = pass * 8 + li;
#pragma unroll
            for (int pc = 0; pc < P; ++pc) {
                u32x4 out;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t hi = v[pc / 2][2 * i + 1], lo = v[pc / 2][2 * i];
                    out[i] = __builtin_amdgcn_perm(hi, lo, (pc & 1) ? 0x07060302u : 0x05040100u);
                }
                o.W[unit_vec_index(rb, kb, kblocks, P, pc, c, rr)] = out;
            }
        }
    }
}

// prepare: both operands of a product in one launch (workgroups [0, a.nblocks) take op(A), the
// rest op(B)).  k-contiguous input: a workgroup takes 32 rows x 64 k, 8 neighbouring lanes read
// 256 contiguous bytes of a row; transposed input: 64 rows x 32 k, a wave reads 256 contiguous
// bytes for each k.
// TAPS: one of the operands may take gather_taps (whose LDS tile and barriers the other launches do
// not pay for).
template <int MODE, bool FTZ, int PS, bool TAPS = false>
__device__ __forceinline__ void prepare_block(const PrepOperand &a, const PrepOperand &b, int K, int kblocks,
                                              const QuantParams &p, unsigned block)
{
    constexpr int P = pieces_of(PS);
    const int tid = threadIdx.x;
    // Each operand owns a run of workgroup ids padded to a multiple of 8.  Consecutive ids go to
    // different XCDs (each with its own L2), so the ids are remapped to give every XCD a contiguous
    // range of rows: a gathered tensor is then read into each L2 once, not eight times.
    const unsigned a_ids = (a.nblocks + 7u) / 8u * 8u;
    const bool second = block >= a_ids;
    const PrepOperand &o = second ? b : a;
    const unsigned lid = block - (second ? a_ids : 0u);
    const unsigned per_xcd = (o.nblocks + 7u) / 8u;
    const unsigned bid = (lid % 8u) * per_xcd + lid / 8u;
    if (bid >= o.nblocks) return;
    if constexpr (TAPS) {
        if (o.g.fast == 2) {                 // block-uniform: every thread takes part in its barriers
            gather_taps<P>(o, bid, K, kblocks);
            return;
        }
    }
    const uint32_t *__restrict__ X = o.X;
    const int64_t ld = o.ld;
    const int rows = o.rows;
    const bool kcontig = o.kcontig != 0;
    const int nslabs = kcontig ? (kblocks + 1) / 2 : kblocks;
    const int bx = bid % nslabs, by = bid / nslabs;
    int row, k0;
    if (kcontig) {
        row = by * 32 + tid / 8;
        k0 = bx * 64 + (tid % 8) * 8;
    } else {
        // the fast gather takes kFastRows groups of 64 rows per workgroup, the other paths one
        row = by * 64 * (o.g.fast == 1 ? kFastRows : 1) + tid % 64;
        k0 = bx * 32 + (tid / 64) * 8;
    }
    if (k0 >= kblocks * kUnitK) return;      // k-contiguous slabs cover two k-blocks; the last may be half
    uint32_t v[8];
    uint32_t w01[8], w2[P >= 3 ? 8 : 1];     // pre-rounded source: pieces 0|1 packed per element, piece 2
    bool packed = false;
    if (o.g.fast == 1) {
        // Patches, lanes along positions: which taps (r, s) fall inside the tensor is a per-lane bit
        // mask, the offset of a tap is per-lane base + a term that depends on k alone, and k is
        // the same in the whole wave, so walking the 8 taps is scalar work.
        // The walk is shared by kFastRows groups of 64 positions (the scalar unit, not the vector unit
        // or memory, bounds this path), each lane owning one position per group.
        const Gather &g = o.g;
        const int hw = g.th * g.tw;
        uint32_t mask[kFastRows];
        int lane_base[kFastRows];
#pragma unroll
        for (int q = 0; q < kFastRows; ++q) {
            const int rq = row + 64 * q;
            int x, t, y, n;
            divmod(g.r0, rq, t, x);
            divmod(g.r1, t, n, y);
            const int by = y * g.mul_y + g.off_y, bx = x * g.mul_x + g.off_x;
            const int lo_r = g.tap > 0 ? max(0, -by) : max(0, by - g.th + 1), hi_r = g.tap > 0 ? min(g.R, g.th - by) : min(g.R, by + 1);
            const int lo_s = g.tap > 0 ? max(0, -bx) : max(0, bx - g.tw + 1), hi_s = g.tap > 0 ? min(g.S, g.tw - bx) : min(g.S, bx + 1);
            const int ns = hi_s - lo_s;
            const uint32_t mx = ns <= 0 ? 0u : ((ns >= 32 ? 0xFFFFFFFFu : (1u << ns) - 1u) << lo_s);
            uint32_t mq = 0u;
            for (int r = 0; r < g.R; ++r)
                if (r >= lo_r && r < hi_r) mq |= mx << (r * g.S);
            mask[q] = rq < rows ? mq : 0u;
            lane_base[q] = n * g.tc * hw + by * g.tw + bx;
        }
        const int ku = __builtin_amdgcn_readfirstlane(k0);
        int s, t2, r, ch;
        divmod(g.k0, ku, t2, s);
        divmod(g.k1, t2, ch, r);
        int rs = r * g.S + s;
        int delta = ch * hw + g.tap * (r * g.tw + s);
        const int zero = g.plane - 1;
        const uint32_t *__restrict__ X2 = X + g.plane;
        uint32_t f01[kFastRows][8], f2[kFastRows][P >= 3 ? 8 : 1];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const bool kin = ku + j < K;
#pragma unroll
            for (int q = 0; q < kFastRows; ++q) {
                const bool ok = kin && ((mask[q] >> rs) & 1u);
                const uint32_t idx = (uint32_t)(ok ? lane_base[q] + delta : zero);
                f01[q][j] = X[idx];
                if (P >= 3) f2[q][j] = X2[idx];
            }
            ++rs;
            delta += g.tap;
            if (++s == g.S) {
                s = 0;
                delta += g.tap * (g.tw - g.S);
                if (++r == g.R) {
                    r = 0;
                    rs = 0;
                    delta += hw - g.tap * g.R * g.tw;
                }
            }
        }
        // two elements' 16-bit halves into one word with a byte permute
        const int kb = k0 / kUnitK, c = (k0 % kUnitK) / 8;
#pragma unroll
        for (int q = 0; q < kFastRows; ++q) {
            const int rq = row + 64 * q;
            const int rb = rq / kUnitRows, rr = rq % kUnitRows;
#pragma unroll
            for (int pc = 0; pc < P; ++pc) {
                u32x4 w;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (pc == 0) w[i] = __builtin_amdgcn_perm(f01[q][2 * i + 1], f01[q][2 * i], 0x05040100u);
                    if (pc == 1) w[i] = __builtin_amdgcn_perm(f01[q][2 * i + 1], f01[q][2 * i], 0x07060302u);
                    if (pc == 2) w[i] = __builtin_amdgcn_perm(f2[q][P >= 3 ? 2 * i + 1 : 0], f2[q][P >= 3 ? 2 * i : 0], 0x05040100u);
                }
                o.W[unit_vec_index(rb, kb, kblocks, P, pc, c, rr)] = w;
            }
        }
        return;
    } else if (o.g.kind != kSrcMatrix) {
        int idx[8];
        gather8(o, row, k0, K, idx);
        if (o.g.pre) {
            // pieces were made beforehand: pure data movement (element plane-1 is a zero)
            const uint32_t *__restrict__ X2 = X + o.g.plane;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint32_t at = (uint32_t)(idx[j] >= 0 ? idx[j] : o.g.plane - 1);
                w01[j] = X[at];
                if (P >= 3) w2[j] = X2[at];
            }
            packed = true;
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = idx[j] >= 0 ? X[(uint32_t)idx[j]] : 0u;
        }
    } else if (kcontig && o.vec4 && row < rows && k0 + 8 <= K) {
        const u32x4 *src = reinterpret_cast<const u32x4 *>(X + (size_t)row * ld + k0);
        const u32x4 lo = __builtin_nontemporal_load(src), hi = __builtin_nontemporal_load(src + 1);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            v[j] = lo[j];
            v[4 + j] = hi[j];
        }
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int k = k0 + j;
            const bool ok = row < rows && k < K;
            const size_t idx = kcontig ? (size_t)row * ld + k : (size_t)k * ld + row;
            v[j] = ok ? X[idx] : 0u;
        }
    }
    const int rb = row / kUnitRows, rr = row % kUnitRows;
    const int kb = k0 / kUnitK, c = (k0 % kUnitK) / 8;
    if (packed) {
        // two elements' 16-bit halves into one word with a byte permute
#pragma unroll
        for (int q = 0; q < P; ++q) {
            u32x4 w;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (q == 0) w[i] = __builtin_amdgcn_perm(w01[2 * i + 1], w01[2 * i], 0x05040100u);
                if (q == 1) w[i] = __builtin_amdgcn_perm(w01[2 * i + 1], w01[2 * i], 0x07060302u);
                if (q == 2) w[i] = __builtin_amdgcn_perm(w2[P >= 3 ? 2 * i + 1 : 0], w2[P >= 3 ? 2 * i : 0], 0x05040100u);
            }
            o.W[unit_vec_index(rb, kb, kblocks, P, q, c, rr)] = w;
        }
        return;
    }
    uint32_t pc[8][P];
#pragma unroll
    for (int j = 0; j < 8; ++j) round_and_split<MODE, FTZ, PS>(v[j], p, pc[j]);
#pragma unroll
    for (int q = 0; q < P; ++q) {
        u32x4 w;
        w[0] = pc[0][q] | (pc[1][q] << 16);
        w[1] = pc[2][q] | (pc[3][q] << 16);
        w[2] = pc[4][q] | (pc[5][q] << 16);
        w[3] = pc[6][q] | (pc[7][q] << 16);
        o.W[unit_vec_index(rb, kb, kblocks, P, q, c, rr)] = w;
    }
}

// Eight rounded values of one thread (fp32 patterns r[], elements k0 .. k0 + 7 of row `row` of operand o) as
// binary16 patterns, two per word: p0 = plane 0, pa / pb = the planes above / below (zero where an element
// does not belong to the plane).  Elements outside plane 0 also leave a record in the list of their row of
// units for the kernel that adds their products.  Returns 2 / 4 if any element went above / below.
template <class OP>
__device__ __forceinline__ uint32_t split_planes(const OP &o, int row, int k0, const uint32_t (&r)[8], u32x4 &p0, u32x4 &pa,
                                                 u32x4 &pb)
{
    const int S = o.pl.S[row];                   // S covers the padded rows
    uint32_t hb[8];
    bool other[8], any = false;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        // r * 2^S (exact: |S| is small) converts to binary16 and back unchanged <=> it is a binary16
        // value -- zeros, the normal and the denormal range, infinities.  NaN (neither below nor above its
        // own conversion) stays in plane 0 as well.
        const float sc = ldexpf(__uint_as_float(r[j]), S);
        const _Float16 h = static_cast<_Float16>(sc);               // round to nearest even
        const float back = static_cast<float>(h);
        other[j] = back < sc || back > sc;
        any |= other[j];
        hb[j] = (uint32_t)__builtin_bit_cast(uint16_t, h);
    }
    pa = pb = u32x4{0u, 0u, 0u, 0u};
    uint32_t mine = 0u;
    if (any) {                                   // rare: the common case does not pay for it element by element
        const int w = o.pl.w;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (other[j]) {
                // too large for plane 0 -> the plane above; bits below 2^-24 -> the plane below (exact there)
                const float rf = __uint_as_float(r[j]);
                const bool up = fabsf(ldexpf(rf, S)) >= 65536.0f;
                const _Float16 g = static_cast<_Float16>(ldexpf(rf, up ? S - w : S + w));
                const uint32_t gb = (uint32_t)__builtin_bit_cast(uint16_t, g) << (16 * (j & 1));
                pa[j / 2] |= up ? gb : 0u;
                pb[j / 2] |= up ? 0u : gb;
                mine |= up ? 2u : 4u;
                hb[j] = 0u;
                const uint32_t slot = atomicAdd(&o.pl.rec_cnt[row / kUnitRows], 1u);
                if (slot < (uint32_t)kRecCap) {
                    uint32_t *rec = o.pl.recs + ((size_t)(row / kUnitRows) * kRecCap + slot) * 2;
                    rec[0] = ((uint32_t)(k0 + j) << 5) | (uint32_t)(row % kUnitRows);
                    rec[1] = r[j];
                }
            }
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) p0[i] = hb[2 * i] | (hb[2 * i + 1] << 16);
    return mine;
}

// Stores what split_planes made: plane 0 always, the planes in `have` (bit 1 above, bit 2 below; agreed on by
// the threads of the unit); the unit's leader writes the mask.
template <class OP>
__device__ __forceinline__ void store_planes(const OP &o, int row, int k0, int kblocks, const u32x4 &p0, const u32x4 &pa,
                                             const u32x4 &pb, uint32_t have, bool leader)
{
    const int rb = row / kUnitRows, rr = row % kUnitRows;
    const int kb = k0 / kUnitK, c = (k0 % kUnitK) / 8;
    const size_t at = unit_vec_index(rb, kb, kblocks, 1, 0, c, rr);
    o.W[at] = p0;
    if (have & 2u) o.W[o.pl.plane + at] = pa;
    if (have & 4u) o.W[2 * o.pl.plane + at] = pb;
    if (leader) o.pl.mask[(size_t)rb * kblocks + kb] = (uint8_t)(1u | have);
}

// Scaled exponent planes of a plain matrix operand (see the top of this file).  Same element-to-thread
// mapping as prepare_block, so a workgroup covers exactly two units; which of them has elements
// outside plane 0 is agreed on through two words of LDS, and only then are the other planes of that
// unit written (the elements that do not belong to a plane are zero there).
template <int MODE, bool FTZ, class OP>
__device__ __forceinline__ void prepare_scaled_block(const OP &o, int K, int kblocks, const QuantParams &p,
                                                     unsigned bid)
{
    __shared__ uint32_t s_planes[2];
    const int tid = threadIdx.x;
    if (tid < 2) s_planes[tid] = 0u;
    const uint32_t *__restrict__ X = o.X;
    const int64_t ld = o.ld;
    const int rows = o.rows;
    const bool kcontig = o.kcontig != 0;
    const int nslabs = kcontig ? (kblocks + 1) / 2 : kblocks;
    const int bx = bid % nslabs, by = bid / nslabs;
    int row, k0, u;                              // u: which of the workgroup's two units this thread works on
    if (kcontig) {
        row = by * 32 + tid / 8;
        k0 = bx * 64 + (tid % 8) * 8;
        u = (tid % 8) / 4;
    } else {
        row = by * 64 + tid % 64;
        k0 = bx * 32 + (tid / 64) * 8;
        u = (tid % 64) / 32;
    }
    const bool live = k0 < kblocks * kUnitK;     // k-contiguous slabs cover two k-blocks; the last may be half
    uint32_t v[8];
    if (live && kcontig && o.vec4 && row < rows && k0 + 8 <= K) {
        const u32x4 *src = reinterpret_cast<const u32x4 *>(X + (size_t)row * ld + k0);
        const u32x4 lo = __builtin_nontemporal_load(src), hi = __builtin_nontemporal_load(src + 1);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            v[j] = lo[j];
            v[4 + j] = hi[j];
        }
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int k = k0 + j;
            const bool ok = live && row < rows && k < K;
            const size_t idx = kcontig ? (size_t)row * ld + k : (size_t)k * ld + row;
            v[j] = ok ? X[idx] : 0u;
        }
    }
    uint32_t r[8];
    u32x4 p0, pa, pb;
#pragma unroll
    for (int j = 0; j < 8; ++j) r[j] = quantize_bits<MODE, FTZ>(v[j], p);
    const uint32_t mine = split_planes(o, row, k0, r, p0, pa, pb);
    __syncthreads();                             // s_planes has been cleared
    if (mine != 0u) atomicOr(&s_planes[u], mine);
    __syncthreads();
    if (!live) return;
    store_planes(o, row, k0, kblocks, p0, pa, pb, s_planes[u],
                 kcontig ? (tid / 8 == 0 && tid % 4 == 0) : (tid / 64 == 0 && tid % 32 == 0));
}

// Both orientations of one tile of a plain matrix X -- 32 rows (32 ty ..) by 64 columns (64 tx ..) -- as scaled
// exponent planes: o0 is X as stored (its rows are X's, k runs along X's columns), o1 is X transposed.  The
// tile is one workgroup's share of either operand in prepare_scaled_block, and the threads keep that function's
// element mappings: the tile is read and rounded once in o0's mapping (a row's eight consecutive columns per
// thread), the rounded patterns cross over to o1's mapping (a column's eight consecutive rows) through LDS.
// A workgroup takes kPairTiles tiles side by side (columns 64 tx0 ..): all their loads are issued before the first
// is worked on (measured: two tiles 2 - 4 % faster than one, four slower than two).
constexpr int kPairTiles = 2;

// ROUND: the pass also does what fmt_quantize does with the tensor -- the rounded values go to Y (leading
// dimension ldy) as fp32 and every element of X is counted in the workgroup's statistics table (tbl, w).
constexpr int kPairCopies = 8;                          // replicas of the statistics table (lane l uses l % 8)
constexpr int kRoundSteps = 4;                          // steps of kPairTiles tiles per workgroup of a ROUND launch, at most

template <int MODE, bool FTZ, bool ROUND, bool DEEP, class OP>
__device__ __forceinline__ void prepare_pair_tile(const OP &o0, const OP &o1, const QuantParams &p, int ty, int tx0,
                                                  uint32_t *Y, int64_t ldy, uint32_t *tbl, Counts &w)
{
    __shared__ __align__(16) uint32_t s_r[32][68];      // 68: rows stay 16-byte aligned, 128-bit writes spread over all banks
    __shared__ uint32_t s_planes[4 * kPairTiles];       // per tile: o0's two units (halves of k), then o1's two (halves of its rows)
    const int tid = threadIdx.x;
    if (tid < 4 * kPairTiles) s_planes[tid] = 0u;
    const int R = o0.rows, C = o1.rows;                 // X is R x C
    const int xr = ty * 32 + tid / 8;
    uint32_t v[kPairTiles][8];
#pragma unroll
    for (int n = 0; n < kPairTiles; ++n) {
        const int xc = (tx0 + n) * 64 + (tid % 8) * 8;
        if (o0.vec4 && xr < R && xc + 8 <= C) {
            const u32x4 *src = reinterpret_cast<const u32x4 *>(o0.X + (size_t)xr * o0.ld + xc);
            const u32x4 lo = __builtin_nontemporal_load(src), hi = __builtin_nontemporal_load(src + 1);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                v[n][j] = lo[j];
                v[n][4 + j] = hi[j];
            }
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) v[n][j] = (xr < R && xc + j < C) ? o0.X[(size_t)xr * o0.ld + xc + j] : 0u;
        }
    }
#pragma unroll
    for (int n = 0; n < kPairTiles; ++n) {
        const int tx = tx0 + n;
        const int xc = tx * 64 + (tid % 8) * 8;
        uint32_t r[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) r[j] = quantize_bits<MODE, FTZ>(v[n][j], p);
        if constexpr (ROUND) {
            const bool row_ok = xr < R;
#pragma unroll
            for (int j = 0; j < 8; ++j)
                account<DEEP, kPairCopies>(v[n][j] & 0x7FFFFFFFu, row_ok && xc + j < C, p, tbl, (uint32_t)tid % kPairCopies, w);
            if (row_ok) {
                uint32_t *dstY = Y + (size_t)xr * ldy + xc;
                if (xc + 8 <= C && ((reinterpret_cast<uintptr_t>(Y) | (uintptr_t)(ldy * 4)) & 15) == 0) {
                    __builtin_nontemporal_store(u32x4{r[0], r[1], r[2], r[3]}, reinterpret_cast<u32x4 *>(dstY));
                    __builtin_nontemporal_store(u32x4{r[4], r[5], r[6], r[7]}, reinterpret_cast<u32x4 *>(dstY) + 1);
                } else {
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if (xc + j < C) dstY[j] = r[j];
                }
            }
        }
        // (the reads of the tile before this one ended before that tile's second barrier)
        u32x4 *dst = reinterpret_cast<u32x4 *>(&s_r[tid / 8][(tid % 8) * 8]);
        dst[0] = u32x4{r[0], r[1], r[2], r[3]};
        dst[1] = u32x4{r[4], r[5], r[6], r[7]};
        __syncthreads();
        // beyond an operand's k-blocks there is nothing of it to write (the other operand's padded rows lie there)
        const bool do0 = tx < (o0.kblocks + 1) / 2, do1 = ty < o1.kblocks;
        const bool live0 = do0 && xc < o0.kblocks * kUnitK;       // the last slab of o0 may hold one k-block only
        const int row1 = tx * 64 + tid % 64, k1 = ty * 32 + (tid / 64) * 8;
        const int u0 = 4 * n + (tid % 8) / 4, u1 = 4 * n + 2 + (tid % 64) / 32;
        // (where an operand has nothing to write the tile holds zeros only and its rows are padded ones, whose
        // scales exist: the split is harmless there and leaves no records)
        uint32_t t[8];
        u32x4 p0a, paa, pba, p0b, pab, pbb;
        const uint32_t mine0 = split_planes(o0, xr, xc, r, p0a, paa, pba);
#pragma unroll
        for (int j = 0; j < 8; ++j) t[j] = s_r[(tid / 64) * 8 + j][tid % 64];
        const uint32_t mine1 = split_planes(o1, row1, k1, t, p0b, pab, pbb);
        if (mine0 != 0u) atomicOr(&s_planes[u0], mine0);
        if (mine1 != 0u) atomicOr(&s_planes[u1], mine1);
        __syncthreads();
        if (live0) store_planes(o0, xr, xc, o0.kblocks, p0a, paa, pba, s_planes[u0], tid / 8 == 0 && tid % 4 == 0);
        if (do1) store_planes(o1, row1, k1, o1.kblocks, p0b, pab, pbb, s_planes[u1], tid / 64 == 0 && tid % 32 == 0);
    }
}

// One launch prepares both operands of a product (or one: b.nblocks == 0).
template <int MODE, bool FTZ, int PS, bool TAPS>
__global__ __launch_bounds__(256) void prepare_kernel(PrepOperand a, PrepOperand b, int K, int kblocks, QuantParams p)
{
    prepare_block<MODE, FTZ, PS, TAPS>(a, b, K, kblocks, p, blockIdx.x);
}

template <int MODE, bool FTZ>
__global__ __launch_bounds__(256) void prepare_scaled_kernel(PrepOperand a, PrepOperand b, int Ka, int kblocks_a, int Kb,
                                                             int kblocks_b, QuantParams p)
{
    // operands own runs of workgroup ids padded to a multiple of 8, remapped XCD by XCD as in prepare_block
    const unsigned a_ids = (a.nblocks + 7u) / 8u * 8u;
    const bool second = blockIdx.x >= a_ids;
    const PrepOperand &o = second ? b : a;
    const unsigned lid = blockIdx.x - (second ? a_ids : 0u);
    const unsigned per_xcd = (o.nblocks + 7u) / 8u;
    const unsigned bid = (lid % 8u) * per_xcd + lid / 8u;
    if (bid >= o.nblocks) return;                // workgroup-uniform: before any barrier
    prepare_scaled_block<MODE, FTZ>(o, second ? Kb : Ka, second ? kblocks_b : kblocks_a, p, bid);
}

// The exponent planes of both orientations of up to kMaxPrepGroup / 2 plain matrices in one launch.  Operands
// 2i (X as stored: rows of X, k along its columns) and 2i + 1 (X transposed) belong to matrix i; the table
// travels by value in the kernel arguments.  A workgroup takes tiles of 32 rows x 64 columns of X and
// prepares them for both operands (prepare_pair_tile): X is read and rounded once.  Every
// matrix owns a run of workgroup ids padded to a multiple of 8 (first[] = the runs' first ids, ascending)
// and remapped XCD by XCD as above.
constexpr int kMaxPrepGroup = 32;

struct PrepPlain {
    const uint32_t *X;
    u32x4 *W;
    int64_t ld;
    int rows;
    int kcontig;
    int vec4;
    int units;
    int K, kblocks;
    Planes pl;
};

struct PrepGroup {
    unsigned first[kMaxPrepGroup / 2];   // 0xFFFFFFFF beyond the last matrix
    unsigned tiles[kMaxPrepGroup / 2];
    PrepPlain o[kMaxPrepGroup];
};

// index of the run that holds workgroup `id`: the number of runs that start at or before it, minus one
// (first[] ascending, 0xFFFFFFFF beyond the last run)
template <int CAP>
__device__ __forceinline__ int run_of(const unsigned (&first)[CAP], unsigned id)
{
    int at = -1;
#pragma unroll
    for (int i = 0; i < CAP; ++i) at += id >= first[i] ? 1 : 0;
    return at;
}

// what the ROUND variant needs of every matrix: the rounded fp32 copy and the partial statistics records
struct RoundGroup {
    uint32_t *Y[kMaxPrepGroup / 2];
    int64_t ldy[kMaxPrepGroup / 2];
    unsigned long long *partials[kMaxPrepGroup / 2];
    int steps;                                   // steps of kPairTiles tiles per workgroup
};

template <int MODE, bool FTZ, bool ROUND, bool DEEP>
__global__ __launch_bounds__(256) void prepare_scaled_group_kernel(PrepGroup grp, RoundGroup rg, QuantParams p)
{
    __shared__ __align__(16) uint32_t tbl[ROUND ? kHistRows * kPairCopies : 4];
    __shared__ uint32_t s_bins[ROUND ? FMT_NBINS : 1], s_cls[ROUND ? 8 : 1];
    const int at = run_of(grp.first, blockIdx.x);
    const PrepPlain &o0 = grp.o[2 * at], &o1 = grp.o[2 * at + 1];
    // ROUND: a workgroup takes up to kRoundSteps consecutive steps of kPairTiles tiles, so that clearing and folding
    // its statistics table is paid once per 16 K elements (as in the stream kernels); fewer when the launch is small
    const unsigned kSteps = ROUND ? (unsigned)rg.steps : 1u;
    const unsigned lid = blockIdx.x - grp.first[at], ntiles = grp.tiles[at];
    const unsigned nwg = (ntiles + kSteps - 1u) / kSteps;
    const unsigned per_xcd = (nwg + 7u) / 8u;
    const unsigned g = (lid % 8u) * per_xcd + lid / 8u;
    if (g >= nwg) return;                        // workgroup-uniform: before any barrier
    // rows of X in 32s: o0's units (rows padded to the tile grid) cover o1's k-blocks; columns of X in 64s:
    // pairs of o1's units cover o0's slabs of two k-blocks
    const int ntx = o1.units / (2 * kPairTiles);
    Counts w;
    if constexpr (ROUND) hist_begin<kPairCopies, 256>(tbl, s_bins, s_cls, threadIdx.x);
#pragma unroll 1
    for (unsigned step = 0; step < kSteps; ++step) {
        const unsigned t = g * kSteps + step;
        if (t >= ntiles) break;                  // workgroup-uniform
        if (step > 0) __syncthreads();           // the step before has read its words of LDS
        const int ty = (int)(t / (unsigned)ntx), tx = (int)(t % (unsigned)ntx) * kPairTiles;
        prepare_pair_tile<MODE, FTZ, ROUND, DEEP>(o0, o1, p, ty, tx, ROUND ? rg.Y[at] : nullptr, ROUND ? rg.ldy[at] : 0, tbl, w);
    }
    if constexpr (ROUND)
        hist_end<kPairCopies, 256>(tbl, s_bins, s_cls, w, p, rg.partials[at], blockIdx.x % kShards, threadIdx.x);
}

// Epilogue of one wave.  The MFMAs are fed operand B's fragment first and A's second, so a 32 x 32 accumulator
// block holds the TRANSPOSE of the usual layout: register v of lane l holds row l % 32 and column
// 8*(v/4) + 4*(l/32) + v%4 of the block of C -- four consecutive columns per group of four registers, which
// leave in one 16-byte store per lane (64 store instructions per wave for a 256 x 256 tile instead of 256;
// nothing is assumed about alignment beyond 4 bytes).
// SCALED: out = acc * 2^-(S_row + S_col), exactly; the scale arrays are padded to the tile grid and 16-byte
// aligned, and all of a lane's scales are fetched together ahead of its stores.
// img > 0: column = (image, position), element (row, col) goes to out[image][row][position] (NCHW with `img`
// positions); the four columns of a group go out together when they fall into one image.
// A wave whose block of C lies inside the matrix (all but the last row and column of tiles) takes a path without
// per-lane tests, in two phases: first every accumulator is scaled in place, then the stores go out straight
// from the accumulator registers.  Measured on a 256 x 256 tile (one wave per SIMD): stores interleaved with
// the arithmetic that refills their data registers take 20 - 25 us per tile when every compute unit stores at
// once (a store holds its data registers until the memory pipeline has taken them), the two phases 8 us, of
// which the stores are 5.
template <int TM, int TN, bool SCALED>
__device__ __forceinline__ void store_tile(floatx16 (&acc)[TM][TN], float *__restrict__ out, int64_t ld, int M, int N, int img,
                                           int row_base, int col_base, int lane, const int *__restrict__ Sa,
                                           const int *__restrict__ Sb)
{
    typedef int i32x4 __attribute__((ext_vector_type(4)));
    typedef float f32x4u __attribute__((ext_vector_type(4), aligned(4)));
    const int r_in = lane & 31, c_half = (lane >> 5) * 4;
    int sa[TM];
    i32x4 sb[TN][4];
    if constexpr (SCALED) {
#pragma unroll
        for (int i = 0; i < TM; ++i) sa[i] = Sa[row_base + i * 32 + r_in];
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) sb[j][g] = -*reinterpret_cast<const i32x4 *>(Sb + col_base + j * 32 + g * 8 + c_half);
    }
    // rows are `rs` elements apart in both output maps
    const size_t rs = img > 0 ? (size_t)img : (size_t)ld;
    float *rowp[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) rowp[i] = out + (size_t)(row_base + i * 32 + r_in) * rs;

    if (row_base + 32 * TM <= M && col_base + 32 * TN <= N && (img & 3) == 0) {      // the same in the whole wave
        if constexpr (SCALED) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[i][j][v] = ldexpf(acc[i][j][v], sb[j][v >> 2][v & 3] - sa[i]);
            __builtin_amdgcn_sched_barrier(0);
        }
        // the four stores that complete the 128-byte lines of a block go out back to back
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            size_t coff[4];
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int col0 = col_base + j * 32 + g * 8 + c_half;
                coff[g] = (size_t)col0;
                if (img > 0) {                   // img is a multiple of 4 and so is col0: one image holds the four columns
                    const int image = col0 / img;
                    coff[g] = (size_t)image * M * img + (col0 - image * img);
                }
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    f32x4u v;
#pragma unroll
                    for (int c = 0; c < 4; ++c) v[c] = acc[i][j][g * 4 + c];
                    *reinterpret_cast<f32x4u *>(rowp[i] + coff[g]) = v;
                }
        }
        return;
    }
    // the last row or column of tiles, and NCHW maps whose images are not a multiple of 4 positions long
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int col0 = col_base + j * 32 + g * 8 + c_half;
            if (col0 >= N) continue;
            // offset of column col0 within a row of the output map; whether its four columns are adjacent there
            size_t coff = (size_t)col0;
            bool together = col0 + 3 < N;
            if (img > 0) {
                const int image = col0 / img, pos = col0 - image * img;
                coff = (size_t)image * M * img + pos;
                together = together && pos + 3 < img;
            }
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                if (row_base + i * 32 + r_in >= M) continue;
                f32x4u v;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    v[c] = acc[i][j][g * 4 + c];
                    if constexpr (SCALED) v[c] = ldexpf(v[c], sb[j][g][c] - sa[i]);
                }
                if (together) {
                    *reinterpret_cast<f32x4u *>(rowp[i] + coff) = v;
                } else {
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        if (col0 + c < N) {
                            size_t off = coff + c;
                            if (img > 0) {
                                const int image = (col0 + c) / img;
                                off = (size_t)image * M * img + (col0 + c - image * img);
                            }
                            rowp[i][off] = v[c];
                        }
                }
            }
        }
}

// product: Aw / Bw are prepared operands (rows padded to a multiple of kRowPad, k to a multiple
// of 32).  A workgroup is 2 x 2 waves; each wave owns TM x TN MFMA tiles of 32 x 32, so the
// workgroup tile is (64*TM) x (64*TN).  Operand stages of KS*16 k go from global memory straight
// into LDS (global_load_lds, 16 bytes per lane) through a ring of NST stage buffers, one barrier
// per stage.  With SPLIT the k range is cut into parts and each part writes its own M x N slab
// of partial sums (summed by reduce_kernel).
// SCALED (single fp16 piece only): the operands are exponent planes with per-row power-of-two scales
// (pa.S / pb.S), undone on the way out; this kernel multiplies plane 0 by plane 0, planes_tail_kernel
// adds the products of the elements that live in the other planes.
// GATHER: operand B is not a prepared operand but a rounded convolution tensor in pixel-major order (`im`,
// Bw unused): a lane's 16-byte load of (position, 8 consecutive k) is 8 consecutive channels of one pixel,
// whose address is a per-lane base (the position's corner pixel) plus a per-stage term (the tap and the
// channel block), or the zero vector where the tap falls outside the tensor (a per-lane bit mask over
// the taps).  The stage image in LDS and everything after it are the same.
// The body is shared by the kernel of one product (bid = blockIdx.x) and the kernel of a group of products
// (bid = the workgroup's index within its product).
template <int PS, int TM, int TN, int KS, int NST, bool SPLIT, bool SCHED, bool SCALED, bool GATHER = false>
__device__ __forceinline__ void product_body(const u32x4 *__restrict__ Aw, const u32x4 *__restrict__ Bw,
                                             float *__restrict__ C, int M, int N, int64_t ldc, int img,
                                             int kblocks, int tiles_m, int tiles_n, int kb_per_split,
                                             const Planes &pa, const Planes &pb, const Implicit &im, const unsigned bid)
{
    constexpr int P = pieces_of(PS);
    constexpr int UA = 2 * TM, UB = 2 * TN;              // 32-row units per operand in the workgroup tile
    constexpr int kHalf = 64;                            // vectors of one piece of one unit per 16 k
    constexpr int SV = kHalf * KS;                       // ... per stage
    constexpr int VA = UA * P * SV, VB = UB * P * SV;    // 16-byte vectors per operand per stage
    constexpr int LA = (VA + 255) / 256, LB = (VB + 255) / 256;   // loads per lane per stage
    constexpr int kWaitLanded = ((NST - 2) * (LA + LB));  // stage loads that may still be in flight
    static_assert(kWaitLanded < 64 && (KS == 1 || KS == 2) && NST >= 2 && NST <= 4, "unsupported pipeline shape");
    static_assert(NST == 2 || (VA % 256 == 0 && VB % 256 == 0), "the wait for a stage counts the same loads in every wave");
    // One LDS array per stage buffer, each addressed with a compile-time index: the compiler then knows
    // which loads-to-LDS an LDS read can depend on and leaves the younger stages in flight.
    constexpr int STV = VA + VB;
    __shared__ u32x4 st0[STV];
    __shared__ u32x4 st1[STV];
    __shared__ u32x4 st2[NST > 2 ? STV : 1];
    __shared__ u32x4 st3[NST > 3 ? STV : 1];
    auto stage = [&](int b) -> u32x4 * { return b == 0 ? st0 : b == 1 ? st1 : b == 2 ? st2 : st3; };
    typedef __attribute__((address_space(3))) void lds_void;
    typedef const __attribute__((address_space(1))) void glb_void;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;

    // Workgroup -> (tile, k part).  Consecutive workgroup ids go to different XCDs (8 of them,
    // each with its own L2), so ids are remapped to give every XCD a contiguous run of tiles.
    const int ntiles = tiles_m * tiles_n;
    const int per_xcd = (ntiles + 7) / 8;
    const int wg = (int)(bid % (unsigned)(per_xcd * 8));
    const int split = (int)(bid / (unsigned)(per_xcd * 8));
    const int tile = (wg % 8) * per_xcd + wg / 8;
    if (tile >= ntiles) return;
    // Within the run, tiles are walked in groups of kGroup tile rows, column by column, so that
    // the 32 tiles an XCD works on at a time cover few distinct operand panels.
    constexpr int kGroup = 16 / TM;                      // 1024 rows of op(A) per group
    const int per_group = kGroup * tiles_n;
    const int group = tile / per_group, in_group = tile % per_group;
    const int rows_here = min(kGroup, tiles_m - group * kGroup);
    const int tm = group * kGroup + in_group % rows_here, tn = in_group / rows_here;
    const int kb0 = SPLIT ? split * kb_per_split : 0;
    const int kb1 = SPLIT ? min(kblocks, kb0 + kb_per_split) : kblocks;
    const int steps = (kb1 - kb0) * (2 / KS);            // stages to consume

    // Stage image per operand = [unit row-block][piece][SV vectors]; in the workspace a unit's
    // piece is 128 vectors (two 16-k halves) and row-blocks are kblocks*P*128 vectors apart.
    const size_t rb_stride = (size_t)kblocks * P * kUnitVec;
    const u32x4 *ga[LA], *gb[LB];
#pragma unroll
    for (int j = 0; j < LA; ++j) {
        const int q = min(j * 256 + tid, VA - 1);
        const int rbl = q / (P * SV), piece = (q % (P * SV)) / SV, v = q % SV;
        ga[j] = Aw + ((size_t)tm * UA + rbl) * rb_stride + (size_t)kb0 * P * kUnitVec + piece * kUnitVec + v;
    }
    int gbase[GATHER ? LB : 1];          // GATHER: vector index of the position's corner pixel (+ piece, + k chunk)
    uint32_t gmask[GATHER ? LB : 1];     // ... and the taps that fall inside the tensor
#pragma unroll
    for (int j = 0; j < LB; ++j) {
        const int q = min(j * 256 + tid, VB - 1);
        const int rbl = q / (P * SV), piece = (q % (P * SV)) / SV, v = q % SV;
        if constexpr (GATHER) {
            const int row = (tn * UB + rbl) * kUnitRows + v % kUnitRows;
            int x, t, y, n;
            divmod(im.r0, min(row, im.rows - 1), t, x);
            divmod(im.r1, t, n, y);
            const int by = y * im.mul_y + im.off_y, bx = x * im.mul_x + im.off_x;
            uint32_t mq = 0u;
            int tap = 0;
            for (int r = 0; r < im.R; ++r)
                for (int s2 = 0; s2 < im.S; ++s2, ++tap) {
                    const int iy = by + im.tap_sign * r, ix = bx + im.tap_sign * s2;
                    if ((unsigned)iy < (unsigned)im.th && (unsigned)ix < (unsigned)im.tw) mq |= 1u << tap;
                }
            gmask[j] = row < im.rows ? mq : 0u;
            gbase[j] = piece * im.piece_vec + ((n * im.th + by) * im.tw + bx) * im.c8 + v / kUnitRows;
            gb[j] = im.T;
        } else {
            gb[j] = Bw + ((size_t)tn * UB + rbl) * rb_stride + (size_t)kb0 * P * kUnitVec + piece * kUnitVec + v;
        }
    }

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    // Loads of stage t (clamped to the last one, so that the number of loads in flight is the
    // same in every trip; a clamped load lands in a buffer nobody reads any more).
    auto issue = [&](int t, int buf) {
        const int tc = min(t, steps - 1);
        u32x4 *sa = stage(buf), *sb = sa + VA;
        const size_t off = KS == 2 ? (size_t)tc * P * kUnitVec : (size_t)(tc >> 1) * P * kUnitVec + (tc & 1) * kHalf;
#pragma unroll
        for (int j = 0; j < LA; ++j)
            if (VA % 256 == 0 || j * 256 + wave * 64 < VA)
                __builtin_amdgcn_global_load_lds((glb_void *)(ga[j] + off), (lds_void *)(sa + j * 256 + wave * 64), 16, 0, 0);
        if constexpr (GATHER) {
            // stage number (in stages of 16*KS k) -> tap and channel block: the same in the whole workgroup
            int tap, cb, r, s2;
            divmod(im.kc, kb0 * (2 / KS) + tc, tap, cb);
            divmod(im.ks, tap, r, s2);
            const int toff = im.tap_sign * (r * im.tw + s2) * im.c8 + cb * (2 * KS);
#pragma unroll
            for (int j = 0; j < LB; ++j)
                if (VB % 256 == 0 || j * 256 + wave * 64 < VB) {
                    const int at = ((gmask[j] >> tap) & 1u) ? gbase[j] + toff : im.zero;
                    __builtin_amdgcn_global_load_lds((glb_void *)(im.T + at), (lds_void *)(sb + j * 256 + wave * 64), 16, 0, 0);
                }
        } else {
#pragma unroll
            for (int j = 0; j < LB; ++j)
                if (VB % 256 == 0 || j * 256 + wave * 64 < VB)
                    __builtin_amdgcn_global_load_lds((glb_void *)(gb[j] + off), (lds_void *)(sb + j * 256 + wave * 64), 16, 0, 0);
        }
    };

    // Operand fragments live in two register sets: while the MFMAs of stage t run on one, the LDS
    // reads of stage t + 1 fill the other, so that no MFMA waits for LDS latency (a workgroup tile
    // of 128 x 128 has one wave per SIMD and nothing else to run meanwhile).
    bf16x8 fa[2][KS][TM][P], fb[2][KS][TN][P];
    auto read_frags = [&](int buf, int set) __attribute__((always_inline)) {
        const u32x4 *sa = stage(buf), *sb = sa + VA;
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int q = 0; q < P; ++q)
                    fa[set][kk][i][q] = __builtin_bit_cast(bf16x8, sa[((wm * TM + i) * P + q) * SV + kk * kHalf + lane]);
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int q = 0; q < P; ++q)
                    fb[set][kk][j][q] = __builtin_bit_cast(bf16x8, sb[((wn * TN + j) * P + q) * SV + kk * kHalf + lane]);
        }
    };
    // The barrier is the bare instruction behind the waits it needs (this wave's LDS reads retired,
    // its stage landed): __syncthreads() would also wait for every load-to-LDS still in flight.
    auto barrier = [&]() __attribute__((always_inline)) { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };

    if (steps > 0) {
#pragma unroll
        for (int t = 0; t < NST; ++t) issue(t, t);
        constexpr int kWaitFirst = (NST - 1) * (LA + LB);
        __builtin_amdgcn_s_waitcnt(0x0F70 | (kWaitFirst & 0xF) | ((kWaitFirst >> 4) << 14));
        barrier();
        read_frags(0, 0);
    }
    // Trip t: stage t is in register set `cur`; stage t + 1 (buffer b + 1) is read into the other set
    // and stage t + NST is loaded into buffer b, which every wave has finished reading once it is past
    // the barrier.  The trips are unrolled over the ring and the two register sets, so that buffer and
    // set are compile-time constants, and the loop over whole turns has a single exit (with early
    // exits the compiler falls back to waiting for all loads at the loop head); the remaining trips
    // follow it.
    auto trip = [&](int t, int b, int cur) __attribute__((always_inline)) {
        // stage t + 1 has landed once at most the loads of the NST-2 younger stages are in flight
        __builtin_amdgcn_sched_barrier(0);       // MFMAs are not memory operations: without this they drift across the barrier
        __builtin_amdgcn_s_waitcnt(0x0F70 | (kWaitLanded & 0xF) | ((kWaitLanded >> 4) << 14));
        barrier();                               // ... for every wave; and every wave holds stage t in registers
        read_frags((b + 1) % NST, cur ^ 1);
        issue(t + NST, b);
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int qa = 0; qa < P; ++qa)
#pragma unroll
                        for (int qb = 0; qb < P; ++qb)
                            // B's fragment first: the block comes out transposed (see store_tile)
                            acc[i][j] = PS == 0 ? __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, fb[cur][kk][j][qb]),
                                                                                         __builtin_bit_cast(f16x8, fa[cur][kk][i][qa]),
                                                                                         acc[i][j], 0, 0, 0)
                                                : __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[cur][kk][j][qb], fa[cur][kk][i][qa], acc[i][j], 0, 0, 0);
        }
        // Issue order inside one trip: the next stage's LDS reads, then its global loads, threaded
        // between the MFMAs so that they issue in the MFMAs' shadow.
        if constexpr (SCHED) {
            constexpr int kMfma = TM * TN * P * P * KS, kReads = (TM + TN) * P * KS, kLoads = LA + LB;
            constexpr int kDsEach = (kReads + kMfma - 1) / kMfma;            // LDS reads behind each of the first MFMAs
            constexpr int kPairs = (kReads + kDsEach - 1) / kDsEach;
#pragma unroll
            for (int r = 0; r < kPairs; ++r) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, kDsEach, 0);
            }
            constexpr int kLeft = kMfma - kPairs;                            // MFMAs left for the global loads
            if constexpr (kLeft > kLoads) {
                constexpr int kPer = kLeft / (kLoads + 1);
#pragma unroll
                for (int r = 0; r < kLoads; ++r) {
                    __builtin_amdgcn_sched_group_barrier(0x008, kPer, 0);
                    __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
                }
            } else if constexpr (kLeft > 0) {
                constexpr int kEach = (kLoads + kLeft - 1) / kLeft;
#pragma unroll
                for (int r = 0; r < kLeft; ++r) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x020, kEach, 0);
                }
            } else {
                __builtin_amdgcn_sched_group_barrier(0x020, kLoads, 0);
            }
        }
    };
    constexpr int kTurn = NST % 2 == 0 ? NST : 2 * NST;      // trips after which buffer and register set repeat
    int t0 = 0;
    for (; t0 + kTurn <= steps; t0 += kTurn) {
#pragma unroll
        for (int u = 0; u < kTurn; ++u) trip(t0 + u, u % NST, u & 1);
    }
#pragma unroll
    for (int u = 0; u < kTurn - 1; ++u)
        if (t0 + u < steps) trip(t0 + u, u % NST, u & 1);
    // every load-to-LDS of this wave must have landed before the workgroup's LDS is handed back
    __builtin_amdgcn_s_waitcnt(0x0F70);

    // plain: C[row][col] with leading dimension ldc; a part of a split k: its own M x N slab; img > 0: NCHW
    float *out = SPLIT ? C + (size_t)split * M * ldc : C;
    store_tile<TM, TN, SCALED>(acc, out, ldc, M, N, SPLIT ? 0 : img, (tm * 2 + wm) * (32 * TM), (tn * 2 + wn) * (32 * TN), lane, pa.S,
                               pb.S);
}

template <int PS, int TM, int TN, int KS, int NST, bool SPLIT, bool SCHED, bool SCALED, bool GATHER = false>
__global__ __launch_bounds__(256) void product_kernel(const u32x4 *__restrict__ Aw, const u32x4 *__restrict__ Bw,
                                                      float *__restrict__ C, int M, int N, int64_t ldc, int img,
                                                      int kblocks, int tiles_m, int tiles_n, int kb_per_split,
                                                      Planes pa, Planes pb, Implicit im)
{
    product_body<PS, TM, TN, KS, NST, SPLIT, SCHED, SCALED, GATHER>(Aw, Bw, C, M, N, ldc, img, kblocks, tiles_m, tiles_n,
                                                                  kb_per_split, pa, pb, im, blockIdx.x);
}

// A group of independent products in one launch (fmt_gemm_prepared_batch): workgroup ids [first, next first)
// belong to product g, each product's run of ids is a multiple of 8 long (so that id % 8, the XCD, means the
// same inside every run), and every product runs the same kernel variant -- no k split, plain row-major output.
// One launch instead of one per product: launch, pipeline fill and drain -- about a third of the time of a
// product with K = 1024 -- are paid once, and the tiles of the next product fill the compute units that the
// last tiles of the previous one leave idle.
constexpr int kMaxGroup = 16;
struct GroupItem {
    const u32x4 *Aw, *Bw;
    float *C;               // the result, or (k in parts) the first of the parts' dense M x N slabs (then ldc = N)
    int64_t ldc;
    int M, N, kblocks, tiles_m, tiles_n;
    int kb_per_part;        // k blocks per part (= kblocks: one part); the product's run of ids holds one run of tiles per part
    unsigned first;
    Planes pa, pb;
};
struct Group {
    int count;
    unsigned first[kMaxGroup];     // p[i].first again, side by side (one scalar load), 0xFFFFFFFF beyond count
    GroupItem p[kMaxGroup];
};

// Which product a workgroup id belongs to: the number of runs that start at or before it, minus one.
__device__ __forceinline__ int group_member(const unsigned (&first)[kMaxGroup], unsigned id)
{
    int g = -1;
#pragma unroll
    for (int i = 0; i < kMaxGroup; ++i) g += id >= first[i] ? 1 : 0;
    return g;
}

template <int PS, int TM, int TN, int KS, int NST, bool SCHED, bool SCALED>
__global__ __launch_bounds__(256) void product_group_kernel(Group grp)
{
    const GroupItem &it = grp.p[group_member(grp.first, blockIdx.x)];      // the same in the whole workgroup
    product_body<PS, TM, TN, KS, NST, true, SCHED, SCALED, false>(it.Aw, it.Bw, it.C, it.M, it.N, it.ldc, 0, it.kblocks, it.tiles_m,
                                                                it.tiles_n, it.kb_per_part, it.pa, it.pb, Implicit{},
                                                                blockIdx.x - it.first);
}

// Half h (0..7) of a 16-byte vector of eight 16-bit patterns, as a float (binary16 -> fp32 is exact).
__device__ __forceinline__ float half_of(const u32x4 &v, int h)
{
    const uint32_t w = (h >> 1) == 0 ? v[0] : (h >> 1) == 1 ? v[1] : (h >> 1) == 2 ? v[2] : v[3];
    return static_cast<float>(__builtin_bit_cast(_Float16, (uint16_t)((h & 1) ? w >> 16 : w & 0xFFFFu)));
}

// Element (row r of the unit, k-chunk c, position h) of the unit whose plane-0 vectors start at W + unit_vec,
// in the scale of plane 0, whichever plane holds it: plane 0 as stored, the plane above times 2^w, the
// plane below times 2^-w (exact: a binary16 value times a power of two, far inside fp32's range).
__device__ __forceinline__ float unit_value(const u32x4 *__restrict__ W, size_t unit_vec, const Planes &pl, uint32_t planes,
                                            int c, int r, int h)
{
    const size_t at = unit_vec + (size_t)(c * kUnitRows + r);
    float x = half_of(W[at], h);
    if (planes & 6u) {                            // rare
        if (planes & 2u) x += ldexpf(half_of(W[pl.plane + at], h), pl.w);
        if (planes & 4u) x += ldexpf(half_of(W[2 * pl.plane + at], h), -pl.w);
    }
    return x;
}

// The products of the elements that live outside plane 0, added to C after the product kernel has stored
// plane 0 x plane 0.  Such elements are rare (a few per million for tensors of neural networks) and each
// contributes to one row or one column of C, so they are added one product at a time with fp32 fused
// multiply-adds on the TRUE values (the binary16 pattern with its plane's and its row's scale undone: a
// value of the format, exactly an fp32) -- exact product, one rounding per accumulation, FMACS.
// One workgroup owns a block of 32 rows (one unit of A) x tail_cols columns (8, 16 or 32 units of B) of C.
// Finding the elements of a row of units (masks, the other planes' vectors, the records) is a chain of dependent
// loads and barriers that costs more than using them, and every block of the same rows repeats it: wide blocks
// when the launch has blocks enough to fill the machine anyway, narrow ones otherwise (tail_cols_for).
//   1. every element a of A's other planes in its rows meets the FULL value of B (all planes) at that k
//      in each of its columns, elements in the order (k block, plane, position in the unit);
//   2. then every element b of B's other planes in its columns meets the plane-0 value of A in each of its
//      rows (an element of A outside plane 0 has met b in step 1), in the same kind of order.
// Every element of C has one owner and a fixed order of additions: the result is reproducible bit for bit.
// A block whose units hold nothing but plane 0 -- the usual case -- leaves after reading its masks.
constexpr int kTailRecs = kUnitRows * kUnitK;    // element records held at a time: one plane of one unit always fits

__device__ __forceinline__ void planes_tail_body(const u32x4 *__restrict__ Aw, const u32x4 *__restrict__ Bw, const Planes &pa,
                                                 const Planes &pb, float *__restrict__ C, int64_t ldc, int M, int N, int kblocks,
                                                 int col_chunks, int tail_cols, const unsigned bid)
{
    __shared__ uint32_t s_rec[kTailRecs];        // row-or-column in the unit (5 bits) | k << 5
    __shared__ float s_val[kTailRecs];           // the element's true value
    __shared__ uint32_t s_list[256];             // k blocks (of one scan of 256) whose unit has other planes | planes << 16
    __shared__ int s_cnt[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int rb = (int)(bid / (unsigned)col_chunks), cc = (int)(bid % (unsigned)col_chunks);
    const int ub0 = cc * (tail_cols / kUnitRows);    // first unit of B of this block
    const int nub = min(tail_cols / kUnitRows, (N + kRowPad - 1) / kRowPad * (kRowPad / kUnitRows) - ub0);   // B is padded to whole groups of 8 units

    // how many elements outside plane 0 A's row of units and B's rows of units hold (counted by the prepare pass)
    const uint32_t cnt_a = pa.rec_cnt[rb];
    const bool do_a = cnt_a != 0u;
    const bool do_b = __syncthreads_or(tid < nub && pb.rec_cnt[ub0 + tid] != 0u ? 1 : 0) != 0;
    if (!do_a && !do_b) return;

    // The records of a row of units whose count fits its list: read, and put into the order (k, row) -- the
    // prepare pass appends them in whatever order its workgroups run, and the additions below must not depend
    // on that.  One barrier before (the record arrays are free), one after.
    auto take_list = [&](const Planes &pl, size_t urow, int n) __attribute__((always_inline)) {
        uint32_t key = 0u, val = 0u;
        if (tid < n) {
            key = pl.recs[(urow * kRecCap + tid) * 2];
            val = pl.recs[(urow * kRecCap + tid) * 2 + 1];
            s_list[tid] = key;
        }
        __syncthreads();
        if (tid < n) {
            int rank = 0;
            for (int i = 0; i < n; ++i) rank += s_list[i] < key ? 1 : 0;
            s_rec[rank] = key;
            s_val[rank] = __uint_as_float(val);
        }
        __syncthreads();
    };

    // Ordered compaction over the workgroup: thread t contributes `have` items; returns the index of its
    // first one and, in total, the number of items.  Two barriers.
    auto place = [&](int have, int &total) __attribute__((always_inline)) {
        int incl = have;                                   // inclusive prefix inside the wave
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int up = __shfl_up(incl, off, 64);
            if (lane >= off) incl += up;
        }
        __syncthreads();                                   // s_cnt is free again
        if (lane == 63) s_cnt[wave] = incl;
        __syncthreads();
        int before = 0;
        total = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            before += q < wave ? s_cnt[q] : 0;
            total += s_cnt[q];
        }
        return before + incl - have;
    };

    // Walks the units of one row of units (mask row urow of operand W / pl, row scales S32) that have
    // other planes, k ascending, four units at a time: the two other planes of a unit are 256 vectors, one
    // per thread (threads 0..127 the plane above, vector tid: k-chunk tid / 32, row tid % 32; threads
    // 128..255 the plane below), all four units' loads are issued together, their non-zero elements become
    // records (row in the unit, k, TRUE value: the pattern with the plane's and the row's scale undone) in a
    // fixed order (thread, unit, position), and `apply(n)` uses up the n records of the group.
    auto walk = [&](const u32x4 *__restrict__ W, const Planes &pl, size_t urow, const int *S32, uint32_t first, bool have_first,
                    auto &&apply) {
        const int q = tid < kUnitVec ? 1 : 2, vec = tid & (kUnitVec - 1);
        const int r = vec & 31, c = vec >> 5;
        const int undo = -(S32[r] + (q == 1 ? -pl.w : pl.w));   // the plane above carries 2^(S - w), the one below 2^(S + w)
        for (int base = 0; base < kblocks; base += 256) {
            const int kb = base + tid;
            const uint32_t m = base == 0 && have_first ? first : (kb < kblocks ? (uint32_t)pl.mask[urow * kblocks + kb] & 6u : 0u);
            int total;
            const int at = place(m != 0u ? 1 : 0, total);
            if (m != 0u) s_list[at] = (uint32_t)tid | (m << 16);
            __syncthreads();
            for (int n0 = 0; n0 < total; n0 += 4) {
                u32x4 v[4];
                int kbn[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const uint32_t e = n0 + u < total ? s_list[n0 + u] : 0u;
                    kbn[u] = base + (int)(e & 0xFFFFu);
                    v[u] = u32x4{0u, 0u, 0u, 0u};
                    if ((e >> (16 + q)) & 1u) v[u] = W[(size_t)q * pl.plane + (urow * kblocks + kbn[u]) * kUnitVec + vec];
                }
                // records of unit u (all four: u < 0) and plane qq (both: qq == 0) of this group, then their use
                auto emit = [&](int only_u, int only_q) {
                    const bool mine = only_q == 0 || only_q == q;
                    int cnt = 0;
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (mine && (only_u < 0 || only_u == u)) {
#pragma unroll
                            for (int t = 0; t < 8; ++t) cnt += (((t & 1) ? v[u][t >> 1] >> 16 : v[u][t >> 1]) & 0x7FFFu) != 0u ? 1 : 0;
                        }
                    int nrec;
                    int at2 = place(cnt, nrec);
                    if (nrec > kTailRecs) return nrec;       // workgroup-uniform: the caller splits the group
                    if (cnt) {
#pragma unroll
                        for (int u = 0; u < 4; ++u)
                            if (only_u < 0 || only_u == u) {
#pragma unroll
                                for (int t = 0; t < 8; ++t) {
                                    const uint32_t hp = ((t & 1) ? v[u][t >> 1] >> 16 : v[u][t >> 1]) & 0xFFFFu;
                                    if (hp & 0x7FFFu) {
                                        s_rec[at2] = (uint32_t)r | ((uint32_t)(kbn[u] * kUnitK + c * 8 + t) << 5);
                                        s_val[at2] = ldexpf(static_cast<float>(__builtin_bit_cast(_Float16, (uint16_t)hp)), undo);
                                        ++at2;
                                    }
                                }
                            }
                    }
                    __syncthreads();
                    apply(nrec);
                    __syncthreads();                         // the records are free again
                    return nrec;
                };
                if (emit(-1, 0) > kTailRecs) {               // rare: many elements outside plane 0 -- one plane of one unit at a time
                    for (int u = 0; u < 4; ++u)
                        for (int qq = 1; qq <= 2; ++qq) (void)emit(u, qq);
                }
            }
        }
    };

    if (do_a) {
        // 1. this block's columns of thread tid, one after the other: C[row][col] += a * b(k, col) for the
        //    records (row, k, a) in order
        auto apply_a = [&](int n) {
#pragma unroll 1
          for (int j = 0; j < tail_cols / 256; ++j) {
            const int col = cc * tail_cols + j * 256 + tid;
            if (col >= N) return;
            const int ub = col / kUnitRows, cr = col % kUnitRows;
            const int sb = pb.S[col];
            // four records at a time: their loads (B's vector and mask, C) are issued together, then the
            // additions follow in record order; a row met earlier in the batch hands its sum on in registers
            for (int i0 = 0; i0 < n; i0 += 4) {
                int row[4], k[4];
                float a[4], c[4];
                u32x4 xv[4];
                uint32_t mk[4];
                size_t uv[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const bool live = i0 + u < n;
                    const uint32_t rec = live ? s_rec[i0 + u] : 0u;
                    row[u] = rb * kUnitRows + (int)(rec & 31u);
                    k[u] = (int)(rec >> 5);
                    a[u] = live ? s_val[i0 + u] : 0.0f;
                    if (!live || row[u] >= M) row[u] = -1;
                    const size_t uidx = (size_t)ub * kblocks + k[u] / kUnitK;
                    uv[u] = uidx * kUnitVec;
                    mk[u] = 0u;
                    xv[u] = u32x4{0u, 0u, 0u, 0u};
                    c[u] = 0.0f;
                    if (row[u] >= 0) {
                        mk[u] = pb.mask[uidx];
                        xv[u] = Bw[uv[u] + (size_t)(((k[u] % kUnitK) / 8) * kUnitRows + cr)];
                        c[u] = C[(size_t)row[u] * ldc + col];
                    }
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if (row[u] < 0) continue;
#pragma unroll
                    for (int v = 0; v < u; ++v)
                        if (row[v] == row[u]) c[u] = c[v];           // the latest sum of that row (v ascending)
                    float x = half_of(xv[u], k[u] % 8);
                    if (mk[u] & 6u) x = unit_value(Bw, uv[u], pb, mk[u], (k[u] % kUnitK) / 8, cr, k[u] % 8);
                    c[u] = __fmaf_rn(a[u], ldexpf(x, -sb), c[u]);
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    bool last = row[u] >= 0;
#pragma unroll
                    for (int v = u + 1; v < 4; ++v) last = last && row[v] != row[u];
                    if (last) C[(size_t)row[u] * ldc + col] = c[u];
                }
            }
          }
        };
        if (cnt_a <= (uint32_t)kRecCap) {
            take_list(pa, (size_t)rb, (int)cnt_a);
            apply_a((int)cnt_a);
            __syncthreads();                                 // the records are free again
        } else {
            walk(Aw, pa, (size_t)rb, pa.S + rb * kUnitRows, 0u, false, apply_a);
        }
    }
    if (do_b) {
        // 2. the rows of this block, one per lane of the first half-wave: C[row][col0] += a0(row, k) * b
        const int row = rb * kUnitRows + (tid & 31);
        const int sa = pa.S[rb * kUnitRows + (tid & 31)];
        for (int u = 0; u < nub; ++u) {
            const int ub = ub0 + u;
            if (ub * kUnitRows >= N) break;                  // workgroup-uniform
            const uint32_t cnt_b = pb.rec_cnt[ub];
            if (cnt_b == 0u) continue;                       // workgroup-uniform
            auto apply_b = [&](int n) {
                if (tid >= 32 || row >= M) return;
                for (int i = 0; i < n; ++i) {
                    const uint32_t rec = s_rec[i];
                    const int col = ub * kUnitRows + (int)(rec & 31u), k = (int)(rec >> 5);
                    if (col >= N) continue;
                    const size_t at = ((size_t)rb * kblocks + k / kUnitK) * kUnitVec + (size_t)(((k % kUnitK) / 8) * kUnitRows + (tid & 31));
                    const float a = ldexpf(half_of(Aw[at], k % 8), -sa);      // plane 0 only
                    float *dst = C + (size_t)row * ldc + col;
                    *dst = __fmaf_rn(a, s_val[i], *dst);
                }
            };
            if (cnt_b <= (uint32_t)kRecCap) {
                take_list(pb, (size_t)ub, (int)cnt_b);
                apply_b((int)cnt_b);
                __syncthreads();
            } else {
                walk(Bw, pb, (size_t)ub, pb.S + ub * kUnitRows, 0u, false, apply_b);
            }
        }
    }
}

__global__ __launch_bounds__(256) void planes_tail_kernel(const u32x4 *__restrict__ Aw, const u32x4 *__restrict__ Bw, Planes pa,
                                                          Planes pb, float *__restrict__ C, int64_t ldc, int M, int N, int kblocks,
                                                          int col_chunks, int tail_cols)
{
    planes_tail_body(Aw, Bw, pa, pb, C, ldc, M, N, kblocks, col_chunks, tail_cols, blockIdx.x);
}

// The tails of a group of products in one launch: blocks [first, next first) belong to product g.
struct TailGroupItem {
    const u32x4 *Aw, *Bw;
    float *C;
    int64_t ldc;
    int M, N, kblocks, col_chunks;
    unsigned first;
    Planes pa, pb;
};
struct TailGroup {
    int count, tail_cols;
    unsigned first[kMaxGroup];
    TailGroupItem p[kMaxGroup];
};

__global__ __launch_bounds__(256) void planes_tail_group_kernel(TailGroup grp)
{
    const TailGroupItem &it = grp.p[group_member(grp.first, blockIdx.x)];  // the same in the whole workgroup
    planes_tail_body(it.Aw, it.Bw, it.pa, it.pb, it.C, it.ldc, it.M, it.N, it.kblocks, it.col_chunks, grp.tail_cols,
                     blockIdx.x - it.first);
}

// Columns per tail block for a launch whose blocks would number `blocks256` at 256 columns each: the widest
// of 1024, 512, 256 that still leaves four blocks per resident slot (three workgroups per compute unit).
static int tail_cols_for(uint64_t blocks256, int cus)
{
    if (const char *env = getenv("FMT_GEMM_TAIL_COLS")) {        // tuning override
        const int t = atoi(env);
        if (t == 256 || t == 512 || t == 1024) return t;
    }
    const uint64_t want = (uint64_t)cus * 12;
    return blocks256 / 4 >= want ? 1024 : blocks256 / 2 >= want ? 512 : 256;
}

// C[r][c] = sum over the k parts of part[s][r][c]  (parts are dense M x N slabs)
__global__ __launch_bounds__(256) void reduce_kernel(const float *__restrict__ part, int nsplit, float *__restrict__ C,
                                                     int M, int N, int64_t ldc, int img)
{
    const size_t total = (size_t)M * N;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        float s = 0.0f;
        for (int q = 0; q < nsplit; ++q) s += part[(size_t)q * total + i];
        const size_t row = i / N, col = i % N;
        if (img > 0)
            C[((col / img) * M + row) * img + col % img] = s;
        else
            C[row * ldc + col] = s;
    }
}

__global__ void zero_fill_kernel(float *__restrict__ C, int M, int N, int64_t ldc, int col_blocks)
{
    const int col = (blockIdx.x % col_blocks) * blockDim.x + threadIdx.x;
    const int row = blockIdx.x / col_blocks;
    if (col < N && row < M) C[(size_t)row * ldc + col] = 0.0f;
}

struct Plan {
    int tm, tn;      // wave tile in MFMA tiles; workgroup tile = 64*tm x 64*tn
    int nsplit;      // k parts
    int sched;       // 1: pin the issue order inside a trip (sched_group_barrier), 0: leave it to the compiler
};

static constexpr size_t lds_bytes(int tm, int tn, int pieces, int ks, int nst)
{
    return (size_t)nst * (2 * tm + 2 * tn) * pieces * 64 * ks * sizeof(u32x4);
}

// Pipeline shape per piece scheme and tile shape: k16 steps per stage, and as many stage buffers (at
// most FMT_GEMM_NST, at least two) as fit the tile's share of the 160 KiB of LDS -- all of it for the
// large tiles, half for 128 x 128 (two resident workgroups), a quarter for 64 x 64.
static constexpr int pipe_ks(int pieces) { return pieces == 1 ? FMT_GEMM_KS : FMT_GEMM_KS_MULTI; }
static constexpr int pipe_nst(int tm, int tn, int pieces, int ks)
{
    if ((tm * pieces * ks) % 2 || (tn * pieces * ks) % 2) return 2;   // stage not a whole number of loads per wave
    const size_t budget = (size_t)160 * 1024 / (tm * tn > 4 ? 1 : tm * tn == 4 ? 2 : 4);
    int n = FMT_GEMM_NST;
    while (n > 2 && lds_bytes(tm, tn, pieces, ks, n) > budget) --n;
    return n;
}
template <int PS, int TM, int TN> struct Pipe {
    static constexpr int ks = pipe_ks(pieces_of(PS)), nst = pipe_nst(TM, TN, pieces_of(PS), ks);
};

// Picks the workgroup tile and the number of k parts from a small cost model fitted to
// measurements on MI355X: large tiles move fewer LDS and L2 bytes per MFMA, small tiles need
// several resident workgroups per compute unit to reach their rate, the busiest compute unit sets
// the time, and cutting k fills the machine at the price of writing and re-reading partial sums.
static Plan make_plan(int M, int N, int kblocks, int cus, int pieces)
{
    // eff1 / effmax: relative MFMA rate of a compute unit with one / with max_occ resident workgroups
    struct Shape { int tm, tn, max_occ; double eff1, effmax; };
    static const Shape multi[] = {
        {4, 4, 1, 1.15, 1.15}, {4, 2, 1, 1.0, 1.0}, {2, 4, 1, 1.03, 1.03}, {2, 2, 2, 0.80, 0.95}, {1, 1, 4, 0.45, 0.78}};
    // one piece: a quarter of the MFMA work per byte, the small tiles lose less
    static const Shape single[] = {
        {4, 4, 1, 1.21, 1.21}, {4, 2, 1, 1.0, 1.0}, {2, 4, 1, 1.03, 1.03}, {2, 2, 2, 0.98, 1.11}, {1, 1, 4, 0.53, 0.68}};
    const Shape(&shapes)[5] = pieces == 1 ? single : multi;
    const double wg_cost = pieces == 1 ? 68.0 : 40.0, split_cost = pieces == 1 ? 5.76 : 2.5;
    if (const char *env = getenv("FMT_GEMM_PLAN")) {      // tuning override: "tm,tn,nsplit[,sched]"
        Plan forced{2, 2, 1, 1};
        if (sscanf(env, "%d,%d,%d,%d", &forced.tm, &forced.tn, &forced.nsplit, &forced.sched) >= 3) {
            for (const auto &sh : shapes)
                if (sh.tm == forced.tm && sh.tn == forced.tn && forced.nsplit >= 1 && forced.nsplit <= 64 &&
                    lds_bytes(sh.tm, sh.tn, pieces, pipe_ks(pieces), 2) <= 160 * 1024)
                    return forced;
        }
    }
    Plan best{2, 2, 1, 1};
    double best_t = 1e300;
    for (const auto &sh : shapes) {
        if (lds_bytes(sh.tm, sh.tn, pieces, pipe_ks(pieces), 2) > 160 * 1024) continue;
        const int bm = 64 * sh.tm, bn = 64 * sh.tn;
        const long tiles = (long)((M + bm - 1) / bm) * ((N + bn - 1) / bn);
        for (int ns = 1; ns <= 32; ns = ns < 4 ? ns + 1 : ns * 2) {
            if (ns > 1 && kblocks / ns < 8) break;
            const int kb_per = (kblocks + ns - 1) / ns;
            const long wgs = tiles * ns;
            const long per_cu = (wgs + cus - 1) / cus;                  // workgroups on the busiest compute unit
            const long resident = per_cu < sh.max_occ ? per_cu : sh.max_occ;
            const double eff = sh.max_occ > 1 ? sh.eff1 + (sh.effmax - sh.eff1) * (resident - 1) / (sh.max_occ - 1) : sh.eff1;
            // MFMA time on that compute unit (arbitrary units) + start-up / epilogue cost per workgroup
            double t = per_cu * ((double)bm * bn * kb_per / eff + wg_cost * bm * bn / 128.0);
            if (ns > 1) t += split_cost * (double)M * N * (ns + 1) / cus * 8.0;   // partial sums out and back
            if (t < best_t) { best_t = t; best = Plan{sh.tm, sh.tn, ns, 1}; }
        }
    }
    return best;
}

template <int PS, int TM, int TN, bool SPLIT, bool SCHED, bool SCALED, bool GATHER = false>
static int launch_product_v2(const u32x4 *Aw, const u32x4 *Bw, float *out, int M, int N, int64_t ld, int img, int kblocks,
                            int nsplit, hipStream_t stream, const Planes &pa, const Planes &pb, const Implicit &im = Implicit{})
{
    constexpr int KS = Pipe<PS, TM, TN>::ks, NST = Pipe<PS, TM, TN>::nst;
    if constexpr (lds_bytes(TM, TN, pieces_of(PS), KS, NST) > 160 * 1024) {
        return FMT_ERR_SHAPE;                            // never planned (make_plan skips such tiles)
    } else {
        const int tiles_m = (M + 64 * TM - 1) / (64 * TM), tiles_n = (N + 64 * TN - 1) / (64 * TN);
        const int64_t per_xcd = ((int64_t)tiles_m * tiles_n + 7) / 8;
        if (per_xcd * 8 * nsplit >= ((int64_t)1 << 31)) return FMT_ERR_SHAPE;
        const int kb_per = (kblocks + nsplit - 1) / nsplit;
        auto kern = product_kernel<PS, TM, TN, KS, NST, SPLIT, SCHED, SCALED, GATHER>;
        Implicit imk = im;
        if (GATHER) imk.kc = make_fastdiv(im.c8 * 8 / (16 * KS));   // stages of 16*KS k per tap
        hipLaunchKernelGGL(kern, dim3((unsigned)(per_xcd * 8 * nsplit)), dim3(256), 0, stream, Aw, Bw, out, M, N, ld, img,
                           kblocks, tiles_m, tiles_n, kb_per, pa, pb, imk);
        FMT_HIP_CHECK(hipGetLastError());
        return FMT_OK;
    }
}

template <int PS, int TM, int TN, bool SPLIT, bool SCHED>
static int launch_product_v(const u32x4 *Aw, const u32x4 *Bw, float *out, int M, int N, int64_t ld, int img, int kblocks,
                            int nsplit, hipStream_t stream, const Planes &pa, const Planes &pb)
{
    if constexpr (PS == 0) {
        if (pa.S != nullptr)
            return launch_product_v2<PS, TM, TN, SPLIT, SCHED, true>(Aw, Bw, out, M, N, ld, img, kblocks, nsplit, stream, pa, pb);
    }
    return launch_product_v2<PS, TM, TN, SPLIT, SCHED, false>(Aw, Bw, out, M, N, ld, img, kblocks, nsplit, stream, pa, pb);
}

template <int PS, int TM, int TN>
static int launch_product(const u32x4 *Aw, const u32x4 *Bw, float *C, int M, int N, int64_t ldc, int img, int kblocks,
                          const Plan &plan, float *part, hipStream_t stream, const Planes &pa, const Planes &pb,
                          const Implicit *im = nullptr)
{
    if (im != nullptr) {
        // operand B gathered inside the product kernel (convolutions); no planes, pinned issue order only
        if (plan.nsplit == 1)
            return launch_product_v2<PS, TM, TN, false, true, false, true>(Aw, nullptr, C, M, N, ldc, img, kblocks, 1, stream, pa,
                                                                          pb, *im);
        int rcg = launch_product_v2<PS, TM, TN, true, true, false, true>(Aw, nullptr, part, M, N, (int64_t)N, 0, kblocks,
                                                                        plan.nsplit, stream, pa, pb, *im);
        if (rcg != FMT_OK) return rcg;
        const size_t total_g = (size_t)M * N;
        const unsigned rgrid_g = (unsigned)((total_g + 1023) / 1024 < 4096 ? (total_g + 1023) / 1024 : 4096);
        hipLaunchKernelGGL(reduce_kernel, dim3(rgrid_g ? rgrid_g : 1), dim3(256), 0, stream, part, plan.nsplit, C, M, N, ldc, img);
        FMT_HIP_CHECK(hipGetLastError());
        return FMT_OK;
    }
    // the elements outside plane 0 of exponent-plane operands follow the product (plain row-major results only)
    auto tail = [&]() -> int {
        if (PS != 0 || pa.S == nullptr) return FMT_OK;
        if (img != 0) return FMT_ERR_SHAPE;
        int cus = 0;
        const int rcc = device_cu_count(&cus);
        if (rcc != FMT_OK) return rcc;
        const int64_t rbs = (M + kUnitRows - 1) / kUnitRows;
        const int tc = tail_cols_for((uint64_t)rbs * ((N + 255) / 256), cus);
        const int64_t col_chunks = (N + tc - 1) / tc, blocks = rbs * col_chunks;
        if (blocks >= ((int64_t)1 << 31)) return FMT_ERR_SHAPE;
        hipLaunchKernelGGL(planes_tail_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, Aw, Bw, pa, pb, C, ldc, M, N, kblocks,
                           (int)col_chunks, tc);
        FMT_HIP_CHECK(hipGetLastError());
        return FMT_OK;
    };
    if (plan.nsplit == 1) {
        int rc1 = plan.sched ? launch_product_v<PS, TM, TN, false, true>(Aw, Bw, C, M, N, ldc, img, kblocks, 1, stream, pa, pb)
                             : launch_product_v<PS, TM, TN, false, false>(Aw, Bw, C, M, N, ldc, img, kblocks, 1, stream, pa, pb);
        return rc1 != FMT_OK ? rc1 : tail();
    }
    int rc = plan.sched
                 ? launch_product_v<PS, TM, TN, true, true>(Aw, Bw, part, M, N, (int64_t)N, 0, kblocks, plan.nsplit, stream, pa, pb)
                 : launch_product_v<PS, TM, TN, true, false>(Aw, Bw, part, M, N, (int64_t)N, 0, kblocks, plan.nsplit, stream, pa, pb);
    if (rc != FMT_OK) return rc;
    const size_t total = (size_t)M * N;
    const unsigned rgrid = (unsigned)((total + 1023) / 1024 < 4096 ? (total + 1023) / 1024 : 4096);
    hipLaunchKernelGGL(reduce_kernel, dim3(rgrid ? rgrid : 1), dim3(256), 0, stream, part, plan.nsplit, C, M, N, ldc, img);
    FMT_HIP_CHECK(hipGetLastError());
    return tail();
}

// One operand of a product as the caller describes it: a plain matrix (kind kSrcMatrix, leading
// dimension ld) or a gathered view of a convolution tensor.
struct OperandSpec {
    const float *X;
    int64_t ld;
    bool kcontig;
    Gather g;
    int64_t pre_elems;   // > 0: round and split the tensor (that many elements) once before gathering from it
};

// Where the M x N result goes: plain row-major with leading dimension ldc, or (img > 0) NCHW with
// columns = (image, position) and `img` positions per image.
struct OutSpec {
    float *C;
    int64_t ldc;
    int img;
};

// How a format's values reach the matrix cores: ps = piece scheme (0: one fp16 piece, 1-3: that many
// bf16 pieces); scaled: ps == 0 with per-row scales and exponent planes (1/6/8 and 1/6/9).
struct Scheme {
    int ps;
    bool scaled;
};

// 0: never scaled planes, 1: whenever the format allows, 2: by size.  Environment override for tests and tuning.
static int window_mode()
{
    if (const char *env = getenv("FMT_GEMM_WINDOW")) return env[0] == '0' ? 0 : (env[0] == '1' ? 1 : 2);
    return 2;
}

static bool planes_possible(fmt_format_t f) { return f.e == 6 && f.m >= 8 && f.m <= 9; }

static Scheme scheme_of(fmt_format_t f, bool want_planes)
{
    if (want_planes && planes_possible(f)) return Scheme{0, true};
    // one fp16 piece for formats inside binary16, else 1-3 bf16 pieces by significand width
    return Scheme{f.m <= 7 ? 1 : (f.e <= 5 && f.m <= 10 ? 0 : (f.m <= 15 ? 2 : 3)), false};
}

// Memory layout of one prepared operand (`rows` x K after op(), padded to kRowPad rows and 32 k):
//   [pieces]  units x kblocks x P units of 128 vectors; with planes: three planes of units x kblocks units
//   [S]       with planes: one int per padded row
//   [mask]    with planes: one byte per unit
// every part 256-byte aligned.
struct OperandLayout {
    Scheme sch;
    int w;                       // planes: binades per plane
    int rows, kblocks, units;
    size_t plane_vec, s_off, mask_off, cnt_off, rec_off, bytes;
};

static int operand_layout(int64_t rows, int64_t K, Scheme sch, int m, OperandLayout *L)
{
    auto up256 = [](size_t b) { return (b + 255) / 256 * 256; };
    L->sch = sch;
    L->w = 40 - m;
    L->rows = (int)rows;
    L->kblocks = (int)((K + kUnitK - 1) / kUnitK);
    L->units = (int)((rows + kRowPad - 1) / kRowPad * (kRowPad / kUnitRows));
    if ((int64_t)L->kblocks * L->units >= ((int64_t)1 << 30)) return FMT_ERR_SHAPE;
    const int P = pieces_of(sch.ps);
    L->plane_vec = (size_t)L->units * L->kblocks * P * kUnitVec;
    const size_t piece_bytes = up256(L->plane_vec * sizeof(u32x4) * (sch.scaled ? 3 : 1));
    L->s_off = piece_bytes;
    L->mask_off = L->s_off + (sch.scaled ? up256((size_t)L->units * kUnitRows * sizeof(int)) : 0);
    L->cnt_off = L->mask_off + (sch.scaled ? up256((size_t)L->units * L->kblocks) : 0);
    L->rec_off = L->cnt_off + (sch.scaled ? up256((size_t)L->units * sizeof(uint32_t)) : 0);
    L->bytes = L->rec_off + (sch.scaled ? up256((size_t)L->units * kRecCap * 2 * sizeof(uint32_t)) : 0);
    return FMT_OK;
}

// A prepared operand in memory at `base`.
struct OperandView {
    u32x4 *W;
    Planes pl;
};

static OperandView view_of(void *base, const OperandLayout &L)
{
    char *b = static_cast<char *>(base);
    OperandView v;
    v.W = reinterpret_cast<u32x4 *>(b);
    v.pl = Planes{nullptr, nullptr, 0, L.w, nullptr, nullptr};
    if (L.sch.scaled) {
        v.pl.S = reinterpret_cast<int *>(b + L.s_off);
        v.pl.mask = reinterpret_cast<uint8_t *>(b + L.mask_off);
        v.pl.plane = L.plane_vec;
        v.pl.rec_cnt = reinterpret_cast<uint32_t *>(b + L.cnt_off);
        v.pl.recs = reinterpret_cast<uint32_t *>(b + L.rec_off);
    }
    return v;
}

// ---- exponent planes: the scale of every row -------------------------------------------------

struct StatOperand {
    const uint32_t *X;
    int64_t ld;
    int rows;
    int rows_pad;
    int kcontig;
    int vec4;                // base 16-byte aligned and ld a multiple of 4: a k-contiguous row is read in 16-byte pieces
    int *S;
    uint32_t *rec_cnt;       // record counts of the operand's rows of units: cleared here, filled by the prepare pass
    unsigned nblocks;
};

// Picks each row's scale S = 15 - T, T the top binade of plane 0, from the binades of a sample of its
// elements (every kstep-th slab of k).  Plane 0 with top T holds the normal values of binades
// [T - wid, T] exactly, and the format's denormal values (multiples of 2^(Emin-m)) exactly iff
// T <= 9 - m.  With hi the largest binade seen (+1: rounding may carry) and lo the smallest binade of
// a value that is normal in the format, every T in [hi + 1, lo + wid] keeps all elements seen in plane 0:
//   - a denormal value was seen: T = 9 - m, the highest choice that keeps the denormals (gradient
//     tensors live here);
//   - otherwise up to three binades above hi + 1 (not beyond the middle of [hi + 1, lo + wid]),
//     which leaves room on both sides for the elements the sample did not see; if the row spans
//     more than a plane, T = lo + wid (the small values stay, the large ones go to the plane above).
// Any T in [kWinTmin, kWinTmax] is correct -- what does not fit plane 0 goes to another plane -- the
// choice only decides how often the other planes are needed, which is why a sample suffices.
__device__ __forceinline__ void window_stats_block(const StatOperand &o, int K, int kstep, int emin, int m, int by)
{
    __shared__ int s_hi[8][32], s_lo[8][32];
    const int tid = threadIdx.x;
    const int wid = 39 - m;                       // binades below the top one that a plane holds with m + 1 significant bits
    int hi = -1000, lo = 1000;
    auto look = [&](uint32_t u) {
        const uint32_t ab = u & 0x7FFFFFFFu;
        const int E = (int)(ab >> 23) - 127;
        if (ab < 0x7F800000u && E >= emin - m - 1) {
            hi = max(hi, E);
            lo = min(lo, max(E, emin - 1));           // emin - 1: a value in the format's denormal range
        }
    };
    // 32 rows per workgroup, 8 lanes per row; eight loads are issued before any is looked at
    const int row = by * 32 + (o.kcontig ? tid / 8 : tid % 32);
    const int kl = o.kcontig ? tid % 8 : tid / 32;
    if (row < o.rows) {
        // at most four slabs are visited (kstep = ceil(slabs / 4)); all their loads are issued first
        uint32_t u[4][8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int k0 = min(kl * 8 + i * 64 * kstep, K - 1);
            if (o.kcontig && o.vec4 && k0 + 8 <= K) {      // k0 is a multiple of 8 here
                const u32x4 *src = reinterpret_cast<const u32x4 *>(o.X + (size_t)row * o.ld + k0);
                const u32x4 a = src[0], b = src[1];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    u[i][j] = a[j];
                    u[i][4 + j] = b[j];
                }
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int k = min(k0 + j, K - 1);      // a repeated element does not change max / min
                    u[i][j] = o.kcontig ? o.X[(size_t)row * o.ld + k] : o.X[(size_t)k * o.ld + row];
                }
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j) look(u[i][j]);
    }
    if (o.kcontig) {
#pragma unroll
        for (int off = 1; off < 8; off <<= 1) {
            hi = max(hi, __shfl_xor(hi, off, 64));
            lo = min(lo, __shfl_xor(lo, off, 64));
        }
        if (kl != 0) return;
    } else {
        s_hi[kl][tid % 32] = hi;
        s_lo[kl][tid % 32] = lo;
        __syncthreads();
        if (kl != 0) return;
#pragma unroll
        for (int q = 1; q < 8; ++q) {
            hi = max(hi, s_hi[q][tid]);
            lo = min(lo, s_lo[q][tid]);
        }
    }
    if (row >= o.rows_pad) return;
    int T = 0;
    if (hi != -1000) {
        const int top = hi + 1, room = lo + wid;
        T = lo < emin ? 9 - m : (top >= room ? room : top + min(3, (room - top) / 2));
    }
    T = max(kWinTmin, min(kWinTmax, T));
    o.S[row] = 15 - T;
    if (row % kUnitRows == 0) o.rec_cnt[row / kUnitRows] = 0u;
}

__global__ __launch_bounds__(256) void window_stats_kernel(StatOperand a, StatOperand b, int Ka, int kstep_a, int Kb,
                                                           int kstep_b, int emin, int m)
{
    const bool second = blockIdx.x >= a.nblocks;
    window_stats_block(second ? b : a, second ? Kb : Ka, second ? kstep_b : kstep_a, emin, m,
                       (int)(blockIdx.x - (second ? a.nblocks : 0u)));
}

// The same for the operands of a prepare group (see prepare_scaled_group_kernel): run i starts at first[i].
struct StatGroup {
    unsigned first[kMaxPrepGroup];   // 0xFFFFFFFF beyond the last operand
    StatOperand o[kMaxPrepGroup];
    int K[kMaxPrepGroup], kstep[kMaxPrepGroup];
};

__global__ __launch_bounds__(256) void window_stats_group_kernel(StatGroup grp, int emin, int m)
{
    const int at = run_of(grp.first, blockIdx.x);
    window_stats_block(grp.o[at], grp.K[at], grp.kstep[at], emin, m, (int)(blockIdx.x - grp.first[at]));
}

// ---- operand preparation ------------------------------------------------------------------------

// Launches what turns the described operands into prepared ones: the pre-rounding of a tensor that is
// gathered from, the row scales of exponent planes, and the prepare kernel.  sb == nullptr: one operand.
// pre_a / pre_b: room for the pre-rounded tensors (only for specs with pre_elems > 0).
template <int MODE, bool FTZ, int PS>
static int prepare_operands(const OperandSpec &sa, const OperandLayout &la, const OperandView &va, uint32_t *pre_a,
                            const OperandSpec *sb, const OperandLayout *lb, const OperandView *vb, uint32_t *pre_b, int K,
                            fmt_format_t f, const QuantParams &p, hipStream_t stream)
{
    const int kblocks = la.kblocks;
    const bool scaled = la.sch.scaled;
    auto operand = [&](const OperandSpec &sp, const OperandLayout &L, const OperandView &v, uint32_t *pre_buf) {
        PrepOperand o;
        o.X = reinterpret_cast<const uint32_t *>(sp.X);
        o.g = sp.g;
        if (sp.pre_elems > 0) {
            const int n = (int)sp.pre_elems;
            const int grid = (n + 1023) / 1024 < 4096 ? (n + 1023) / 1024 : 4096;
            hipLaunchKernelGGL((round_split_kernel<MODE, FTZ, PS>), dim3(grid), dim3(256), 0, stream, o.X, pre_buf, n, p);
            o.X = pre_buf;
            o.g.pre = 1;
            o.g.plane = n + 1;
            const bool simple = o.g.den_y == 1 && o.g.den_x == 1 && o.g.R * o.g.S <= 32;
            o.g.fast = simple && o.g.kind == kSrcPatchRows && !sp.kcontig ? 1
                       : simple && o.g.kind == kSrcPatchK && sp.kcontig && o.g.tap > 0 ? 2 : 0;
        }
        o.W = v.W;
        o.ld = sp.ld;
        o.rows = L.rows;
        o.kcontig = sp.kcontig;
        o.vec4 = (reinterpret_cast<uintptr_t>(sp.X) & 15) == 0 && sp.ld % 4 == 0;
        o.nblocks = o.g.fast == 2 ? (unsigned)((kblocks + 7) / 8) * L.units            // 32 taps x 256 positions each
                    : sp.kcontig ? (unsigned)((kblocks + 1) / 2) * L.units
                                 : (unsigned)kblocks * (L.units / (o.g.fast ? 2 * kFastRows : 2));
        o.pl = v.pl;
        return o;
    };
    const PrepOperand oa = operand(sa, la, va, pre_a);
    PrepOperand ob = oa;
    ob.nblocks = 0u;
    if (sb != nullptr) ob = operand(*sb, *lb, *vb, pre_b);
    FMT_HIP_CHECK(hipGetLastError());
    const unsigned prep_grid = (oa.nblocks + 7u) / 8u * 8u + (ob.nblocks + 7u) / 8u * 8u;
    if (scaled) {
        if constexpr (PS == 0 && MODE == kModeMagic) {
            auto stat = [&](const PrepOperand &o, const OperandLayout &L, bool present) {
                StatOperand t;
                t.X = o.X;
                t.ld = o.ld;
                t.rows = L.rows;
                t.rows_pad = L.units * kUnitRows;
                t.kcontig = o.kcontig;
                t.vec4 = o.vec4;
                t.S = o.pl.S;
                t.rec_cnt = o.pl.rec_cnt;
                t.nblocks = present ? (unsigned)L.units : 0u;
                return t;
            };
            const StatOperand ta = stat(oa, la, true), tb = stat(ob, sb ? *lb : la, sb != nullptr);
            // a sample of at most 4 slabs of 64 k per row (256 elements): the scale only has to be a good guess
            const int slabs = (K + 63) / 64;
            const int bias = (1 << (f.e - 1)) - 1;
            hipLaunchKernelGGL(window_stats_kernel, dim3(ta.nblocks + tb.nblocks), dim3(256), 0, stream, ta, tb, K,
                               (slabs + 3) / 4, K, (slabs + 3) / 4, 1 - bias, f.m);
            FMT_HIP_CHECK(hipGetLastError());
            hipLaunchKernelGGL((prepare_scaled_kernel<MODE, FTZ>), dim3(prep_grid), dim3(256), 0, stream, oa, ob, K, kblocks, K,
                               kblocks, p);
        } else {
            return FMT_ERR_FORMAT;               // planes exist for e == 6 formats only (rounding mode kModeMagic)
        }
    } else if (oa.g.fast == 2 || ob.g.fast == 2) {
        hipLaunchKernelGGL((prepare_kernel<MODE, FTZ, PS, true>), dim3(prep_grid), dim3(256), 0, stream, oa, ob, K, kblocks, p);
    } else {
        hipLaunchKernelGGL((prepare_kernel<MODE, FTZ, PS, false>), dim3(prep_grid), dim3(256), 0, stream, oa, ob, K, kblocks, p);
    }
    FMT_HIP_CHECK(hipGetLastError());
    return FMT_OK;
}

// Room for the split-k partial sums of a plan.
static size_t part_bytes_of(const Plan &plan, int M, int N)
{
    return plan.nsplit > 1 ? ((size_t)plan.nsplit * M * N * sizeof(float) + 255) / 256 * 256 : 0;
}

template <int PS>
static int product_of_views(const OperandView &va, const OperandView &vb, int M, int N, int kblocks, const OutSpec &out,
                            const Plan &plan, float *part, hipStream_t stream)
{
#define FMT_PRODUCT(TMV, TNV) \
    launch_product<PS, TMV, TNV>(va.W, vb.W, out.C, M, N, out.ldc, out.img, kblocks, plan, part, stream, va.pl, vb.pl)
    if (plan.tm == 4 && plan.tn == 4) return FMT_PRODUCT(4, 4);
    if (plan.tm == 4 && plan.tn == 2) return FMT_PRODUCT(4, 2);
    if (plan.tm == 2 && plan.tn == 4) return FMT_PRODUCT(2, 4);
    if (plan.tm == 2 && plan.tn == 2) return FMT_PRODUCT(2, 2);
    return FMT_PRODUCT(1, 1);
#undef FMT_PRODUCT
}

static int product_dispatch(int ps, const OperandView &va, const OperandView &vb, int M, int N, int kblocks,
                            const OutSpec &out, const Plan &plan, float *part, hipStream_t stream)
{
    switch (ps) {
        case 0: return product_of_views<0>(va, vb, M, N, kblocks, out, plan, part, stream);
        case 1: return product_of_views<1>(va, vb, M, N, kblocks, out, plan, part, stream);
        case 2: return product_of_views<2>(va, vb, M, N, kblocks, out, plan, part, stream);
        default: return product_of_views<3>(va, vb, M, N, kblocks, out, plan, part, stream);
    }
}

// Prepare + product (+ reduction) of described operands in library scratch.
template <int MODE, bool FTZ, int PS>
static int run(int M, int N, int K, const OperandSpec &sa, const OperandSpec &sb, const OutSpec &out, fmt_format_t f,
               const QuantParams &p, hipStream_t stream, bool scaled)
{
    const Scheme sch{PS, scaled};
    OperandLayout la, lb;
    int rc = operand_layout(M, K, sch, f.m, &la);
    if (rc != FMT_OK) return rc;
    rc = operand_layout(N, K, sch, f.m, &lb);
    if (rc != FMT_OK) return rc;
    int cus = 0;
    rc = device_cu_count(&cus);
    if (rc != FMT_OK) return rc;
    const Plan plan = make_plan(M, N, la.kblocks, cus, pieces_of(PS));
    auto up256 = [](size_t b) { return (b + 255) / 256 * 256; };
    const int words = (pieces_of(PS) + 1) / 2;
    const size_t pre_a = sa.pre_elems ? up256((size_t)(sa.pre_elems + 1) * words * sizeof(uint32_t)) : 0;
    const size_t pre_b = sb.pre_elems ? up256((size_t)(sb.pre_elems + 1) * words * sizeof(uint32_t)) : 0;
    const size_t part = part_bytes_of(plan, M, N);
    Scratch s;
    rc = get_scratch(stream, 0, la.bytes + lb.bytes + part + pre_a + pre_b, &s);
    if (rc != FMT_OK) return rc;
    char *ws = static_cast<char *>(s.gemm_ws);
    const OperandView va = view_of(ws, la), vb = view_of(ws + la.bytes, lb);
    float *partp = reinterpret_cast<float *>(ws + la.bytes + lb.bytes);
    uint32_t *pa = reinterpret_cast<uint32_t *>(ws + la.bytes + lb.bytes + part);
    uint32_t *pb = reinterpret_cast<uint32_t *>(ws + la.bytes + lb.bytes + part + pre_a);
    rc = prepare_operands<MODE, FTZ, PS>(sa, la, va, pa, &sb, &lb, &vb, pb, K, f, p, stream);
    if (rc != FMT_OK) return rc;
    return product_of_views<PS>(va, vb, M, N, la.kblocks, out, plan, partp, stream);
}

template <int MODE, bool FTZ>
static int run_p(Scheme sch, int M, int N, int K, const OperandSpec &sa, const OperandSpec &sb, const OutSpec &out,
                 fmt_format_t f, const QuantParams &p, hipStream_t stream)
{
    switch (sch.ps) {
        case 0: return run<MODE, FTZ, 0>(M, N, K, sa, sb, out, f, p, stream, sch.scaled);
        case 1: return run<MODE, FTZ, 1>(M, N, K, sa, sb, out, f, p, stream, false);
        case 2: return run<MODE, FTZ, 2>(M, N, K, sa, sb, out, f, p, stream, false);
        default: return run<MODE, FTZ, 3>(M, N, K, sa, sb, out, f, p, stream, false);
    }
}

// Product of two described operands (K > 0): picks the piece scheme and the rounding variant.
static int run_product(int M, int N, int K, const OperandSpec &sa, const OperandSpec &sb, const OutSpec &out,
                       fmt_format_t f, const QuantParams &p, hipStream_t stream)
{
    const bool ftz = f.denorm == 0;
    // 1/6/9 and 1/6/8: exponent planes (a quarter of the MFMA work of two bf16 pieces) for plain matrix
    // operands, when the product is large enough to pay for the launch that picks the row scales
    const int wmode = window_mode();
    const bool planes = sa.g.kind == kSrcMatrix && sb.g.kind == kSrcMatrix && out.img == 0 &&
                        K < (1 << 27) && (wmode == 1 || (wmode == 2 && 2.0 * M * N * K >= 1e9 && K >= 128));
    const Scheme sch = scheme_of(f, planes);
#define FMT_RUN(MD)                                                                     \
    (ftz ? run_p<MD, true>(sch, M, N, K, sa, sb, out, f, p, stream)                      \
         : run_p<MD, false>(sch, M, N, K, sa, sb, out, f, p, stream))
    if (p.mode == kModeMagic) return FMT_RUN(kModeMagic);
    if (p.mode == kModeInteger) return FMT_RUN(kModeInteger);
    return FMT_RUN(kModeMixed);
#undef FMT_RUN
}

// ---- prepared operands in caller-owned memory ---------------------------------------------------

// (the tail's element records hold k in 27 bits: longer sums take the bf16 pieces)
static Scheme api_scheme(fmt_format_t f, int64_t K) { return scheme_of(f, window_mode() != 0 && K < ((int64_t)1 << 27)); }

int prepared_operand_bytes(int64_t rows, int64_t K, fmt_format_t f, size_t *bytes, int *scheme)
{
    OperandLayout L;
    const Scheme sch = api_scheme(f, K);
    int rc = operand_layout(rows, K, sch, f.m, &L);
    if (rc != FMT_OK) return rc;
    *bytes = L.bytes;
    *scheme = sch.ps + (sch.scaled ? 16 : 0);
    return FMT_OK;
}

template <int MODE, bool FTZ>
static int prepare_one_p(Scheme sch, const OperandSpec &sp, const OperandLayout &L, const OperandView &v, int K,
                         fmt_format_t f, const QuantParams &p, hipStream_t stream)
{
    switch (sch.ps) {
        case 0: return prepare_operands<MODE, FTZ, 0>(sp, L, v, nullptr, nullptr, nullptr, nullptr, nullptr, K, f, p, stream);
        case 1: return prepare_operands<MODE, FTZ, 1>(sp, L, v, nullptr, nullptr, nullptr, nullptr, nullptr, K, f, p, stream);
        case 2: return prepare_operands<MODE, FTZ, 2>(sp, L, v, nullptr, nullptr, nullptr, nullptr, nullptr, K, f, p, stream);
        default: return prepare_operands<MODE, FTZ, 3>(sp, L, v, nullptr, nullptr, nullptr, nullptr, nullptr, K, f, p, stream);
    }
}

// X is `rows` x K after op(): trans == 0: X[r*ld + k], trans != 0: X[k*ld + r].  rows, K > 0.
int launch_prepare_operand(const float *X, int64_t ld, int trans, int64_t rows, int64_t K, fmt_format_t f,
                           const QuantParams &p, void *buf, hipStream_t stream)
{
    const Scheme sch = api_scheme(f, K);
    OperandLayout L;
    int rc = operand_layout(rows, K, sch, f.m, &L);
    if (rc != FMT_OK) return rc;
    const OperandView v = view_of(buf, L);
    const OperandSpec sp{X, ld, trans == 0, Gather{}, 0};
    const bool ftz = f.denorm == 0;
#define FMT_PREP(MD)                                                                \
    (ftz ? prepare_one_p<MD, true>(sch, sp, L, v, (int)K, f, p, stream)              \
         : prepare_one_p<MD, false>(sch, sp, L, v, (int)K, f, p, stream))
    if (p.mode == kModeMagic) return FMT_PREP(kModeMagic);
    if (p.mode == kModeInteger) return FMT_PREP(kModeInteger);
    return FMT_PREP(kModeMixed);
#undef FMT_PREP
}

// Both orientations of several matrices (buf0 = X as stored, buf1 = X transposed) with shared launches:
// matrices whose two operands take exponent planes are gathered, up to kMaxPrepGroup / 2 at a time, into one
// statistics launch and one prepare launch; the others are prepared operand by operand.  The operands equal
// those of two launch_prepare_operand calls (the same block functions on the same blocks; only the order of
// the records within a list may differ, which the product's tail sorts away).
// round != nullptr: the same launch also writes every matrix rounded to fp32 (round[i].Y) and counts its elements
// into round[i].hist, as fmt_quantize does (window from p.exp_lo); planes formats only (FMT_ERR_FORMAT otherwise).
static_assert(sizeof(PrepGroup) + sizeof(RoundGroup) + sizeof(QuantParams) <= 4096 && sizeof(StatGroup) + 8 <= 4096,
              "group tables travel in the kernel arguments");

int launch_prepare_pair_batch(int64_t count, const PrepPairItem *items, fmt_format_t f, const QuantParams &p, hipStream_t stream,
                              const RoundItem *round)
{
    StatGroup sg;
    PrepGroup pg;
    RoundGroup rg{};
    FinalizeGroup fg{};
    unsigned long long *records = nullptr;
    if (round != nullptr) {
        for (int64_t i = 0; i < count; ++i)
            if (!(api_scheme(f, items[i].cols).scaled && api_scheme(f, items[i].rows).scaled && p.mode == kModeMagic))
                return FMT_ERR_FORMAT;
        Scratch sc;
        const int rc = get_scratch(stream, (size_t)(kMaxPrepGroup / 2) * kHistScratchBytes, 0, &sc);
        if (rc != FMT_OK) return rc;
        records = static_cast<unsigned long long *>(sc.hist_partials);
        // steps per workgroup: as many as leave every compute unit four workgroups (measured on 12 tensors of 4 M to 16 M
        // elements: one step 267 us, four 242 us, eight 258 us; one tensor of 4 M elements: four 36 us)
        int cus = 0;
        const int rc2 = device_cu_count(&cus);
        if (rc2 != FMT_OK) return rc2;
        uint64_t all_tiles = 0;
        for (int64_t i = 0; i < count; ++i)
            all_tiles += (uint64_t)((items[i].rows + 31) / 32) * (uint64_t)((items[i].cols + 64 * kPairTiles - 1) / (64 * kPairTiles));
        rg.steps = kRoundSteps;
        while (rg.steps > 1 && all_tiles / (uint64_t)rg.steps < (uint64_t)cus * 4) rg.steps /= 2;
    }
    int n = 0;
    unsigned stat_ids = 0, prep_ids = 0;
    const int bias = (1 << (f.e - 1)) - 1;
    auto flush = [&]() -> int {
        if (n == 0) return FMT_OK;
        for (int i = n; i < kMaxPrepGroup; ++i) {
            sg.first[i] = 0xFFFFFFFFu;
            sg.o[i] = StatOperand{};
            sg.K[i] = sg.kstep[i] = 0;
            pg.o[i] = PrepPlain{};
        }
        for (int i = n / 2; i < kMaxPrepGroup / 2; ++i) {
            pg.first[i] = 0xFFFFFFFFu;
            pg.tiles[i] = 0u;
        }
        hipLaunchKernelGGL(window_stats_group_kernel, dim3(stat_ids), dim3(256), 0, stream, sg, 1 - bias, f.m);
        FMT_HIP_CHECK(hipGetLastError());
#define FMT_PAIR_LAUNCH(FTZV, ROUNDV, DEEPV)                                                                           \
    hipLaunchKernelGGL((prepare_scaled_group_kernel<kModeMagic, FTZV, ROUNDV, DEEPV>), dim3(prep_ids), dim3(256), 0, stream, pg, \
                       rg, p)
        const bool ftz = f.denorm == 0, deep = p.exp_lo < -126;
        if (round == nullptr) {
            if (ftz) FMT_PAIR_LAUNCH(true, false, false); else FMT_PAIR_LAUNCH(false, false, false);
        } else if (deep) {
            if (ftz) FMT_PAIR_LAUNCH(true, true, true); else FMT_PAIR_LAUNCH(false, true, true);
        } else {
            if (ftz) FMT_PAIR_LAUNCH(true, true, false); else FMT_PAIR_LAUNCH(false, true, false);
        }
#undef FMT_PAIR_LAUNCH
        FMT_HIP_CHECK(hipGetLastError());
        if (round != nullptr) {
            const int rc = launch_hist_finalize_group(fg, n / 2, stream);     // sums and clears the records
            if (rc != FMT_OK) return rc;
        }
        n = 0;
        stat_ids = prep_ids = 0;
        return FMT_OK;
    };
    auto add = [&](const PrepPairItem &it, bool kcontig, const OperandLayout &L, const OperandView &v, int K) {
        PrepPlain &o = pg.o[n];
        o.X = reinterpret_cast<const uint32_t *>(it.X);
        o.W = v.W;
        o.ld = it.ld;
        o.rows = L.rows;
        o.kcontig = kcontig;
        o.vec4 = (reinterpret_cast<uintptr_t>(it.X) & 15) == 0 && it.ld % 4 == 0;
        o.units = L.units;
        o.K = K;
        o.kblocks = L.kblocks;
        o.pl = v.pl;
        StatOperand &t = sg.o[n];
        t.X = o.X;
        t.ld = o.ld;
        t.rows = L.rows;
        t.rows_pad = L.units * kUnitRows;
        t.kcontig = kcontig;
        t.vec4 = o.vec4;
        t.S = v.pl.S;
        t.rec_cnt = v.pl.rec_cnt;
        t.nblocks = (unsigned)L.units;
        sg.K[n] = K;
        sg.kstep[n] = ((K + 63) / 64 + 3) / 4;
        sg.first[n] = stat_ids;
        stat_ids += t.nblocks;
        ++n;
    };
    for (int64_t i = 0; i < count; ++i) {
        const PrepPairItem &it = items[i];
        const Scheme s0 = api_scheme(f, it.cols), s1 = api_scheme(f, it.rows);
        if (!(s0.scaled && s1.scaled && p.mode == kModeMagic)) {
            int rc = launch_prepare_operand(it.X, it.ld, 0, it.rows, it.cols, f, p, it.buf0, stream);
            if (rc == FMT_OK) rc = launch_prepare_operand(it.X, it.ld, 1, it.cols, it.rows, f, p, it.buf1, stream);
            if (rc != FMT_OK) return rc;
            continue;
        }
        OperandLayout L0, L1;
        int rc = operand_layout(it.rows, it.cols, s0, f.m, &L0);
        if (rc != FMT_OK) return rc;
        rc = operand_layout(it.cols, it.rows, s1, f.m, &L1);
        if (rc != FMT_OK) return rc;
        if (n + 2 > kMaxPrepGroup || prep_ids > 0x40000000u) {
            rc = flush();
            if (rc != FMT_OK) return rc;
        }
        // workgroups: kPairTiles tiles of 32 rows x 64 columns of X each; L0's units by pairs of L1's units cover X (and
        // either operand's k)
        const unsigned tiles = (unsigned)L0.units * (unsigned)(L1.units / (2 * kPairTiles));
        pg.first[n / 2] = prep_ids;
        pg.tiles[n / 2] = tiles;
        if (round != nullptr) {
            const int slot = n / 2;
            rg.Y[slot] = reinterpret_cast<uint32_t *>(round[i].Y);
            rg.ldy[slot] = round[i].ldy;
            rg.partials[slot] = records + (size_t)slot * kShards * kSlots;
            fg.partials[slot] = rg.partials[slot];
            fg.n[slot] = (unsigned long long)it.rows * (unsigned long long)it.cols;
            fg.hist[slot] = reinterpret_cast<unsigned long long *>(round[i].hist);
        }
        const unsigned steps = round != nullptr ? (unsigned)rg.steps : 1u;
        prep_ids += ((tiles + steps - 1u) / steps + 7u) / 8u * 8u;
        add(it, true, L0, view_of(it.buf0, L0), (int)it.cols);
        add(it, false, L1, view_of(it.buf1, L1), (int)it.rows);
    }
    return flush();
}

// Both orientations of one matrix X (rows x cols, X[r*ld + c]) as prepared operands: buf0 = X as stored
// (rows, k = cols), buf1 = X transposed (cols, k = rows).  Exponent planes: one statistics launch and one
// prepare launch that reads X once serve both (launch_prepare_pair_batch); other schemes: two prepare calls.
int launch_prepare_pair(const float *X, int64_t ld, int64_t rows, int64_t cols, fmt_format_t f, const QuantParams &p, void *buf0,
                        void *buf1, hipStream_t stream)
{
    const Scheme s0 = api_scheme(f, cols), s1 = api_scheme(f, rows);
    if (s0.scaled && s1.scaled && p.mode == kModeMagic) {
        const PrepPairItem it{X, ld, rows, cols, buf0, buf1};
        return launch_prepare_pair_batch(1, &it, f, p, stream, nullptr);
    }
    const int rc = launch_prepare_operand(X, ld, 0, rows, cols, f, p, buf0, stream);
    return rc != FMT_OK ? rc : launch_prepare_operand(X, ld, 1, cols, rows, f, p, buf1, stream);
}

// C = A B^T on two prepared operands (A: M rows, B: N rows, both with the same K and scheme).
int launch_gemm_prepared(const void *A, const void *B, int64_t M64, int64_t N64, int64_t K64, int scheme, fmt_format_t f,
                         float *C, int64_t ldc, hipStream_t stream)
{
    const int M = (int)M64, N = (int)N64;
    const Scheme sch{scheme & 15, (scheme & 16) != 0};
    OperandLayout la, lb;
    int rc = operand_layout(M64, K64, sch, f.m, &la);
    if (rc != FMT_OK) return rc;
    rc = operand_layout(N64, K64, sch, f.m, &lb);
    if (rc != FMT_OK) return rc;
    int cus = 0;
    rc = device_cu_count(&cus);
    if (rc != FMT_OK) return rc;
    const Plan plan = make_plan(M, N, la.kblocks, cus, pieces_of(sch.ps));
    float *part = nullptr;
    if (plan.nsplit > 1) {
        Scratch s;
        rc = get_scratch(stream, 0, part_bytes_of(plan, M, N), &s);
        if (rc != FMT_OK) return rc;
        part = static_cast<float *>(s.gemm_ws);
    }
    const OperandView va = view_of(const_cast<void *>(A), la), vb = view_of(const_cast<void *>(B), lb);
    return product_dispatch(sch.ps, va, vb, M, N, la.kblocks, OutSpec{C, ldc, 0}, plan, part, stream);
}

template <int PS, bool SCALED, int T>
static int launch_group_t(const Group &grp, unsigned grid, hipStream_t stream)
{
    constexpr int KS = Pipe<PS, T, T>::ks, NST = Pipe<PS, T, T>::nst;
    if constexpr (lds_bytes(T, T, pieces_of(PS), KS, NST) > 160 * 1024) {
        return FMT_ERR_SHAPE;                            // never chosen (group_tile checks the same bound)
    } else {
        hipLaunchKernelGGL((product_group_kernel<PS, T, T, KS, NST, true, SCALED>), dim3(grid), dim3(256), 0, stream, grp);
        FMT_HIP_CHECK(hipGetLastError());
        return FMT_OK;
    }
}

template <int PS, bool SCALED>
static int launch_group(const Group &grp, unsigned grid, int t, hipStream_t stream)
{
    return t == 4 ? launch_group_t<PS, SCALED, 4>(grp, grid, stream) : launch_group_t<PS, SCALED, 2>(grp, grid, stream);
}

// Workgroup tile of a shared launch: 64 t x 64 t with t = 2 or 4.  The 256 x 256 tile runs one workgroup per
// compute unit, the 128 x 128 tile two; per unit of k both keep the matrix cores about equally busy when every
// slot has work, so what decides is how the tiles fill the slots.  A tile of kb blocks of 32 k takes about
// 9.5 + 0.89 kb us (large) or 9.8 + 0.47 kb us (small, two to a compute unit) on one fp16 piece -- fitted to
// per-workgroup timestamps on MI355X -- and P x P times the k term on P bf16 pieces.  Workgroups start in
// id order, longest tiles first, so the launch takes about as long as the larger of: all tile time spread
// over all slots; for each product, the rounds that the tiles up to and including its own need, times its
// tile time.  The shape with the smaller estimate is taken.
struct GroupEntry {
    int item;            // index into the batch
    int nparts;          // k parts (1: the product writes its result itself)
    int kb_per_part;     // k blocks per part
    size_t part_off;     // bytes from the start of the scratch to this product's slabs
};

// time estimate (us) of a shared launch of entries [g0, g0 + n) with workgroup tiles of 64 t x 64 t
static double group_estimate(const BatchItem *items, const std::vector<GroupEntry> &e, size_t g0, int n, int cus, int pieces, int t)
{
    const double fixed = t == 4 ? 9.5 : 9.8, per_kb = (t == 4 ? 0.89 : 0.47) * pieces * pieces;
    const double slots = (double)cus * (t == 4 ? 1 : 2);
    double work = 0.0, tiles = 0.0, rounds_bound = 0.0;
    for (int j = 0; j < n; ++j) {                            // longest parts first
        const BatchItem &it = items[e[g0 + j].item];
        const double tile_time = fixed + per_kb * e[g0 + j].kb_per_part;
        const double nt = (double)((it.M + 64 * t - 1) / (64 * t)) * (double)((it.N + 64 * t - 1) / (64 * t)) * e[g0 + j].nparts;
        tiles += nt;
        work += nt * tile_time;
        rounds_bound = std::max(rounds_bound, std::ceil(tiles / slots) * tile_time);
    }
    return std::max(work / slots, rounds_bound);
}

static int group_tile(const BatchItem *items, const std::vector<GroupEntry> &e, size_t g0, int n, int cus, int pieces)
{
    if (const char *env = getenv("FMT_GEMM_GROUP_TILE")) {      // tuning override: "2" or "4"
        const int t = atoi(env);
        if (t == 2 || (t == 4 && lds_bytes(4, 4, pieces, pipe_ks(pieces), 2) <= 160 * 1024)) return t;
    }
    if (lds_bytes(4, 4, pieces, pipe_ks(pieces), 2) > 160 * 1024) return 2;
    return group_estimate(items, e, g0, n, cus, pieces, 4) < group_estimate(items, e, g0, n, cus, pieces, 2) ? 4 : 2;
}

// Several products on prepared operands (all of one format and scheme).  A product joins a shared launch when
// it needs no split over k: its own plan has none, or one of its tiles is no longer than the work the whole
// batch leaves to each compute unit (then the other products fill the machine while its few long tiles run).
// A product that does need its k in parts (few tiles, long k) joins with its parts -- each part a run of tiles
// of its own that writes a slab of partial sums, summed by reduce_kernel after the launch -- when a part's
// tile takes no longer than the launch is estimated to take without it.  Shared launches hold up to kMaxGroup
// products, longest parts first (their tiles take longest and workgroups start in id order); what is left
// runs one by one as launch_gemm_prepared runs it.
int launch_gemm_prepared_batch(int count, const BatchItem *items, int scheme, fmt_format_t f, hipStream_t stream)
{
    const Scheme sch{scheme & 15, (scheme & 16) != 0};
    const int pieces = pieces_of(sch.ps);
    int cus = 0;
    int rc = device_cu_count(&cus);
    if (rc != FMT_OK) return rc;
    std::vector<GroupEntry> grouped;
    std::vector<int> alone, parted;
    std::vector<Plan> plans((size_t)count);
    double load = 0.0;                                   // 256 x 256 x 32 blocks of multiplications per compute unit
    for (int i = 0; i < count; ++i)
        load += (double)((items[i].M + 255) / 256) * (double)((items[i].N + 255) / 256) * (double)((items[i].K + kUnitK - 1) / kUnitK);
    load /= cus;
    for (int i = 0; i < count; ++i) {
        const int kblocks = (int)((items[i].K + kUnitK - 1) / kUnitK);
        plans[(size_t)i] = make_plan((int)items[i].M, (int)items[i].N, kblocks, cus, pieces);
        if (plans[(size_t)i].nsplit == 1 || kblocks <= load) grouped.push_back(GroupEntry{i, 1, kblocks, 0});
        else parted.push_back(i);
    }
    size_t part_bytes = 0;
    if (!grouped.empty() && !parted.empty()) {
        const int n0 = (int)std::min<size_t>(kMaxGroup, grouped.size());
        const int t0 = group_tile(items, grouped, 0, n0, cus, pieces);
        const double base = group_estimate(items, grouped, 0, n0, cus, pieces, t0);
        const double fixed = t0 == 4 ? 9.5 : 9.8, per_kb = (t0 == 4 ? 0.89 : 0.47) * pieces * pieces;
        for (int i : parted) {
            const int kblocks = (int)((items[i].K + kUnitK - 1) / kUnitK);
            const int ns = plans[(size_t)i].nsplit, kb_per = (kblocks + ns - 1) / ns;
            if (fixed + per_kb * kb_per <= base) {
                grouped.push_back(GroupEntry{i, ns, kb_per, part_bytes});
                part_bytes += ((size_t)ns * items[i].M * items[i].N * sizeof(float) + 255) / 256 * 256;
            } else {
                alone.push_back(i);
            }
        }
    } else {
        alone = parted;
    }
    if (grouped.size() == 1 && grouped[0].nparts == 1) {
        alone.push_back(grouped[0].item);
        grouped.clear();
    }
    // the scratch for every slab of partial sums of the call, before anything is launched (growing it waits for the device)
    size_t need = part_bytes;
    for (int i : alone) need = std::max(need, part_bytes_of(plans[(size_t)i], (int)items[i].M, (int)items[i].N));
    char *scratch = nullptr;
    if (need > 0) {
        Scratch sc;
        rc = get_scratch(stream, 0, need, &sc);
        if (rc != FMT_OK) return rc;
        scratch = static_cast<char *>(sc.gemm_ws);
    }
    std::stable_sort(grouped.begin(), grouped.end(),
                     [&](const GroupEntry &a, const GroupEntry &b) { return a.kb_per_part > b.kb_per_part; });

    for (size_t g0 = 0; g0 < grouped.size(); g0 += kMaxGroup) {
        const int n = (int)std::min<size_t>(kMaxGroup, grouped.size() - g0);
        const int gt = group_tile(items, grouped, g0, n, cus, pieces);
        Group grp{};
        TailGroup tg{};
        grp.count = tg.count = n;
        for (int j = 0; j < kMaxGroup; ++j) grp.first[j] = tg.first[j] = 0xFFFFFFFFu;
        uint64_t ids = 0, blocks = 0, blocks256 = 0;
        for (int j = 0; j < n; ++j) {
            const BatchItem &it = items[grouped[g0 + j].item];
            blocks256 += (uint64_t)((it.M + kUnitRows - 1) / kUnitRows) * (uint64_t)((it.N + 255) / 256);
        }
        tg.tail_cols = tail_cols_for(blocks256, cus);
        for (int j = 0; j < n; ++j) {
            const GroupEntry &ge = grouped[g0 + j];
            const BatchItem &it = items[ge.item];
            OperandLayout la, lb;
            rc = operand_layout(it.M, it.K, sch, f.m, &la);
            if (rc != FMT_OK) return rc;
            rc = operand_layout(it.N, it.K, sch, f.m, &lb);
            if (rc != FMT_OK) return rc;
            const OperandView va = view_of(const_cast<void *>(it.A), la), vb = view_of(const_cast<void *>(it.B), lb);
            const int M = (int)it.M, N = (int)it.N;
            GroupItem &p = grp.p[j];
            p.Aw = va.W; p.Bw = vb.W;
            p.C = ge.nparts > 1 ? reinterpret_cast<float *>(scratch + ge.part_off) : it.C;
            p.ldc = ge.nparts > 1 ? (int64_t)N : it.ldc;
            p.M = M; p.N = N; p.kblocks = la.kblocks; p.kb_per_part = ge.kb_per_part;
            p.tiles_m = (M + 64 * gt - 1) / (64 * gt); p.tiles_n = (N + 64 * gt - 1) / (64 * gt);
            p.first = grp.first[j] = (unsigned)ids;
            p.pa = va.pl; p.pb = vb.pl;
            ids += ((uint64_t)p.tiles_m * p.tiles_n + 7) / 8 * 8 * (uint64_t)ge.nparts;
            TailGroupItem &t = tg.p[j];
            t.Aw = va.W; t.Bw = vb.W; t.C = it.C; t.ldc = it.ldc;
            t.M = M; t.N = N; t.kblocks = la.kblocks; t.col_chunks = (N + tg.tail_cols - 1) / tg.tail_cols;
            t.first = tg.first[j] = (unsigned)blocks;
            t.pa = va.pl; t.pb = vb.pl;
            blocks += (uint64_t)((M + kUnitRows - 1) / kUnitRows) * t.col_chunks;
            if (ids >= ((uint64_t)1 << 31) || blocks >= ((uint64_t)1 << 31)) return FMT_ERR_SHAPE;
        }
        switch (sch.ps) {
            case 0: rc = sch.scaled ? launch_group<0, true>(grp, (unsigned)ids, gt, stream) : launch_group<0, false>(grp, (unsigned)ids, gt, stream); break;
            case 1: rc = launch_group<1, false>(grp, (unsigned)ids, gt, stream); break;
            case 2: rc = launch_group<2, false>(grp, (unsigned)ids, gt, stream); break;
            default: rc = launch_group<3, false>(grp, (unsigned)ids, gt, stream); break;
        }
        if (rc != FMT_OK) return rc;
        for (int j = 0; j < n; ++j) {                        // the sums of the parts, in part order
            const GroupEntry &ge = grouped[g0 + j];
            if (ge.nparts == 1) continue;
            const BatchItem &it = items[ge.item];
            const size_t total = (size_t)it.M * it.N;
            const unsigned rgrid = (unsigned)((total + 1023) / 1024 < 4096 ? (total + 1023) / 1024 : 4096);
            hipLaunchKernelGGL(reduce_kernel, dim3(rgrid ? rgrid : 1), dim3(256), 0, stream,
                               reinterpret_cast<const float *>(scratch + ge.part_off), ge.nparts, it.C, (int)it.M, (int)it.N, it.ldc, 0);
            FMT_HIP_CHECK(hipGetLastError());
        }
        if (sch.scaled) {
            hipLaunchKernelGGL(planes_tail_group_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, tg);
            FMT_HIP_CHECK(hipGetLastError());
        }
    }
    for (int i : alone) {
        rc = launch_gemm_prepared(items[i].A, items[i].B, items[i].M, items[i].N, items[i].K, scheme, f, items[i].C, items[i].ldc,
                                  stream);
        if (rc != FMT_OK) return rc;
    }
    return FMT_OK;
}

static int zero_fill(float *C, int64_t rows, int64_t cols, int64_t ldc, hipStream_t stream)
{
    if (rows == 0 || cols == 0) return FMT_OK;
    const int64_t col_blocks = (cols + 255) / 256;
    if (col_blocks * rows >= ((int64_t)1 << 31)) return FMT_ERR_SHAPE;
    hipLaunchKernelGGL(zero_fill_kernel, dim3((unsigned)(col_blocks * rows)), dim3(256), 0, stream, C, (int)rows, (int)cols,
                       ldc, (int)col_blocks);
    FMT_HIP_CHECK(hipGetLastError());
    return FMT_OK;
}

int launch_gemm(int transA, int transB, int64_t M64, int64_t N64, int64_t K64, const float *A, int64_t lda,
                const float *B, int64_t ldb, float *C, int64_t ldc, fmt_format_t f, const QuantParams &p,
                hipStream_t stream)
{
    const int M = (int)M64, N = (int)N64, K = (int)K64;
    if (K == 0) return zero_fill(C, M, N, ldc, stream);
    // op(A) is M x K: k-contiguous unless transposed.  op(B) is K x N, consumed as N rows of K:
    // k-contiguous when B is stored transposed (N x K).
    const OperandSpec sa{A, lda, !transA, Gather{}, 0};
    const OperandSpec sb{B, ldb, transB != 0, Gather{}, 0};
    return run_product(M, N, K, sa, sb, OutSpec{C, ldc, 0}, f, p, stream);
}

// Forward and dgrad with the patches gathered inside the product kernel: the tensor behind the patches is
// rounded once into pixel-major 16-bit pieces (2P bytes per tensor element), the filter into an ordinary
// prepared operand whose k runs (tap, channel), and no patch-sized operand exists anywhere.
template <int MODE, bool FTZ, int PS>
static int run_implicit(int M, int N, int K, const OperandSpec &sa, const float *tensor, int64_t tensor_elems, int HW,
                        Implicit im, const OutSpec &out, fmt_format_t f, const QuantParams &p, hipStream_t stream)
{
    constexpr int P = pieces_of(PS);
    const Scheme sch{PS, false};
    OperandLayout la;
    int rc = operand_layout(M, K, sch, f.m, &la);
    if (rc != FMT_OK) return rc;
    int cus = 0;
    rc = device_cu_count(&cus);
    if (rc != FMT_OK) return rc;
    const Plan plan = make_plan(M, N, la.kblocks, cus, P);
    auto up256 = [](size_t b) { return (b + 255) / 256 * 256; };
    const int C = im.c8 * 8;
    const int npix = (int)(tensor_elems / C);
    const size_t piece_vec = (size_t)npix * im.c8;
    const size_t nhwc = up256((P * piece_vec + 1) * sizeof(u32x4));
    const size_t part = part_bytes_of(plan, M, N);
    Scratch s;
    rc = get_scratch(stream, 0, la.bytes + nhwc + part, &s);
    if (rc != FMT_OK) return rc;
    char *ws = static_cast<char *>(s.gemm_ws);
    const OperandView va = view_of(ws, la);
    u32x4 *T = reinterpret_cast<u32x4 *>(ws + la.bytes);
    float *partp = reinterpret_cast<float *>(ws + la.bytes + nhwc);
    rc = prepare_operands<MODE, FTZ, PS>(sa, la, va, nullptr, nullptr, nullptr, nullptr, nullptr, K, f, p, stream);
    if (rc != FMT_OK) return rc;
    hipLaunchKernelGGL((nhwc_split_kernel<MODE, FTZ, PS>), dim3((unsigned)((npix + 63) / 64), (unsigned)(C / 32)), dim3(256), 0,
                       stream, reinterpret_cast<const uint32_t *>(tensor), T, C, HW, npix, p);
    FMT_HIP_CHECK(hipGetLastError());
    im.T = T;
    im.piece_vec = (int)piece_vec;
    im.zero = (int)(P * piece_vec);
    const Planes none{nullptr, nullptr, 0, 0, nullptr, nullptr};
#define FMT_PRODUCT(TMV, TNV) \
    launch_product<PS, TMV, TNV>(va.W, nullptr, out.C, M, N, out.ldc, out.img, la.kblocks, plan, partp, stream, none, none, &im)
    if (plan.tm == 4 && plan.tn == 4) return FMT_PRODUCT(4, 4);
    if (plan.tm == 4 && plan.tn == 2) return FMT_PRODUCT(4, 2);
    if (plan.tm == 2 && plan.tn == 4) return FMT_PRODUCT(2, 4);
    if (plan.tm == 2 && plan.tn == 2) return FMT_PRODUCT(2, 2);
    return FMT_PRODUCT(1, 1);
#undef FMT_PRODUCT
}

// In-kernel gather for forward (which == 0) and dgrad (which == 1): returns FMT_OK after launching, or 1 when
// the geometry is not covered (channels of the gathered tensor not a multiple of 32, more than 32 taps, dgrad
// with a stride, index ranges), in which case the caller takes the route through a gathered operand.
static int conv_implicit(int which, const fmt_conv2d_t &g, int64_t P, int64_t Q, const float *tensor, const float *filt,
                         float *out, fmt_format_t f, const QuantParams &p, hipStream_t stream)
{
    if (const char *env = getenv("FMT_CONV_IMPLICIT"))
        if (env[0] == '0') return 1;
    const int tc = which == 0 ? g.c : g.k;                       // channels of the gathered tensor
    const int64_t th = which == 0 ? g.h : P, tw = which == 0 ? g.w : Q;
    const int64_t elems = (int64_t)g.n * tc * th * tw;
    if (tc % 32 != 0 || g.r * g.s > 32 || elems >= ((int64_t)1 << 31)) return 1;
    if (which == 1 && (g.stride_h != 1 || g.stride_w != 1)) return 1;
    const Scheme sch = scheme_of(f, false);
    if ((elems / 8) * pieces_of(sch.ps) + (int64_t)(g.r * tw + g.s) * (tc / 8) >= ((int64_t)1 << 31)) return 1;
    const int rs = g.r * g.s;
    const int64_t M = which == 0 ? g.k : g.c, K = (int64_t)tc * rs;
    const int64_t gy = which == 0 ? P : g.h, gx = which == 0 ? Q : g.w;
    const int64_t N = (int64_t)g.n * gy * gx;
    Implicit im{};
    im.c8 = tc / 8;
    im.th = (int)th; im.tw = (int)tw; im.gy = (int)gy; im.gx = (int)gx;
    im.mul_y = which == 0 ? g.stride_h : 1; im.mul_x = which == 0 ? g.stride_w : 1;
    im.off_y = which == 0 ? -g.pad_h : g.pad_h; im.off_x = which == 0 ? -g.pad_w : g.pad_w;
    im.tap_sign = which == 0 ? 1 : -1;
    im.R = g.r; im.S = g.s;
    im.rows = (int)N;
    im.r0 = make_fastdiv((int)gx); im.r1 = make_fastdiv((int)gy);
    im.ks = make_fastdiv(g.s);
    Gather ft{};
    ft.kind = kSrcFilterTap;
    ft.k0 = make_fastdiv(tc);
    // filter [K][C][R][S]: forward row = filter, k = (tap, c); dgrad row = c, k = (tap, filter)
    ft.th = which == 0 ? g.c * rs : rs;
    ft.tw = which == 0 ? rs : g.c * rs;
    const OperandSpec sa{filt, 0, true, ft, 0};
    const OutSpec os{out, 0, (int)(gy * gx)};
    const bool ftz = f.denorm == 0;
#define FMT_IMPL2(MD, FZ)                                                                                                     \
    (sch.ps == 0   ? run_implicit<MD, FZ, 0>((int)M, (int)N, (int)K, sa, tensor, elems, (int)(th * tw), im, os, f, p, stream) \
     : sch.ps == 1 ? run_implicit<MD, FZ, 1>((int)M, (int)N, (int)K, sa, tensor, elems, (int)(th * tw), im, os, f, p, stream) \
     : sch.ps == 2 ? run_implicit<MD, FZ, 2>((int)M, (int)N, (int)K, sa, tensor, elems, (int)(th * tw), im, os, f, p, stream) \
                   : run_implicit<MD, FZ, 3>((int)M, (int)N, (int)K, sa, tensor, elems, (int)(th * tw), im, os, f, p, stream))
#define FMT_IMPL(MD) (ftz ? FMT_IMPL2(MD, true) : FMT_IMPL2(MD, false))
    if (p.mode == kModeMagic) return FMT_IMPL(kModeMagic);
    if (p.mode == kModeInteger) return FMT_IMPL(kModeInteger);
    return FMT_IMPL(kModeMixed);
#undef FMT_IMPL
#undef FMT_IMPL2
}

// Convolutions (Sec. IV-A) as products on patches that are never materialised in fp32.
//   forward  Y[n][k][p][q]:  M = K filters (rows of the filter matrix), N = n*P*Q output positions
//            (patches of X), k = C*R*S, result stored NCHW
//   dgrad    dX[n][c][h][w]: M = C (filter seen from the input channel), N = n*H*W input positions
//            (patches of dY through the taps that reach them), k = K*R*S, result stored NCHW
//   wgrad    dW[k][c][r][s]: M = K (dY as [K][n*P*Q]), N = C*R*S (patches of X, transposed),
//            k = n*P*Q, result is the plain [K][C*R*S] matrix
// Forward and (stride 1) dgrad with a channel count that is a multiple of 32 and at most 32 taps gather
// the patches inside the product kernel from the once-rounded tensor (conv_implicit: scratch is 2P bytes
// per TENSOR element); the other cases, and wgrad, go through a prepare pass that gathers from the once
// rounded tensor into a patch-sized 16-bit prepared operand.
int launch_conv2d(int which, const fmt_conv2d_t &g, const float *a, const float *b, float *out, fmt_format_t f,
                  const QuantParams &p, hipStream_t stream)
{
    const int64_t P = (g.h + 2 * g.pad_h - g.r) / g.stride_h + 1, Q = (g.w + 2 * g.pad_w - g.s) / g.stride_w + 1;
    Gather patch{};
    patch.R = g.r;
    patch.S = g.s;
    Gather none{};
    if (which == 0) {
        const int64_t M = g.k, N = (int64_t)g.n * P * Q, K = (int64_t)g.c * g.r * g.s;
        if (M == 0 || N == 0) return FMT_OK;
        patch.kind = kSrcPatchRows;
        patch.tc = g.c; patch.th = g.h; patch.tw = g.w;
        patch.gy = (int)P; patch.gx = (int)Q;
        patch.mul_y = g.stride_h; patch.mul_x = g.stride_w; patch.off_y = -g.pad_h; patch.off_x = -g.pad_w;
        patch.tap = 1; patch.den_y = 1; patch.den_x = 1;
        patch.r0 = make_fastdiv(patch.gx); patch.r1 = make_fastdiv(patch.gy);
        patch.k0 = make_fastdiv(g.s); patch.k1 = make_fastdiv(g.r);
        if (K == 0) return zero_fill(out, (int64_t)g.n * M, P * Q, P * Q, stream);
        {
            const int rci = conv_implicit(0, g, P, Q, a, b, out, f, p, stream);
            if (rci <= 0) return rci;
        }
        const OperandSpec sa{b, K, true, none, 0};                 // filter [K][C*R*S]
        const OperandSpec sb{a, 0, false, patch, (int64_t)g.n * g.c * g.h * g.w};   // patches of X, lanes along positions
        return run_product((int)M, (int)N, (int)K, sa, sb, OutSpec{out, 0, (int)(P * Q)}, f, p, stream);
    }
    if (which == 1) {
        const int64_t M = g.c, N = (int64_t)g.n * g.h * g.w, K = (int64_t)g.k * g.r * g.s;
        if (M == 0 || N == 0) return FMT_OK;
        patch.kind = kSrcPatchRows;
        patch.tc = g.k; patch.th = (int)P; patch.tw = (int)Q;
        patch.gy = g.h; patch.gx = g.w;
        patch.mul_y = 1; patch.mul_x = 1; patch.off_y = g.pad_h; patch.off_x = g.pad_w;
        patch.tap = -1; patch.den_y = g.stride_h; patch.den_x = g.stride_w;
        patch.r0 = make_fastdiv(patch.gx); patch.r1 = make_fastdiv(patch.gy);
        patch.k0 = make_fastdiv(g.s); patch.k1 = make_fastdiv(g.r);
        if (K == 0) return zero_fill(out, (int64_t)g.n * M, (int64_t)g.h * g.w, (int64_t)g.h * g.w, stream);
        {
            const int rci = conv_implicit(1, g, P, Q, a, b, out, f, p, stream);
            if (rci <= 0) return rci;
        }
        Gather ft{};
        ft.kind = kSrcFilterT;
        ft.tc = g.c; ft.R = g.r; ft.S = g.s;
        ft.k0 = make_fastdiv(g.r * g.s);
        const OperandSpec sa{b, 0, true, ft, 0};                   // filter as [C][K*R*S]
        const OperandSpec sb{a, 0, false, patch, (int64_t)g.n * g.k * P * Q};       // patches of dY
        return run_product((int)M, (int)N, (int)K, sa, sb, OutSpec{out, 0, g.h * g.w}, f, p, stream);
    }
    const int64_t M = g.k, N = (int64_t)g.c * g.r * g.s, K = (int64_t)g.n * P * Q;
    if (M == 0 || N == 0) return FMT_OK;
    if (K == 0) return zero_fill(out, M, N, N, stream);
    Gather ch{};
    ch.kind = kSrcChannelRows;
    ch.tc = g.k; ch.th = (int)P; ch.tw = (int)Q;
    ch.k0 = make_fastdiv((int)(P * Q));
    patch.kind = kSrcPatchK;
    patch.tc = g.c; patch.th = g.h; patch.tw = g.w;
    patch.gy = (int)P; patch.gx = (int)Q;
    patch.mul_y = g.stride_h; patch.mul_x = g.stride_w; patch.off_y = -g.pad_h; patch.off_x = -g.pad_w;
    patch.tap = 1; patch.den_y = 1; patch.den_x = 1;
    patch.r0 = make_fastdiv(g.s); patch.r1 = make_fastdiv(g.r);
    patch.k0 = make_fastdiv(patch.gx); patch.k1 = make_fastdiv(patch.gy);
    const OperandSpec sa{a, 0, true, ch, 0};                       // dY as [K][n*P*Q]
    const OperandSpec sb{b, 0, true, patch, (int64_t)g.n * g.c * g.h * g.w};      // patches of X, k along positions
    return run_product((int)M, (int)N, (int)K, sa, sb, OutSpec{out, N, 0}, f, p, stream);
}

}  // namespace fmt
