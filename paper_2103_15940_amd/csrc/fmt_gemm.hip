// fmt_gemm: C = Q(op(A)) * Q(op(B)) with exact products and fp32 accumulation -- the FMACS
// instruction of Sec. III-B applied to the matrix products of Sec. IV-A.
//
// The matrix cores have no 1/6/9 (or general 1/e/m) operand type, so each rounded operand
// value r is split exactly into P bf16 pieces r = p0 + p1 (+ p2): p0 is r truncated to bf16's
// 8 significant bits, p1 the (exactly representable) remainder, and so on.  bf16 has fp32's
// exponent range, so every piece of a format with e <= 8 fits.  A product r*s is then the sum
// of the P*P piece products, each exact inside the bf16 MFMA, accumulated in its fp32
// accumulator: exact products, fp32 accumulation -- FMACS.  P = 1 for m <= 7 (bfloat16),
// P = 2 for m <= 15 (1/6/9, binary16), P = 3 up to m = 23.
//
// Two kernels:
//   prepare  reads one fp32 operand (either layout), rounds it to the format, splits it and
//            writes the pieces into a library-owned workspace, zero-padded and already in the
//            order the product kernel consumes: units of 32 rows x 32 k per piece, each unit
//            stored as [k-chunk of 8][row][8 x bf16] so that a wave's MFMA operand fetch is one
//            contiguous 1 KiB read.
//   product  a 128x128 workgroup tile, 4 waves each owning 64x64 (2x2 MFMA 32x32x16 tiles),
//            register-prefetched global loads, one LDS stage of 32 k.
#include "fmt_internal.h"
#include "fmt_quant.h"

namespace fmt {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kUnitRows = 32;                 // rows per unit (one MFMA fragment)
constexpr int kUnitK = 32;                    // k per unit (two MFMA steps of 16)
constexpr int kUnitVec = kUnitRows * kUnitK * 2 / 16;   // 16-byte vectors per unit per piece = 128
constexpr int kTile = 128;                    // workgroup tile edge (rows of op(A), columns of op(B))
constexpr int kTileUnits = kTile / kUnitRows; // 4

// Rounds one fp32 pattern to the format and splits the result into P bf16 patterns.
template <int MODE, bool FTZ, int P>
__device__ __forceinline__ void round_and_split(uint32_t u, const QuantParams &p, uint32_t (&piece)[P])
{
    const uint32_t r = quantize_bits<MODE, FTZ>(u, p);
    const uint32_t hi = r & 0xFFFF0000u;
    piece[0] = hi >> 16;
    if (P >= 2) {
        // infinities and NaN stay in the first piece alone
        const bool finite = (r & 0x7F800000u) != 0x7F800000u;
        const float rem = finite ? __uint_as_float(r) - __uint_as_float(hi) : 0.0f;   // exact
        const uint32_t rb = __float_as_uint(rem);
        piece[1] = rb >> 16;
        if (P >= 3) {
            const float rem2 = rem - __uint_as_float(rb & 0xFFFF0000u);                // exact
            piece[2] = __float_as_uint(rem2) >> 16;
        }
    }
}

// Workspace address (in 16-byte vectors) of chunk c (8 consecutive k) of row `row` in unit
// (rb, kb), piece `piece`.
__device__ __forceinline__ size_t unit_vec_index(int rb, int kb, int kblocks, int P, int piece, int c, int row)
{
    return (((size_t)rb * kblocks + kb) * P + piece) * kUnitVec + c * kUnitRows + row;
}

// prepare: X is the fp32 operand, `rows` x K after op(); element (r, k) sits at X[r*ld + k]
// (KCONTIG) or X[k*ld + r].  1-D grid of nslabs * (row groups): slab = 64 k (KCONTIG) or 32 k.
template <int MODE, bool FTZ, int P, bool KCONTIG>
__global__ __launch_bounds__(256) void prepare_kernel(const uint32_t *__restrict__ X, int64_t ld, int rows, int K,
                                                      int kblocks, int nslabs, QuantParams p, u32x4 *__restrict__ W)
{
    const int tid = threadIdx.x;
    const int bx = blockIdx.x % nslabs, by = blockIdx.x / nslabs;
    int row, k0;
    if (KCONTIG) {
        // 32 rows x 64 k per workgroup; 8 neighbouring lanes read 256 contiguous bytes of one row
        row = by * 32 + tid / 8;
        k0 = bx * 64 + (tid % 8) * 8;
    } else {
        // 64 rows x 32 k per workgroup; a wave reads 256 contiguous bytes for each k
        row = by * 64 + tid % 64;
        k0 = bx * 32 + (tid / 64) * 8;
    }
    if (k0 >= kblocks * kUnitK) return;      // KCONTIG slabs cover two k-blocks; the last may be half
    uint32_t v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int k = k0 + j;
        const bool ok = row < rows && k < K;
        const size_t idx = KCONTIG ? (size_t)row * ld + k : (size_t)k * ld + row;
        v[j] = ok ? X[idx] : 0u;
    }
    uint32_t pc[8][P];
#pragma unroll
    for (int j = 0; j < 8; ++j) round_and_split<MODE, FTZ, P>(v[j], p, pc[j]);
    const int rb = row / kUnitRows, rr = row % kUnitRows;
    const int kb = k0 / kUnitK, c = (k0 % kUnitK) / 8;
#pragma unroll
    for (int q = 0; q < P; ++q) {
        u32x4 o;
        o[0] = pc[0][q] | (pc[1][q] << 16);
        o[1] = pc[2][q] | (pc[3][q] << 16);
        o[2] = pc[4][q] | (pc[5][q] << 16);
        o[3] = pc[6][q] | (pc[7][q] << 16);
        W[unit_vec_index(rb, kb, kblocks, P, q, c, rr)] = o;
    }
}

// product: Aw / Bw are prepared operands (rows padded to a multiple of 128, k to a multiple of 32).
template <int P>
__global__ __launch_bounds__(256) void product_kernel(const u32x4 *__restrict__ Aw, const u32x4 *__restrict__ Bw,
                                                      float *__restrict__ C, int M, int N, int64_t ldc, int kblocks,
                                                      int tiles_n)
{
    constexpr int kStageVec = kTileUnits * P * kUnitVec;     // 16-byte vectors per operand per stage
    constexpr int kLoads = kStageVec / 256;                   // per thread per operand (2 * P)
    __shared__ u32x4 sA[kStageVec];
    __shared__ u32x4 sB[kStageVec];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int tm = blockIdx.x / tiles_n, tn = blockIdx.x % tiles_n;

    // Stage image = [unit row-block 0..3][piece][128 vectors]; in the workspace the four row-blocks
    // of one k-block are kblocks*P*128 vectors apart.
    const size_t rb_stride = (size_t)kblocks * P * kUnitVec;
    const u32x4 *ga[kLoads], *gb[kLoads];
#pragma unroll
    for (int j = 0; j < kLoads; ++j) {
        const int q = j * 256 + tid;
        const int rbl = q / (P * kUnitVec), rest = q % (P * kUnitVec);
        ga[j] = Aw + ((size_t)tm * kTileUnits + rbl) * rb_stride + rest;
        gb[j] = Bw + ((size_t)tn * kTileUnits + rbl) * rb_stride + rest;
    }

    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    u32x4 ra[kLoads], rb[kLoads];
#pragma unroll
    for (int j = 0; j < kLoads; ++j) {
        ra[j] = ga[j][0];
        rb[j] = gb[j][0];
    }

    for (int kb = 0; kb < kblocks; ++kb) {
#pragma unroll
        for (int j = 0; j < kLoads; ++j) {
            sA[j * 256 + tid] = ra[j];
            sB[j * 256 + tid] = rb[j];
        }
        __syncthreads();
        if (kb + 1 < kblocks) {
            const size_t off = (size_t)(kb + 1) * P * kUnitVec;
#pragma unroll
            for (int j = 0; j < kLoads; ++j) {
                ra[j] = ga[j][off];
                rb[j] = gb[j][off];
            }
        }
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            bf16x8 fa[2][P], fb[2][P];
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int q = 0; q < P; ++q) {
                    fa[i][q] = __builtin_bit_cast(bf16x8, sA[((wm * 2 + i) * P + q) * kUnitVec + kk * 64 + lane]);
                    fb[i][q] = __builtin_bit_cast(bf16x8, sB[((wn * 2 + i) * P + q) * kUnitVec + kk * 64 + lane]);
                }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int qa = 0; qa < P; ++qa)
#pragma unroll
                        for (int qb = 0; qb < P; ++qb)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i][qa], fb[j][qb], acc[i][j], 0, 0, 0);
        }
        __syncthreads();
    }

    // 32x32 accumulator layout: register v of lane l holds row 8*(v/4) + 4*(l/32) + v%4, column l%32
    const int col_in = lane & 31, row_half = (lane >> 5) * 4;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int col = tn * kTile + wn * 64 + j * 32 + col_in;
            const int row0 = tm * kTile + wm * 64 + i * 32 + row_half;
            if (col < N) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = row0 + (v >> 2) * 8 + (v & 3);
                    if (row < M) C[(size_t)row * ldc + col] = acc[i][j][v];
                }
            }
        }
}

__global__ void zero_fill_kernel(float *__restrict__ C, int M, int N, int64_t ldc, int col_blocks)
{
    const int col = (blockIdx.x % col_blocks) * blockDim.x + threadIdx.x;
    const int row = blockIdx.x / col_blocks;
    if (col < N && row < M) C[(size_t)row * ldc + col] = 0.0f;
}

template <int MODE, bool FTZ, int P>
static int run(int transA, int transB, int M, int N, int K, const float *A, int64_t lda, const float *B, int64_t ldb,
               float *C, int64_t ldc, const QuantParams &p, hipStream_t stream)
{
    const int kblocks = (K + kUnitK - 1) / kUnitK;
    const int tiles_m = (M + kTile - 1) / kTile, tiles_n = (N + kTile - 1) / kTile;
    const size_t a_vec = (size_t)tiles_m * kTileUnits * kblocks * P * kUnitVec;
    const size_t b_vec = (size_t)tiles_n * kTileUnits * kblocks * P * kUnitVec;
    Scratch s;
    int rc = get_scratch(stream, 0, (a_vec + b_vec) * sizeof(u32x4), &s);
    if (rc != FMT_OK) return rc;
    u32x4 *Aw = static_cast<u32x4 *>(s.gemm_ws);
    u32x4 *Bw = Aw + a_vec;
    const uint32_t *Au = reinterpret_cast<const uint32_t *>(A), *Bu = reinterpret_cast<const uint32_t *>(B);

    // op(A) is M x K: k-contiguous unless transposed.  op(B) is K x N, consumed as N rows of K:
    // k-contiguous when B is stored transposed (N x K).
    const int slabs64 = (kblocks + 1) / 2;
    const int64_t lim = (int64_t)1 << 31;
    if ((int64_t)slabs64 * tiles_m * kTileUnits >= lim || (int64_t)slabs64 * tiles_n * kTileUnits >= lim ||
        (int64_t)kblocks * tiles_m * 2 >= lim || (int64_t)kblocks * tiles_n * 2 >= lim)
        return FMT_ERR_SHAPE;
    if (!transA) {
        hipLaunchKernelGGL((prepare_kernel<MODE, FTZ, P, true>), dim3(slabs64 * tiles_m * kTileUnits), dim3(256), 0,
                           stream, Au, lda, M, K, kblocks, slabs64, p, Aw);
    } else {
        hipLaunchKernelGGL((prepare_kernel<MODE, FTZ, P, false>), dim3(kblocks * tiles_m * kTileUnits / 2), dim3(256), 0,
                           stream, Au, lda, M, K, kblocks, kblocks, p, Aw);
    }
    FMT_HIP_CHECK(hipGetLastError());
    if (transB) {
        hipLaunchKernelGGL((prepare_kernel<MODE, FTZ, P, true>), dim3(slabs64 * tiles_n * kTileUnits), dim3(256), 0,
                           stream, Bu, ldb, N, K, kblocks, slabs64, p, Bw);
    } else {
        hipLaunchKernelGGL((prepare_kernel<MODE, FTZ, P, false>), dim3(kblocks * tiles_n * kTileUnits / 2), dim3(256), 0,
                           stream, Bu, ldb, N, K, kblocks, kblocks, p, Bw);
    }
    FMT_HIP_CHECK(hipGetLastError());
    hipLaunchKernelGGL((product_kernel<P>), dim3(tiles_m * tiles_n), dim3(256), 0, stream, Aw, Bw, C, M, N, ldc, kblocks,
                       tiles_n);
    FMT_HIP_CHECK(hipGetLastError());
    return FMT_OK;
}

template <int MODE, bool FTZ>
static int run_p(int pieces, int transA, int transB, int M, int N, int K, const float *A, int64_t lda, const float *B,
                 int64_t ldb, float *C, int64_t ldc, const QuantParams &p, hipStream_t stream)
{
    switch (pieces) {
        case 1: return run<MODE, FTZ, 1>(transA, transB, M, N, K, A, lda, B, ldb, C, ldc, p, stream);
        case 2: return run<MODE, FTZ, 2>(transA, transB, M, N, K, A, lda, B, ldb, C, ldc, p, stream);
        default: return run<MODE, FTZ, 3>(transA, transB, M, N, K, A, lda, B, ldb, C, ldc, p, stream);
    }
}

int launch_gemm(int transA, int transB, int64_t M64, int64_t N64, int64_t K64, const float *A, int64_t lda,
                const float *B, int64_t ldb, float *C, int64_t ldc, fmt_format_t f, const QuantParams &p,
                hipStream_t stream)
{
    const int M = (int)M64, N = (int)N64, K = (int)K64;
    if (K == 0) {
        const int col_blocks = (N + 255) / 256;
        if ((int64_t)col_blocks * M >= ((int64_t)1 << 31)) return FMT_ERR_SHAPE;
        hipLaunchKernelGGL(zero_fill_kernel, dim3(col_blocks * M), dim3(256), 0, stream, C, M, N, ldc, col_blocks);
        FMT_HIP_CHECK(hipGetLastError());
        return FMT_OK;
    }
    if ((int64_t)((M + kTile - 1) / kTile) * ((N + kTile - 1) / kTile) >= ((int64_t)1 << 31)) return FMT_ERR_SHAPE;
    const int pieces = f.m <= 7 ? 1 : (f.m <= 15 ? 2 : 3);
    const bool ftz = f.denorm == 0;
#define FMT_RUN(MD)                                                                                       \
    (ftz ? run_p<MD, true>(pieces, transA, transB, M, N, K, A, lda, B, ldb, C, ldc, p, stream)              \
         : run_p<MD, false>(pieces, transA, transB, M, N, K, A, lda, B, ldb, C, ldc, p, stream))
    if (p.mode == kModeMagic) return FMT_RUN(kModeMagic);
    if (p.mode == kModeInteger) return FMT_RUN(kModeInteger);
    return FMT_RUN(kModeMixed);
#undef FMT_RUN
}

}  // namespace fmt
