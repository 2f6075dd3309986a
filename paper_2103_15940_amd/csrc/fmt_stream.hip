// Stream kernels of libfmt: the rounding kernel of Sec. IV-A (fp32 -> 1/e/m, result kept as
// fp32) and the per-tensor statistics of Sec. V, separately or fused in one pass over x.
//
// Both are HBM streams: 4 B read (+ 4 B written) per element, 128-bit non-temporal accesses.
// A workgroup walks over tiles of 16 KiB of consecutive input (tile b, b+grid, ...): contiguous
// tiles handed out in launch order measured faster on MI355X than a thread-granular grid stride.  The rounding works on the fp32 bit pattern:
//   * e < 8: the format's grid around |x| has spacing 2^(max(E,Emin)-m), E = floor(log2|x|), and
//     (|x| + C) - C with C = 2^(max(E,Emin)+23-m) lands on it with the hardware's own RNE --
//     exact, since the addition is one correctly rounded fp32 operation whose ulp is that
//     spacing and the subtraction is exact.  C comes from the exponent field of |x| with two
//     integer operations.  fp32-denormal inputs are far below minD/2 there, so a flush of
//     them could only give the same zero;
//   * e = 8: fp32's own denormal grid is the format's, so round-to-nearest-even is done on the
//     integer pattern (add "half minus one plus the last kept bit", clear the dropped bits; a
//     mantissa carry walks into the exponent by itself), fp32-denormal inputs included;
//   * overflow, zero and flush decisions are comparisons of |x|'s pattern with thresholds
//     computed on the host (the ties at minD/2, minN - minD/2 and maxN + ulp/2 all go to the
//     even neighbour).
// Statistics: each element adds one to an LDS table indexed by its 8-bit fp32 exponent field,
// replicated 32 times so that lane l only ever touches bank l%32 (no bank or address
// conflicts, however concentrated the distribution); the class counts are per-lane
// compare-and-add counters.  Each workgroup folds its table into 64 bins and adds them, with one
// 64-bit atomic per non-zero slot, into one of 64 partial records in library scratch; a second
// tiny kernel sums the 64 records into the caller's fmt_hist_t and clears them again.
#include <mutex>

#include "fmt_hist.h"
#include "fmt_internal.h"
#include "fmt_quant.h"

#ifndef FMT_STREAM_BLOCK
#define FMT_STREAM_BLOCK 256
#endif
#ifndef FMT_STREAM_UNROLL
#define FMT_STREAM_UNROLL 4
#endif
#ifndef FMT_STREAM_GRID_PER_CU
#define FMT_STREAM_GRID_PER_CU 16
#endif

namespace fmt {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kBlock = FMT_STREAM_BLOCK;  // threads per workgroup
// Replicas of the exponent table in LDS, lane l uses replica l % copies.  The fused kernel that writes fp32 keeps
// one replica per bank (32: 35 KiB, 4 workgroups per compute unit); the statistics-only kernel and the one that writes
// 16-bit codes run 8 to 12 % faster with 16 (17.5 KiB, 8 workgroups per compute unit), the fused fp32 one does not.
constexpr int kCopiesFused = 32;
constexpr int kCopiesLight = 16;
constexpr int kUnroll = FMT_STREAM_UNROLL;  // independent 128-bit loads in flight per thread
constexpr int kGridPerCU = FMT_STREAM_GRID_PER_CU;   // workgroups launched per compute unit (at most): statistics only
constexpr int kGridFused = 64;           // ... fused quantize + statistics, fp32 out
constexpr int kGridPack = 128;           // ... fused quantize + statistics, 16-bit codes out
constexpr int kGridStore = 256;          // ... quantize only
template <int MODE, bool STORE, bool FTZ, bool HIST, bool DEEP, int kCopies>
__device__ __forceinline__ u32x4 do_vec(u32x4 v, bool valid, const QuantParams &p, uint32_t *tbl, uint32_t lane32,
                                        Counts &w)
{
    u32x4 o = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t u = v[j];
        if (HIST) account<DEEP, kCopies>(u & 0x7FFFFFFFu, valid, p, tbl, lane32, w);
        if (STORE) o[j] = quantize_bits<MODE, FTZ>(u, p);
    }
    return o;
}

// x, y: element pointers.  The vector body covers elements [head, head + 4*nvec) and needs
// x + head (and y + head when STORE) 16-byte aligned; the at most 6 remaining elements at both
// ends are handled one per lane by the first wave of workgroup 0.  VEC = false is the fallback
// for x and y misaligned relative to each other: the whole range goes one dword per lane.
// PACK: y holds the format's 16-bit codes instead of fp32 values (two bytes written per element; the
// vector body then needs y + head 8-byte aligned).
template <int MODE, bool STORE, bool FTZ, bool HIST, bool DEEP, bool VEC, bool PACK>
__global__ __launch_bounds__(kBlock) void stream_kernel(const uint32_t *__restrict__ x, uint32_t *__restrict__ y,
                                                        size_t n, size_t head, size_t nvec, QuantParams p,
                                                        unsigned long long *__restrict__ partials)
{
    constexpr int EM = MODE == kModeInteger ? kModeInteger : kModeMagic;   // encode_bits' variant
    constexpr int kCopies = (STORE && !PACK) ? kCopiesFused : kCopiesLight;
    uint16_t *__restrict__ y16 = reinterpret_cast<uint16_t *>(y);
    auto put = [&](size_t vec_index, u32x4 o) {
        if (PACK) {
            u32x2 c;
            c[0] = encode_bits<EM>(o[0], p) | (encode_bits<EM>(o[1], p) << 16);
            c[1] = encode_bits<EM>(o[2], p) | (encode_bits<EM>(o[3], p) << 16);
            __builtin_nontemporal_store(c, reinterpret_cast<u32x2 *>(y16 + head) + vec_index);
        } else {
            __builtin_nontemporal_store(o, reinterpret_cast<u32x4 *>(y + head) + vec_index);
        }
    };
    auto put_one = [&](size_t idx, uint32_t r) {
        if (PACK)
            y16[idx] = (uint16_t)encode_bits<EM>(r, p);
        else
            y[idx] = r;
    };
    __shared__ __attribute__((aligned(16))) uint32_t tbl[HIST ? kHistRows * kCopies : 4];
    __shared__ uint32_t s_bins[FMT_NBINS];
    __shared__ uint32_t s_cls[8];
    const uint32_t tid = threadIdx.x;
    const uint32_t lane32 = tid & (kCopies - 1);
    Counts w;

    if (HIST) hist_begin<kCopies, kBlock>(tbl, s_bins, s_cls, tid);

    if (VEC) {
        const u32x4 *xv = reinterpret_cast<const u32x4 *>(x + head);
        // A tile is kBlock*kUnroll consecutive vectors; workgroup b takes tiles b, b+grid, ...
        // Every lane of the workgroup runs the same trips, and all tiles but the last are full.
        constexpr size_t kTileVec = (size_t)kBlock * kUnroll;
        const size_t full_tiles = nvec / kTileVec;
        for (size_t t = blockIdx.x; t < full_tiles; t += gridDim.x) {
            const size_t i = t * kTileVec + tid;
            u32x4 v[kUnroll];
#pragma unroll
            for (int k = 0; k < kUnroll; ++k) v[k] = __builtin_nontemporal_load(xv + i + k * kBlock);
            uint32_t amax = 0u;
#pragma unroll
            for (int k = 0; k < kUnroll; ++k) {
                u32x4 o = {0u, 0u, 0u, 0u};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t u = v[k][j];
                    if (HIST) account_run<DEEP, kCopies>(u & 0x7FFFFFFFu, p, tbl, lane32, w, amax);
                    if (STORE) o[j] = quantize_bits<MODE, FTZ>(u, p);
                }
                if (STORE) put(i + k * kBlock, o);
            }
            if (HIST) {
                uint32_t flat[4 * kUnroll];
#pragma unroll
                for (int k = 0; k < kUnroll; ++k)
#pragma unroll
                    for (int j = 0; j < 4; ++j) flat[4 * k + j] = v[k][j];
                account_run_top(flat, amax, p, w);
            }
        }
        if (blockIdx.x == full_tiles % gridDim.x && full_tiles * kTileVec < nvec) {
            // the ragged last tile, lane by lane
#pragma unroll
            for (int k = 0; k < kUnroll; ++k) {
                const size_t i = full_tiles * kTileVec + k * kBlock + tid;
                const bool valid = i < nvec;
                u32x4 v = {0u, 0u, 0u, 0u};
                if (valid) v = __builtin_nontemporal_load(xv + i);
                u32x4 o = do_vec<MODE, STORE, FTZ, HIST, DEEP, kCopies>(v, valid, p, tbl, lane32, w);
                if (STORE && valid) put(i, o);
            }
        }
        if (blockIdx.x == 0 && tid < 64) {
            // leftovers: [0, head) and [head + 4*nvec, n)
            const size_t body_end = head + 4 * nvec;
            const size_t ntail = n - body_end;
            size_t idx = tid < head ? tid : body_end + (tid - head);
            const bool valid = tid < head + ntail;
            if (!valid) idx = 0;
            const uint32_t u = valid ? x[idx] : 0u;
            if (HIST) account<DEEP, kCopies>(u & 0x7FFFFFFFu, valid, p, tbl, lane32, w);
            if (STORE && valid) put_one(idx, quantize_bits<MODE, FTZ>(u, p));
        }
    } else {
        const size_t stride = (size_t)gridDim.x * kBlock;
        // every lane runs the same number of trips
        const size_t trips = (n + stride - 1) / stride;
        size_t i = (size_t)blockIdx.x * kBlock + tid;
        for (size_t t = 0; t < trips; ++t, i += stride) {
            const bool valid = i < n;
            const uint32_t u = valid ? x[i] : 0u;
            if (HIST) account<DEEP, kCopies>(u & 0x7FFFFFFFu, valid, p, tbl, lane32, w);
            if (STORE && valid) put_one(i, quantize_bits<MODE, FTZ>(u, p));
        }
    }

    if (HIST) hist_end<kCopies, kBlock>(tbl, s_bins, s_cls, w, p, partials, blockIdx.x % kShards, tid);
}

// Sums the shard records into the caller's fmt_hist_t and clears them for the next call (one
// workgroup; the stream orders it after the kernel that filled them).
constexpr int kFinSplit = 14;
__device__ __forceinline__ void finalize_body(unsigned long long *__restrict__ partials, int nrec, unsigned long long n,
                                              unsigned long long *__restrict__ hist)
{
    __shared__ unsigned long long acc[kSlots * kFinSplit];
    __shared__ unsigned long long tot[kSlots];
    const int tid = threadIdx.x;
    const int slot = tid % kSlots, part = tid / kSlots;
    if (part < kFinSplit) {
        unsigned long long s = 0;
        for (int r = part; r < nrec; r += kFinSplit) {
            s += partials[(size_t)r * kSlots + slot];
            partials[(size_t)r * kSlots + slot] = 0;
        }
        acc[part * kSlots + slot] = s;
    }
    __syncthreads();
    if (tid < kSlots) {
        unsigned long long s = 0;
        for (int q = 0; q < kFinSplit; ++q) s += acc[q * kSlots + tid];
        tot[tid] = s;
    }
    __syncthreads();
    if (tid < kSlots) {
        unsigned long long v;
        const unsigned long long z = tot[P_Z], zu = tot[P_ZU], zud = tot[P_ZUD], top = tot[P_TOP],
                                 infnan = tot[P_INFNAN], nan = tot[P_NAN];
        switch (tid) {
            case 0: v = n; break;                    // total
            case 1: v = z; break;                    // zero
            case 2: v = zu - z; break;               // underflow
            case 3: v = zud - zu; break;             // denormal
            case 4: v = n - zud - top; break;        // normal
            case 5: v = top - infnan; break;         // overflow
            case 6: v = infnan - nan; break;         // inf
            case 7: v = nan; break;                  // nan
            default: v = tot[tid]; break;            // bins
        }
        hist[tid] = v;
    }
}

__global__ __launch_bounds__(1024) void finalize_kernel(unsigned long long *__restrict__ partials, int nrec,
                                                        unsigned long long n, unsigned long long *__restrict__ hist)
{
    finalize_body(partials, nrec, n, hist);
}

// The same for up to kFinalizeGroup tensors in one launch: workgroup i sums the records of tensor i.
__global__ __launch_bounds__(1024) void finalize_group_kernel(FinalizeGroup g)
{
    finalize_body(g.partials[blockIdx.x], kShards, g.n[blockIdx.x], g.hist[blockIdx.x]);
}

int launch_hist_finalize_group(const FinalizeGroup &g, int count, hipStream_t stream)
{
    if (count < 1 || count > kFinalizeGroup) return FMT_ERR_SHAPE;
    hipLaunchKernelGGL(finalize_group_kernel, dim3(count), dim3(1024), 0, stream, g);
    FMT_HIP_CHECK(hipGetLastError());
    return FMT_OK;
}

int launch_hist_finalize(unsigned long long *partials, size_t n, fmt_hist_t *hist, hipStream_t stream)
{
    hipLaunchKernelGGL(finalize_kernel, dim3(1), dim3(1024), 0, stream, partials, partials ? kShards : 0,
                       (unsigned long long)n, reinterpret_cast<unsigned long long *>(hist));
    FMT_HIP_CHECK(hipGetLastError());
    return FMT_OK;
}

template <int MODE, bool STORE, bool FTZ, bool HIST, bool DEEP, bool VEC, bool PACK>
static int launch_variant(const float *x, void *y, size_t n, size_t head, size_t nvec, const QuantParams &p,
                          fmt_hist_t *hist, hipStream_t stream, unsigned long long *fixed_partials)
{
    auto kern = stream_kernel<MODE, STORE, FTZ, HIST, DEEP, VEC, PACK>;
    int cus = 0;
    int rc = device_cu_count(&cus);
    if (rc != FMT_OK) return rc;
    const size_t per_block = (size_t)kBlock * (VEC ? 4 * kUnroll : 4);
    const size_t want = (n + per_block - 1) / per_block;
    // Workgroups per compute unit, measured on 2^28 elements: a pure stream likes one 16 KiB tile per
    // workgroup (6.4 TB/s against 5.9 with 16 per CU: the hardware balances the tail); every workgroup
    // of a statistics pass pays for clearing and folding its LDS table, so the read-only pass keeps 16
    // per CU (6.3 TB/s) and the fused pass settles in between (64 per CU: 6.07 against 5.77 TB/s; 128 per
    // CU when it writes 16-bit codes, where 8 workgroups fit a compute unit).
    const size_t cap = (size_t)cus * (HIST ? (STORE ? (PACK ? kGridPack : kGridFused) : kGridPerCU) : kGridStore);
    size_t g = want;
    if (HIST) {
        // mid-size tensors: at least four tiles per workgroup (one tile does not pay for the table),
        // but no fewer workgroups than the four per compute unit that the LDS table lets run at once
        const size_t resident = (size_t)cus * 4;
        g = (want + 3) / 4;
        if (g < resident) g = want < resident ? want : resident;
    }
    int grid = (int)(g < cap ? g : cap);
    if (grid < 1) grid = 1;
    unsigned long long *partials = fixed_partials;
    if (HIST && partials == nullptr) {
        Scratch s;
        rc = get_scratch(stream, kHistScratchBytes, 0, &s);
        if (rc != FMT_OK) return rc;
        partials = static_cast<unsigned long long *>(s.hist_partials);
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kBlock), 0, stream, reinterpret_cast<const uint32_t *>(x),
                       reinterpret_cast<uint32_t *>(y), n, head, nvec, p, partials);
    FMT_HIP_CHECK(hipGetLastError());
    if (HIST) return launch_hist_finalize(partials, n, hist, stream);
    return FMT_OK;
}

int launch_stream(const float *x, void *y, size_t n, const QuantParams &p, bool ftz, fmt_hist_t *hist,
                  hipStream_t stream, bool pack16, unsigned long long *fixed_partials)
{
    const bool store = y != nullptr;
    const bool do_hist = hist != nullptr;
    const bool deep = do_hist && p.exp_lo < -126;
    if (n == 0) {
        if (do_hist) return launch_hist_finalize(nullptr, 0, hist, stream);
        return FMT_OK;
    }
    // elements before the first 16-byte boundary of x, and before the first 16-byte (codes: 8-byte)
    // boundary of y: both must agree for the vector path
    const size_t hx = ((16 - (reinterpret_cast<uintptr_t>(x) & 15)) & 15) / 4;
    const size_t hy = !store ? hx
                      : pack16 ? ((8 - (reinterpret_cast<uintptr_t>(y) & 7)) & 7) / 2
                               : ((16 - (reinterpret_cast<uintptr_t>(y) & 15)) & 15) / 4;
    const bool vec = hx == hy;
    size_t head = hx < n ? hx : n;
    size_t nvec = vec ? (n - head) / 4 : 0;
    if (!vec) head = 0;

#define FMT_LAUNCH_M(MD, S, F, H, D, PK)                                                                     \
    (vec ? launch_variant<MD, S, F, H, D, true, PK>(x, y, n, head, nvec, p, hist, stream, fixed_partials)           \
         : launch_variant<MD, S, F, H, D, false, PK>(x, y, n, head, nvec, p, hist, stream, fixed_partials))
#define FMT_LAUNCH(S, F, H, D)                                                                               \
    (p.mode == kModeMagic ? FMT_LAUNCH_M(kModeMagic, S, F, H, D, false)                                      \
     : p.mode == kModeInteger ? FMT_LAUNCH_M(kModeInteger, S, F, H, D, false)                                \
                              : FMT_LAUNCH_M(kModeMixed, S, F, H, D, false))
    // formats with a 16-bit code have m <= 14: never the m == 23 variant
#define FMT_LAUNCH_PACK(F, H, D)                                                                             \
    (p.mode == kModeInteger ? FMT_LAUNCH_M(kModeInteger, true, F, H, D, true) : FMT_LAUNCH_M(kModeMagic, true, F, H, D, true))
    if (pack16) {
        if (!store || p.mode == kModeMixed) return FMT_ERR_FORMAT;
        if (!do_hist) return ftz ? FMT_LAUNCH_PACK(true, false, false) : FMT_LAUNCH_PACK(false, false, false);
        if (deep) return ftz ? FMT_LAUNCH_PACK(true, true, true) : FMT_LAUNCH_PACK(false, true, true);
        return ftz ? FMT_LAUNCH_PACK(true, true, false) : FMT_LAUNCH_PACK(false, true, false);
    }
    // the statistics do not depend on how the rounding is carried out: one instantiation serves all
    if (!store)
        return deep ? FMT_LAUNCH_M(kModeMagic, false, false, true, true, false)
                    : FMT_LAUNCH_M(kModeMagic, false, false, true, false, false);
    if (!do_hist) return ftz ? FMT_LAUNCH(true, true, false, false) : FMT_LAUNCH(true, false, false, false);
    if (deep) return ftz ? FMT_LAUNCH(true, true, true, true) : FMT_LAUNCH(true, false, true, true);
    return ftz ? FMT_LAUNCH(true, true, true, false) : FMT_LAUNCH(true, false, true, false);
#undef FMT_LAUNCH_PACK
#undef FMT_LAUNCH_M
#undef FMT_LAUNCH
}

// ---- fmt_quantize_static: the partial records in a file-scope device array instead of allocated scratch
//
// Every GPU that loads the library holds its own copy of this array (36 KiB) until the process ends.
// In host code the array's name is only a handle for hipGetSymbolAddress: the address kernels and
// fills use is looked up once per device, with that device current, and kept.
static __device__ __align__(256) unsigned long long scratch[kShards * kSlots];

constexpr int kMaxDevices = 64;
static std::mutex g_static_mu;
static unsigned long long *g_static_ptr[kMaxDevices];

static int static_partials(unsigned long long **out)
{
    int dev = 0;
    FMT_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return FMT_ERR_HIP;
    std::lock_guard<std::mutex> lk(g_static_mu);
    if (g_static_ptr[dev] == nullptr) {
        void *ptr = nullptr;
        FMT_HIP_CHECK(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (ptr == nullptr) return FMT_ERR_HIP;
        g_static_ptr[dev] = static_cast<unsigned long long *>(ptr);
    }
    *out = g_static_ptr[dev];
    return FMT_OK;
}

__global__ __launch_bounds__(256) void clear_records_kernel(unsigned long long *__restrict__ rec, int n)
{
    for (int i = blockIdx.x * 256 + threadIdx.x; i < n; i += gridDim.x * 256) rec[i] = 0ull;
}

int launch_stream_static(const float *x, float *y, size_t n, const QuantParams &p, bool ftz, fmt_hist_t *hist,
                         hipStream_t stream)
{
    unsigned long long *rec = nullptr;
    if (hist != nullptr) {
        int rc = static_partials(&rec);
        if (rc != FMT_OK) return rc;
        // The array keeps whatever the last call on this GPU left in it.  A completed call leaves zeros
        // (its last kernel clears what it has summed), a call that failed half-way may not have: start clean.
        // A kernel, not a memset, so that the call can be recorded into a graph.
        if (n > 0) {
            hipLaunchKernelGGL(clear_records_kernel, dim3(kShards * kSlots / 256), dim3(256), 0, stream, rec, kShards * kSlots);
            FMT_HIP_CHECK(hipGetLastError());
        }
    }
    return launch_stream(x, y, n, p, ftz, hist, stream, false, rec);
}

// codes -> fp32: 2 bytes read, 4 written per element.  In the vector body a lane turns four codes (one
// 64-bit load) into four values (one 128-bit store), four such units per trip, consecutive lanes on
// consecutive units so that loads and stores of a wave are contiguous; the at most 6 elements around
// the body go one per lane.
template <bool INTEGER, bool VEC>
__global__ __launch_bounds__(kBlock) void unpack16_kernel(const uint16_t *__restrict__ codes, uint32_t *__restrict__ y,
                                                          size_t n, size_t head, size_t nvec, QuantParams p)
{
    const uint32_t tid = threadIdx.x;
    if (VEC) {
        const u32x2 *cv = reinterpret_cast<const u32x2 *>(codes + head);
        u32x4 *yv = reinterpret_cast<u32x4 *>(y + head);
        constexpr int kU = 4;
        for (size_t base = (size_t)blockIdx.x * kBlock * kU; base < nvec; base += (size_t)gridDim.x * kBlock * kU) {
            u32x2 c[kU];
#pragma unroll
            for (int k = 0; k < kU; ++k) {
                const size_t i = base + (size_t)k * kBlock + tid;
                c[k] = u32x2{0u, 0u};
                if (i < nvec) c[k] = __builtin_nontemporal_load(cv + i);
            }
#pragma unroll
            for (int k = 0; k < kU; ++k) {
                const size_t i = base + (size_t)k * kBlock + tid;
                u32x4 o;
                o[0] = decode_bits<INTEGER>(c[k][0] & 0xFFFFu, p);
                o[1] = decode_bits<INTEGER>(c[k][0] >> 16, p);
                o[2] = decode_bits<INTEGER>(c[k][1] & 0xFFFFu, p);
                o[3] = decode_bits<INTEGER>(c[k][1] >> 16, p);
                if (i < nvec) __builtin_nontemporal_store(o, yv + i);
            }
        }
        if (blockIdx.x == 0 && tid < 64) {
            const size_t body_end = head + 4 * nvec;
            const size_t ntail = n - body_end;
            const size_t idx = tid < head ? tid : body_end + (tid - head);
            if (tid < head + ntail) y[idx] = decode_bits<INTEGER>(codes[idx], p);
        }
    } else {
        for (size_t i = (size_t)blockIdx.x * kBlock + tid; i < n; i += (size_t)gridDim.x * kBlock)
            y[i] = decode_bits<INTEGER>(codes[i], p);
    }
}

int launch_unpack16(const uint16_t *codes, float *y, size_t n, const QuantParams &p, hipStream_t stream)
{
    if (n == 0) return FMT_OK;
    if (p.mode == kModeMixed) return FMT_ERR_FORMAT;
    int cus = 0;
    int rc = device_cu_count(&cus);
    if (rc != FMT_OK) return rc;
    // codes before the first 8-byte boundary of the codes, values before the first 16-byte boundary of y:
    // both must agree for the vector body
    const size_t hc = ((8 - (reinterpret_cast<uintptr_t>(codes) & 7)) & 7) / 2;        // 0..3
    const size_t hy = ((16 - (reinterpret_cast<uintptr_t>(y) & 15)) & 15) / 4;         // 0..3
    const bool vec = hc == hy;
    const size_t head = vec ? (hc < n ? hc : n) : 0;
    const size_t nvec = vec ? (n - head) / 4 : 0;
    const size_t per_block = (size_t)kBlock * (vec ? 16 : 1);
    const size_t want = (n + per_block - 1) / per_block;
    const size_t cap = (size_t)cus * kGridStore;
    const int grid = (int)(want < cap ? (want ? want : 1) : cap);
    uint32_t *yo = reinterpret_cast<uint32_t *>(y);
    const bool integer = p.mode == kModeInteger;
    if (vec) {
        if (integer)
            hipLaunchKernelGGL((unpack16_kernel<true, true>), dim3(grid), dim3(kBlock), 0, stream, codes, yo, n, head, nvec, p);
        else
            hipLaunchKernelGGL((unpack16_kernel<false, true>), dim3(grid), dim3(kBlock), 0, stream, codes, yo, n, head, nvec, p);
    } else {
        if (integer)
            hipLaunchKernelGGL((unpack16_kernel<true, false>), dim3(grid), dim3(kBlock), 0, stream, codes, yo, n, head, nvec, p);
        else
            hipLaunchKernelGGL((unpack16_kernel<false, false>), dim3(grid), dim3(kBlock), 0, stream, codes, yo, n, head, nvec, p);
    }
    FMT_HIP_CHECK(hipGetLastError());
    return FMT_OK;
}

}  // namespace fmt
