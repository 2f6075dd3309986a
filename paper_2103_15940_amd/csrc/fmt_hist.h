// Device-side pieces of the per-tensor statistics (Sec. V), shared by the stream kernels and the
// Linear-layer epilogue: the replicated exponent table in LDS, the per-lane class counters, and
// the fold of a workgroup's table into one of the partial records in global memory.
#pragma once

#include "fmt_internal.h"

namespace fmt {

constexpr int kHistRows = 256 + 24;      // exponent fields 0..255, then the 23 binades of fp32 denormals
constexpr int kSlots = 72;               // uint64 per partial record (8 class slots + 64 bins)
constexpr int kShards = 64;              // partial records in global memory (workgroup b adds into b % 64)
// slots of a partial record
enum { P_Z = 0, P_ZU, P_ZUD, P_TOP, P_INFNAN, P_NAN, P_BINS = 8 };

struct Counts {                          // per-lane counters, reduced once at the end
    uint32_t z = 0, zu = 0, zud = 0, top = 0, infnan = 0, nan = 0;
};

// Statistics of one element (a = pattern of |x|): one LDS increment and four compare-and-count
// steps (six when the wave holds an overflowing or non-finite element).  COPIES replicas of the
// table, lane l uses replica l % COPIES (with 32 replicas no two lanes share a bank).
template <bool DEEP, int COPIES>
__device__ __forceinline__ void account(uint32_t a, bool valid, const QuantParams &p, uint32_t *tbl, uint32_t copy,
                                        Counts &w)
{
    uint32_t row = a >> 23;
    if (DEEP) {
        // fp32-denormal inputs get a row per binade so that windows reaching below 2^-126 stay exact
        if (a - 1u < 0x007FFFFFu) row = 256u + (31u - (uint32_t)__builtin_clz(a));
    }
    if (valid) __hip_atomic_fetch_add(&tbl[row * COPIES + copy], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    w.z += (valid && a == 0u) ? 1u : 0u;
    w.zu += (valid && a <= p.t_zero) ? 1u : 0u;
    w.zud += (valid && a < p.t_den) ? 1u : 0u;
    const bool top = valid && a >= p.t_ovf;
    if (__ballot(top)) {                 // wave-uniform: rare for real tensors
        w.top += top ? 1u : 0u;
        w.infnan += (valid && a >= 0x7F800000u) ? 1u : 0u;
        w.nan += (valid && a > 0x7F800000u) ? 1u : 0u;
    }
}

// The same statistics for a run of elements that are all valid, in two parts.  account_run does the
// table increment and the three counters every element needs, and keeps the largest pattern seen in
// amax; after the run, account_run_top looks at amax once and recounts the run's elements for the
// overflow / infinity / NaN counters only if one of them can be non-zero anywhere in the wave.
template <bool DEEP, int COPIES>
__device__ __forceinline__ void account_run(uint32_t a, const QuantParams &p, uint32_t *tbl, uint32_t copy, Counts &w,
                                            uint32_t &amax)
{
    uint32_t row = a >> 23;
    if (DEEP) {
        if (a - 1u < 0x007FFFFFu) row = 256u + (31u - (uint32_t)__builtin_clz(a));
    }
    __hip_atomic_fetch_add(&tbl[row * COPIES + copy], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    w.z += a == 0u ? 1u : 0u;
    w.zu += a <= p.t_zero ? 1u : 0u;
    w.zud += a < p.t_den ? 1u : 0u;
    amax = a > amax ? a : amax;
}

template <int N>
__device__ __forceinline__ void account_run_top(const uint32_t (&u)[N], uint32_t amax, const QuantParams &p, Counts &w)
{
    if (__ballot(amax >= p.t_ovf)) {     // wave-uniform: rare for real tensors
#pragma unroll
        for (int j = 0; j < N; ++j) {
            const uint32_t a = u[j] & 0x7FFFFFFFu;
            w.top += a >= p.t_ovf ? 1u : 0u;
            w.infnan += a >= 0x7F800000u ? 1u : 0u;
            w.nan += a > 0x7F800000u ? 1u : 0u;
        }
    }
}

// Zeroes the table and the two small arrays; ends with a barrier.  tbl must be 16-byte aligned.
template <int COPIES, int BLOCK>
__device__ __forceinline__ void hist_begin(uint32_t *tbl, uint32_t *s_bins, uint32_t *s_cls, uint32_t tid)
{
    typedef uint32_t v4 __attribute__((ext_vector_type(4)));
    for (int i = tid; i < kHistRows * COPIES / 4; i += BLOCK) reinterpret_cast<v4 *>(tbl)[i] = v4{0u, 0u, 0u, 0u};
    if (tid < FMT_NBINS) s_bins[tid] = 0;
    if (tid < 8) s_cls[tid] = 0;
    __syncthreads();
}

// Folds the workgroup's counters and table into 64 bins and adds the 72 counts, one 64-bit atomic
// per non-zero slot, into partial record `shard` (< kShards).  All BLOCK threads call it.
template <int COPIES, int BLOCK>
__device__ __forceinline__ void hist_end(uint32_t *tbl, uint32_t *s_bins, uint32_t *s_cls, const Counts &w,
                                         const QuantParams &p, unsigned long long *partials, uint32_t shard,
                                         uint32_t tid)
{
    uint32_t c[6] = {w.z, w.zu, w.zud, w.top, w.infnan, w.nan};
#pragma unroll
    for (int q = 0; q < 6; ++q) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) c[q] += __shfl_xor(c[q], off, 64);
    }
    if ((tid & 63) == 0) {
#pragma unroll
        for (int q = 0; q < 6; ++q)
            if (c[q]) atomicAdd(&s_cls[q], c[q]);
    }
    __syncthreads();
    for (int row = tid; row < kHistRows; row += BLOCK) {
        uint32_t sum = 0;
#pragma unroll 8
        for (int k = 0; k < COPIES; ++k) sum += tbl[row * COPIES + ((k + row) & (COPIES - 1))];
        int E;
        if (row < 256) {
            E = row - 127;
            if (row == 0) sum -= s_cls[P_Z];      // zeros are not binned; what is left are fp32 denormals
            if (row == 255) { sum -= s_cls[P_NAN]; E = 1 << 20; }   // infinities -> top bin, NaN not binned
        } else {
            E = row - 256 - 149;                  // binade of an fp32 denormal with leading bit row-256
        }
        int b = E - p.exp_lo;
        b = b < 0 ? 0 : (b > FMT_NBINS - 1 ? FMT_NBINS - 1 : b);
        if (sum) atomicAdd(&s_bins[b], sum);
    }
    __syncthreads();
    unsigned long long *rec = partials + (size_t)shard * kSlots;
    if (tid < kSlots) {
        const uint32_t v = tid < 8 ? s_cls[tid] : s_bins[tid - 8];
        if (v) atomicAdd(&rec[tid], (unsigned long long)v);
    }
}

// Sums the partial records into the caller's fmt_hist_t and clears them (fmt_stream.hip).
int launch_hist_finalize(unsigned long long *partials, size_t n, fmt_hist_t *hist, hipStream_t stream);

// ... for several tensors in one launch: partial records, element count and result of each (fmt_stream.hip).
constexpr int kFinalizeGroup = 16;
struct FinalizeGroup {
    unsigned long long *partials[kFinalizeGroup];
    unsigned long long n[kFinalizeGroup];
    unsigned long long *hist[kFinalizeGroup];
};
int launch_hist_finalize_group(const FinalizeGroup &g, int count, hipStream_t stream);

// Scratch bytes the partial records need.
constexpr size_t kHistScratchBytes = (size_t)kShards * kSlots * sizeof(unsigned long long);

}  // namespace fmt
