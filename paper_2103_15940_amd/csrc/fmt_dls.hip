// Loss-scale controller and denormal-fraction monitor (Sec. II loss scaling / dynamic loss
// scaling; Sec. V highest denormal fraction over all tensors), one tiny kernel per training step so
// that the decision "skip this step / change the scale" never leaves the device.
#include <cmath>

#include "fmt_internal.h"

namespace fmt {

namespace {

constexpr int kDlsBlock = 256;

struct Best {               // candidate for the largest denormal fraction
    double frac;            // -1: none
    long long idx;
};

__device__ __forceinline__ Best better(Best a, Best b)
{
    // larger fraction wins; equal fractions go to the lower index
    if (b.frac > a.frac || (b.frac == a.frac && b.idx < a.idx)) return b;
    return a;
}

__global__ void dls_init_kernel(fmt_dls_state_t *st, float scale)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        fmt_dls_state_t s = {};
        s.loss_scale = scale;
        s.worst_tensor = -1;
        s.peak_tensor = -1;
        s.peak_step = -1;
        *st = s;
    }
}

__global__ __launch_bounds__(kDlsBlock) void dls_step_kernel(const fmt_hist_t *__restrict__ hists, long long count,
                                                             fmt_dls_params_t prm, fmt_dls_state_t *__restrict__ st)
{
    __shared__ unsigned long long s_bad[kDlsBlock];
    __shared__ Best s_best[kDlsBlock];
    const int tid = threadIdx.x;
    unsigned long long bad = 0;
    Best best{-1.0, -1};
    for (long long i = tid; i < count; i += kDlsBlock) {
        const fmt_hist_t &h = hists[i];
        bad += h.overflow + h.inf + h.nan;
        if (h.total > 0) best = better(best, Best{(double)h.denormal / (double)h.total, i});
    }
    s_bad[tid] = bad;
    s_best[tid] = best;
    __syncthreads();
    for (int off = kDlsBlock / 2; off > 0; off >>= 1) {
        if (tid < off) {
            s_bad[tid] += s_bad[tid + off];
            s_best[tid] = better(s_best[tid], s_best[tid + off]);
        }
        __syncthreads();
    }
    if (tid != 0) return;
    fmt_dls_state_t s = *st;
    const unsigned long long nonfinite = s_bad[0];
    const Best w = s_best[0];
    s.nonfinite = nonfinite;
    s.worst_tensor = w.idx;
    s.worst_denormal = w.idx >= 0 ? hists[w.idx].denormal : 0;
    s.worst_total = w.idx >= 0 ? hists[w.idx].total : 0;
    if (nonfinite > 0) {
        s.skip = 1;
        const float v = __fmul_rn(s.loss_scale, prm.backoff);
        s.loss_scale = v < prm.min_scale ? prm.min_scale : v;
        s.good_steps = 0;
    } else {
        s.skip = 0;
        s.good_steps += 1;
        if (s.good_steps >= prm.interval) {
            const float v = __fmul_rn(s.loss_scale, prm.growth);
            s.loss_scale = v > prm.max_scale ? prm.max_scale : v;
            s.good_steps = 0;
        }
    }
    if (w.idx >= 0) {
        const double peak = s.peak_total > 0 ? (double)s.peak_denormal / (double)s.peak_total : -1.0;
        if (w.frac > peak) {
            s.peak_tensor = w.idx;
            s.peak_step = s.steps;
            s.peak_denormal = s.worst_denormal;
            s.peak_total = s.worst_total;
        }
    }
    s.steps += 1;
    *st = s;
}

}  // namespace

int launch_dls_init(fmt_dls_state_t *state, float loss_scale, hipStream_t stream)
{
    hipLaunchKernelGGL(dls_init_kernel, dim3(1), dim3(64), 0, stream, state, loss_scale);
    FMT_HIP_CHECK(hipGetLastError());
    return FMT_OK;
}

int launch_dls_step(const fmt_hist_t *hists, int64_t count, fmt_dls_params_t prm, fmt_dls_state_t *state,
                    hipStream_t stream)
{
    hipLaunchKernelGGL(dls_step_kernel, dim3(1), dim3(kDlsBlock), 0, stream, hists, (long long)count, prm, state);
    FMT_HIP_CHECK(hipGetLastError());
    return FMT_OK;
}

}  // namespace fmt
