#include "fmt_internal.h"
namespace fmt {
int launch_gemm(int, int, int64_t, int64_t, int64_t, const float *, int64_t, const float *, int64_t, float *, int64_t,
                fmt_format_t, const QuantParams &, hipStream_t)
{
    return FMT_ERR_HIP;
}
}  // namespace fmt
