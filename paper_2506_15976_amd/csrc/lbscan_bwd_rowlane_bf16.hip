// Row-per-lane backward kernels, bf16 storage (fp32 arithmetic).
#include "lbscan_device.h"
#include "lbscan_internal.h"
#include "lbscan_bwd_rowlane.inc"
#include "lbscan_bwd_local.inc"

namespace lbscan {
hipError_t launch_bwd_rowlane_bf16(const BwdParams& p, hipStream_t stream)
{
    return launch_bwd_t<bf16_t>(p, stream);
}
hipError_t launch_bwd_local_bf16(const BwdParams& p, hipStream_t stream)
{
    return launch_bwd_local_t<bf16_t>(p, stream);
}
hipError_t launch_convert_bf16(const float* src, void* dst, long n, hipStream_t stream)
{
    return launch_convert_t<bf16_t>(src, dst, n, stream);
}
}  // namespace lbscan
