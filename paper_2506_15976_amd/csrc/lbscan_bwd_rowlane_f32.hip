// Row-per-lane backward kernels, fp32 storage.
#include "lbscan_device.h"
#include "lbscan_internal.h"
#include "lbscan_bwd_rowlane.inc"
#include "lbscan_bwd_local.inc"

namespace lbscan {
hipError_t launch_bwd_rowlane_f32(const BwdParams& p, hipStream_t stream)
{
    return launch_bwd_t<float>(p, stream);
}
hipError_t launch_bwd_local_f32(const BwdParams& p, hipStream_t stream)
{
    return launch_bwd_local_t<float>(p, stream);
}
hipError_t launch_convert_f32(const float* src, void* dst, long n, hipStream_t stream)
{
    return launch_convert_t<float>(src, dst, n, stream);
}
}  // namespace lbscan
