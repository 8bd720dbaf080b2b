// Row-per-lane forward kernels, fp32 storage.
#include "lbscan_device.h"
#include "lbscan_internal.h"
#include "lbscan_fwd_rowlane.inc"

namespace lbscan {
hipError_t launch_fwd_rowlane_f32(const FwdParams& p, int waves_log2, hipStream_t stream)
{
    return launch_rowlane_t<float>(p, waves_log2, stream);
}
}  // namespace lbscan
