// Row-per-lane forward kernels, bf16 storage (fp32 arithmetic).
#include "lbscan_device.h"
#include "lbscan_internal.h"
#include "lbscan_fwd_rowlane.inc"

namespace lbscan {
hipError_t launch_fwd_rowlane_bf16(const FwdParams& p, int waves_log2, hipStream_t stream)
{
    return launch_rowlane_t<bf16_t>(p, waves_log2, stream);
}
}  // namespace lbscan
