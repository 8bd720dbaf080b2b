// Row-per-lane backward kernels, bf16 storage (fp32 arithmetic).
#include "lbscan_device.h"
#include "lbscan_internal.h"
#include "lbscan_bwd_rowlane.inc"

namespace lbscan {
hipError_t launch_bwd_rowlane_bf16(const BwdParams& p, hipStream_t stream)
{
    return launch_bwd_t<bf16_t>(p, stream);
}
hipError_t launch_reduce_bf16(const float* part, void* dB, void* dC, long bnl, int nbx, hipStream_t stream)
{
    return launch_reduce_t<bf16_t>(part, dB, dC, bnl, nbx, stream);
}
}  // namespace lbscan
