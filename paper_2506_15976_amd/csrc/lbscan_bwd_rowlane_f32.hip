// Row-per-lane backward kernels, fp32 storage.
#include "lbscan_device.h"
#include "lbscan_internal.h"
#include "lbscan_bwd_rowlane.inc"

namespace lbscan {
hipError_t launch_bwd_rowlane_f32(const BwdParams& p, hipStream_t stream)
{
    return launch_bwd_t<float>(p, stream);
}
hipError_t launch_reduce_f32(const float* part, void* dB, void* dC, long bnl, int nbx, hipStream_t stream)
{
    return launch_reduce_t<float>(part, dB, dC, bnl, nbx, stream);
}
}  // namespace lbscan
