// Launch-shape heuristics of the forward path.
#include "lbscan_internal.h"

namespace lbscan {

// The row-per-lane kernel runs one wave per 64 rows and state group.  MI355X
// has 256 CUs x 4 SIMDs; the scan is bound by VALU issue, which needs a few
// waves per SIMD to overlap LDS and memory latency.  Split the states over
// more waves until there are about 4 waves per SIMD (splitting duplicates the
// per-token work of a row in every wave, so no further than needed).
static int pick_waves_log2(const FwdParams& p)
{
    const long row_blocks = (long)((p.dim + 63) / 64) * p.batch;
    const int max_log2 = p.dstate > 8 ? 3 : (p.dstate > 4 ? 2 : (p.dstate > 2 ? 1 : 0));
    if (p.force_waves_log2 >= 0) return p.force_waves_log2 < max_log2 ? p.force_waves_log2 : max_log2;
    int w = 0;
    while (w < max_log2 && (row_blocks << w) < 4096) ++w;
    return w;
}

hipError_t launch_fwd(const FwdParams& p, hipStream_t stream)
{
    if (p.batch == 0 || p.dim == 0 || p.seqlen == 0) return hipSuccess;
    const int w = pick_waves_log2(p);
    return p.dtype == 0 ? launch_fwd_rowlane_f32(p, w, stream) : launch_fwd_rowlane_bf16(p, w, stream);
}

}  // namespace lbscan
