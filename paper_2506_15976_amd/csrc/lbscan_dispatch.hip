// Launch-shape heuristics of the forward path.
#include "lbscan_internal.h"

namespace lbscan {
namespace {

struct Shape { int waves_log2, nseg, seg_tiles; };

// The row-per-lane kernel runs one wave per (64 rows, state group, segment).
// MI355X has 256 CUs x 4 SIMDs; the kernel needs a few waves per SIMD to cover
// LDS and memory latency.
//  * The N states of a row are split over 4 waves of the block (4 states each):
//    measured best at every workload shape (one wave with all 16 states needs
//    256 registers; 8 waves repeat too much per-token work).
//  * If the rows alone cannot fill the chip even with 8 waves per 64 rows, they
//    are cut into segments scanned in parallel: a summary launch, the carry
//    chain, then the full pass started from the carried-in states.  That costs a
//    second read of x, delta, Bm and ~60% more arithmetic, so only when rows are
//    scarce.
Shape pick_shape(const FwdParams& p)
{
    const long nrb = (long)((p.dim + 63) / 64) * p.batch;
    const int max_log2 = p.dstate > 8 ? 3 : (p.dstate > 4 ? 2 : (p.dstate > 2 ? 1 : 0));
    const int ntiles = (p.seqlen + kFwdTileTokens - 1) / kFwdTileTokens;
    Shape s{0, 1, ntiles};
    s.waves_log2 = max_log2 < 2 ? max_log2 : 2;
    long want_seg = 1;
    if ((nrb << max_log2) < 2048) {
        const int wl = max_log2 < 2 ? max_log2 : 2;
        s.waves_log2 = wl;
        want_seg = (2560 + (nrb << wl) - 1) / (nrb << wl);       // about 2.5 waves per SIMD (measured best)
    }
    if (p.force_waves_log2 >= 0) s.waves_log2 = p.force_waves_log2 < max_log2 ? p.force_waves_log2 : max_log2;
    if (p.force_nseg >= 1) want_seg = p.force_nseg;
    if (want_seg > 1) {
        int st = (int)((ntiles + want_seg - 1) / want_seg);
        if (p.force_nseg < 1 && st < 2) st = 2;               // at least 64 tokens per segment
        if (st < 1) st = 1;
        s.seg_tiles = st;
        s.nseg = (ntiles + st - 1) / st;
    }
    return s;
}

size_t carry_floats(const FwdParams& p, int nseg)
{
    return (size_t)nseg * p.batch * p.dim * (size_t)p.dstate;
}

}  // namespace

size_t fwd_workspace_bytes(const FwdParams& p)
{
    if (p.batch == 0 || p.dim == 0 || p.seqlen == 0) return 0;
    const Shape s = pick_shape(p);
    if (s.nseg <= 1) return 0;
    return (carry_floats(p, s.nseg) + (size_t)s.nseg * p.batch * p.dim) * sizeof(float);
}

hipError_t launch_fwd(FwdParams p, void* workspace, hipStream_t stream)
{
    if (p.batch == 0 || p.dim == 0 || p.seqlen == 0) return hipSuccess;
    const Shape s = pick_shape(p);
    auto launch = [&](const FwdParams& q) {
        return q.dtype == 0 ? launch_fwd_rowlane_f32(q, s.waves_log2, stream)
                            : launch_fwd_rowlane_bf16(q, s.waves_log2, stream);
    };
    p.nseg = s.nseg;
    p.seg_tiles = s.seg_tiles;
    p.summary_only = 0;
    p.carry = nullptr;
    p.dsum = nullptr;
    if (s.nseg > 1) {
        if (!workspace) return hipErrorInvalidValue;
        p.carry = static_cast<float*>(workspace);
        p.dsum = p.carry + carry_floats(p, s.nseg);
        FwdParams q = p;
        q.summary_only = 1;
        hipError_t e = launch(q);
        if (e != hipSuccess) return e;
        e = launch_carry_chain(p, stream);
        if (e != hipSuccess) return e;
    }
    return launch(p);
}

// ---- backward ----------------------------------------------------------------

static size_t ckpt_floats(const FwdParams& f)
{
    const size_t ntiles = (f.seqlen + kTileTokens - 1) / kTileTokens;
    return ntiles * f.batch * f.dim * (size_t)f.dstate;
}

size_t bwd_workspace_bytes(const FwdParams& f)
{
    if (f.batch == 0 || f.dim == 0 || f.seqlen == 0) return 0;
    const size_t ntiles = (f.seqlen + kTileTokens - 1) / kTileTokens;
    size_t fl = ckpt_floats(f) + ntiles * f.batch * f.dim;           // ckpt + cum
    if (f.dtype != 0) fl += 2 * (size_t)f.batch * f.dstate * f.seqlen;   // fp32 dBm, dCm
    return fl * sizeof(float);
}

hipError_t launch_bwd(const FwdParams& f, BwdParams p, void* dBm, void* dCm, void* workspace,
                      hipStream_t stream)
{
    if (f.batch == 0 || f.dim == 0 || f.seqlen == 0) return hipSuccess;
    if (!workspace) return hipErrorInvalidValue;
    const size_t ntiles = (f.seqlen + kTileTokens - 1) / kTileTokens;
    const long bnl = (long)f.batch * f.dstate * f.seqlen;
    float* ckpt = static_cast<float*>(workspace);
    float* cum = ckpt + ckpt_floats(f);
    float* acc = cum + ntiles * f.batch * f.dim;
    p.dBacc = f.dtype == 0 ? static_cast<float*>(dBm) : acc;
    p.dCacc = f.dtype == 0 ? static_cast<float*>(dCm) : acc + bnl;
    p.ckpt = ckpt;

    hipError_t e;
    if ((e = launch_zero(p.dBacc, bnl, stream)) != hipSuccess) return e;
    if ((e = launch_zero(p.dCacc, bnl, stream)) != hipSuccess) return e;
    if ((e = launch_zero(p.dA, (long)f.dim * f.dstate, stream)) != hipSuccess) return e;
    if ((e = launch_zero(p.dDskip, f.dim, stream)) != hipSuccess) return e;
    if ((e = launch_zero(p.dbias, f.dim, stream)) != hipSuccess) return e;

    // checkpoint pass: the forward kernel in summary mode over whole rows
    FwdParams q = f;
    q.force_nseg = 1;
    const Shape s = pick_shape(q);
    q.nseg = 1;
    q.seg_tiles = (f.seqlen + kFwdTileTokens - 1) / kFwdTileTokens;
    q.summary_only = 1;
    q.carry = nullptr;
    q.dsum = nullptr;
    q.ckpt = ckpt;
    q.cum = cum;
    e = q.dtype == 0 ? launch_fwd_rowlane_f32(q, s.waves_log2, stream)
                     : launch_fwd_rowlane_bf16(q, s.waves_log2, stream);
    if (e != hipSuccess) return e;

    e = f.dtype == 0 ? launch_bwd_rowlane_f32(p, stream) : launch_bwd_rowlane_bf16(p, stream);
    if (e != hipSuccess) return e;
    if (f.dtype != 0) {
        if ((e = launch_convert_bf16(p.dBacc, dBm, bnl, stream)) != hipSuccess) return e;
        if ((e = launch_convert_bf16(p.dCacc, dCm, bnl, stream)) != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace lbscan
