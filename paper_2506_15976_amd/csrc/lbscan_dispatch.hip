// Launch-shape heuristics of the forward path.
#include "lbscan_internal.h"

namespace lbscan {
namespace {

struct Shape { int waves_log2, nseg, seg_tiles; };

// Up to this many segments the full forward pass folds the carry chain itself.
constexpr int kFoldChainSegments = 16;

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
        // three blocks per CU are resident (LDS): aim at 3 x 256 blocks in all
        s.waves_log2 = max_log2 < 2 ? max_log2 : 2;
        want_seg = (768 + nrb - 1) / nrb;
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

// The chunk-per-lane kernel (one wave per row, 1024-token chunks) against the
// row-per-lane kernels, measured on MI355X (us, row-per-lane / chunk-per-lane):
//   B x D = 8 x 768,  L = 4096, bf16: 213 / 161      fp32: 217 / 180
//   32 x 768, L = 2048, bf16: 368 / 287               16 x 768, L = 2048, fp32: 204 / 186
//   8 x 384,  L = 4096, bf16: 132 / 83                16 x 768, L = 1024, fp32: 111 / 94
//   2 x 768,  L = 8192, bf16: 139 / 129               fp32: 138 / 150
//   64 x 384, L = 1024, fp32: 187 / 187 (rows not cut by the row-per-lane path)
// It needs rows enough for a wave each (four rows per block, three blocks per CU),
// and chunks that are mostly full.  With fp32 storage it wins where the row-per-lane
// kernels would have to cut rows into segments; with bf16 storage always.  It leaves
// no checkpoints for a backward call.
bool use_chunk_mapping(const FwdParams& p, const Shape& s, const float* saved)
{
    if (p.force_mapping == 1) return false;
    FwdParams q = p;
    q.ckpt = nullptr; q.summary_only = 0;
    if (!fwd_chunk_supported(q)) return false;
    if (saved && s.nseg == 1) return false;
    if (p.force_mapping == 2) return true;
    const long rows = (long)p.batch * p.dim;
    const long chunk = 1024, nchunks = (p.seqlen + chunk - 1) / chunk;
    if (p.seqlen * 5 < nchunks * chunk * 4) return false;             // chunks less than 80% full
    if (p.dtype != 0) return rows >= 1536;
    return rows >= 3072 && s.nseg > 1;
}

}  // namespace

size_t fwd_workspace_bytes(const FwdParams& p)
{
    if (p.batch == 0 || p.dim == 0 || p.seqlen == 0) return 0;
    const Shape s = pick_shape(p);
    if (s.nseg <= 1) return 0;
    return (carry_floats(p, s.nseg) + (size_t)s.nseg * p.batch * p.dim) * sizeof(float);
}

size_t saved_state_bytes(const FwdParams& p)
{
    if (p.batch == 0 || p.dim == 0 || p.seqlen == 0) return 0;
    if (pick_shape(p).nseg > 1) return 0;
    const size_t ntiles16 = (p.seqlen + kTileTokens - 1) / kTileTokens;
    return ntiles16 * p.batch * p.dim * (size_t)p.dstate * sizeof(float);
}

hipError_t launch_fwd(FwdParams p, void* workspace, float* saved, hipStream_t stream)
{
    if (p.batch == 0 || p.dim == 0 || p.seqlen == 0) return hipSuccess;
    const Shape s = pick_shape(p);
    if (use_chunk_mapping(p, s, saved)) return launch_fwd_chunk(p, stream);
    p.ckpt = (saved && s.nseg == 1) ? saved : nullptr;
    p.cum = nullptr;
    auto launch = [&](const FwdParams& q) {
        return q.dtype == 0 ? launch_fwd_rowlane_f32(q, s.waves_log2, stream)
                            : launch_fwd_rowlane_bf16(q, s.waves_log2, stream);
    };
    p.nseg = s.nseg;
    p.seg_tiles = s.seg_tiles;
    p.summary_only = 0;
    // (uncut rows read the entering state from h0)
    p.carry = nullptr;
    p.dsum = nullptr;
    p.fold_chain = 0;
    if (s.nseg > 1) {
        if (!workspace) return hipErrorInvalidValue;
        p.carry = static_cast<float*>(workspace);
        p.dsum = p.carry + carry_floats(p, s.nseg);
        FwdParams q = p;
        q.summary_only = 1;
        hipError_t e = launch(q);
        if (e != hipSuccess) return e;
        // few segments: the full pass folds the chain itself (one launch less);
        // many: the chain kernel, a shuffle scan over the segments
        p.fold_chain = s.nseg <= kFoldChainSegments;
        if (!p.fold_chain) {
            e = launch_carry_chain(p, stream);
            if (e != hipSuccess) return e;
        }
    }
    return launch(p);
}

// ---- window lengths without a compiled kernel ---------------------------------
//
// Eq. 8 splits into the plain forward scan (sum_n Cm f + Dskip x: the kernel
// compiled for window 1, entering and leaving states included) and the local
// backward part sum_n Cm g, which never crosses a window end.  Pass 1 leaves the
// first in fp32 (in y itself when y is fp32, else at the start of the
// workspace); pass 2 adds the second for any window length, gates and writes y.

size_t fwd_generic_workspace_bytes(const FwdParams& p)
{
    if (p.batch == 0 || p.dim == 0 || p.seqlen == 0) return 0;
    FwdParams p1 = p;
    p1.window = 1;
    const size_t partial = p.dtype == 0 ? 0 : (size_t)p.batch * p.dim * p.seqlen * sizeof(float);
    return partial + fwd_workspace_bytes(p1);
}

hipError_t launch_fwd_generic(FwdParams p, void* workspace, hipStream_t stream)
{
    if (p.batch == 0 || p.dim == 0 || p.seqlen == 0) return hipSuccess;
    float* partial = static_cast<float*>(p.y);
    char* scratch = static_cast<char*>(workspace);
    if (p.dtype != 0) {
        if (!workspace) return hipErrorInvalidValue;
        partial = static_cast<float*>(workspace);
        scratch += (size_t)p.batch * p.dim * p.seqlen * sizeof(float);
    }
    FwdParams p1 = p;
    p1.window = 1; p1.z = nullptr; p1.y = partial; p1.y_is_f32 = 1;
    hipError_t e = launch_fwd(p1, scratch, nullptr, stream);
    if (e != hipSuccess) return e;

    FwdParams p2 = p;
    p2.generic_window = 1; p2.Dskip = nullptr; p2.yprev = partial;
    p2.h0 = nullptr; p2.hT = nullptr; p2.carry = nullptr; p2.dsum = nullptr;
    p2.ckpt = nullptr; p2.cum = nullptr; p2.summary_only = 0; p2.seg_tiles = 0;
    // segments of whole windows, at least 64 steps each, enough of them to fill the chip
    const long nrb = (long)((p.dim + 63) / 64) * p.batch;
    const long M = p.window, L = p.seqlen;
    const long nw = (L + M - 1) / M;
    long want_seg = nrb < 768 ? (768 + nrb - 1) / nrb : 1;
    if (p.force_nseg >= 1) want_seg = p.force_nseg;
    long wps = (nw + want_seg - 1) / want_seg;
    if (p.force_nseg < 1 && wps * M < 64) wps = (64 + M - 1) / M;
    if (wps < 1) wps = 1;
    p2.seg_tokens = (int)(wps * M);
    p2.nseg = (int)((L + p2.seg_tokens - 1) / p2.seg_tokens);
    const int wl = pick_shape(p).waves_log2;
    return p2.dtype == 0 ? launch_fwd_rowlane_f32(p2, wl, stream)
                         : launch_fwd_rowlane_bf16(p2, wl, stream);
}

// ---- backward ----------------------------------------------------------------

namespace {

// A window that straddles the start of a 16-token tile needs the part of the adjoint
// of the local backward state that enters the tile from the left (BwdParams::gck).
bool needs_gamma_checkpoints(const FwdParams& f)
{
    return f.seqlen > kTileTokens && kTileTokens % f.window != 0;
}

struct BwdLayout {
    Shape shape;            // segments in forward tiles (32 tokens)
    size_t ntiles16;        // backward tiles (16 tokens) per row
    size_t ckpt, cum, gck, carry, dsum, psi, part;   // float offsets into the workspace
    size_t total;           // floats
};

BwdLayout bwd_layout(const FwdParams& f)
{
    BwdLayout l;
    l.shape = pick_shape(f);
    if (l.shape.nseg > 1 && f.force_nseg < 1) {
        // the backward kernel runs two blocks per CU: one round of 512 blocks (measured:
        // 4096-token shape 5 segments 841 us, 8: 878, 16: 838; whole-slide shape 128
        // segments 515 us, 192: 558, 256: 538)
        const long nrb = (long)((f.dim + 63) / 64) * f.batch;
        const long ntiles = (f.seqlen + kFwdTileTokens - 1) / kFwdTileTokens;
        long want = 512 / nrb;
        if (want < 1) want = 1;
        long st = (ntiles + want - 1) / want;
        if (st < 2) st = 2;
        if (st > ntiles) st = ntiles;
        l.shape.seg_tiles = (int)st;
        l.shape.nseg = (int)((ntiles + st - 1) / st);
    }
    const bool gamma = needs_gamma_checkpoints(f);
    if (gamma && l.shape.nseg > 1) {
        // segments must start at window starts: whole windows per segment
        long g = f.window, r = kFwdTileTokens;
        while (r) { const long t = g % r; g = r; r = t; }          // gcd(window, 32)
        const long unit = f.window / g;                            // forward tiles per window period
        const long ntiles = (f.seqlen + kFwdTileTokens - 1) / kFwdTileTokens;
        long st = ((l.shape.seg_tiles + unit - 1) / unit) * unit;
        if (st >= ntiles) st = ntiles;
        l.shape.seg_tiles = (int)st;
        l.shape.nseg = (int)((ntiles + st - 1) / st);
    }
    const size_t rows = (size_t)f.batch * f.dim, N = f.dstate;
    l.ntiles16 = (f.seqlen + kTileTokens - 1) / kTileTokens;
    size_t o = 0;
    l.ckpt = o; o += l.ntiles16 * rows * N;
    l.cum = o;  o += l.ntiles16 * rows;
    l.gck = o;  if (gamma) o += l.ntiles16 * rows * N;
    const size_t ns = l.shape.nseg > 1 ? l.shape.nseg : 0;
    l.carry = o; o += ns * rows * N;
    l.dsum = o;  o += ns * rows;
    l.psi = o;   o += ns * rows * N;
    l.part = o;                                // per block of 64 channels: fp32 dBm, dCm
    o += 2 * (size_t)((f.dim + 63) / 64) * f.batch * N * f.seqlen;
    l.total = o;
    return l;
}

}  // namespace

size_t bwd_workspace_bytes(const FwdParams& f)
{
    if (f.batch == 0 || f.dim == 0 || f.seqlen == 0) return 0;
    return bwd_layout(f).total * sizeof(float);
}

hipError_t launch_bwd(const FwdParams& f, BwdParams p, void* dBm, void* dCm, void* workspace,
                      const float* saved, const float* dhT, hipStream_t stream)
{
    if (f.batch == 0 || f.dim == 0 || f.seqlen == 0) return hipSuccess;
    if (!workspace) return hipErrorInvalidValue;
    const BwdLayout l = bwd_layout(f);
    const Shape& s = l.shape;
    const bool gamma = needs_gamma_checkpoints(f);
    float* ws = static_cast<float*>(workspace);
    const long bnl = (long)f.batch * f.dstate * f.seqlen;
    p.dBpart = ws + l.part;
    p.ckpt = ws + l.ckpt;
    p.cum = ws + l.cum;
    p.gck = gamma ? ws + l.gck : nullptr;
    p.nseg = s.nseg;
    p.seg_tiles = s.seg_tiles * (kFwdTileTokens / kTileTokens);
    // uncut rows: the entering state and the gradient arriving at the leaving state
    // take the places of the chained values
    p.carry = s.nseg > 1 ? ws + l.carry : f.h0;
    p.psi_in = s.nseg > 1 ? ws + l.psi : dhT;

    hipError_t e;
    const ZeroMany z{{p.dA, p.dDskip, p.dbias, nullptr, nullptr},
                     {(long)f.dim * f.dstate, f.dim, f.dim, 0, 0}};
    if ((e = launch_zero_many(z, stream)) != hipSuccess) return e;

    // after the backward kernel: dBm, dCm from the per-block partial sums
    auto finish = [&]() -> hipError_t {
        const int nbx = (f.dim + 63) / 64;
        return f.dtype == 0 ? launch_reduce_f32(p.dBpart, dBm, dCm, bnl, nbx, stream)
                            : launch_reduce_bf16(p.dBpart, dBm, dCm, bnl, nbx, stream);
    };

    if (saved && s.nseg == 1 && !gamma) {
        // the forward call left the checkpoints (entering state included): no summary pass
        p.ckpt = saved;
        p.cum = nullptr;
        p.carry = nullptr;
        e = f.dtype == 0 ? launch_bwd_rowlane_f32(p, stream) : launch_bwd_rowlane_bf16(p, stream);
        return e != hipSuccess ? e : finish();
    }

    // summary pass (the forward kernel in summary mode): checkpoints of f for every
    // 16-token tile and, when the rows are cut, the per-segment summaries of the
    // forward and of the right-to-left recurrence; for windows that straddle tile
    // starts also the checkpoints of the adjoint of the local backward state
    FwdParams q = f;
    q.nseg = s.nseg;
    q.seg_tiles = s.seg_tiles;
    q.summary_only = 1;
    q.ckpt = ws + l.ckpt;
    q.cum = ws + l.cum;
    q.gck = gamma ? ws + l.gck : nullptr;
    q.carry = s.nseg > 1 ? ws + l.carry : nullptr;
    q.dsum = s.nseg > 1 ? ws + l.dsum : nullptr;
    q.psi = s.nseg > 1 ? ws + l.psi : nullptr;
    q.dout = p.dout;
    e = q.dtype == 0 ? launch_fwd_rowlane_f32(q, s.waves_log2, stream)
                     : launch_fwd_rowlane_bf16(q, s.waves_log2, stream);
    if (e != hipSuccess) return e;
    if (s.nseg > 1) {
        if ((e = launch_carry_chain(q, stream)) != hipSuccess) return e;
        if ((e = launch_carry_chain_reverse(q, q.psi, dhT, stream)) != hipSuccess) return e;
    }

    e = f.dtype == 0 ? launch_bwd_rowlane_f32(p, stream) : launch_bwd_rowlane_bf16(p, stream);
    return e != hipSuccess ? e : finish();
}

}  // namespace lbscan
