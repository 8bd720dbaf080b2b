// Host-side declarations shared by the lbscan translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "lbscan_device.h"

namespace lbscan {

// Arguments of one forward launch, already validated by the C entry points.
struct FwdParams {
    int batch, dim, dstate, seqlen;
    int window;
    int dtype;     // LBSCAN_FP32 / LBSCAN_BF16
    int softplus;
    int reverse;
    TokenOrder order;   // scan order of a row's tokens (kind 0: as stored)
    const void* x;
    const void* delta;
    const void* Bm;
    const void* Cm;
    const void* z;        // nullable
    const float* A;
    const float* Dskip;   // nullable
    const float* bias;    // nullable
    const float* yprev;   // nullable, fp32 (B,D,L): added to y before the gate
    void* y;              // element type = dtype, or fp32 when y_is_f32
    int y_is_f32;         // write y as fp32 whatever dtype says (first pass of the two-pass scan)
    int force_waves_log2; // >= 0: override the state-split heuristic (tests, tuning)
    int force_nseg;       // >= 1: override the number of segments a row is cut into
    int force_mapping;    // 0: heuristic; 1: row-per-lane kernels; 2: chunk-per-lane kernel where it applies
    // Long rows are cut into nseg segments of seg_tiles forward tiles (kFwdTileTokens tokens each), one
    // block per (64 rows, segment).  carry: (nseg, N, B*D) states entering each
    // segment (read by the full pass; written by the summary pass as the states a
    // segment reaches from zero); dsum: (nseg, B*D) sum of time steps per segment.
    int nseg, seg_tiles;
    int summary_only;
    int fold_chain;       // full pass: fold the chain over the summaries in the kernel
    float* carry;         // nullable when nseg == 1
    float* dsum;
    // summary pass only: per-tile checkpoints for the backward pass (nullable):
    // ckpt (ntiles, N, B*D) state at the start of each tile, cum (ntiles, B*D)
    // time-step sum up to there, both counted from the start of the segment
    float* ckpt;
    float* cum;
    // summary pass for a segmented backward pass (nullable): dout (B,D,L) in, and
    // psi (nseg, B*D, N) out: the segment's summary of the right-to-left recurrence
    const void* dout;
    float* psi;
    // summary pass for window lengths that 16 is not a multiple of (nullable):
    // gck (ntiles16, N, B*D), see lbscan_fwd_rowlane.inc MODE 2
    float* gck;
    // forward state entering the row (nullable: zeros) and leaving it (nullable), (B*D, N)
    const float* h0;
    float* hT;
    // second pass of the path for window lengths without a compiled kernel: only
    // the local backward part, added to yprev; window is then the run-time window
    // length and the grid has one block per (64 rows, seg_tokens logical steps)
    int generic_window;
    int seg_tokens;
};

// Arguments of one backward launch: the forward inputs plus the gradient tensors.
struct BwdParams {
    int batch, dim, dstate, seqlen;
    int window;
    int dtype;
    int softplus;
    int reverse;
    TokenOrder order;
    const void* x;
    const void* delta;
    const void* Bm;
    const void* Cm;
    const void* z;        // nullable
    const float* A;
    const float* Dskip;   // nullable
    const float* bias;    // nullable
    const void* dout;
    void* dx;
    void* ddelta;
    void* dz;             // nullable iff z is
    float* dBpart;        // fp32 partial sums [dBm | dCm][block of 64 channels][B][N][L]: every
                          // block of the backward kernel writes its own share
    float* dA;            // (D,N) zeroed
    float* dDskip;        // (D) zeroed, nullable
    float* dbias;         // (D) zeroed, nullable
    const float* ckpt;    // (ntiles, N, B*D): f at the first step of every tile, counted
                          // from the start of the tile's segment
    // rows cut into nseg segments of seg_tiles backward tiles (16 tokens each):
    int nseg, seg_tiles;
    const float* cum;     // (ntiles, B*D): time-step sum from the segment start to the tile
    const float* carry;   // (nseg, B*D, N): forward state entering each segment (null: zeros)
    const float* psi_in;  // (nseg, B*D, N): psi entering each segment from the right
    const float* gck;     // (ntiles, N, B*D), nullable: abar_{t-1} gamma_{t-1} entering each tile
                          // (windows that straddle tile starts)
    float* dh0;           // (B*D, N), nullable: psi leaving the row on the left
};

// Arguments of the pre-scan convolution kernels (lbscan_conv.hip).
struct ConvParams {
    int batch, dim, seqlen, width;
    int dtype, activation, reverse;
    const void* x;
    const float* weight;
    const float* bias;    // nullable
    void* y;              // forward only
    const void* dy;       // backward only
    void* dx;
    float* dweight;       // (D,K), zeroed by the launcher
    float* dbias;         // (D), nullable
    int items_per_wave;   // set by the launcher
};

#ifndef LBSCAN_BWD_TILE
#define LBSCAN_BWD_TILE 16
#endif
constexpr int kTileTokens = LBSCAN_BWD_TILE;      // tokens per tile of the backward kernel = checkpoint spacing
#ifndef LBSCAN_FWD_TILE
#define LBSCAN_FWD_TILE 32
#endif
constexpr int kFwdTileTokens = LBSCAN_FWD_TILE;   // tokens per tile of the forward kernel (32: 128 bytes of an fp32 row)

// Window lengths with a compiled kernel.
inline bool window_supported(int M) { return M == 1 || M == 2 || M == 4 || M == 8 || M == 16; }

// Row-per-lane forward kernel family (lbscan_fwd_rowlane.inc), one translation
// unit per storage type.  waves_log2: log2 of the waves the states are split over.
hipError_t launch_fwd_rowlane_f32(const FwdParams& p, int waves_log2, hipStream_t stream);
hipError_t launch_fwd_rowlane_bf16(const FwdParams& p, int waves_log2, hipStream_t stream);

// Chunk-per-lane forward kernel (lbscan_fwd_chunk.hip): one wave per row, 16 tokens
// per lane, no workspace.  fwd_chunk_supported: p is within what it implements.
bool fwd_chunk_supported(const FwdParams& p);
hipError_t launch_fwd_chunk(const FwdParams& p, hipStream_t stream);

// Picks the launch shape for the sizes in p and launches the forward pass
// (several kernels when rows are cut into segments).  workspace must hold
// fwd_workspace_bytes(p) bytes when that is non-zero.
// saved (nullable): buffer of saved_state_bytes(p) bytes to fill with checkpoints for
// a backward call (ignored when that size is 0).
hipError_t launch_fwd(FwdParams p, void* workspace, float* saved, hipStream_t stream);
size_t fwd_workspace_bytes(const FwdParams& p);
// The same for a window length without a compiled kernel (p.window <= p.seqlen, any
// value): two launches, the plain forward scan and the local backward part.
hipError_t launch_fwd_generic(FwdParams p, void* workspace, hipStream_t stream);
size_t fwd_generic_workspace_bytes(const FwdParams& p);
// Bytes of the saved-state buffer, 0 when rows are cut into segments (the backward
// pass then needs its own summary pass anyway).
size_t saved_state_bytes(const FwdParams& p);

// Backward kernels (lbscan_bwd_rowlane.inc), one translation unit per storage type.
hipError_t launch_bwd_rowlane_f32(const BwdParams& p, hipStream_t stream);
hipError_t launch_bwd_rowlane_bf16(const BwdParams& p, hipStream_t stream);
// dBm, dCm (storage type) = the partial sums of BwdParams::dBpart added over the nbx
// blocks of 64 channels; bnl = B * N * L.
hipError_t launch_reduce_f32(const float* part, void* dB, void* dC, long bnl, int nbx, hipStream_t stream);
hipError_t launch_reduce_bf16(const float* part, void* dB, void* dC, long bnl, int nbx, hipStream_t stream);
// Sets n floats to zero with a kernel (a memset node must not be recorded into
// a captured graph).
hipError_t launch_zero(float* dst, long n, hipStream_t stream);
// The same for several buffers in one launch (null or empty entries are skipped).
constexpr int kZeroMany = 5;
struct ZeroMany { float* dst[kZeroMany]; long n[kZeroMany]; };
hipError_t launch_zero_many(ZeroMany z, hipStream_t stream);

// Whole backward pass: zero the accumulators, checkpoint pass, backward kernel,
// conversion of dBm / dCm when the storage type is not fp32.  dBm / dCm are the
// caller's outputs; workspace must hold bwd_workspace_bytes(f) bytes.  f.window is
// any window length >= 1 (1, 2, 4 run with a compiled window structure, all others
// with run-time window masks).
// saved (nullable): checkpoints left by launch_fwd on the same inputs.
// dhT (nullable): gradient arriving at the state that leaves the row.
hipError_t launch_bwd(const FwdParams& f, BwdParams p, void* dBm, void* dCm, void* workspace,
                      const float* saved, const float* dhT, hipStream_t stream);
size_t bwd_workspace_bytes(const FwdParams& f);

// Depthwise causal convolution + SiLU along the sequence and its gradient.
hipError_t launch_conv1d_fwd(const ConvParams& p, hipStream_t stream);
hipError_t launch_conv1d_bwd(const ConvParams& p, hipStream_t stream);

// Chains the per-segment summaries into the states entering each segment
// (lbscan_carry.hip): carry[s] <- exclusive scan over s of (exp(A*dsum), carry),
// started from p.h0 (zeros when null).
hipError_t launch_carry_chain(const FwdParams& p, hipStream_t stream);
// The same chain over `buf` (nseg, B*D, N) walking the segments right to left,
// started from init (B*D, N), zeros when null.
hipError_t launch_carry_chain_reverse(const FwdParams& p, float* buf, const float* init,
                                      hipStream_t stream);
// dst[i] = src[i] (zeros when src is null), n floats.
hipError_t launch_copy(float* dst, const float* src, long n, hipStream_t stream);

}  // namespace lbscan
