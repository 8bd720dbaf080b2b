/*
 * lbscan - locally bi-directional selective scan (LBMamba, arXiv 2506.15976)
 *          for AMD MI355X (gfx950).  C ABI, no C++ or framework types.
 *
 * Notation: B = batch, D = channels (the paper's E), N = state size,
 * L = sequence length, M = window length.
 *
 * Per (b, d, n), with the time step of Sec. 3.1 Eq. 3 / Algorithm 1
 *     dt_t   = softplus?(delta[b,d,t] + delta_bias[d])
 *     abar_t = exp(dt_t * A[d,n])           u_t = dt_t * Bm[b,n,t] * x[b,d,t]
 * the library computes
 *     f_t = abar_t f_{t-1} + u_t,  f_{-1} = h0 or 0     global forward scan (Eq. 1)
 *     g_t = 0 at the last step of each window [kM, kM+M-1] (and at t = L-1),
 *           abar_t (g_{t+1} + u_{t+1}) otherwise        local backward scan (Eq. 7,
 *           without its own input term: the "B x" counted once, Eq. 8)
 *     y_t = sum_n Cm[b,n,t] (f_t + g_t) + Dskip[d] x_t  (Eq. 8)
 *     out_t = y_t * SiLU(z_t) when z is given            (Algorithm 1, gate line)
 *
 * Memory layout: every tensor is dense with the last index contiguous:
 *     x, delta, z, y, dout, dx, ddelta, dz : (B, D, L)     element type = dtype
 *     Bm, Cm, dBm, dCm                     : (B, N, L)     element type = dtype
 *     A, dA                                : (D, N)        fp32
 *     Dskip, delta_bias and their grads    : (D)           fp32
 *     h0, hT, dh0, dhT                     : (B, D, N)     fp32
 * One B/C group is shared by all channels (Algorithm 1: B, C have shape
 * (B, L, N)); A is real.
 *
 * Ownership: every data pointer is a caller-owned DEVICE pointer.  The library
 * never allocates, frees or synchronises; it enqueues work on the HIP stream
 * passed in (a hipStream_t cast to void*, NULL = default stream) and returns.
 * Outputs are fully overwritten.  Calls are re-entrant as long as
 * lbscan_set_option is not called concurrently: the only global state is a
 * thread-local last-error string and the process-wide tuning options.
 *
 * Errors: 0 on success, a negative LBSCAN_E* code otherwise; nothing is
 * enqueued when an error is returned before launch.
 */
#ifndef LBSCAN_H
#define LBSCAN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LBSCAN_OK            0
#define LBSCAN_EINVAL       (-1)  /* null required pointer, negative size, window < 1        */
#define LBSCAN_EUNSUPPORTED (-2)  /* dtype, state size or window the GPU path does not cover  */
#define LBSCAN_EWORKSPACE   (-3)  /* workspace missing or smaller than lbscan_workspace_bytes */
#define LBSCAN_EHIP         (-4)  /* HIP launch error; text via lbscan_last_error()           */

#define LBSCAN_FP32 0
#define LBSCAN_BF16 1

#define LBSCAN_MAX_DSTATE 16

typedef struct lbscan_args {
    int32_t batch, dim, dstate, seqlen;  /* B, D, N, L.  B, D or L may be 0: nothing is computed
                                            (the state passes through, reduced gradients are
                                            zero).  N = 0 with B*D*L > 0 is LBSCAN_EUNSUPPORTED
                                            (the result would be Dskip x SiLU(z); no kernel) */
    int32_t window;           /* M >= 1, any value (Sec. 3.2 leaves the window length free;
                                 M >= L is one window).  lbscan_fwd: M in {1,2,4,8,16} (and any
                                 M >= L when L <= 16) runs one fused pass, any other M two
                                 passes over HBM (the plain scan with window 1, then the local
                                 backward part).  lbscan_bwd: one backward kernel for every M;
                                 when 16 is not a multiple of M its checkpoint pass also reads
                                 dout, z, Cm and needs N floats more scratch per 16 tokens */
    int32_t dtype;            /* LBSCAN_FP32 or LBSCAN_BF16: storage type of the (B,D,L) and
                                 (B,N,L) tensors; arithmetic is fp32 either way                */
    int32_t delta_softplus;   /* 0/1: apply softplus to delta + delta_bias (Algorithm 1)      */
    int32_t reverse;          /* 0: as defined above.  1: the same operator applied to the
                                 time-reversed sequence, result reversed back (global scan
                                 runs right to left, windows are anchored at t = L-1); this is
                                 the per-encoder sequence reversal of Sec. 3.3 without a copy  */
    const void  *x;           /* (B,D,L) */
    const void  *delta;       /* (B,D,L) raw: before bias and softplus */
    const void  *Bm;          /* (B,N,L) */
    const void  *Cm;          /* (B,N,L) */
    const void  *z;           /* (B,D,L) or NULL: no gate */
    const float *A;           /* (D,N) */
    const float *Dskip;       /* (D) or NULL: treated as 0 */
    const float *delta_bias;  /* (D) or NULL: treated as 0 */
    void        *y;           /* (B,D,L) out */
    void        *workspace;   /* device scratch of lbscan_workspace_bytes() bytes, or NULL if 0 */
    size_t       workspace_bytes;
    void        *saved_state; /* optional device buffer of lbscan_workspace_bytes(args,
                                 LBSCAN_WS_SAVED) bytes shared by a forward call and the
                                 backward call that follows it.  lbscan_fwd fills it with
                                 checkpoints of the forward states (when the size is not 0
                                 for these shapes); lbscan_bwd given the same buffer starts
                                 from them instead of recomputing them.  NULL: not used. */
    size_t       saved_state_bytes;
    /* Forward state entering and leaving the call, for sequences processed in
       chunks (Algorithm 1 starts from zero: both NULL).  The local backward state
       never crosses a call, so chunk lengths must be multiples of the window for
       the chunks to add up to the whole sequence.  With reverse = 1 the state
       enters at t = L-1 and leaves after t = 0.  Not used by lbscan_bidir_fwd. */
    const float *h0;          /* (B,D,N) or NULL: zeros */
    float       *hT;          /* (B,D,N) out of lbscan_fwd, or NULL: not wanted */
    /* Scan order of a row's tokens (the multi-direction models of Sec. 4.5 / Appendix D
       scan a 2-D token grid also vertically).  LBSCAN_ORDER_SEQUENCE (0, the default of a
       zeroed struct): the tokens as stored.  LBSCAN_ORDER_COLUMNS: the tokens
       [grid_prefix, grid_prefix + grid_h * grid_w) are a grid_h x grid_w grid stored row by
       row and are scanned column by column, top to bottom; tokens before and after the
       grid (class tokens) are scanned in place, before and after it.  The operator is
       applied to the sequence in that order and every (B,D,L) / (B,N,L) tensor, inputs
       and outputs alike, stays in stored order: no reordered copy exists.  reverse = 1
       reverses the scanned sequence.  Kernels then gather token by token.  lbscan_fwd
       with a window length outside {1,2,4,8,16} and lbscan_bidir_fwd support only the
       stored order (LBSCAN_EUNSUPPORTED otherwise); lbscan_bwd supports every window. */
    int32_t scan_order;
    int32_t grid_h, grid_w, grid_prefix;
} lbscan_args;

#define LBSCAN_ORDER_SEQUENCE 0
#define LBSCAN_ORDER_COLUMNS  1

#define LBSCAN_WS_FWD   0
#define LBSCAN_WS_BWD   1
#define LBSCAN_WS_BIDIR 2
#define LBSCAN_WS_SAVED 3   /* size of lbscan_args.saved_state (0: these shapes do not use it) */

/* Forward pass of the locally bi-directional scan (Sec. 3.2, Eq. 7-8, on top of
 * the global forward scan of Eq. 1-3; gate and skip of Algorithm 1 fused in). */
int lbscan_fwd(const lbscan_args *args, void *hip_stream);

/* lbscan_fwd for callers that cannot allocate or hand over scratch: code under HIP
 * graph capture, tight serving loops, harnesses that forbid allocation.  The same
 * computation and the same kernels, with the scratch of long rows (carried states of
 * the row segments) in a fixed device array of LBSCAN_STATIC_SCRATCH_BYTES that the
 * library holds on every GPU it runs on until the process ends; args->workspace is
 * ignored.  Nothing is allocated or freed, here or in the runtime (the array's
 * address is looked up once per device, on the first call there).  Sizes that need
 * more scratch than the array holds (lbscan_workspace_bytes(args, LBSCAN_WS_FWD))
 * return LBSCAN_EWORKSPACE, with the two sizes in lbscan_last_error().  Every call on
 * a GPU shares that GPU's array: calls that overlap on one GPU (different streams)
 * race; calls on one stream are ordered.  Nothing in the array needs clearing
 * between calls (each call writes what it reads). */
#define LBSCAN_STATIC_SCRATCH_BYTES (8u << 20)
int lbscan_fwd_static(const lbscan_args *args, void *hip_stream);

/* Gradients of lbscan_fwd with respect to every input (the paper reports only
 * training throughput, Appendix B; the formulas are the reverse-mode derivative
 * of the forward definition above).  fwd_args names the forward inputs
 * (fwd_args->y is not read; fwd_args->saved_state, if given, must have been filled
 * by lbscan_fwd on the same inputs).  dout is the upstream gradient of out.  dz may be
 * NULL iff fwd_args->z is NULL.  dDskip / ddelta_bias may be NULL iff the
 * corresponding input is NULL.  All outputs are overwritten (not accumulated).
 * dBm and dCm are summed in a fixed order (the same bits on every run); dA, dDskip
 * and ddelta_bias use fp32 atomics and may differ in their last bits between runs. */
int lbscan_bwd(const lbscan_args *fwd_args, const void *dout,
               void *dx, void *ddelta, void *dz,
               void *dBm, void *dCm,
               float *dA, float *dDskip, float *ddelta_bias,
               void *hip_stream);

/* lbscan_bwd for chunked sequences: dhT (B,D,N) fp32, nullable, is the gradient
 * arriving at the state that left the forward call (fwd_args->hT); dh0 (B,D,N)
 * fp32, nullable, receives the gradient with respect to fwd_args->h0 (it is
 * defined, and written, also when h0 is NULL).  fwd_args->hT is not read. */
int lbscan_bwd_state(const lbscan_args *fwd_args, const void *dout, const float *dhT,
                     void *dx, void *ddelta, void *dz,
                     void *dBm, void *dCm,
                     float *dA, float *dDskip, float *ddelta_bias, float *dh0,
                     void *hip_stream);

/* The comparison method: global bi-directional scan (Sec. 3.1, Eq. 4-6) as two
 * full passes over HBM.  Pass 1 scans fwd_set left to right (Eq. 1-2); pass 2
 * scans bwd_set right to left (Eq. 4-5) and adds; each direction adds its own
 * Dskip x term; the sum is gated once with fwd_set->z and written to
 * fwd_set->y.  window / reverse / z / y of bwd_set are ignored.  bwd_set may
 * alias fwd_set. */
int lbscan_bidir_fwd(const lbscan_args *fwd_set, const lbscan_args *bwd_set, void *hip_stream);

/* Pre-scan step of the block (Algorithm 1: x' = SiLU(Conv1d(x)), the line before
 * B, C and Delta are projected from x').  The paper names the operation only; as
 * in the Mamba block it extends, the convolution is depthwise and causal:
 *     pre[b,d,t] = bias[d] + sum_{k<K} weight[d,k] x[b,d,t-(K-1)+k]   (x before 0 is 0)
 *     y = pre * sigmoid(pre)          (y = pre when activation is 0)
 * reverse = 1: the same operator on the time-reversed sequence (output t sees
 * inputs t .. t+K-1), for blocks that scan right to left.  K = width in 1..4. */
typedef struct lbscan_conv_args {
    int32_t batch, dim, seqlen;   /* B, D, L; any may be 0 */
    int32_t width;                /* K, 1..4 (else LBSCAN_EUNSUPPORTED) */
    int32_t dtype;                /* storage type of x, y (and dy, dx); arithmetic is fp32 */
    int32_t activation;           /* 1: SiLU, 0: none */
    int32_t reverse;              /* 0/1 */
    const void  *x;               /* (B,D,L) */
    const float *weight;          /* (D,K) */
    const float *bias;            /* (D) or NULL: 0 */
    void        *y;               /* (B,D,L) out (not read by the backward call) */
} lbscan_conv_args;

int lbscan_conv1d_fwd(const lbscan_conv_args *args, void *hip_stream);

/* Gradients of lbscan_conv1d_fwd: dx (B,D,L) in the storage type, dweight (D,K)
 * and dbias (D; NULL iff bias is NULL) in fp32, all overwritten; the two sums
 * over batch and time are accumulated with fp32 atomics.  No workspace. */
int lbscan_conv1d_bwd(const lbscan_conv_args *fwd_args, const void *dy,
                      void *dx, float *dweight, float *dbias, void *hip_stream);

/* Bytes of device scratch the call named by `which` (LBSCAN_WS_*) needs for
 * these sizes; 0 means workspace may be NULL. */
size_t lbscan_workspace_bytes(const lbscan_args *args, int which);

/* Window length the paper uses for a sequence length (Sec. 4, first paragraph):
 * L > 256 -> 16, 128 < L <= 256 -> 8, otherwise 4. */
int lbscan_default_window(int32_t seqlen);

/* Process-wide launch-shape override, for tuning and for tests that must reach
 * every kernel variant; results do not depend on it beyond rounding order.
 * NOT thread-safe with respect to the other entry points: "segments" changes what
 * lbscan_workspace_bytes returns and what the calls expect, so set options before
 * other threads query sizes or launch, never between a thread's size query and its
 * call.
 *   "waves_log2": -1 (default) lets the library choose over how many waves of
 *                 a block the N states of a row are split; 0..3 forces 1, 2, 4
 *                 or 8 (clamped to what the state size allows).
 *   "segments":   0 (default) lets the library choose into how many segments a
 *                 row is cut for parallel scanning (long rows, few channels);
 *                 k >= 1 asks for k (rounded so that segments are whole 32-token tiles).  It
 *                 changes lbscan_workspace_bytes: query after setting it.
 *   "mapping":    0 (default) lets lbscan_fwd choose between its two kernel
 *                 families: one lane per row (rows walked in tiles; cut into
 *                 segments when rows are few) and one wave per row with 16 tokens
 *                 per lane (the tile-per-thread organisation of Sec. 3.4; picked
 *                 for long bf16 rows that are many).  1 forces the first, 2 the
 *                 second wherever it applies (compiled window lengths, stored
 *                 order, rows that allow 16-byte accesses); other
 *                 calls are not affected.  Results agree within the tolerance of
 *                 the arithmetic; workspace sizes do not change.
 * Returns LBSCAN_EINVAL for an unknown name or a value out of range. */
int lbscan_set_option(const char *name, int value);

const char *lbscan_strerror(int code);
/* Text of the last HIP error seen by this thread ("" if none). */
const char *lbscan_last_error(void);
/* Library version, e.g. "0.1.0". */
const char *lbscan_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LBSCAN_H */
