// C entry points of liblbscan: argument validation and kernel dispatch.
// Every step of the computation runs in the HIP kernels; nothing here touches
// tensor data on the host, allocates or synchronises.
#include "../../include/lbscan.h"
#include "lbscan_internal.h"

#include <atomic>
#include <mutex>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

namespace {

thread_local char g_last_error[256] = "";

int hip_fail(hipError_t e, const char* where)
{
    snprintf(g_last_error, sizeof(g_last_error), "%s: %s", where, hipGetErrorString(e));
    return LBSCAN_EHIP;
}

// Scratch missing or too small; for the fixed array the text says what was asked for.
int scratch_too_small(size_t need, size_t have, bool fixed)
{
    if (fixed)
        snprintf(g_last_error, sizeof(g_last_error),
                 "lbscan_fwd_static: these sizes need %zu bytes of scratch, the fixed array holds %zu",
                 need, have);
    return LBSCAN_EWORKSPACE;
}

// Launch-shape overrides set through lbscan_set_option (tuning and tests).
std::atomic<int> g_waves_log2{-1};
std::atomic<int> g_nseg{0};
int tuning_waves_log2() { return g_waves_log2.load(std::memory_order_relaxed); }
std::atomic<int> g_mapping{0};
int tuning_nseg() { return g_nseg.load(std::memory_order_relaxed); }

bool aligned4(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 3u) == 0; }

// Size and flag checks.  *empty is set when there is nothing to compute.
int check_args_sizes(const lbscan_args* a, bool* empty)
{
    *empty = false;
    if (!a) return LBSCAN_EINVAL;
    if (a->batch < 0 || a->dim < 0 || a->dstate < 0 || a->seqlen < 0) return LBSCAN_EINVAL;
    if (a->window < 1) return LBSCAN_EINVAL;
    if (a->dtype != LBSCAN_FP32 && a->dtype != LBSCAN_BF16) return LBSCAN_EUNSUPPORTED;
    if (a->dstate > LBSCAN_MAX_DSTATE) return LBSCAN_EUNSUPPORTED;
    if (a->reverse != 0 && a->reverse != 1) return LBSCAN_EINVAL;
    if (a->seqlen > (1 << 24)) return LBSCAN_EUNSUPPORTED;   // 64 rows * L is indexed in 32 bits
    if (a->scan_order != LBSCAN_ORDER_SEQUENCE && a->scan_order != LBSCAN_ORDER_COLUMNS) return LBSCAN_EINVAL;
    if (a->scan_order == LBSCAN_ORDER_COLUMNS) {
        if (a->grid_h < 1 || a->grid_w < 1 || a->grid_prefix < 0) return LBSCAN_EINVAL;
        if ((long)a->grid_prefix + (long)a->grid_h * a->grid_w > (long)a->seqlen) return LBSCAN_EINVAL;
    }
    if ((long)a->batch * a->dim * a->seqlen == 0) *empty = true;
    // a state size of zero with steps to take (y = Dskip x SiLU(z)) has no kernel
    if (!*empty && a->dstate == 0) return LBSCAN_EUNSUPPORTED;
    return LBSCAN_OK;
}

// Shape / pointer checks common to all entry points.
int check_args(const lbscan_args* a, bool need_y, bool* empty)
{
    int rc = check_args_sizes(a, empty);
    if (rc != LBSCAN_OK || *empty) return rc;
    if (!a->x || !a->delta || (need_y && !a->y)) return LBSCAN_EINVAL;
    if (!a->A || !a->Bm || !a->Cm) return LBSCAN_EINVAL;
    const void* ptrs[] = {a->x, a->delta, a->Bm, a->Cm, a->z, a->A, a->Dskip, a->delta_bias, a->y,
                          a->h0, a->hT};
    for (const void* p : ptrs)
        if (p && !aligned4(p)) return LBSCAN_EINVAL;
    return LBSCAN_OK;
}

// Window length the kernels run with: a window that covers the whole row is
// the same as any longer one, and the kernels pad the row with identity steps,
// so every M >= L maps to the smallest compiled window >= L.
int effective_window(int M, int L)
{
    if (lbscan::window_supported(M)) return M;
    if (M >= L) {
        for (int m = 1; m <= 16; m *= 2)
            if (m >= L) return m;
    }
    return 0;
}

lbscan::FwdParams to_params(const lbscan_args* a, int window)
{
    lbscan::FwdParams p;
    p.batch = a->batch; p.dim = a->dim; p.dstate = a->dstate; p.seqlen = a->seqlen;
    p.window = window; p.dtype = a->dtype; p.softplus = a->delta_softplus; p.reverse = a->reverse;
    p.order.kind = a->scan_order;
    p.order.prefix = a->grid_prefix;
    p.order.H = a->scan_order ? a->grid_h : 1;
    p.order.W = a->scan_order ? a->grid_w : 1;
    p.order.HW = p.order.H * p.order.W;
    p.order.rH = 1.0f / (float)p.order.H;
    p.x = a->x; p.delta = a->delta; p.Bm = a->Bm; p.Cm = a->Cm; p.z = a->z;
    p.A = a->A; p.Dskip = a->Dskip; p.bias = a->delta_bias;
    p.yprev = nullptr; p.y = a->y; p.y_is_f32 = 0;
    p.force_waves_log2 = tuning_waves_log2();
    p.force_nseg = tuning_nseg();
    p.force_mapping = g_mapping.load(std::memory_order_relaxed);
    p.nseg = 1; p.seg_tiles = 0; p.summary_only = 0; p.fold_chain = 0; p.carry = nullptr; p.dsum = nullptr;
    p.ckpt = nullptr; p.cum = nullptr; p.dout = nullptr; p.psi = nullptr; p.gck = nullptr;
    p.h0 = a->h0; p.hT = a->hT;
    p.generic_window = 0; p.seg_tokens = 0;
    return p;
}

int check_conv_args(const lbscan_conv_args* a, bool* empty)
{
    *empty = false;
    if (!a) return LBSCAN_EINVAL;
    if (a->batch < 0 || a->dim < 0 || a->seqlen < 0 || a->width < 1) return LBSCAN_EINVAL;
    if (a->dtype != LBSCAN_FP32 && a->dtype != LBSCAN_BF16) return LBSCAN_EUNSUPPORTED;
    if (a->width > 4) return LBSCAN_EUNSUPPORTED;
    if ((a->reverse != 0 && a->reverse != 1) || (a->activation != 0 && a->activation != 1)) return LBSCAN_EINVAL;
    if (a->seqlen > (1 << 28)) return LBSCAN_EUNSUPPORTED;     // token offsets are 32-bit
    if ((long)a->batch * a->dim * a->seqlen == 0) { *empty = true; return LBSCAN_OK; }
    if (!a->x || !a->weight) return LBSCAN_EINVAL;
    if (!aligned4(a->x) || !aligned4(a->weight) || (a->bias && !aligned4(a->bias))) return LBSCAN_EINVAL;
    return LBSCAN_OK;
}

lbscan::ConvParams to_conv_params(const lbscan_conv_args* a)
{
    lbscan::ConvParams p;
    p.batch = a->batch; p.dim = a->dim; p.seqlen = a->seqlen; p.width = a->width;
    p.dtype = a->dtype; p.activation = a->activation; p.reverse = a->reverse;
    p.x = a->x; p.weight = a->weight; p.bias = a->bias; p.y = a->y;
    p.dy = nullptr; p.dx = nullptr; p.dweight = nullptr; p.dbias = nullptr;
    p.items_per_wave = 1;
    return p;
}

// ---- scratch of lbscan_fwd_static ----------------------------------------------
// A fixed device array that every GPU the library runs on holds until the process
// ends.  In host code the array's name is only a handle for hipGetSymbolAddress: the
// device address is looked up once per device and that pointer, never the name, is
// what the kernels get.
static __device__ __align__(256) unsigned char g_static_scratch[LBSCAN_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_static_mutex;
void* g_static_ptr[kMaxDevices] = {};

// Device address of the scratch array on the current device (nullptr and *err set on
// failure).  The first call on a device asks the runtime; no allocation either way.
void* static_scratch(hipError_t* err)
{
    int dev = -1;
    *err = hipGetDevice(&dev);
    if (*err != hipSuccess) return nullptr;
    if (dev < 0 || dev >= kMaxDevices) { *err = hipErrorInvalidDevice; return nullptr; }
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (!g_static_ptr[dev]) {
        void* ptr = nullptr;
        *err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_static_scratch));
        if (*err != hipSuccess) return nullptr;
        g_static_ptr[dev] = ptr;
    }
    return g_static_ptr[dev];
}

// lbscan_fwd with the scratch given explicitly (bytes available at `scratch`).
int fwd_with_scratch(const lbscan_args* args, void* scratch, size_t scratch_bytes, bool fixed, void* hip_stream);

}  // namespace

extern "C" {

int lbscan_fwd(const lbscan_args* args, void* hip_stream)
{
    return fwd_with_scratch(args, args ? args->workspace : nullptr, args ? args->workspace_bytes : 0, false,
                            hip_stream);
}

int lbscan_fwd_static(const lbscan_args* args, void* hip_stream)
{
    hipError_t e = hipSuccess;
    void* ptr = static_scratch(&e);
    if (!ptr) return hip_fail(e, "lbscan_fwd_static: address of the scratch array");
    return fwd_with_scratch(args, ptr, LBSCAN_STATIC_SCRATCH_BYTES, true, hip_stream);
}

}  // extern "C"

namespace {

int fwd_with_scratch(const lbscan_args* args, void* scratch, size_t scratch_bytes, bool fixed, void* hip_stream)
{
    bool empty;
    int rc = check_args(args, true, &empty);
    if (rc != LBSCAN_OK) return rc;
    if (empty) {
        // no steps: the state passes through
        if (!args->hT) return LBSCAN_OK;
        if ((args->h0 && !aligned4(args->h0)) || !aligned4(args->hT)) return LBSCAN_EINVAL;
        hipError_t e = lbscan::launch_copy(args->hT, args->h0, (long)args->batch * args->dim * args->dstate,
                                           static_cast<hipStream_t>(hip_stream));
        return e == hipSuccess ? LBSCAN_OK : hip_fail(e, "lbscan_fwd");
    }
    const int M = effective_window(args->window, args->seqlen);
    if (M == 0) {
        // no compiled kernel for this window length: the two-launch path
        if (args->scan_order != LBSCAN_ORDER_SEQUENCE) return LBSCAN_EUNSUPPORTED;
        lbscan::FwdParams p = to_params(args, args->window < args->seqlen ? args->window : args->seqlen);
        const size_t need = lbscan::fwd_generic_workspace_bytes(p);
        if (need && (!scratch || scratch_bytes < need || !aligned4(scratch)))
            return scratch_too_small(need, scratch_bytes, fixed);
        hipError_t e = lbscan::launch_fwd_generic(p, scratch, static_cast<hipStream_t>(hip_stream));
        return e == hipSuccess ? LBSCAN_OK : hip_fail(e, "lbscan_fwd");
    }
    lbscan::FwdParams p = to_params(args, M);
    const size_t need = lbscan::fwd_workspace_bytes(p);
    if (need && (!scratch || scratch_bytes < need || !aligned4(scratch)))
        return scratch_too_small(need, scratch_bytes, fixed);
    float* saved = nullptr;
    if (args->saved_state) {
        const size_t sneed = lbscan::saved_state_bytes(p);
        if (sneed && (args->saved_state_bytes < sneed || !aligned4(args->saved_state))) return LBSCAN_EWORKSPACE;
        if (sneed) saved = static_cast<float*>(args->saved_state);
    }
    hipError_t e = lbscan::launch_fwd(p, scratch, saved, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? LBSCAN_OK : hip_fail(e, "lbscan_fwd");
}

}  // namespace

extern "C" {

int lbscan_bidir_fwd(const lbscan_args* fs, const lbscan_args* bs, void* hip_stream)
{
    bool empty_f, empty_b;
    int rc = check_args(fs, true, &empty_f);
    if (rc != LBSCAN_OK) return rc;
    rc = check_args(bs, false, &empty_b);
    if (rc != LBSCAN_OK) return rc;
    if (fs->batch != bs->batch || fs->dim != bs->dim || fs->dstate != bs->dstate ||
        fs->seqlen != bs->seqlen || fs->dtype != bs->dtype) return LBSCAN_EINVAL;
    if (fs->h0 || fs->hT || bs->h0 || bs->hT) return LBSCAN_EINVAL;   // whole sequences only
    if (fs->scan_order != LBSCAN_ORDER_SEQUENCE || bs->scan_order != LBSCAN_ORDER_SEQUENCE)
        return LBSCAN_EUNSUPPORTED;
    if (empty_f) return LBSCAN_OK;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);

    // Pass 1 leaves the ungated forward result in fp32: in y itself when y is
    // fp32, else at the start of the workspace.  Pass 2 reads it back, adds the
    // reverse scan, gates and writes y.  Both passes share the scratch the
    // forward kernels need for long rows (they run one after the other).
    lbscan::FwdParams p1 = to_params(fs, 1);
    lbscan::FwdParams p2 = to_params(bs, 1);
    const size_t need = lbscan_workspace_bytes(fs, LBSCAN_WS_BIDIR);
    if (need && (!fs->workspace || fs->workspace_bytes < need || !aligned4(fs->workspace)))
        return LBSCAN_EWORKSPACE;
    const size_t bdl = (size_t)fs->batch * fs->dim * fs->seqlen;
    float* partial;
    char* scratch = static_cast<char*>(fs->workspace);
    if (fs->dtype == LBSCAN_FP32) {
        partial = static_cast<float*>(fs->y);
    } else {
        partial = static_cast<float*>(fs->workspace);
        scratch += bdl * sizeof(float);
    }
    p1.reverse = 0; p1.z = nullptr; p1.y = partial; p1.y_is_f32 = 1;
    hipError_t e = lbscan::launch_fwd(p1, scratch, nullptr, s);
    if (e != hipSuccess) return hip_fail(e, "lbscan_bidir_fwd pass 1");
    p2.reverse = 1; p2.z = fs->z; p2.yprev = partial; p2.y = fs->y; p2.y_is_f32 = 0;
    e = lbscan::launch_fwd(p2, scratch, nullptr, s);
    return e == hipSuccess ? LBSCAN_OK : hip_fail(e, "lbscan_bidir_fwd pass 2");
}

int lbscan_bwd(const lbscan_args* a, const void* dout,
               void* dx, void* ddelta, void* dz, void* dBm, void* dCm,
               float* dA, float* dDskip, float* ddelta_bias, void* hip_stream)
{
    return lbscan_bwd_state(a, dout, nullptr, dx, ddelta, dz, dBm, dCm, dA, dDskip, ddelta_bias,
                            nullptr, hip_stream);
}

int lbscan_bwd_state(const lbscan_args* a, const void* dout, const float* dhT,
                     void* dx, void* ddelta, void* dz, void* dBm, void* dCm,
                     float* dA, float* dDskip, float* ddelta_bias, float* dh0, void* hip_stream)
{
    bool empty;
    int rc = check_args(a, false, &empty);
    if (rc != LBSCAN_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (!dA || !dBm || !dCm) {
        if ((long)a->dim * a->dstate > 0 && !dA) return LBSCAN_EINVAL;
        if ((long)a->batch * a->dstate * a->seqlen > 0 && (!dBm || !dCm)) return LBSCAN_EINVAL;
    }
    if ((a->Dskip && !dDskip) || (a->delta_bias && !ddelta_bias)) return LBSCAN_EINVAL;
    if (empty) {
        // nothing flows back: the per-channel sums are still overwritten (with zeros)
        hipError_t e = lbscan::launch_zero(dA, (long)a->dim * a->dstate, s);
        if (e == hipSuccess) e = lbscan::launch_zero(dDskip, a->dim, s);
        if (e == hipSuccess) e = lbscan::launch_zero(ddelta_bias, a->dim, s);
        // no steps: the gradient of the leaving state is that of the entering state
        if (e == hipSuccess && dh0 && aligned4(dh0) && (!dhT || aligned4(dhT)))
            e = lbscan::launch_copy(dh0, dhT, (long)a->batch * a->dim * a->dstate, s);
        return e == hipSuccess ? LBSCAN_OK : hip_fail(e, "lbscan_bwd");
    }
    if (!dout || !dx || !ddelta || (a->z && !dz)) return LBSCAN_EINVAL;
    const void* ptrs[] = {dout, dx, ddelta, dz, dBm, dCm, dA, dDskip, ddelta_bias, dhT, dh0};
    for (const void* q : ptrs)
        if (q && !aligned4(q)) return LBSCAN_EINVAL;
    // one backward kernel covers every window length (1, 2, 4 with a compiled window
    // structure, all others with run-time window masks); a window that covers the
    // whole row is the same as any longer one
    const int fwdM = effective_window(a->window, a->seqlen);
    const int M = fwdM ? fwdM : (a->window < a->seqlen ? a->window : a->seqlen);
    lbscan::FwdParams f = to_params(a, M);
    const size_t need = lbscan::bwd_workspace_bytes(f);
    if (need && (!a->workspace || a->workspace_bytes < need || !aligned4(a->workspace)))
        return LBSCAN_EWORKSPACE;
    lbscan::BwdParams p;
    p.batch = f.batch; p.dim = f.dim; p.dstate = f.dstate; p.seqlen = f.seqlen;
    p.window = M; p.dtype = f.dtype; p.softplus = f.softplus; p.reverse = f.reverse;
    p.order = f.order;
    p.x = f.x; p.delta = f.delta; p.Bm = f.Bm; p.Cm = f.Cm; p.z = f.z;
    p.A = f.A; p.Dskip = f.Dskip; p.bias = f.bias;
    p.dout = dout; p.dx = dx; p.ddelta = ddelta; p.dz = a->z ? dz : nullptr;
    p.dBpart = nullptr;
    p.dA = dA; p.dDskip = a->Dskip ? dDskip : nullptr; p.dbias = a->delta_bias ? ddelta_bias : nullptr;
    p.ckpt = nullptr; p.nseg = 1; p.seg_tiles = 0; p.cum = nullptr; p.carry = nullptr; p.psi_in = nullptr;
    p.dh0 = dh0; p.gck = nullptr;
    f.hT = nullptr;
    const float* saved = nullptr;
    if (a->saved_state && fwdM != 0) {
        const size_t sneed = lbscan::saved_state_bytes(f);
        if (sneed && (a->saved_state_bytes < sneed || !aligned4(a->saved_state))) return LBSCAN_EWORKSPACE;
        if (sneed) saved = static_cast<const float*>(a->saved_state);
    }
    hipError_t e = lbscan::launch_bwd(f, p, dBm, dCm, a->workspace, saved, dhT, s);
    return e == hipSuccess ? LBSCAN_OK : hip_fail(e, "lbscan_bwd");
}

int lbscan_conv1d_fwd(const lbscan_conv_args* a, void* hip_stream)
{
    bool empty;
    int rc = check_conv_args(a, &empty);
    if (rc != LBSCAN_OK || empty) return rc;
    if (!a->y || !aligned4(a->y)) return LBSCAN_EINVAL;
    hipError_t e = lbscan::launch_conv1d_fwd(to_conv_params(a), static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? LBSCAN_OK : hip_fail(e, "lbscan_conv1d_fwd");
}

int lbscan_conv1d_bwd(const lbscan_conv_args* a, const void* dy, void* dx, float* dweight, float* dbias,
                      void* hip_stream)
{
    bool empty;
    int rc = check_conv_args(a, &empty);
    if (rc != LBSCAN_OK) return rc;
    if ((long)a->dim * a->width > 0 && (!dweight || !aligned4(dweight))) return LBSCAN_EINVAL;
    if (a->bias && (!dbias || !aligned4(dbias))) return LBSCAN_EINVAL;
    if (!empty && (!dy || !dx || !aligned4(dy) || !aligned4(dx))) return LBSCAN_EINVAL;
    lbscan::ConvParams p = to_conv_params(a);
    p.y = nullptr; p.dy = dy; p.dx = dx; p.dweight = dweight; p.dbias = a->bias ? dbias : nullptr;
    hipError_t e = lbscan::launch_conv1d_bwd(p, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? LBSCAN_OK : hip_fail(e, "lbscan_conv1d_bwd");
}

size_t lbscan_workspace_bytes(const lbscan_args* a, int which)
{
    bool empty;
    if (check_args_sizes(a, &empty) != LBSCAN_OK || empty) return 0;
    const size_t bdl = (size_t)a->batch * a->dim * a->seqlen;
    int M = effective_window(a->window, a->seqlen);
    if (M == 0) {
        // two launches each way: the plain scan with window 1 and the local backward part
        if (which == LBSCAN_WS_FWD)
            return lbscan::fwd_generic_workspace_bytes(to_params(a, a->window < a->seqlen ? a->window : a->seqlen));
        if (which == LBSCAN_WS_SAVED) return 0;
        if (which == LBSCAN_WS_BWD)
            return lbscan::bwd_workspace_bytes(to_params(a, a->window < a->seqlen ? a->window : a->seqlen));
        M = 1;
    }
    switch (which) {
        case LBSCAN_WS_FWD:
            return lbscan::fwd_workspace_bytes(to_params(a, M));
        case LBSCAN_WS_BWD:
            return lbscan::bwd_workspace_bytes(to_params(a, M));
        case LBSCAN_WS_SAVED:
            return lbscan::saved_state_bytes(to_params(a, M));
        case LBSCAN_WS_BIDIR:
            return (a->dtype == LBSCAN_FP32 ? 0 : bdl * sizeof(float)) +
                   lbscan::fwd_workspace_bytes(to_params(a, 1));
        default: return 0;
    }
}

int lbscan_default_window(int32_t seqlen)
{
    if (seqlen > 256) return 16;
    if (seqlen > 128) return 8;
    return 4;
}

const char* lbscan_strerror(int code)
{
    switch (code) {
        case LBSCAN_OK: return "ok";
        case LBSCAN_EINVAL: return "invalid argument";
        case LBSCAN_EUNSUPPORTED: return "unsupported dtype, state size or window";
        case LBSCAN_EWORKSPACE: return "workspace missing or too small";
        case LBSCAN_EHIP: return "HIP error";
        default: return "unknown error";
    }
}

int lbscan_set_option(const char* name, int value)
{
    if (!name) return LBSCAN_EINVAL;
    if (strcmp(name, "waves_log2") == 0) {
        if (value < -1 || value > 3) return LBSCAN_EINVAL;
        g_waves_log2.store(value, std::memory_order_relaxed);
        return LBSCAN_OK;
    }
    if (strcmp(name, "segments") == 0) {
        if (value < 0 || value > (1 << 20)) return LBSCAN_EINVAL;
        g_nseg.store(value, std::memory_order_relaxed);
        return LBSCAN_OK;
    }
    if (strcmp(name, "mapping") == 0) {
        if (value < 0 || value > 2) return LBSCAN_EINVAL;
        g_mapping.store(value, std::memory_order_relaxed);
        return LBSCAN_OK;
    }
    return LBSCAN_EINVAL;
}

const char* lbscan_last_error(void) { return g_last_error; }
const char* lbscan_version(void) { return "0.1.0"; }

}  // extern "C"
