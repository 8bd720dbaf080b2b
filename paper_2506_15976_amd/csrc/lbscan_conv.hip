// Pre-scan step of the LBMamba block (Algorithm 1: x' = SiLU(Conv1d(x))):
// depthwise causal convolution along the sequence, then SiLU, and its gradient.
//
//     pre[b,d,t] = bias[d] + sum_{k<K} w[d,k] x[b,d,t-(K-1)+k]     (inputs before 0 are zero)
//     y = pre * sigmoid(pre)          reverse: output t sees inputs t .. t+K-1 instead
//
// Both kernels are bound by HBM traffic, so the mapping serves the memory system:
// a wave takes chunks of 64 consecutive quads (256 tokens) of one row, every lane
// loads its quad once with one 16-byte load, and the K-1 neighbouring inputs an
// output needs from the quad next to it come from the neighbouring lane through a
// wave shuffle instead of a second load; only the lane at the end of the wave loads
// its three halo elements itself.  A wave works on one channel and walks several
// (batch entry, chunk) items of it, so that the filter is read once, waves live
// long enough to keep loads in flight, and the backward kernel's sums over batch
// and time are folded in registers before they reach an atomic.
#include "lbscan_device.h"
#include "lbscan_internal.h"

namespace lbscan {
namespace {

constexpr int kConvWaves = 4;          // waves per block
constexpr int kConvUnroll = 4;         // items whose loads a wave issues together

// x[row, t] for t in [0, L), 0 outside
template <typename T>
__device__ __forceinline__ float load_or_zero(const T* __restrict__ row, int t, int L)
{
    const int tc = t < 0 ? 0 : (t >= L ? L - 1 : t);
    const float v = to_f32(row[tc]);
    return t == tc ? v : 0.0f;
}

// A lane's quad is fetched in two steps so that a wave can have the loads of
// several items in flight.  quad_issue is one unconditional 16-byte load from an
// address clamped into the row (no load sits behind a divergent branch);
// quad_finish turns it into the four values x[t0 .. t0+3], zero outside the row,
// and only the lane holding a ragged last quad (and every lane when quads cannot
// be loaded whole: rows shorter than 4, or 2-byte rows starting at odd elements)
// goes back to memory element by element.
template <typename T>
__device__ __forceinline__ Quad<T> quad_issue(const T* __restrict__ row, int t0, int L, bool vec_ok)
{
    if (!vec_ok) return Quad<T>{};                               // uniform
    const int tc = t0 < 0 ? 0 : (t0 > L - 4 ? L - 4 : t0);
    return quad_raw_fast<T>(row, tc);
}

template <typename T>
__device__ __forceinline__ void quad_finish(const Quad<T>& raw, const T* __restrict__ row, int t0, int L,
                                            bool vec_ok, float (&cur)[4])
{
    const bool whole = vec_ok && t0 >= 0 && t0 + 4 <= L;
    float slow[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (!whole && t0 >= 0 && t0 < L) {
#pragma unroll
        for (int e = 0; e < 4; ++e) slow[e] = load_or_zero<T>(row, t0 + e, L);
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) cur[e] = whole ? to_f32(raw.v[e]) : slow[e];
}

// The lane's own quad and the three inputs on the side the filter reaches to:
// win[0..2] = x[t0-3 .. t0-1], win[3..6] = x[t0 .. t0+3] (forward direction), or
// win[0..3] = x[t0 .. t0+3], win[4..6] = x[t0+4 .. t0+6] (reversed direction).
// Lanes whose quad lies outside the row hold zeros.  Every lane of the wave calls it.
template <typename T, bool REV>
__device__ __forceinline__ void make_window(const float (&cur)[4], const T* __restrict__ row, int t0, int L,
                                            int lane, float (&win)[7])
{
    const bool active = t0 >= 0 && t0 < L;
    float halo[3];
    if (!REV) {
#pragma unroll
        for (int j = 0; j < 3; ++j) halo[j] = __shfl_up(cur[1 + j], 1, 64);
        if (lane == 0) {
#pragma unroll
            for (int j = 0; j < 3; ++j) halo[j] = active ? load_or_zero<T>(row, t0 - 3 + j, L) : 0.0f;
        }
#pragma unroll
        for (int j = 0; j < 3; ++j) win[j] = halo[j];
#pragma unroll
        for (int e = 0; e < 4; ++e) win[3 + e] = cur[e];
    } else {
#pragma unroll
        for (int j = 0; j < 3; ++j) halo[j] = __shfl_down(cur[j], 1, 64);
        if (lane == 63) {
#pragma unroll
            for (int j = 0; j < 3; ++j) halo[j] = active ? load_or_zero<T>(row, t0 + 4 + j, L) : 0.0f;
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) win[e] = cur[e];
#pragma unroll
        for (int j = 0; j < 3; ++j) win[4 + j] = halo[j];
    }
}

// pre-activation of output e of the quad from the window above
template <int K, bool REV>
__device__ __forceinline__ float conv_at(const float (&win)[7], const float (&w)[K], float bias, int e)
{
    float pre = bias;
#pragma unroll
    for (int k = 0; k < K; ++k)
        pre = fmaf(w[k], REV ? win[e + (K - 1) - k] : win[3 + e - (K - 1) + k], pre);
    return pre;
}

// The (batch entry, chunk) items of a channel are numbered b * chunks + chunk; wave
// `wid` takes channel wid % D and the items [g * per_wave, (g + 1) * per_wave) of
// group g = wid / D, so that waves launched together work on neighbouring rows.
// Item counts fit 32 bits (checked by the launcher).
struct ConvWave {
    bool any;      // the wave has work
    int d;         // channel
    int n;         // items
    int b, ch;     // first item: batch entry and chunk
};
__device__ __forceinline__ ConvWave conv_wave(const ConvParams& p, int chunks)
{
    const unsigned items = (unsigned)p.batch * (unsigned)chunks;
    const unsigned per = (unsigned)p.items_per_wave;
    const unsigned groups = (items + per - 1) / per;
    const unsigned wid = blockIdx.x * kConvWaves + (threadIdx.x >> 6);
    ConvWave w;
    w.any = wid < (unsigned)p.dim * groups;
    w.d = (int)(wid % (unsigned)p.dim);
    const unsigned i0 = (wid / (unsigned)p.dim) * per;
    w.n = (int)(i0 + per <= items ? per : items - i0);
    w.b = (int)(i0 / (unsigned)chunks);
    w.ch = (int)(i0 % (unsigned)chunks);
    return w;
}

template <typename T, int K, bool REV>
__global__ void __launch_bounds__(64 * kConvWaves)
conv1d_fwd_kernel(const ConvParams p)
{
    constexpr int U = kConvUnroll;
    const int lane = threadIdx.x & 63;
    const int L = p.seqlen;
    const int chunks = ((L + 3) / 4 + 63) / 64;
    const ConvWave cw = conv_wave(p, chunks);
    if (!cw.any) return;                                        // whole wave
    const int d = cw.d;
    const bool vec_ok = L >= 4 && (sizeof(T) == 4 || L % 2 == 0);   // quads can be loaded whole
    const bool act = p.activation != 0;
    const T* __restrict__ xg = static_cast<const T*>(p.x);
    T* __restrict__ yg = static_cast<T*>(p.y);

    float w[K];
#pragma unroll
    for (int k = 0; k < K; ++k) w[k] = p.weight[(long)d * K + k];
    const float bias = p.bias ? p.bias[d] : 0.0f;

    int b = cw.b, ch = cw.ch;
    for (int i = 0; i < cw.n; i += U) {
        long roff[U];
        int t0[U];
        Quad<T> raw[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            roff[u] = ((long)b * p.dim + d) * L;
            t0[u] = (ch * 64 + lane) * 4;
            raw[u] = quad_issue<T>(xg + roff[u], t0[u], L, vec_ok);
            if (i + u + 1 < cw.n) {                             // uniform; else repeat the last item
                if (++ch == chunks) { ch = 0; ++b; }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (i + u < cw.n) {                                 // uniform
                float cur[4], win[7];
                quad_finish<T>(raw[u], xg + roff[u], t0[u], L, vec_ok, cur);
                make_window<T, REV>(cur, xg + roff[u], t0[u], L, lane, win);
                if (t0[u] < L) {
                    float out[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float pre = conv_at<K, REV>(win, w, bias, e);
                        out[e] = act ? pre * sigmoid_f32(pre) : pre;
                    }
                    quad_store<T>(yg + roff[u], t0[u], vec_ok && t0[u] + 4 <= L, t0[u], L, out);
                }
            }
        }
    }
}

// Gradient.  dpre_t = dy_t * dSiLU(pre_t); an input s collects w[k] dpre_t from the
// K outputs that read it, which lie in the lane's own quad and in the quad on the
// other side than the forward halo, so dpre of the neighbouring lane is shuffled
// in.  For that, consecutive chunks of a row overlap by one quad: 63 lanes own
// their quad (write dx, add to the filter and bias sums), the 64th only supplies
// dpre.  The filter and bias sums are folded over the wave's items in registers,
// then over the wave, and added with one atomic per wave and tap.
template <typename T, int K, bool REV>
__global__ void __launch_bounds__(64 * kConvWaves)
conv1d_bwd_kernel(const ConvParams p)
{
    constexpr int U = kConvUnroll;
    const int lane = threadIdx.x & 63;
    const int L = p.seqlen;
    const int chunks = ((L + 3) / 4 + 62) / 63;
    const ConvWave cw = conv_wave(p, chunks);
    if (!cw.any) return;                                        // whole wave
    const int d = cw.d;
    const bool vec_ok = L >= 4 && (sizeof(T) == 4 || L % 2 == 0);   // quads can be loaded whole
    const bool act = p.activation != 0;
    const bool owner_lane = REV ? lane >= 1 : lane <= 62;
    const T* __restrict__ xg = static_cast<const T*>(p.x);
    const T* __restrict__ gg = static_cast<const T*>(p.dy);
    T* __restrict__ dxg = static_cast<T*>(p.dx);

    float w[K];
#pragma unroll
    for (int k = 0; k < K; ++k) w[k] = p.weight[(long)d * K + k];
    const float bias = p.bias ? p.bias[d] : 0.0f;

    float acc[K + 1];                                           // filter taps, then bias
#pragma unroll
    for (int k = 0; k <= K; ++k) acc[k] = 0.0f;

    int b = cw.b, ch = cw.ch;
    for (int i = 0; i < cw.n; i += U) {
        long roff[U];
        int t0s[U];
        Quad<T> rawx[U], rawg[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            roff[u] = ((long)b * p.dim + d) * L;
            t0s[u] = (ch * 63 - (REV ? 1 : 0) + lane) * 4;
            rawx[u] = quad_issue<T>(xg + roff[u], t0s[u], L, vec_ok);
            rawg[u] = quad_issue<T>(gg + roff[u], t0s[u], L, vec_ok);
            if (i + u + 1 < cw.n) {                             // uniform; else repeat the last item
                if (++ch == chunks) { ch = 0; ++b; }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (i + u < cw.n) {                                 // uniform
                const int t0 = t0s[u];
                const bool own = owner_lane && t0 >= 0 && t0 < L;
                float cur[4], win[7], dy[4];
                quad_finish<T>(rawx[u], xg + roff[u], t0, L, vec_ok, cur);
                make_window<T, REV>(cur, xg + roff[u], t0, L, lane, win);
                quad_finish<T>(rawg[u], gg + roff[u], t0, L, vec_ok, dy);

                // dpre of the own quad (zero past the end of the row: dy is zero there)
                float dpre[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float pre = conv_at<K, REV>(win, w, bias, e);
                    float g = dy[e];
                    if (act) {
                        const float sg = sigmoid_f32(pre);
                        g *= sg * fmaf(pre, 1.0f - sg, 1.0f);
                    }
                    dpre[e] = g;
                }
                // dwin: dpre around the own quad, on the side where the outputs that read it lie
                float dwin[7];
                if (!REV) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) dwin[e] = dpre[e];
#pragma unroll
                    for (int j = 0; j < 3; ++j) dwin[4 + j] = __shfl_down(dpre[j], 1, 64);
                } else {
#pragma unroll
                    for (int j = 0; j < 3; ++j) dwin[j] = __shfl_up(dpre[1 + j], 1, 64);
#pragma unroll
                    for (int e = 0; e < 4; ++e) dwin[3 + e] = dpre[e];
                }
                if (own) {
                    float dx[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        // input t0+e is read through tap k by output t0+e+(K-1)-k (forward
                        // direction) or t0+e-(K-1)+k (reversed)
                        float sum = 0.0f;
#pragma unroll
                        for (int k = 0; k < K; ++k)
                            sum = fmaf(w[k], REV ? dwin[3 + e - (K - 1) + k] : dwin[e + (K - 1) - k], sum);
                        dx[e] = sum;
#pragma unroll
                        for (int k = 0; k < K; ++k)
                            acc[k] = fmaf(dpre[e], REV ? win[e + (K - 1) - k] : win[3 + e - (K - 1) + k], acc[k]);
                        acc[K] += dpre[e];
                    }
                    quad_store<T>(dxg + roff[u], t0, vec_ok && t0 + 4 <= L, t0, L, dx);
                }
            }
        }
    }
#pragma unroll
    for (int k = 0; k <= K; ++k) {
#pragma unroll
        for (int s = 1; s < 64; s *= 2) acc[k] += __shfl_xor(acc[k], s, 64);
    }
    if (lane == 0) {
#pragma unroll
        for (int k = 0; k < K; ++k) unsafeAtomicAdd(&p.dweight[(long)d * K + k], acc[k]);
        if (p.dbias) unsafeAtomicAdd(&p.dbias[d], acc[K]);
    }
}

template <typename T, int K, bool REV>
hipError_t launch_conv_kr(ConvParams p, bool bwd, hipStream_t s)
{
    const long nq = (p.seqlen + 3) / 4;
    const long chunks = bwd ? (nq + 62) / 63 : (nq + 63) / 64;
    // items per wave: about 8 waves per SIMD of the chip in all, at most 64 items
    const long items = (long)p.batch * chunks;
    if (items > 0x7fffffffL) return hipErrorInvalidConfiguration;
    long per_wave = ((long)p.dim * items + 8191) / 8192;
    per_wave = per_wave < 1 ? 1 : (per_wave > 64 ? 64 : per_wave);
    p.items_per_wave = (int)per_wave;
    const long waves = (long)p.dim * ((items + per_wave - 1) / per_wave);
    const long blocks = (waves + kConvWaves - 1) / kConvWaves;
    if (blocks > 0x3fffffffL) return hipErrorInvalidConfiguration;     // wave ids fit 32 bits
    if (bwd)
        hipLaunchKernelGGL((conv1d_bwd_kernel<T, K, REV>), dim3((unsigned)blocks), dim3(64 * kConvWaves), 0, s, p);
    else
        hipLaunchKernelGGL((conv1d_fwd_kernel<T, K, REV>), dim3((unsigned)blocks), dim3(64 * kConvWaves), 0, s, p);
    return hipGetLastError();
}

template <typename T, int K>
hipError_t launch_conv_k(const ConvParams& p, bool bwd, hipStream_t s)
{
    return p.reverse ? launch_conv_kr<T, K, true>(p, bwd, s) : launch_conv_kr<T, K, false>(p, bwd, s);
}

template <typename T>
hipError_t launch_conv_t(const ConvParams& p, bool bwd, hipStream_t s)
{
    switch (p.width) {
        case 1: return launch_conv_k<T, 1>(p, bwd, s);
        case 2: return launch_conv_k<T, 2>(p, bwd, s);
        case 3: return launch_conv_k<T, 3>(p, bwd, s);
        case 4: return launch_conv_k<T, 4>(p, bwd, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

hipError_t launch_conv1d_fwd(const ConvParams& p, hipStream_t stream)
{
    if ((long)p.batch * p.dim * p.seqlen == 0) return hipSuccess;
    return p.dtype == 0 ? launch_conv_t<float>(p, false, stream) : launch_conv_t<bf16_t>(p, false, stream);
}

hipError_t launch_conv1d_bwd(const ConvParams& p, hipStream_t stream)
{
    hipError_t e = launch_zero(p.dweight, (long)p.dim * p.width, stream);
    if (e == hipSuccess) e = launch_zero(p.dbias, p.dim, stream);
    if (e != hipSuccess || (long)p.batch * p.dim * p.seqlen == 0) return e;
    return p.dtype == 0 ? launch_conv_t<float>(p, true, stream) : launch_conv_t<bf16_t>(p, true, stream);
}

}  // namespace lbscan
