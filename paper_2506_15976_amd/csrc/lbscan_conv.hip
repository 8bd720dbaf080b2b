// Pre-scan step of the LBMamba block (Algorithm 1: x' = SiLU(Conv1d(x))):
// depthwise causal convolution along the sequence, then SiLU, and its gradient.
//
//     pre[b,d,t] = bias[d] + sum_{k<K} w[d,k] x[b,d,t-(K-1)+k]     (inputs before 0 are zero)
//     y = pre * sigmoid(pre)          reverse: output t sees inputs t .. t+K-1 instead
//
// Both kernels are bound by HBM traffic, so the mapping serves the memory system:
// a wave takes 64 consecutive quads (256 tokens) of one row, every lane loads its
// quad once with one 16-byte load, and the K-1 neighbouring inputs an output needs
// from the quad next to it come from the neighbouring lane through a wave shuffle
// instead of a second load; only the lane at the end of the wave loads its three
// halo elements itself.
#include "lbscan_device.h"
#include "lbscan_internal.h"

namespace lbscan {
namespace {

constexpr int kConvWaves = 4;          // waves per block, one chunk of a row each

// x[row, t] for t in [0, L), 0 outside
template <typename T>
__device__ __forceinline__ float load_or_zero(const T* __restrict__ row, int t, int L)
{
    const int tc = t < 0 ? 0 : (t >= L ? L - 1 : t);
    const float v = to_f32(row[tc]);
    return t == tc ? v : 0.0f;
}

// The lane's own quad and the three inputs on the side the filter reaches to:
// win[0..2] = x[t0-3 .. t0-1], win[3..6] = x[t0 .. t0+3] (forward direction), or
// win[0..3] = x[t0 .. t0+3], win[4..6] = x[t0+4 .. t0+6] (reversed direction).
// Lanes whose quad lies outside the row hold zeros.
template <typename T>
__device__ __forceinline__ void load_window(const T* __restrict__ row, int t0, int L, bool vec_ok,
                                            bool rev, int lane, float win[7])
{
    float cur[4];
    const bool active = t0 >= 0 && t0 < L;
    if (active && vec_ok && t0 + 4 <= L) {
        quad_load_fast<T>(row, t0, cur);
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) cur[e] = active ? load_or_zero<T>(row, t0 + e, L) : 0.0f;
    }
    float halo[3];
    if (!rev) {
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
template <int K>
__device__ __forceinline__ float conv_at(const float win[7], const float (&w)[K], float bias, bool rev, int e)
{
    float pre = bias;
#pragma unroll
    for (int k = 0; k < K; ++k)
        pre = fmaf(w[k], rev ? win[e + (K - 1) - k] : win[3 + e - (K - 1) + k], pre);
    return pre;
}

template <typename T, int K>
__global__ void __launch_bounds__(64 * kConvWaves)
conv1d_fwd_kernel(const ConvParams p)
{
    const int lane = threadIdx.x & 63;
    const int L = p.seqlen;
    const long nq = (L + 3) / 4, chunks = (nq + 63) / 64;
    const long c = (long)blockIdx.x * kConvWaves + (threadIdx.x >> 6);
    if (c >= (long)p.batch * p.dim * chunks) return;            // whole wave
    const long r = c / chunks;
    const int t0 = (int)(((c % chunks) * 64 + lane) * 4);
    const int d = (int)(r % p.dim);
    const bool rev = p.reverse != 0;
    const bool vec_ok = sizeof(T) == 4 || (L % 2 == 0);
    const T* __restrict__ xr = static_cast<const T*>(p.x) + r * L;
    T* __restrict__ yr = static_cast<T*>(p.y) + r * L;

    float w[K];
#pragma unroll
    for (int k = 0; k < K; ++k) w[k] = p.weight[(long)d * K + k];
    const float bias = p.bias ? p.bias[d] : 0.0f;

    float win[7];
    load_window<T>(xr, t0, L, vec_ok, rev, lane, win);
    if (t0 >= L) return;
    float out[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float pre = conv_at<K>(win, w, bias, rev, e);
        out[e] = p.activation ? pre * sigmoid_f32(pre) : pre;
    }
    quad_store<T>(yr, t0, vec_ok && t0 + 4 <= L, t0, L, out);
}

// Gradient.  dpre_t = dy_t * dSiLU(pre_t); an input s collects w[k] dpre_t from the
// K outputs that read it, which lie in the lane's own quad and in the quad on the
// other side than the forward halo, so dpre of the neighbouring lane is shuffled
// in.  For that, consecutive chunks of a row overlap by one quad: 63 lanes own
// their quad (write dx, add to the filter and bias sums), the 64th only supplies
// dpre.  The filter and bias sums are folded over the wave and added with one
// atomic per wave and tap.
template <typename T, int K>
__global__ void __launch_bounds__(64 * kConvWaves)
conv1d_bwd_kernel(const ConvParams p)
{
    const int lane = threadIdx.x & 63;
    const int L = p.seqlen;
    const long nq = (L + 3) / 4, chunks = (nq + 62) / 63;
    const long c = (long)blockIdx.x * kConvWaves + (threadIdx.x >> 6);
    if (c >= (long)p.batch * p.dim * chunks) return;            // whole wave
    const long r = c / chunks;
    const bool rev = p.reverse != 0;
    const long q = (c % chunks) * 63 - (rev ? 1 : 0) + lane;
    const int t0 = (int)(q * 4);
    const int d = (int)(r % p.dim);
    const bool vec_ok = sizeof(T) == 4 || (L % 2 == 0);
    const bool active = t0 >= 0 && t0 < L;
    const bool own = active && (rev ? lane >= 1 : lane <= 62);
    const T* __restrict__ xr = static_cast<const T*>(p.x) + r * L;
    const T* __restrict__ gr = static_cast<const T*>(p.dy) + r * L;
    T* __restrict__ dxr = static_cast<T*>(p.dx) + r * L;

    float w[K];
#pragma unroll
    for (int k = 0; k < K; ++k) w[k] = p.weight[(long)d * K + k];
    const float bias = p.bias ? p.bias[d] : 0.0f;

    float win[7], dy[4];
    load_window<T>(xr, t0, L, vec_ok, rev, lane, win);
    if (active && vec_ok && t0 + 4 <= L) {
        quad_load_fast<T>(gr, t0, dy);
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) dy[e] = active ? load_or_zero<T>(gr, t0 + e, L) : 0.0f;
    }

    // dpre of the own quad (zero past the end of the row: dy is zero there)
    float dpre[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float pre = conv_at<K>(win, w, bias, rev, e);
        float g = dy[e];
        if (p.activation) {
            const float sg = sigmoid_f32(pre);
            g *= sg * fmaf(pre, 1.0f - sg, 1.0f);
        }
        dpre[e] = g;
    }
    // dwin[j]: dpre around the own quad on the side the outputs that read it lie
    float dwin[7];
    if (!rev) {
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

    float acc[K + 1];
#pragma unroll
    for (int k = 0; k <= K; ++k) acc[k] = 0.0f;
    if (own) {
        float dx[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            // input t0+e is read through tap k by output t0+e+(K-1)-k (forward
            // direction) or t0+e-(K-1)+k (reversed)
            float s = 0.0f;
#pragma unroll
            for (int k = 0; k < K; ++k)
                s = fmaf(w[k], rev ? dwin[3 + e - (K - 1) + k] : dwin[e + (K - 1) - k], s);
            dx[e] = s;
#pragma unroll
            for (int k = 0; k < K; ++k)
                acc[k] = fmaf(dpre[e], rev ? win[e + (K - 1) - k] : win[3 + e - (K - 1) + k], acc[k]);
            acc[K] += dpre[e];
        }
        quad_store<T>(dxr, t0, vec_ok && t0 + 4 <= L, t0, L, dx);
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

template <typename T, int K>
hipError_t launch_conv_k(const ConvParams& p, bool bwd, hipStream_t s)
{
    const long nq = (p.seqlen + 3) / 4;
    const long chunks = bwd ? (nq + 62) / 63 : (nq + 63) / 64;
    const long waves = (long)p.batch * p.dim * chunks;
    const long blocks = (waves + kConvWaves - 1) / kConvWaves;
    if (blocks > 0x7fffffffL) return hipErrorInvalidConfiguration;
    if (bwd)
        hipLaunchKernelGGL((conv1d_bwd_kernel<T, K>), dim3((unsigned)blocks), dim3(64 * kConvWaves), 0, s, p);
    else
        hipLaunchKernelGGL((conv1d_fwd_kernel<T, K>), dim3((unsigned)blocks), dim3(64 * kConvWaves), 0, s, p);
    return hipGetLastError();
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
