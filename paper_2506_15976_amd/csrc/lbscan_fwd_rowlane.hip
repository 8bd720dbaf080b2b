// Forward kernel, "row per lane" mapping.
//
// Each lane owns one (batch, channel) row and walks it left to right with the
// N states in registers, so the global forward recurrence (Sec. 3.1, Eq. 1)
// needs no cross-lane scan at all, and the local backward recurrence of each
// M-token window (Sec. 3.2, Eq. 7) runs in registers right after the forward
// steps of that window, on the same abar and u values.  The output of Eq. 8
// with the skip term, and the SiLU gate of Algorithm 1, are fused in.
//
// All lanes of a block belong to one batch entry, so Bm[b,n,t] and Cm[b,n,t]
// are the same for every lane: they are staged once per block in LDS and read
// back as broadcasts.  The (B,D,L) tensors are contiguous along L, which is the
// wrong way round for a lane-per-row walk, so a tile of TT tokens of all rows
// of the block is loaded with coalesced quad loads, transformed (bias,
// softplus) and transposed through LDS; y goes back the same way and is gated
// on the way out.  Tokens past the end of the row are staged as dt = 0, x = 0,
// which leaves the states untouched (abar = 1, u = 0) and makes the ragged last
// window an ordinary short window.
//
// reverse = 1 stages the tile mirrored (logical token j <-> physical L-1-j), so
// the scan phase is the same code for both directions.
#include "lbscan_device.h"
#include "lbscan_internal.h"

namespace lbscan {
namespace {

constexpr int kTT = 16;            // tokens per tile
constexpr int kTS = kTT + 1;       // LDS row stride in floats (odd: conflict-free column walks)
constexpr int kQ = kTT / 4;        // quads per row per tile
constexpr int kMaxRows = 256;      // lanes (rows) per block

template <typename T, int NS, int M, bool REV>
__global__ void __launch_bounds__(kMaxRows)
rowlane_fwd_kernel(const FwdParams p)
{
    constexpr int GT = M > 4 ? M : 4;   // tokens handled per register group
    static_assert(kTT % GT == 0, "tile must hold whole groups");
    __shared__ float sx[kMaxRows * kTS];   // x, later y
    __shared__ float sd[kMaxRows * kTS];   // time step dt
    __shared__ __attribute__((aligned(16))) float sB[NS * kTT];
    __shared__ __attribute__((aligned(16))) float sC[NS * kTT];

    const int R = blockDim.x, tid = threadIdx.x;
    const int L = p.seqlen, D = p.dim, N = p.dstate;
    const int nbx = (D + R - 1) / R;             // blocks per batch entry
    const int b = blockIdx.x / nbx, d0 = (blockIdx.x % nbx) * R;
    const int d = d0 + tid;
    const bool row_ok = d < D;

    const T* __restrict__ xg = static_cast<const T*>(p.x);
    const T* __restrict__ dg = static_cast<const T*>(p.delta);
    const T* __restrict__ zg = static_cast<const T*>(p.z);
    const T* __restrict__ Bg = static_cast<const T*>(p.Bm);
    const T* __restrict__ Cg = static_cast<const T*>(p.Cm);

    float A2[NS], f[NS];
#pragma unroll
    for (int n = 0; n < NS; ++n) {
        A2[n] = (row_ok && n < N) ? p.A[(long)d * N + n] * kLog2e : 0.0f;
        f[n] = 0.0f;
    }
    const float Dd = (row_ok && p.Dskip) ? p.Dskip[d] : 0.0f;

    const int ntiles = (L + kTT - 1) / kTT;
    for (int tile = 0; tile < ntiles; ++tile) {
        const int j0 = tile * kTT;   // first logical token of the tile

        // ---- load phase: x, delta -> (bias, softplus) -> LDS, transposed ----
        for (int k = tid; k < R * kQ; k += R) {
            const int row = k / kQ, q = k % kQ;
            const int dd = d0 + row;
            float xv[4] = {0.f, 0.f, 0.f, 0.f}, dv[4] = {0.f, 0.f, 0.f, 0.f};
            const int jq = j0 + 4 * q;
            const int i0 = REV ? (L - 4 - jq) : jq;   // physical token of quad element 0
            if (dd < D) {
                const long rowbase = ((long)b * D + dd) * L;
                const bool vec_ok = sizeof(T) == 4 || (((rowbase + i0) & 1) == 0);
                load_quad<T>(xg, rowbase + i0, rowbase, rowbase + L, vec_ok, xv);
                load_quad<T>(dg, rowbase + i0, rowbase, rowbase + L, vec_ok, dv);
                const float bias = p.bias ? p.bias[dd] : 0.0f;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int ph = i0 + e;
                    float v = dv[e] + bias;
                    v = p.softplus ? softplus_f32(v) : v;
                    dv[e] = (ph >= 0 && ph < L) ? v : 0.0f;
                }
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int pos = 4 * q + (REV ? 3 - e : e);
                sx[row * kTS + pos] = xv[e];
                sd[row * kTS + pos] = dv[e];
            }
        }
        // ---- Bm, Cm tile -> LDS as [n][t] ----
        for (int k = tid; k < 2 * NS * kQ; k += R) {
            const int which = k / (NS * kQ);
            const int n = (k / kQ) % NS, q = k % kQ;
            float v[4] = {0.f, 0.f, 0.f, 0.f};
            const int jq = j0 + 4 * q;
            const int i0 = REV ? (L - 4 - jq) : jq;
            if (n < N) {
                const long rowbase = ((long)b * N + n) * L;
                const bool vec_ok = sizeof(T) == 4 || (((rowbase + i0) & 1) == 0);
                load_quad<T>(which ? Cg : Bg, rowbase + i0, rowbase, rowbase + L, vec_ok, v);
            }
            float* dst = which ? sC : sB;
#pragma unroll
            for (int e = 0; e < 4; ++e) dst[n * kTT + 4 * q + (REV ? 3 - e : e)] = v[e];
        }
        __syncthreads();

        // ---- scan phase: this lane's row, kTT tokens, all states in registers ----
#pragma unroll
        for (int g0 = 0; g0 < kTT; g0 += GT) {
            float dl[GT], dx[GT], yv[GT];
#pragma unroll
            for (int t = 0; t < GT; ++t) {
                dl[t] = sd[tid * kTS + g0 + t];
                const float xx = sx[tid * kTS + g0 + t];
                dx[t] = dl[t] * xx;
                yv[t] = Dd * xx;
            }
#pragma unroll
            for (int n = 0; n < NS; ++n) {
                float a[GT], u[GT], cc[GT];
#pragma unroll
                for (int t = 0; t < GT; ++t) {
                    a[t] = fast_exp2(dl[t] * A2[n]);
                    u[t] = dx[t] * sB[n * kTT + g0 + t];
                    cc[t] = sC[n * kTT + g0 + t];
                }
                // global forward recurrence (Eq. 1) and its share of Eq. 8
                float fn = f[n];
#pragma unroll
                for (int t = 0; t < GT; ++t) {
                    fn = fmaf(a[t], fn, u[t]);
                    yv[t] = fmaf(cc[t], fn, yv[t]);
                }
                f[n] = fn;
                // local backward recurrence (Eq. 7) per window, carried without
                // the current input term so that B x is counted once (Eq. 8)
                if constexpr (M > 1) {
#pragma unroll
                    for (int w0 = 0; w0 < GT; w0 += M) {
                        // g is zero at the last step of the window
                        float g = a[w0 + M - 2] * u[w0 + M - 1];
                        yv[w0 + M - 2] = fmaf(cc[w0 + M - 2], g, yv[w0 + M - 2]);
#pragma unroll
                        for (int t = M - 3; t >= 0; --t) {
                            g = a[w0 + t] * (g + u[w0 + t + 1]);
                            yv[w0 + t] = fmaf(cc[w0 + t], g, yv[w0 + t]);
                        }
                    }
                }
            }
#pragma unroll
            for (int t = 0; t < GT; ++t) sx[tid * kTS + g0 + t] = yv[t];
        }
        __syncthreads();

        // ---- store phase: y from LDS, gate, coalesced store ----
        for (int k = tid; k < R * kQ; k += R) {
            const int row = k / kQ, q = k % kQ;
            const int dd = d0 + row;
            if (dd >= D) continue;
            const int jq = j0 + 4 * q;
            const int i0 = REV ? (L - 4 - jq) : jq;
            const long rowbase = ((long)b * D + dd) * L;
            const bool vec_ok = sizeof(T) == 4 || (((rowbase + i0) & 1) == 0);
            float yv[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) yv[e] = sx[row * kTS + 4 * q + (REV ? 3 - e : e)];
            if (p.yprev) {
                float pv[4];
                load_quad<float>(p.yprev, rowbase + i0, rowbase, rowbase + L, true, pv);
#pragma unroll
                for (int e = 0; e < 4; ++e) yv[e] += pv[e];
            }
            if (zg) {
                float zv[4];
                load_quad<T>(zg, rowbase + i0, rowbase, rowbase + L, vec_ok, zv);
#pragma unroll
                for (int e = 0; e < 4; ++e) yv[e] *= zv[e] * sigmoid_f32(zv[e]);
            }
            if (p.y_is_f32)
                store_quad<float>(static_cast<float*>(p.y), rowbase + i0, rowbase, rowbase + L, true, yv);
            else
                store_quad<T>(static_cast<T*>(p.y), rowbase + i0, rowbase, rowbase + L, vec_ok, yv);
        }
        __syncthreads();
    }
}

template <typename T, int NS, int M>
hipError_t launch_rev(const FwdParams& p, dim3 grid, dim3 block, hipStream_t s)
{
    if (p.reverse) hipLaunchKernelGGL((rowlane_fwd_kernel<T, NS, M, true>), grid, block, 0, s, p);
    else           hipLaunchKernelGGL((rowlane_fwd_kernel<T, NS, M, false>), grid, block, 0, s, p);
    return hipGetLastError();
}

template <typename T, int NS>
hipError_t launch_m(const FwdParams& p, dim3 grid, dim3 block, hipStream_t s)
{
    switch (p.window) {
        case 1:  return launch_rev<T, NS, 1>(p, grid, block, s);
        case 2:  return launch_rev<T, NS, 2>(p, grid, block, s);
        case 4:  return launch_rev<T, NS, 4>(p, grid, block, s);
        case 8:  return launch_rev<T, NS, 8>(p, grid, block, s);
        case 16: return launch_rev<T, NS, 16>(p, grid, block, s);
        default: return hipErrorInvalidValue;
    }
}

template <typename T>
hipError_t launch_n(const FwdParams& p, dim3 grid, dim3 block, hipStream_t s)
{
    if (p.dstate <= 8) return launch_m<T, 8>(p, grid, block, s);
    return launch_m<T, 16>(p, grid, block, s);
}

}  // namespace

// Rows per block: the largest multiple of 64 up to 256 that divides D, so that
// no lane idles; otherwise 256 (or D rounded up to a wave when D < 256).
static int pick_rows_per_block(int D)
{
    for (int k = 4; k >= 1; --k)
        if (D % (64 * k) == 0) return 64 * k;
    if (D >= kMaxRows) return kMaxRows;
    return ((D + 63) / 64) * 64;
}

hipError_t launch_fwd_rowlane(const FwdParams& p, hipStream_t stream)
{
    if (p.batch == 0 || p.dim == 0 || p.seqlen == 0) return hipSuccess;
    const int R = pick_rows_per_block(p.dim);
    const long nblocks = (long)((p.dim + R - 1) / R) * p.batch;
    if (nblocks > 0x7fffffffL) return hipErrorInvalidConfiguration;
    dim3 block(R), grid((unsigned)nblocks);
    if (p.dtype == 0) return launch_n<float>(p, grid, block, stream);
    return launch_n<bf16_t>(p, grid, block, stream);
}

}  // namespace lbscan
