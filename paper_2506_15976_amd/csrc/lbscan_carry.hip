// Carry chain of the segmented forward pass.
//
// When a row is cut into segments that different blocks scan at the same time,
// a first launch leaves, per segment s, row and state n, the state e_s the
// segment reaches from a zero state, and the sum S_s of its time steps.  The
// recurrence of Eq. 1 (Sec. 3.1) is linear, so the state entering segment s+1
// is  c_{s+1} = exp(A S_s) c_s + e_s  with c_0 = 0: the product of the
// segment's abar factors is exp(A * sum of dt).  A step of that chain is the
// affine map c -> P c + e, and affine maps compose associatively, so a group of
// G lanes (G a power of two, at most a wave) takes G consecutive segments of one
// (row, n) pair, forms the running composition with a shuffle scan, and each
// lane overwrites its e_s by the state c_s entering its segment.  Chains longer
// than G are walked in chunks of G with the carried state passed along.  The
// backward pass's right-to-left recurrence psi_t = abar_t (e_t + psi_{t+1})
// chains the same way with the segments walked from the last to the first.
#include "lbscan_device.h"
#include "lbscan_internal.h"

namespace lbscan {
namespace {

__global__ void __launch_bounds__(256)
carry_chain_kernel(float* __restrict__ carry, const float* __restrict__ dsum,
                   const float* __restrict__ A, const float* __restrict__ init,
                   int rows, int D, int N, int nseg, int nsum, int reverse, int G)
{
    const long npairs = (long)rows * N;
    const long t = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const int g = (int)(t % G);                       // segment within the chunk
    const long pair = t / G;                          // (row, n)
    const bool valid = pair < npairs;
    const long i = valid ? pair : npairs - 1;         // clamped: every lane shuffles
    const int row = (int)(i / N), n = (int)(i % N);
    const float a2 = A[(long)(row % D) * N + n] * kLog2e;
    float cin = init ? init[i] : 0.0f;                // state entering the chunk
    for (int base = 0; base < nseg; base += G) {
        const int ss = base + g;
        const bool on = ss < nseg;
        const int s = reverse ? nseg - 1 - (on ? ss : 0) : (on ? ss : 0);
        const long k = ((long)s * N + n) * rows + row;        // (segment, n, row)
        // lanes past the end of the chain, and segments whose summary was not
        // computed (ss >= nsum: the last one, which nothing follows), hold the
        // identity map
        const bool have = on && ss < nsum;
        float e = have ? carry[k] : 0.0f;
        float P = have ? fast_exp2(a2 * dsum[(long)s * rows + row]) : 1.0f;
        // inclusive scan: lane g ends with the composition of segments base..base+g
        for (int d = 1; d < G; d <<= 1) {
            const float Pp = __shfl_up(P, d, G), ep = __shfl_up(e, d, G);
            if (g >= d) { e = fmaf(P, ep, e); P *= Pp; }
        }
        const float Pm = __shfl_up(P, 1, G), em = __shfl_up(e, 1, G);
        const float c = g == 0 ? cin : fmaf(Pm, cin, em);
        if (on && valid) carry[k] = c;
        const float Pl = __shfl(P, G - 1, G), el = __shfl(e, G - 1, G);
        cin = fmaf(Pl, cin, el);
    }
}

__global__ void __launch_bounds__(256) zero_kernel(float* __restrict__ dst, long n)
{
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = 0.0f;
}

// Clears up to kZeroMany buffers in one launch: block x belongs to the buffer whose
// range of blocks contains it.
__global__ void __launch_bounds__(256) zero_many_kernel(const ZeroMany z)
{
    long blk = blockIdx.x;
#pragma unroll
    for (int k = 0; k < kZeroMany; ++k) {
        const long nb = (z.n[k] + 255) / 256;
        if (blk < nb) {
            const long i = blk * 256 + threadIdx.x;
            if (i < z.n[k]) z.dst[k][i] = 0.0f;
            return;
        }
        blk -= nb;
    }
}

__global__ void __launch_bounds__(256)
copy_kernel(float* __restrict__ dst, const float* __restrict__ src, long n)
{
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src[i];
}

// lanes per (row, n) pair: the smallest power of two that covers the chain, one
// wave at most
int chain_group(int nseg)
{
    int G = 1;
    while (G < nseg && G < 64) G <<= 1;
    return G;
}

}  // namespace

hipError_t launch_zero(float* dst, long n, hipStream_t stream)
{
    if (n <= 0 || !dst) return hipSuccess;
    hipLaunchKernelGGL(zero_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, dst, n);
    return hipGetLastError();
}

hipError_t launch_zero_many(ZeroMany z, hipStream_t stream)
{
    long blocks = 0;
    for (int k = 0; k < kZeroMany; ++k) {
        if (!z.dst[k] || z.n[k] < 0) z.n[k] = 0;
        blocks += (z.n[k] + 255) / 256;
    }
    if (blocks == 0) return hipSuccess;
    if (blocks > 0x7fffffffL) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(zero_many_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, z);
    return hipGetLastError();
}

hipError_t launch_copy(float* dst, const float* src, long n, hipStream_t stream)
{
    if (!src) return launch_zero(dst, n, stream);
    if (n <= 0 || !dst) return hipSuccess;
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, dst, src, n);
    return hipGetLastError();
}

hipError_t launch_carry_chain(const FwdParams& p, hipStream_t stream)
{
    const int rows = p.batch * p.dim;
    const long n = (long)rows * p.dstate;
    if (n == 0) return hipSuccess;
    const int G = chain_group(p.nseg);
    const unsigned blocks = (unsigned)((n * G + 255) / 256);
    hipLaunchKernelGGL(carry_chain_kernel, dim3(blocks), dim3(256), 0, stream,
                       p.carry, p.dsum, p.A, p.h0, rows, p.dim, p.dstate, p.nseg,
                       p.ckpt ? p.nseg : p.nseg - 1, 0, G);
    return hipGetLastError();
}

hipError_t launch_carry_chain_reverse(const FwdParams& p, float* buf, const float* init,
                                      hipStream_t stream)
{
    const int rows = p.batch * p.dim;
    const long n = (long)rows * p.dstate;
    if (n == 0) return hipSuccess;
    const int G = chain_group(p.nseg);
    const unsigned blocks = (unsigned)((n * G + 255) / 256);
    hipLaunchKernelGGL(carry_chain_kernel, dim3(blocks), dim3(256), 0, stream,
                       buf, p.dsum, p.A, init, rows, p.dim, p.dstate, p.nseg, p.nseg, 1, G);
    return hipGetLastError();
}

}  // namespace lbscan
