// Carry chain of the segmented forward pass.
//
// When a row is cut into segments that different blocks scan at the same time,
// a first launch leaves, per segment s, row and state n, the state e_s the
// segment reaches from a zero state, and the sum S_s of its time steps.  The
// recurrence of Eq. 1 (Sec. 3.1) is linear, so the state entering segment s+1
// is  c_{s+1} = exp(A S_s) c_s + e_s  with c_0 = 0: the product of the
// segment's abar factors is exp(A * sum of dt).  One lane per (row, n) walks
// the segments in order and overwrites e_s by c_s in place.  The backward pass's
// right-to-left recurrence psi_t = abar_t (e_t + psi_{t+1}) chains the same way
// with the segments walked from the last to the first.
#include "lbscan_device.h"
#include "lbscan_internal.h"

namespace lbscan {
namespace {

__global__ void __launch_bounds__(256)
carry_chain_kernel(float* __restrict__ carry, const float* __restrict__ dsum,
                   const float* __restrict__ A, int rows, int D, int N, int nseg, int reverse)
{
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;   // (row, n)
    if (i >= (long)rows * N) return;
    const int row = (int)(i / N), n = (int)(i % N);
    const float a2 = A[(long)(row % D) * N + n] * kLog2e;
    float c = 0.0f;
    for (int ss = 0; ss < nseg; ++ss) {
        const int s = reverse ? nseg - 1 - ss : ss;
        const long k = (long)s * rows * N + i;
        const float e = carry[k];
        carry[k] = c;
        c = fmaf(fast_exp2(a2 * dsum[(long)s * rows + row]), c, e);
    }
}

__global__ void __launch_bounds__(256) zero_kernel(float* __restrict__ dst, long n)
{
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = 0.0f;
}

}  // namespace

hipError_t launch_zero(float* dst, long n, hipStream_t stream)
{
    if (n <= 0 || !dst) return hipSuccess;
    hipLaunchKernelGGL(zero_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, dst, n);
    return hipGetLastError();
}

hipError_t launch_carry_chain(const FwdParams& p, hipStream_t stream)
{
    const int rows = p.batch * p.dim;
    const long n = (long)rows * p.dstate;
    if (n == 0) return hipSuccess;
    const unsigned blocks = (unsigned)((n + 255) / 256);
    hipLaunchKernelGGL(carry_chain_kernel, dim3(blocks), dim3(256), 0, stream,
                       p.carry, p.dsum, p.A, rows, p.dim, p.dstate, p.nseg, 0);
    return hipGetLastError();
}

hipError_t launch_carry_chain_reverse(const FwdParams& p, float* buf, hipStream_t stream)
{
    const int rows = p.batch * p.dim;
    const long n = (long)rows * p.dstate;
    if (n == 0) return hipSuccess;
    const unsigned blocks = (unsigned)((n + 255) / 256);
    hipLaunchKernelGGL(carry_chain_kernel, dim3(blocks), dim3(256), 0, stream,
                       buf, p.dsum, p.A, rows, p.dim, p.dstate, p.nseg, 1);
    return hipGetLastError();
}

}  // namespace lbscan
