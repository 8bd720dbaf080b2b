// Issue-rate probes for the ALU bound of the scan kernels: dependent chains of one
// instruction kind (fp32 fma, v_exp_f32, v_rcp_f32), eight independent chains per
// lane, so that the measured rate is the issue rate of that instruction and not
// its latency.  The caller times the launch (bench.py --alu-rates).
#include "lbscan_device.h"
#include "lbscan_internal.h"

namespace lbscan {
namespace {

constexpr int kChains = 8;        // independent chains per lane
constexpr int kUnroll = 16;       // steps of every chain per loop iteration

template <int WHICH>
__global__ void __launch_bounds__(256) probe_kernel(float* __restrict__ out, int iters, float a, float b)
{
    float x[kChains];
#pragma unroll
    for (int i = 0; i < kChains; ++i) x[i] = 1.0f + threadIdx.x * 0.001f + i * 0.01f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < kUnroll; ++r) {
#pragma unroll
            for (int i = 0; i < kChains; ++i) {
                if (WHICH == 0) x[i] = fmaf(x[i], a, b);
                if (WHICH == 1) x[i] = fast_exp2(-x[i]);
                if (WHICH == 2) x[i] = fast_rcp(x[i]);
            }
        }
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < kChains; ++i) s += x[i];
    out[(long)blockIdx.x * blockDim.x + threadIdx.x] = s;      // keeps the chains alive
}

}  // namespace

long probe_ops_per_lane(int iters) { return (long)iters * kUnroll * kChains; }

hipError_t launch_probe(int which, int blocks, int iters, float* out, hipStream_t stream)
{
    if (blocks <= 0 || iters <= 0 || !out) return hipErrorInvalidValue;
    dim3 grid((unsigned)blocks), block(256);
    switch (which) {
        case 0: hipLaunchKernelGGL(probe_kernel<0>, grid, block, 0, stream, out, iters, 0.999f, 0.001f); break;
        case 1: hipLaunchKernelGGL(probe_kernel<1>, grid, block, 0, stream, out, iters, 0.0f, 0.0f); break;
        case 2: hipLaunchKernelGGL(probe_kernel<2>, grid, block, 0, stream, out, iters, 0.0f, 0.0f); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace lbscan
