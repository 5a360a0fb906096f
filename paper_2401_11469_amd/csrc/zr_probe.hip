// Measuring aid: what the matrix cores of this chip sustain with nothing else
// in the way -- bf16 MFMAs on register operands, no memory traffic -- so that
// the GEMM kernels' rates can be set against the clock the chip actually holds
// under this load, next to the published peak.
#include "zr_common.h"

namespace zr {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int CHAINS = 8;      // independent accumulators per wavefront: no MFMA waits for another

__global__ __launch_bounds__(256) void mfma_rate_kernel(int iters, float* sink)
{
    const int lane = threadIdx.x & 63;
    bf16x8 a, b;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        // small, lane-dependent values of both signs (not all-zero operands, which would draw less power)
        a[q] = (__bf16)((float)(((lane * 7 + q * 3) % 13) - 6) * 0.125f);
        b[q] = (__bf16)((float)(((lane * 5 + q) % 11) - 5) * 0.0078125f);
    }
    f32x16 acc[CHAINS];
#pragma unroll
    for (int c = 0; c < CHAINS; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[c][r] = 0.f;
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int c = 0; c < CHAINS; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[c], 0, 0, 0);
    }
    float sum = 0.f;
#pragma unroll
    for (int c = 0; c < CHAINS; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) sum += acc[c][r];
    // one word per workgroup, so that the work cannot be removed
    if (threadIdx.x == 0) sink[blockIdx.x] = sum;
}

}  // namespace

double mfma_rate_flops(int blocks, int iters)
{
    // 4 wavefronts per workgroup, CHAINS MFMAs of 32 x 32 x 16 per iteration
    return (double)blocks * 4.0 * (double)iters * CHAINS * 2.0 * 32.0 * 32.0 * 16.0;
}

int launch_mfma_rate(int blocks, int iters, float* sink, hipStream_t stream)
{
    hipLaunchKernelGGL(mfma_rate_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, iters, sink);
    return hip_status(hipGetLastError());
}

}  // namespace zr
