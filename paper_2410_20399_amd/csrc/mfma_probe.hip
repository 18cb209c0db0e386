// Measurement aid: a bare stream of v_mfma_f32_32x32x16_bf16 on caller-supplied operands.
//
// The attention kernels are priced against the published dense bf16 rate (2.5 PFLOP/s at
// 2.4 GHz).  What the matrix pipe sustains depends on the clock the chip holds under the load,
// and that clock depends on the operand VALUES (constant operands toggle few wires).  This
// kernel has nothing but MFMAs in its loop, so its rate is the ceiling for any kernel fed with
// the same kind of data.
#include "tk_common.h"
#include "tk_launch.h"

namespace tk {

// One wave per SIMD (256 threads, one workgroup per compute unit); every wave keeps four
// independent accumulators, so the pipe never waits on a dependency.
__global__ __launch_bounds__(256, 1)
void mfma_probe_kernel(const bf16x8* __restrict__ operands, float* __restrict__ sink, int iters)
{
    // operands: 16 fragments of 256 lanes x 16 bytes
    bf16x8 a[8], b[8];
#pragma unroll
    for (int i = 0; i < 8; i++) {
        a[i] = operands[(size_t)i * 256 + threadIdx.x];
        b[i] = operands[(size_t)(8 + i) * 256 + threadIdx.x];
    }
    f32x16 c[4];
#pragma unroll
    for (int j = 0; j < 4; j++)
#pragma unroll
        for (int r = 0; r < 16; r++) c[j][r] = 0.f;
#pragma unroll 1
    for (int it = 0; it < iters; it++) {
#pragma unroll
        for (int i = 0; i < 8; i++)
#pragma unroll
            for (int j = 0; j < 4; j++) c[j] = mfma32(a[i], b[(i + j) & 7], c[j]);
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 4; j++)
#pragma unroll
        for (int r = 0; r < 16; r++) s += c[j][r];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

hipError_t launch_mfma_probe(const void* operands, float* sink, int workgroups, int iters, hipStream_t stream)
{
    hipLaunchKernelGGL(mfma_probe_kernel, dim3(workgroups), dim3(256), 0, stream,
                       (const bf16x8*)operands, sink, iters);
    return hipGetLastError();
}

}  // namespace tk
