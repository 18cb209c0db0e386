// Rotary positional encoding for gfx950 (MI355X): o1 = x1 cos - x2 sin, o2 = x2 cos + x1 sin with
// x1, x2 the two halves of each row (the rotary kernel of the paper's appendix, head dimension D).
//
// The operation moves 4*D bytes per row against 3*D flops: it is bound by HBM.  One thread owns
// 8 consecutive columns of x1 and the matching 8 of x2 (two 16-byte loads, two 16-byte stores),
// so a wave reads and writes whole 128-byte segments; sin and cos are [N, D/2] and are re-read by
// every head from L2.  Arithmetic in fp32, one round-to-nearest-even to bf16.
#include "tk_common.h"
#include "tk_launch.h"

namespace tk {

template <int D>
__global__ __launch_bounds__(256)
void rotary_kernel(const bf16* X, const bf16* __restrict__ Sin, const bf16* __restrict__ Cos,   // X and O may be the same buffer
                   bf16* O, int N, size_t n_items)
{
    constexpr int kChunks = D / 16;                      // 8-column chunks per half row
    const size_t item = (size_t)blockIdx.x * 256 + threadIdx.x;   // (row, chunk)
    if (item >= n_items) return;
    const size_t row = item / kChunks;
    const int chunk = (int)(item % kChunks);
    const int pos = (int)(row % N);
    const bf16* xr = X + row * D + chunk * 8;
    const bf16x8 a = *(const bf16x8*)xr;
    const bf16x8 b = *(const bf16x8*)(xr + D / 2);
    const bf16x8 sn = *(const bf16x8*)(Sin + (size_t)pos * (D / 2) + chunk * 8);
    const bf16x8 cs = *(const bf16x8*)(Cos + (size_t)pos * (D / 2) + chunk * 8);
    float o1[8], o2[8];
#pragma unroll
    for (int e = 0; e < 8; e++) {
        const float x1 = (float)a[e], x2 = (float)b[e], s = (float)sn[e], c = (float)cs[e];
        o1[e] = __builtin_fmaf(x1, c, -(x2 * s));
        o2[e] = __builtin_fmaf(x2, c, x1 * s);
    }
    bf16* orow = O + row * D + chunk * 8;
    *(bf16x8*)orow = cvt8(o1[0], o1[1], o1[2], o1[3], o1[4], o1[5], o1[6], o1[7]);
    *(bf16x8*)(orow + D / 2) = cvt8(o2[0], o2[1], o2[2], o2[3], o2[4], o2[5], o2[6], o2[7]);
}

hipError_t launch_rotary(const void* x, const void* sn, const void* cs, void* o,
                         int B, int H, int N, int D, hipStream_t stream)
{
    const size_t n_items = (size_t)B * H * N * (D / 16);
    const dim3 grid((unsigned)((n_items + 255) / 256));
    if (D == 128) hipLaunchKernelGGL((rotary_kernel<128>), grid, dim3(256), 0, stream, (const bf16*)x, (const bf16*)sn, (const bf16*)cs, (bf16*)o, N, n_items);
    else          hipLaunchKernelGGL((rotary_kernel<64>), grid, dim3(256), 0, stream, (const bf16*)x, (const bf16*)sn, (const bf16*)cs, (bf16*)o, N, n_items);
    return hipGetLastError();
}

}  // namespace tk
