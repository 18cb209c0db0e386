// Host-side launchers implemented by the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

namespace tk {

hipError_t launch_attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse,
                           int B, int H, int N, int D, int causal, float scale, hipStream_t stream);

// Delta_i = sum_d dO_id O_id; optionally also clears the fp32 dQ accumulator rows it walks over.
hipError_t launch_attn_bwd_delta(const void* o, const void* d_o, float* delta, float* dq_acc_or_null,
                                 int B, int H, int N, int D, hipStream_t stream);

hipError_t launch_attn_bwd_main(const void* q, const void* k, const void* v, const void* d_o,
                                const float* lse, const float* delta, float* dq_acc,
                                void* dk, void* dv,
                                int B, int H, int N, int D, int causal, float scale, hipStream_t stream);

// dq = bf16(scale * dq_acc)
hipError_t launch_attn_bwd_dq_convert(const float* dq_acc, void* dq, size_t n_elems, float scale,
                                      hipStream_t stream);

}  // namespace tk
