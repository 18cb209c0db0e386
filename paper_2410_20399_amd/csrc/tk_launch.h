// Host-side launchers implemented by the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

#include <atomic>

namespace tk {

// Compute units of the current device (persistent kernels size their grid by it).  The attribute is
// queried once per device and cached; a launch then costs one hipGetDevice (a thread-local read).
inline hipError_t compute_unit_count(int* cus) {
    constexpr int kMaxDevices = 64;
    static std::atomic<int> cache[kMaxDevices];      // 0 = not queried yet
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < kMaxDevices) {
        const int hit = cache[dev].load(std::memory_order_relaxed);
        if (hit > 0) { *cus = hit; return hipSuccess; }
    }
    e = hipDeviceGetAttribute(cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e == hipSuccess && dev >= 0 && dev < kMaxDevices) cache[dev].store(*cus, std::memory_order_relaxed);
    return e;
}

// H query heads share Hkv key/value heads in groups of H / Hkv consecutive heads (Hkv == H: plain
// multi-head attention); Nq queries, Nk keys per head (causal: aligned at their ends, Nq <= Nk).
// q, o, d_o, dq: [B,H,Nq,D]; k, v, dk, dv: [B,Hkv,Nk,D]; lse, delta: [B,H,Nq].
hipError_t launch_attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse,
                           int B, int H, int Hkv, int Nq, int Nk, int D, int causal, float scale, hipStream_t stream);

// The same forward, non-causal, with the keys split n_splits (>= 2) ways and a merge kernel behind it
// (decode-shaped calls).  o_part: fp32 [n_splits][B*H][Nq][D]; lse_part: fp32 [n_splits][B*H][Nq];
// tiles_per_split: even number of 64-key tiles per split, (n_splits - 1) * tiles_per_split * 64 < Nk.
hipError_t launch_attn_fwd_splitk(const void* q, const void* k, const void* v, void* o, float* lse,
                                  float* o_part, float* lse_part,
                                  int B, int H, int Hkv, int Nq, int Nk, int D, float scale,
                                  int n_splits, int tiles_per_split, hipStream_t stream);

// Delta_i = sum_d dO_id O_id
hipError_t launch_attn_bwd_delta(const void* o, const void* d_o, float* delta,
                                 int B, int H, int N, int D, hipStream_t stream);

// The dS blocks that the dK/dV kernel can leave behind for launch_attn_bwd_dq_from_ds: one 2 KB block per
// (query head, 128-key tile, 32-query block, wave of 32 keys).  Query blocks per head: the dK/dV kernel walks
// them in pairs from a multiple of 32, so up to two past the last real one.
inline int ds_query_blocks(int Nq) { return Nq / 32 + 2; }
inline size_t ds_spill_bytes(int B, int H, int Nq, int Nk) {
    return (size_t)B * H * (size_t)((Nk + 127) / 128) * (size_t)ds_query_blocks(Nq) * 8192;
}

// dK, dV (key-tile parallel).  ds != nullptr: also store the dS blocks there (ds_spill_bytes(B, H, Nq, Nk) bytes).
hipError_t launch_attn_bwd_dkdv(const void* q, const void* k, const void* v, const void* d_o,
                                const float* lse, const float* delta, void* dk, void* dv,
                                int B, int H, int Hkv, int Nq, int Nk, int D, int causal, float scale, hipStream_t stream,
                                void* ds = nullptr);

// dQ = scale * dS K from the blocks a launch_attn_bwd_dkdv call with the same shape arguments stored
hipError_t launch_attn_bwd_dq_from_ds(const void* k, const void* ds, void* dq,
                                      int B, int H, int Hkv, int Nq, int Nk, int D, int causal, float scale, hipStream_t stream);

// dQ (query-tile parallel).  With o != nullptr the kernel computes Delta itself from o and d_o, writes it to
// delta_out (for the dK/dV kernel launched after it) and does not read delta.
hipError_t launch_attn_bwd_dq(const void* q, const void* k, const void* v, const void* d_o,
                              const float* lse, const float* delta, void* dq,
                              int B, int H, int Hkv, int Nq, int Nk, int D, int causal, float scale, hipStream_t stream,
                              const void* o = nullptr, float* delta_out = nullptr);

// bf16 matrix multiply C = A B: A [M,K], B [K,N], C [M,N] row-major; M >= 1, N and K multiples of 8
hipError_t launch_gemm(const void* a, const void* b, void* c, int M, int N, int K, hipStream_t stream);

// rotary positional encoding: x, o [B,H,N,D]; sin, cos [N, D/2]
hipError_t launch_rotary(const void* x, const void* sn, const void* cs, void* o,
                         int B, int H, int N, int D, hipStream_t stream);

// bare MFMA stream (measurement aid): 32 MFMAs per wave per iteration
hipError_t launch_mfma_probe(const void* operands, float* sink, int workgroups, int iters, hipStream_t stream);

}  // namespace tk
