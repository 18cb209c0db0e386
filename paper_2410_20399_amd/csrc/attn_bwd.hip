// Fused exact softmax attention, backward pass, for gfx950 (MI355X).
//
// The paper reports the backward kernel's speed only (Section 4.1, Table 3); the algorithm
// here is the chain rule with P recomputed from the saved log-sum-exp:
//
//   kernel 1  Delta_i = sum_d dO_id O_id          (HBM stream; also clears the fp32 dQ accumulator)
//   kernel 2  one workgroup per 128-key tile, wave w owns keys 32w..32w+31, loop over 32-query blocks:
//               S  = Q_i K_j^T            P  = 2^(S*c - LSE_i*log2e)
//               dP = dO_i V_j^T           dS = P (dP - Delta_i)
//               dV_j^T += dO_i^T P        dK_j^T += Q_i^T dS
//               dQ_i   += dS K_j          (dS goes through LDS so that the contraction can run
//                                          over keys; partial dQ added to fp32 with atomics)
//   kernel 3  dQ = bf16(scale * accumulator)
//
// S and dP are produced with the KEY index on lanes and the query index on registers, so P and
// dS in accumulator layout are directly the B operands of the two products contracted over
// queries; their A operands (dO^T, Q^T) come from row-major LDS tiles via transposing reads.
#include "tk_common.h"
#include "tk_launch.h"

namespace tk {

// ------------------------------------------------------------------------------------------
// kernel 1: Delta, and zero-fill of the dQ accumulator
// ------------------------------------------------------------------------------------------
template <int D, bool ZERO>
__global__ __launch_bounds__(256)
void attn_bwd_delta_kernel(const bf16* __restrict__ O, const bf16* __restrict__ dO,
                           float* __restrict__ delta, float* __restrict__ dq_acc, size_t n_chunks)
{
    constexpr int kLanesPerRow = D / 8;
    const size_t chunk = (size_t)blockIdx.x * 256 + threadIdx.x;   // one 8-element chunk per thread
    if (chunk >= n_chunks) return;                                  // n_chunks is a multiple of 256: never taken
    bf16x8 a = *(const bf16x8*)(O + chunk * 8);
    bf16x8 b = *(const bf16x8*)(dO + chunk * 8);
    float acc = 0.f;
#pragma unroll
    for (int e = 0; e < 8; e++) acc = __builtin_fmaf((float)a[e], (float)b[e], acc);
#pragma unroll
    for (int off = kLanesPerRow / 2; off >= 1; off >>= 1) acc += __shfl_xor(acc, off);
    if ((threadIdx.x & (kLanesPerRow - 1)) == 0) delta[chunk / kLanesPerRow] = acc;
    if (ZERO) {
        f32x4 z = {0.f, 0.f, 0.f, 0.f};
        *(f32x4*)(dq_acc + chunk * 8) = z;
        *(f32x4*)(dq_acc + chunk * 8 + 4) = z;
    }
}

hipError_t launch_attn_bwd_delta(const void* o, const void* d_o, float* delta, float* dq_acc,
                                 int B, int H, int N, int D, hipStream_t stream)
{
    const size_t n_chunks = (size_t)B * H * N * D / 8;   // N % 128 == 0, so a multiple of 256
    const dim3 grid((unsigned)(n_chunks / 256));
    if (D == 128) {
        if (dq_acc) hipLaunchKernelGGL((attn_bwd_delta_kernel<128, true>), grid, dim3(256), 0, stream, (const bf16*)o, (const bf16*)d_o, delta, dq_acc, n_chunks);
        else        hipLaunchKernelGGL((attn_bwd_delta_kernel<128, false>), grid, dim3(256), 0, stream, (const bf16*)o, (const bf16*)d_o, delta, dq_acc, n_chunks);
    } else {
        if (dq_acc) hipLaunchKernelGGL((attn_bwd_delta_kernel<64, true>), grid, dim3(256), 0, stream, (const bf16*)o, (const bf16*)d_o, delta, dq_acc, n_chunks);
        else        hipLaunchKernelGGL((attn_bwd_delta_kernel<64, false>), grid, dim3(256), 0, stream, (const bf16*)o, (const bf16*)d_o, delta, dq_acc, n_chunks);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// kernel 3: dQ = bf16(scale * accumulator)
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256)
void attn_bwd_dq_convert_kernel(const float* __restrict__ acc, bf16* __restrict__ dq, size_t n_chunks, float scale)
{
    const size_t chunk = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (chunk >= n_chunks) return;
    f32x4 a = *(const f32x4*)(acc + chunk * 8);
    f32x4 b = *(const f32x4*)(acc + chunk * 8 + 4);
    *(bf16x8*)(dq + chunk * 8) = cvt8(a[0] * scale, a[1] * scale, a[2] * scale, a[3] * scale,
                                      b[0] * scale, b[1] * scale, b[2] * scale, b[3] * scale);
}

hipError_t launch_attn_bwd_dq_convert(const float* dq_acc, void* dq, size_t n_elems, float scale, hipStream_t stream)
{
    const size_t n_chunks = n_elems / 8;
    hipLaunchKernelGGL(attn_bwd_dq_convert_kernel, dim3((unsigned)((n_chunks + 255) / 256)), dim3(256), 0, stream,
                       dq_acc, (bf16*)dq, n_chunks, scale);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// kernel 2: dK, dV (and dQ partials)
// ------------------------------------------------------------------------------------------
template <int D>
struct BwdShape {
    static constexpr int kWaves = 4;
    static constexpr int kThreads = 256;
    static constexpr int kTileKV = 128;                 // keys per workgroup (32 per wave)
    static constexpr int kTileQ = 32;                   // queries per loop iteration
    static constexpr int kRowBytes = D * 2;
    static constexpr int kChunksPerRow = D / 8;
    static constexpr int kQTileBytes = kTileQ * kRowBytes;
    static constexpr int kStageBytes = 2 * kQTileBytes + 256;      // Q, dO, LSE[32], Delta[32]
    static constexpr int kKTileBytes = kTileKV * kRowBytes;
    static constexpr int kDsBytes = kTileKV * kTileQ * 2;          // dS^T [128 keys][32 queries] bf16
    static constexpr int kOffDs = 0;
    static constexpr int kOffStage = kOffDs + kDsBytes;
    static constexpr int kOffK = kOffStage + 2 * kStageBytes;
    static constexpr int kLdsBytes = kOffK + kKTileBytes;
    static constexpr int kQLoads = kTileQ * kChunksPerRow / kThreads;   // per thread, per tensor
    static constexpr int kKLoads = kTileKV * kChunksPerRow / kThreads;
    static constexpr int kDBlocksPerWave = 1;
    static constexpr int kKeyStepsPerWave = (D == 128) ? 8 : 4;    // 16-key MFMA steps of the dQ product
};

// Chunk swizzle of every row-major bf16 tile in this kernel (rows of D elements): spreads both a
// 16-row same-chunk read (MFMA operand rows) and a 4-row x 64-byte transposing read over the banks.
template <int D> __device__ __forceinline__ int swz(int row) {
    return D == 128 ? (((row & 3) << 2) | ((row >> 2) & 3)) : ((((row >> 1) & 1) << 2) | ((row >> 2) & 3));
}

template <int D, bool CAUSAL>
__global__ __launch_bounds__(256, (D == 128 ? 1 : 2))
void attn_bwd_main_kernel(const bf16* __restrict__ Q, const bf16* __restrict__ K, const bf16* __restrict__ V,
                          const bf16* __restrict__ dO, const float* __restrict__ LSE, const float* __restrict__ Delta,
                          float* __restrict__ dQacc, bf16* __restrict__ dK, bf16* __restrict__ dV,
                          int N, int num_kv_tiles, int total_wg, float scale)
{
    using S = BwdShape<D>;
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int l32 = lane & 31;
    const int h = lane >> 5;
    const int j16 = lane & 15;
    const int ghalf = (lane >> 4) & 1;

    const int logical = xcd_remap(blockIdx.x, total_wg);
    const int bh = logical / num_kv_tiles;
    const int kt = logical % num_kv_tiles;         // early key tiles have the most work when causal: first
    const int j0 = kt * S::kTileKV;
    const int jw0 = j0 + wave * 32;                // first key of this wave
    const int my_j = jw0 + l32;

    const size_t head = (size_t)bh * N * D;
    const bf16* Qh = Q + head;
    const bf16* dOh = dO + head;
    const float* LSEh = LSE + (size_t)bh * N;
    const float* Deltah = Delta + (size_t)bh * N;
    float* dQh = dQacc + head;

    const float c = scale * kLog2e;

    // ---- K tile of the workgroup -> LDS (for the dQ product)
    {
        const bf16* Kt = K + head + (size_t)j0 * D;
#pragma unroll
        for (int it = 0; it < S::kKLoads; it++) {
            int s = it * S::kThreads + tid;
            int row = s / S::kChunksPerRow, pc = s % S::kChunksPerRow;
            load_global_to_lds16(Kt + row * D + ((pc ^ swz<D>(row)) * 8),
                                 smem + S::kOffK + it * (S::kThreads * 16) + wave * 1024);
        }
    }
    // ---- K, V fragments of this wave's 32 keys (B operands of S = Q K^T and dP = dO V^T)
    bf16x8 kf[D / 16], vf[D / 16];
#pragma unroll
    for (int kb = 0; kb < D / 16; kb++) {
        kf[kb] = *(const bf16x8*)(K + head + (size_t)my_j * D + kb * 16 + h * 8);
        vf[kb] = *(const bf16x8*)(V + head + (size_t)my_j * D + kb * 16 + h * 8);
    }

    // ---- Q / dO / LSE / Delta block loads
    int q_src[S::kQLoads];
#pragma unroll
    for (int it = 0; it < S::kQLoads; it++) {
        int s = it * S::kThreads + tid;
        int row = s / S::kChunksPerRow, pc = s % S::kChunksPerRow;
        q_src[it] = row * D + ((pc ^ swz<D>(row)) * 8);
    }
    auto issue_block = [&](int stage, int i0) {
        char* base = smem + S::kOffStage + stage * S::kStageBytes;
#pragma unroll
        for (int it = 0; it < S::kQLoads; it++)
            load_global_to_lds16(Qh + (size_t)i0 * D + q_src[it], base + it * (S::kThreads * 16) + wave * 1024);
#pragma unroll
        for (int it = 0; it < S::kQLoads; it++)
            load_global_to_lds16(dOh + (size_t)i0 * D + q_src[it],
                                 base + S::kQTileBytes + it * (S::kThreads * 16) + wave * 1024);
        if (wave == 0 && lane < 16) {   // 8 lanes fetch LSE[i0..i0+31], 8 lanes Delta[i0..i0+31]
            const float* src = (lane < 8) ? (LSEh + i0 + lane * 4) : (Deltah + i0 + (lane - 8) * 4);
            load_global_to_lds16(src, base + 2 * S::kQTileBytes);
        }
    };

    // ---- per-lane LDS offsets
    // row operand (A of S and dP): row l32, logical chunk 2*kb + h
    const int row_lane = l32 * S::kRowBytes + ((h ^ swz<D>(l32)) << 4);
    // transposed operand from a 32-row Q/dO block (A of dV^T, dK^T): rows 16*ks + 4h + j16/4 (+8)
    const int trq_row = 4 * h + (j16 >> 2);
    const int trq_lane = trq_row * S::kRowBytes + (((2 * ghalf + ((j16 & 3) >> 1)) ^ swz<D>(trq_row)) << 4) + ((j16 & 1) << 3);
    // transposed operand from the K tile (B of dQ): rows 16*ks + 8h + j16/4 (+4)
    const int trk_row = 8 * h + (j16 >> 2);
    const int trk_lane = trk_row * S::kRowBytes + (((2 * ghalf + ((j16 & 3) >> 1)) ^ swz<D>(trk_row)) << 4) + ((j16 & 1) << 3);
    // dS^T buffer: row = key (64 bytes = 32 queries), 8-byte slot index XOR ((key >> 2) & 7)
    //   write: key = 32*wave + l32, slot = 2g + h
    const int ds_wr_lane = (wave * 32 + l32) * 64 + ((h ^ (((wave * 32 + l32) >> 2) & 7)) << 3);
    //   transposing read (A of dQ): rows 16*ks + 8h + j16/4 (+4), slot 4*ghalf + (j16 & 3)
    const int ds_rd_lane = trk_row * 64 + (((4 * ghalf + (j16 & 3)) ^ (2 * h)) << 3);

    // dQ work split: D=128 -> wave w takes columns 32w..32w+31 over all 128 keys;
    //                D=64  -> wave w takes columns 32*(w&1).. over keys 64*(w>>1)..
    const int dq_db = (D == 128) ? wave : (wave & 1);
    const int dq_ks0 = (D == 128) ? 0 : (wave >> 1) * 4;

    f32x16 dk_acc[D / 32], dv_acc[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; db++)
#pragma unroll
        for (int r = 0; r < 16; r++) { dk_acc[db][r] = 0.f; dv_acc[db][r] = 0.f; }

    auto compute_block = [&](int stage, int i0) {
        const char* qs = smem + S::kOffStage + stage * S::kStageBytes;
        const char* dos = qs + S::kQTileBytes;
        const f32x4* stat = (const f32x4*)(qs + 2 * S::kQTileBytes);

        f32x16 s, dp;
#pragma unroll
        for (int r = 0; r < 16; r++) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
        for (int kb = 0; kb < D / 16; kb++) {
            bf16x8 a = lds_read_b128(qs, row_lane ^ ((2 * kb) << 4));
            s = mfma32(a, kf[kb], s);
        }
#pragma unroll
        for (int kb = 0; kb < D / 16; kb++) {
            bf16x8 a = lds_read_b128(dos, row_lane ^ ((2 * kb) << 4));
            dp = mfma32(a, vf[kb], dp);
        }
        // P and dS; register r <-> query i0 + 8*(r/4) + 4h + r%4, lane <-> key my_j
        const bool diag = CAUSAL && (i0 < jw0 + 31);
#pragma unroll
        for (int g = 0; g < 4; g++) {
            f32x4 lse4 = stat[2 * g + h];
            f32x4 dl4 = stat[8 + 2 * g + h];
#pragma unroll
            for (int t = 0; t < 4; t++) {
                const int r = 4 * g + t;
                float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], c, -lse4[t] * kLog2e));
                if (diag && (i0 + 8 * g + 4 * h + t < my_j)) p = 0.f;
                s[r] = p;
                dp[r] = p * (dp[r] - dl4[t]);
            }
        }
        bf16x8 pb[2], dsb[2];
#pragma unroll
        for (int ks = 0; ks < 2; ks++) {
            const int r0 = 8 * ks;
            pb[ks] = cvt8(s[r0], s[r0 + 1], s[r0 + 2], s[r0 + 3], s[r0 + 4], s[r0 + 5], s[r0 + 6], s[r0 + 7]);
            dsb[ks] = cvt8(dp[r0], dp[r0 + 1], dp[r0 + 2], dp[r0 + 3], dp[r0 + 4], dp[r0 + 5], dp[r0 + 6], dp[r0 + 7]);
        }
        // dS^T -> LDS (4 queries = 8 bytes per write)
#pragma unroll
        for (int g = 0; g < 4; g++) {
            bf16x8 src = dsb[g >> 1];
            bf16x4 v4 = (g & 1) ? __builtin_shufflevector(src, src, 4, 5, 6, 7) : __builtin_shufflevector(src, src, 0, 1, 2, 3);
            *(bf16x4*)(smem + S::kOffDs + (ds_wr_lane ^ ((2 * g) << 3))) = v4;
        }
        // dV^T += dO^T P ; dK^T += Q^T dS   (16 queries per MFMA)
#pragma unroll
        for (int ks = 0; ks < 2; ks++) {
            const int row_off = 16 * ks * S::kRowBytes;
#pragma unroll
            for (int db = 0; db < D / 32; db++) {
                const int x0 = (4 * db) << 4, x1 = ((4 * db) ^ 2) << 4;
                bf16x4 a0 = lds_read_tr16(dos, (trq_lane ^ x0) + row_off);
                bf16x4 a1 = lds_read_tr16(dos, (trq_lane ^ x1) + row_off + 8 * S::kRowBytes);
                dv_acc[db] = mfma32(concat(a0, a1), pb[ks], dv_acc[db]);
                bf16x4 b0 = lds_read_tr16(qs, (trq_lane ^ x0) + row_off);
                bf16x4 b1 = lds_read_tr16(qs, (trq_lane ^ x1) + row_off + 8 * S::kRowBytes);
                dk_acc[db] = mfma32(concat(b0, b1), dsb[ks], dk_acc[db]);
            }
        }
        wait_vmcnt<0>();      // next block's loads (issued before this block's math) have landed
        __syncthreads();      // dS^T of all four waves visible

        // dQ[i][d] partial = sum over this workgroup's keys of dS[i][key] K[key][d]
        f32x16 dq;
#pragma unroll
        for (int r = 0; r < 16; r++) dq[r] = 0.f;
        const char* kt_s = smem + S::kOffK;
        const char* ds_s = smem + S::kOffDs;
#pragma unroll
        for (int kk = 0; kk < S::kKeyStepsPerWave; kk++) {
            const int ks = dq_ks0 + kk;   // dq_ks0 is 0 or 4: (ks & 1) == (kk & 1)
            const int xa0 = (4 * (kk & 1)) << 3, xa1 = (4 * (kk & 1) + 1) << 3;
            bf16x4 a0 = lds_read_tr16(ds_s, (ds_rd_lane ^ xa0) + ks * 16 * 64);
            bf16x4 a1 = lds_read_tr16(ds_s, (ds_rd_lane ^ xa1) + ks * 16 * 64 + 4 * 64);
            const int xb0 = (4 * dq_db) << 4, xb1 = ((4 * dq_db) ^ 1) << 4;
            bf16x4 b0 = lds_read_tr16(kt_s, (trk_lane ^ xb0) + ks * 16 * S::kRowBytes);
            bf16x4 b1 = lds_read_tr16(kt_s, (trk_lane ^ xb1) + ks * 16 * S::kRowBytes + 4 * S::kRowBytes);
            dq = mfma32(concat(a0, a1), concat(b0, b1), dq);
        }
        float* dst = dQh + (size_t)i0 * D + 32 * dq_db + l32;
#pragma unroll
        for (int r = 0; r < 16; r++)
            unsafeAtomicAdd(dst + (8 * (r >> 2) + 4 * h + (r & 3)) * D, dq[r]);
        __syncthreads();      // dS^T and this stage may be overwritten
    };

    const int i_begin = CAUSAL ? j0 : 0;
    issue_block(0, i_begin);
    wait_vmcnt<0>();
    __syncthreads();
    for (int i0 = i_begin; i0 < N; i0 += 2 * S::kTileQ) {     // (N - i_begin) / 32 is even
        issue_block(1, i0 + S::kTileQ);
        compute_block(0, i0);
        if (i0 + 2 * S::kTileQ < N) issue_block(0, i0 + 2 * S::kTileQ);
        compute_block(1, i0 + S::kTileQ);
    }

    // ---- epilogue: lane <-> key my_j, register r of block db <-> column 32db + 8*(r/4) + 4h + r%4
    bf16* dKr = dK + head + (size_t)my_j * D;
    bf16* dVr = dV + head + (size_t)my_j * D;
#pragma unroll
    for (int db = 0; db < D / 32; db++)
#pragma unroll
        for (int g = 0; g < 4; g++) {
            const int col = 32 * db + 8 * g + 4 * h;
            bf16x2 a = cvt2(dk_acc[db][4 * g] * scale, dk_acc[db][4 * g + 1] * scale);
            bf16x2 b = cvt2(dk_acc[db][4 * g + 2] * scale, dk_acc[db][4 * g + 3] * scale);
            *(bf16x4*)(dKr + col) = __builtin_shufflevector(a, b, 0, 1, 2, 3);
            bf16x2 e = cvt2(dv_acc[db][4 * g], dv_acc[db][4 * g + 1]);
            bf16x2 f = cvt2(dv_acc[db][4 * g + 2], dv_acc[db][4 * g + 3]);
            *(bf16x4*)(dVr + col) = __builtin_shufflevector(e, f, 0, 1, 2, 3);
        }
}

template <int D, bool CAUSAL>
static hipError_t launch_bwd_main_t(const void* q, const void* k, const void* v, const void* d_o,
                                    const float* lse, const float* delta, float* dq_acc, void* dk, void* dv,
                                    int B, int H, int N, float scale, hipStream_t stream)
{
    using S = BwdShape<D>;
    auto kern = attn_bwd_main_kernel<D, CAUSAL>;
    static bool configured = false;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, S::kLdsBytes);
        if (e != hipSuccess) return e;
        configured = true;
    }
    const int num_kv_tiles = N / S::kTileKV;
    const int total = B * H * num_kv_tiles;
    hipLaunchKernelGGL(kern, dim3(total), dim3(S::kThreads), S::kLdsBytes, stream,
                       (const bf16*)q, (const bf16*)k, (const bf16*)v, (const bf16*)d_o, lse, delta,
                       dq_acc, (bf16*)dk, (bf16*)dv, N, num_kv_tiles, total, scale);
    return hipGetLastError();
}

hipError_t launch_attn_bwd_main(const void* q, const void* k, const void* v, const void* d_o,
                                const float* lse, const float* delta, float* dq_acc, void* dk, void* dv,
                                int B, int H, int N, int D, int causal, float scale, hipStream_t stream)
{
    if (D == 128) return causal ? launch_bwd_main_t<128, true>(q, k, v, d_o, lse, delta, dq_acc, dk, dv, B, H, N, scale, stream)
                                : launch_bwd_main_t<128, false>(q, k, v, d_o, lse, delta, dq_acc, dk, dv, B, H, N, scale, stream);
    return causal ? launch_bwd_main_t<64, true>(q, k, v, d_o, lse, delta, dq_acc, dk, dv, B, H, N, scale, stream)
                  : launch_bwd_main_t<64, false>(q, k, v, d_o, lse, delta, dq_acc, dk, dv, B, H, N, scale, stream);
}

}  // namespace tk
