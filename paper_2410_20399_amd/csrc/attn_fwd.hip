// Fused exact softmax attention, forward pass, for gfx950 (MI355X).
//
// One workgroup = 4 waves = 128 query rows of one (batch, head); each wave owns 32 query rows.
// K and V are streamed in tiles of 64 keys through a two-stage LDS ring filled by direct
// global->LDS loads.  Per tile each wave computes, with v_mfma_f32_32x32x16_bf16:
//
//   S^T = K Q^T          (so that a lane owns ONE query: softmax statistics are lane-local)
//   online softmax in base 2 with the temperature folded into the exponent
//                        (the streaming recurrence of the paper's Appendix B.3 listing)
//   O^T += V^T P^T       (P^T in accumulator layout IS a valid B operand; V^T comes from
//                         row-major V in LDS through transposing reads)
//
// Epilogue: O = O / l -> bf16, LSE = m*scale + ln l.
#include "tk_common.h"
#include "tk_launch.h"

namespace tk {

template <int D>
struct FwdShape {
    static constexpr int kWaves = 4;
    static constexpr int kThreads = kWaves * 64;
    static constexpr int kTileQ = kWaves * 32;          // query rows per workgroup
    static constexpr int kTileKV = 64;                  // keys per LDS stage
    static constexpr int kRowBytes = D * 2;
    static constexpr int kChunksPerRow = D / 8;         // 16-byte chunks
    static constexpr int kTileBytes = kTileKV * kRowBytes;
    static constexpr int kStageBytes = 2 * kTileBytes;  // K tile then V tile
    static constexpr int kLdsBytes = 2 * kStageBytes;
    static constexpr int kLoadsPerTile = kTileKV * kChunksPerRow / kThreads;  // per thread
};

// LDS layout of a [64 x D] bf16 tile: row-major, with the 16-byte chunk index XOR-ed by a
// function of the row so that the two read patterns below spread over all 64 banks.
//   K tile, read as MFMA A operand: 16 consecutive lanes read the same chunk of 16 consecutive rows.
//   V tile, read through ds_read_b64_tr_b16: 32 lanes read a 4-row x 64-byte block.
template <int D> __device__ __forceinline__ int swizzle_k(int row) {
    return D == 128 ? (row & 15) : ((row >> 1) & 7);
}
template <int D> __device__ __forceinline__ int swizzle_v(int row) {
    return D == 128 ? (((row & 3) << 2) | ((row >> 2) & 3)) : ((((row >> 1) & 1) << 2) | ((row >> 2) & 3));
}

// Nq queries, Nk keys.  TAIL: the general case (Nq != Nk, or a length that is not a multiple of
// 128); the aligned square case compiles without any of the tail code.  With the causal mask the
// sequences are aligned at their ends: query i sees keys j <= i + (Nk - Nq); the host has checked
// Nq <= Nk for that case, so every query sees key 0.
template <int D, bool CAUSAL, bool TAIL>
__global__ __launch_bounds__(256, 2)
void attn_fwd_kernel(const bf16* __restrict__ Q, const bf16* __restrict__ K, const bf16* __restrict__ V,
                     bf16* __restrict__ O, float* __restrict__ LSE,
                     int Nq, int Nk, int num_q_tiles, int total_wg, float scale, int hq, int hkv,
                     int n_splits, int tiles_per_split, float* __restrict__ O_part, float* __restrict__ LSE_part)
{
    using S = FwdShape<D>;
    // One array per ring stage: distinct LDS objects let the compiler see that reads of the stage
    // being consumed cannot alias the direct-to-LDS loads in flight into the other stage (otherwise
    // it drains every outstanding load before the first LDS read that follows them).
    __shared__ __attribute__((aligned(1024))) char smem0[S::kStageBytes];
    __shared__ __attribute__((aligned(1024))) char smem1[S::kStageBytes];

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int l32 = lane & 31;
    const int h = lane >> 5;

    // workgroup -> (head, query tile); heavy (late) query tiles first when causal
    // Split over the keys (general-case variant, no mask; used for decode-shaped calls where heads and
    // query tiles alone cannot fill the chip): n_splits workgroups share one query tile, each takes
    // tiles_per_split (even) consecutive key tiles and leaves a normalised fp32 partial O and its LSE.
    const int logical = xcd_remap(blockIdx.x, total_wg);
    const int split = (TAIL && !CAUSAL) ? logical % n_splits : 0;
    const int tile_id = (TAIL && !CAUSAL) ? logical / n_splits : logical;
    const int bh = tile_id / num_q_tiles;
    int qt = tile_id % num_q_tiles;
    if (CAUSAL) qt = num_q_tiles - 1 - qt;

    // grouped-query attention: query head h of a batch entry reads key/value head h / (hq / hkv)
    const size_t head = (size_t)bh * Nq * D;
    const size_t kv_head = (size_t)((bh / hq) * hkv + (bh % hq) / (hq / hkv)) * Nk * D;
    const bf16* Qh = Q + head;
    const bf16* Kh = K + kv_head;
    const bf16* Vh = V + kv_head;
    const int q0 = qt * S::kTileQ + wave * 32;   // first query row of this wave
    const int my_q = q0 + l32;
    // The lengths need not be multiples of the tile sizes: the kernel works on padded sequences,
    // reads of rows past the end are redirected to the last row, keys >= Nk are masked, query rows
    // >= Nq are not stored.
    const int my_q_ld = (!TAIL || my_q < Nq) ? my_q : Nq - 1;
    const int off = TAIL ? Nk - Nq : 0;          // causal: query i sees keys <= i + off

    const float c = scale * kLog2e;              // base-2 temperature

    // ---- Q fragments (B operand of S^T = K Q^T): lane holds Q[my_q][16*kb + 8*h .. +7]
    bf16x8 qf[D / 16];
#pragma unroll
    for (int kb = 0; kb < D / 16; kb++)
        qf[kb] = *(const bf16x8*)(Qh + (size_t)my_q_ld * D + kb * 16 + h * 8);

    // ---- per-thread source offsets of the direct-to-LDS tile loads
    // LDS slot s = it*256 + tid holds (row = s / chunks_per_row, physical chunk = s % chunks_per_row).
    int k_src[S::kLoadsPerTile], v_src[S::kLoadsPerTile];
#pragma unroll
    for (int it = 0; it < S::kLoadsPerTile; it++) {
        int s = it * S::kThreads + tid;
        int row = s / S::kChunksPerRow, pc = s % S::kChunksPerRow;
        k_src[it] = row * D + ((pc ^ swizzle_k<D>(row)) * 8);
        v_src[it] = row * D + ((pc ^ swizzle_v<D>(row)) * 8);
    }
    auto issue_tile = [&](int stage, int tile) {
        const int j0 = tile * S::kTileKV;
        const bf16* kt = Kh + (size_t)j0 * D;
        const bf16* vt = Vh + (size_t)j0 * D;
        char* base = (stage ? smem1 : smem0) + wave * 1024;
        if (!TAIL || j0 + S::kTileKV <= Nk) {
#pragma unroll
            for (int it = 0; it < S::kLoadsPerTile; it++)
                load_global_to_lds16(kt + k_src[it], base + it * (S::kThreads * 16));
#pragma unroll
            for (int it = 0; it < S::kLoadsPerTile; it++)
                load_global_to_lds16(vt + v_src[it], base + S::kTileBytes + it * (S::kThreads * 16));
        } else {
            // the tile runs past the last key: rows >= Nk fetch row Nk-1 instead (they are masked later)
#pragma unroll
            for (int it = 0; it < S::kLoadsPerTile; it++) {
                const int row = j0 + (it * S::kThreads + tid) / S::kChunksPerRow;
                const int back = (row < Nk ? 0 : row - (Nk - 1)) * D;     // elements to step back
                load_global_to_lds16(kt + k_src[it] - back, base + it * (S::kThreads * 16));
            }
#pragma unroll
            for (int it = 0; it < S::kLoadsPerTile; it++) {
                const int row = j0 + (it * S::kThreads + tid) / S::kChunksPerRow;
                const int back = (row < Nk ? 0 : row - (Nk - 1)) * D;
                load_global_to_lds16(vt + v_src[it] - back, base + S::kTileBytes + it * (S::kThreads * 16));
            }
        }
        __builtin_amdgcn_sched_barrier(0);   // keep the prefetch ahead of the math it overlaps with
    };

    // ---- per-lane LDS read offsets (the XOR with a compile-time chunk index is applied at use)
    // K: row = 32*b + l32, logical chunk 2*kb + h
    const int k_lane = l32 * S::kRowBytes + ((h ^ swizzle_k<D>(l32)) << 4);
    // V (transposing read): 16-lane group G = lane/16 -> (d half = G%2, key half = G/2);
    //   lane j of the group addresses row 4*(G/2) + j/4, columns 32*db + 16*(G%2) + 4*(j%4)
    const int j16 = lane & 15;
    const int v_row = 4 * h + (j16 >> 2);
    const int v_chunk = 2 * ((lane >> 4) & 1) + ((j16 & 3) >> 1);
    const int v_lane = v_row * S::kRowBytes + ((v_chunk ^ swizzle_v<D>(v_row)) << 4) + ((j16 & 1) << 3);

    f32x16 o_acc[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; db++)
#pragma unroll
        for (int r = 0; r < 16; r++) o_acc[db][r] = 0.f;
    float m_run = -INFINITY;   // running max of raw scores (shared by both half-waves)
    float l_run = 0.f;         // running sum, partial: this lane's 32 of the 64 keys per tile

    auto compute_tile = [&](int stage, int tile) {
        const int j0 = tile * S::kTileKV;
        if (CAUSAL && j0 > q0 + 31 + off) return;    // every key of the tile is masked for this wave
        if (TAIL && q0 >= Nq) return;                // a wave of padding rows only (few queries, e.g. decode)
        const char* ks = stage ? smem1 : smem0;
        const char* vs = ks + S::kTileBytes;

        // S^T[key][query] for two 32-key blocks
        f32x16 s[2];
#pragma unroll
        for (int b = 0; b < 2; b++) {
#pragma unroll
            for (int r = 0; r < 16; r++) s[b][r] = 0.f;
#pragma unroll
            for (int kb = 0; kb < D / 16; kb++) {
                bf16x8 kf = lds_read_b128(ks, (k_lane ^ ((2 * kb) << 4)) + b * 32 * S::kRowBytes);
                s[b] = mfma32(kf, qf[kb], s[b]);
            }
        }
        // tile crosses the diagonal for some row of this wave, or runs past the last key
        if ((CAUSAL && j0 + S::kTileKV - 1 > q0 + off) || (TAIL && j0 + S::kTileKV > Nk)) {
#pragma unroll
            for (int b = 0; b < 2; b++)
#pragma unroll
                for (int r = 0; r < 16; r++) {
                    int key = j0 + 32 * b + 8 * (r >> 2) + 4 * h + (r & 3);
                    if ((CAUSAL && key > my_q + off) || (TAIL && key >= Nk)) s[b][r] = -INFINITY;
                }
        }
        // running max
        float mx = s[0][0];
#pragma unroll
        for (int r = 1; r < 16; r++) mx = __builtin_fmaxf(mx, s[0][r]);
#pragma unroll
        for (int r = 0; r < 16; r++) mx = __builtin_fmaxf(mx, s[1][r]);
        mx = half_max(mx);
        // The running max is only raised when some row of the wave outgrows it by more than
        // kMaxSlack in the base-2 exponent: with a stale max every exponent stays <= kMaxSlack,
        // so P <= 2^kMaxSlack is still exactly representable work for fp32/bf16, and O and l
        // carry the same factor, which the final division removes.  Saves the O rescale on
        // almost every tile.
        constexpr float kMaxSlack = 8.0f;
        const bool raise = (mx - m_run) * c > kMaxSlack;          // true on the first tile (m_run = -inf)
        if (__builtin_amdgcn_ballot_w64(raise) != 0) {
            const float m_new = __builtin_fmaxf(m_run, mx);
            const float corr = __builtin_amdgcn_exp2f((m_run - m_new) * c);
            m_run = m_new;
            l_run *= corr;
#pragma unroll
            for (int db = 0; db < D / 32; db++)
#pragma unroll
                for (int r = 0; r < 16; r++) o_acc[db][r] *= corr;
        }
        const float mc = m_run * c;
        // P = 2^(S*c - m*c), partial row sums
        float psum = 0.f;
#pragma unroll
        for (int b = 0; b < 2; b++)
#pragma unroll
            for (int r = 0; r < 16; r++) {
                float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[b][r], c, -mc));
                s[b][r] = p;
                psum += p;
            }
        l_run += psum;

        // O^T += V^T P^T, 16 keys per MFMA
#pragma unroll
        for (int kk = 0; kk < 4; kk++) {
            const int b = kk >> 1, r0 = 8 * (kk & 1);
            bf16x8 pb = cvt8(s[b][r0 + 0], s[b][r0 + 1], s[b][r0 + 2], s[b][r0 + 3],
                             s[b][r0 + 4], s[b][r0 + 5], s[b][r0 + 6], s[b][r0 + 7]);
#pragma unroll
            for (int db = 0; db < D / 32; db++) {
                // rows 16*kk + 4*h + (0..3) and +8; the +8 flips bit 1 of swizzle_v's low field
                const int row_off = 16 * kk * S::kRowBytes;
                const int x0 = (4 * db) << 4;
                const int x1 = ((4 * db) ^ 2) << 4;
                bf16x4 v0 = lds_read_tr16(vs, (v_lane ^ x0) + row_off);
                bf16x4 v1 = lds_read_tr16(vs, (v_lane ^ x1) + row_off + 8 * S::kRowBytes);
                o_acc[db] = mfma32(concat(v0, v1), pb, o_acc[db]);
            }
        }
    };

    // key tiles this workgroup visits: an even count that covers every key visible to its last query
    int n_tiles;
    if (!TAIL) {
        n_tiles = (CAUSAL ? qt * S::kTileQ + S::kTileQ : num_q_tiles * S::kTileQ) / S::kTileKV;
    } else {
        int n_keys = Nk;
        if (CAUSAL && qt * S::kTileQ + S::kTileQ + off < n_keys) n_keys = qt * S::kTileQ + S::kTileQ + off;
        n_tiles = 2 * ((n_keys + 2 * S::kTileKV - 1) / (2 * S::kTileKV));
    }

    int t_begin = 0;
    if (TAIL && !CAUSAL && n_splits > 1) {
        t_begin = split * tiles_per_split;
        if (t_begin + tiles_per_split < n_tiles) n_tiles = t_begin + tiles_per_split;
    }
    issue_tile(0, t_begin);
    wait_vmcnt<0>();
    __syncthreads();
    for (int t = t_begin; t < n_tiles; t += 2) {
        issue_tile(1, t + 1);
        compute_tile(0, t);
        wait_vmcnt<0>();
        __syncthreads();
        if (t + 2 < n_tiles) issue_tile(0, t + 2);
        compute_tile(1, t + 1);
        wait_vmcnt<0>();
        __syncthreads();
    }

    // ---- epilogue
    const float l_tot = half_sum(l_run);
    const float inv = 1.0f / l_tot;
    if (TAIL && !CAUSAL && n_splits > 1) {
        if (my_q < Nq) {
            const size_t prow = ((size_t)split * (total_wg / n_splits / num_q_tiles) + bh) * Nq + my_q;   // [split][head][query]
            float* Op = O_part + prow * D;
#pragma unroll
            for (int db = 0; db < D / 32; db++)
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    f32x4 v4 = {o_acc[db][4 * g + 0] * inv, o_acc[db][4 * g + 1] * inv, o_acc[db][4 * g + 2] * inv, o_acc[db][4 * g + 3] * inv};
                    *(f32x4*)(Op + 32 * db + 8 * g + 4 * h) = v4;
                }
            if (h == 0) LSE_part[prow] = m_run * scale + __builtin_logf(l_tot);
        }
    } else if (!TAIL || my_q < Nq) {
        bf16* Oh = O + head + (size_t)my_q * D;
#pragma unroll
        for (int db = 0; db < D / 32; db++)
#pragma unroll
            for (int g = 0; g < 4; g++) {
                bf16x2 a = cvt2(o_acc[db][4 * g + 0] * inv, o_acc[db][4 * g + 1] * inv);
                bf16x2 b = cvt2(o_acc[db][4 * g + 2] * inv, o_acc[db][4 * g + 3] * inv);
                *(bf16x4*)(Oh + 32 * db + 8 * g + 4 * h) = __builtin_shufflevector(a, b, 0, 1, 2, 3);
            }
        if (h == 0) LSE[(size_t)bh * Nq + my_q] = m_run * scale + __builtin_logf(l_tot);
    }
}

template <int D, bool CAUSAL, bool TAIL>
static hipError_t launch_fwd_tt(const void* q, const void* k, const void* v, void* o, float* lse,
                                int B, int H, int Hkv, int Nq, int Nk, float scale, hipStream_t stream,
                                int n_splits = 1, int tiles_per_split = 0, float* o_part = nullptr, float* lse_part = nullptr)
{
    using S = FwdShape<D>;
    auto kern = attn_fwd_kernel<D, CAUSAL, TAIL>;
    const int num_q_tiles = (Nq + S::kTileQ - 1) / S::kTileQ;
    const int total = B * H * num_q_tiles * n_splits;
    hipLaunchKernelGGL(kern, dim3(total), dim3(S::kThreads), 0, stream,
                       (const bf16*)q, (const bf16*)k, (const bf16*)v, (bf16*)o, lse,
                       Nq, Nk, num_q_tiles, total, scale, H, Hkv, n_splits, tiles_per_split, o_part, lse_part);
    return hipGetLastError();
}

template <int D, bool CAUSAL>
static hipError_t launch_fwd_t(const void* q, const void* k, const void* v, void* o, float* lse,
                               int B, int H, int Hkv, int Nq, int Nk, float scale, hipStream_t stream)
{
    using S = FwdShape<D>;
    return (Nq != Nk || Nq % S::kTileQ) ? launch_fwd_tt<D, CAUSAL, true>(q, k, v, o, lse, B, H, Hkv, Nq, Nk, scale, stream)
                                        : launch_fwd_tt<D, CAUSAL, false>(q, k, v, o, lse, B, H, Hkv, Nq, Nk, scale, stream);
}

hipError_t launch_attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse,
                           int B, int H, int Hkv, int Nq, int Nk, int D, int causal, float scale, hipStream_t stream)
{
    if (D == 128) return causal ? launch_fwd_t<128, true>(q, k, v, o, lse, B, H, Hkv, Nq, Nk, scale, stream)
                                : launch_fwd_t<128, false>(q, k, v, o, lse, B, H, Hkv, Nq, Nk, scale, stream);
    return causal ? launch_fwd_t<64, true>(q, k, v, o, lse, B, H, Hkv, Nq, Nk, scale, stream)
                  : launch_fwd_t<64, false>(q, k, v, o, lse, B, H, Hkv, Nq, Nk, scale, stream);
}

// ------------------------------------------------------------------------------------------
// merge of the partial results of a split over the keys
// ------------------------------------------------------------------------------------------
// O = sum_s w_s O_s / sum_s w_s with w_s = exp(LSE_s - max_s LSE_s), LSE = max + ln sum_s w_s: the
// partials are softmax results over disjoint key ranges, each normalised by its own sum.
template <int D>
__global__ __launch_bounds__(256)
void attn_fwd_combine_kernel(const float* __restrict__ O_part, const float* __restrict__ LSE_part,
                             bf16* __restrict__ O, float* __restrict__ LSE, size_t rows, int n_splits)
{
    constexpr int kLanesPerRow = D / 4;                 // one float4 per lane
    const size_t row = (size_t)blockIdx.x * (256 / kLanesPerRow) + threadIdx.x / kLanesPerRow;
    if (row >= rows) return;
    const int col = (threadIdx.x % kLanesPerRow) * 4;
    float m = -INFINITY;
    for (int s = 0; s < n_splits; s++) m = __builtin_fmaxf(m, LSE_part[(size_t)s * rows + row]);
    float wsum = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < n_splits; s++) {
        const float w = __builtin_expf(LSE_part[(size_t)s * rows + row] - m);
        const f32x4 v = *(const f32x4*)(O_part + ((size_t)s * rows + row) * D + col);
        wsum += w;
        acc += v * w;
    }
    const float inv = 1.0f / wsum;
    bf16x2 lo = cvt2(acc[0] * inv, acc[1] * inv), hi = cvt2(acc[2] * inv, acc[3] * inv);
    *(bf16x4*)(O + row * D + col) = __builtin_shufflevector(lo, hi, 0, 1, 2, 3);
    if (col == 0) LSE[row] = m + __builtin_logf(wsum);
}

// Non-causal forward with the keys split n_splits ways (n_splits >= 2, every split holds at least one
// key: (n_splits - 1) * tiles_per_split * 64 < Nk, tiles_per_split even).  o_part: fp32
// [n_splits][B*H][Nq][D], lse_part: fp32 [n_splits][B*H][Nq].
hipError_t launch_attn_fwd_splitk(const void* q, const void* k, const void* v, void* o, float* lse,
                                  float* o_part, float* lse_part,
                                  int B, int H, int Hkv, int Nq, int Nk, int D, float scale,
                                  int n_splits, int tiles_per_split, hipStream_t stream)
{
    hipError_t e = D == 128
        ? launch_fwd_tt<128, false, true>(q, k, v, o, lse, B, H, Hkv, Nq, Nk, scale, stream, n_splits, tiles_per_split, o_part, lse_part)
        : launch_fwd_tt<64, false, true>(q, k, v, o, lse, B, H, Hkv, Nq, Nk, scale, stream, n_splits, tiles_per_split, o_part, lse_part);
    if (e != hipSuccess) return e;
    const size_t rows = (size_t)B * H * Nq;
    if (D == 128) {
        const unsigned grid = (unsigned)((rows + 7) / 8);
        hipLaunchKernelGGL((attn_fwd_combine_kernel<128>), dim3(grid), dim3(256), 0, stream, o_part, lse_part, (bf16*)o, lse, rows, n_splits);
    } else {
        const unsigned grid = (unsigned)((rows + 15) / 16);
        hipLaunchKernelGGL((attn_fwd_combine_kernel<64>), dim3(grid), dim3(256), 0, stream, o_part, lse_part, (bf16*)o, lse, rows, n_splits);
    }
    return hipGetLastError();
}

}  // namespace tk
