// Fused exact softmax attention, backward pass, for gfx950 (MI355X).
//
// The paper reports the backward kernel's speed only (the attention plots of Section 4.1 and the profile table of Section 4.2); the algorithm
// here is the chain rule with P recomputed from the saved log-sum-exp:
//
//   kernel 1  Delta_i = sum_d dO_id O_id          (HBM stream)
//   kernel 2  dK, dV: persistent workgroups walk the 128-key tiles; wave w owns keys 32w..32w+31 and keeps
//             their dK^T, dV^T accumulators in registers while it loops over 32-query blocks:
//               S  = Q_i K_j^T            P  = 2^(S*c - LSE_i*log2e)
//               dP = dO_i V_j^T           dS = P (dP - Delta_i)
//               dV_j^T += dO_i^T P        dK_j^T += Q_i^T dS
//   kernel 3  dQ: one workgroup per 128-query tile, wave w owns queries 32w..32w+31 and keeps
//             their dQ^T accumulator in registers while it loops over 64-key tiles:
//               S^T = K_j Q_i^T, dP^T = V_j dO_i^T, dS^T as above, dQ_i^T += K_j^T dS^T
//
// dQ gets a kernel of its own (recomputing S and dP) instead of fp32 atomics from kernel 2: the
// L2 atomic units retire about one fp32 lane per clock per channel (measured ~0.33 T lane-adds/s
// for the whole chip), and a 128-key tile needs N/128 partial sums per dQ element, which made
// the atomics alone as long as all the matrix work.  The split is also deterministic.
//
// With a large workspace (the chip has 288 GB) the recomputation goes away as well: kernel 2 then
// also stores its bf16 dS blocks, 2 bytes per (query, key) pair, exactly as its lanes hold them
// (SPILL), and dQ becomes one product per pair,
//   kernel 4  dQ_i = scale * sum_j dS_ij K_j  from the stored blocks (attn_bwd_dq_from_ds_kernel),
// which is bound by reading dS back from HBM instead of by 6*D flops per pair.  10*D flops per
// pair are executed instead of 14*D; Delta then comes from kernel 1.
//
// In kernel 2, S and dP are produced with the KEY index on lanes and the query index on
// registers, so P and dS in accumulator layout are directly the B operands of the two products
// contracted over queries; their A operands (dO^T, Q^T) come from row-major LDS tiles via
// transposing reads.  Kernel 3 mirrors the forward kernel: QUERY index on lanes, so LSE_i and
// Delta_i are lane scalars and dS^T is directly the B operand of the product contracted over keys.
#include "tk_common.h"
#include "tk_launch.h"

#include <type_traits>

namespace tk {

// ------------------------------------------------------------------------------------------
// kernel 1: Delta
// ------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256)
void attn_bwd_delta_kernel(const bf16* __restrict__ O, const bf16* __restrict__ dO,
                           float* __restrict__ delta, size_t n_chunks)
{
    constexpr int kLanesPerRow = D / 8;
    const size_t chunk = (size_t)blockIdx.x * 256 + threadIdx.x;   // one 8-element chunk per thread
    if (chunk >= n_chunks) return;                                  // (whole rows: n_chunks is a multiple of D/8)
    bf16x8 a = *(const bf16x8*)(O + chunk * 8);
    bf16x8 b = *(const bf16x8*)(dO + chunk * 8);
    float acc = 0.f;
#pragma unroll
    for (int e = 0; e < 8; e++) acc = __builtin_fmaf((float)a[e], (float)b[e], acc);
#pragma unroll
    for (int off = kLanesPerRow / 2; off >= 1; off >>= 1) acc += __shfl_xor(acc, off);
    if ((threadIdx.x & (kLanesPerRow - 1)) == 0) delta[chunk / kLanesPerRow] = acc;
}

hipError_t launch_attn_bwd_delta(const void* o, const void* d_o, float* delta,
                                 int B, int H, int N, int D, hipStream_t stream)
{
    const size_t n_chunks = (size_t)B * H * N * D / 8;
    const dim3 grid((unsigned)((n_chunks + 255) / 256));
    if (D == 128) hipLaunchKernelGGL((attn_bwd_delta_kernel<128>), grid, dim3(256), 0, stream, (const bf16*)o, (const bf16*)d_o, delta, n_chunks);
    else          hipLaunchKernelGGL((attn_bwd_delta_kernel<64>), grid, dim3(256), 0, stream, (const bf16*)o, (const bf16*)d_o, delta, n_chunks);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// kernel 2: dK, dV
// ------------------------------------------------------------------------------------------
// LSE stand-in for query rows past the end of a sequence: P = 2^(s - inf) = 0 for them.
__device__ float g_lse_pad[1] = {INFINITY};

template <int D>
struct DkdvShape {
    static constexpr int kWaves = 4;
    static constexpr int kThreads = 256;
    static constexpr int kTileKV = 128;                 // keys per workgroup (32 per wave)
    static constexpr int kTileQ = 32;                   // queries per loop iteration
    // LDS ring of query blocks.  D = 64: four stages, filled three blocks ahead.  D = 128 (the pipelined
    // step, see the kernel): seven stages, six of them filled at the start; step n then fetches block n + 6
    // into the stage of block n - 1, which nobody reads any more.
    static constexpr bool kPipe = (D == 128);
    static constexpr int kStages = kPipe ? 7 : 4;
    static constexpr int kAhead = kStages - 1;
    static constexpr int kRowBytes = D * 2;
    static constexpr int kChunksPerRow = D / 8;
    static constexpr int kQTileBytes = kTileQ * kRowBytes;
    static constexpr int kStageBytes = 2 * kQTileBytes + 256;      // Q, dO, LSE[32], Delta[32]; a multiple of 256
    static constexpr int kQLoads = kTileQ * kChunksPerRow / kThreads;   // per thread, per tensor
    static constexpr int kLoadsPerBlock = 2 * kQLoads;  // per thread, of Q and dO rows (one more load fetches the statistics)
    static constexpr int kEpiPitch = kRowBytes + 8;     // row pitch of the epilogue staging tile: the odd multiple of 8 bytes spreads
                                                        // both the 8-byte column-piece writes and the row reads over the banks
};

// Chunk swizzle of every row-major bf16 tile in the backward kernels (rows of D elements): spreads
// both a 16-row same-chunk read (MFMA operand rows) and a 4-row x 64-byte transposing read over
// the banks.
template <int D> __device__ __forceinline__ int swz(int row) {
    return D == 128 ? (((row & 3) << 2) | ((row >> 2) & 3)) : ((((row >> 1) & 1) << 2) | ((row >> 2) & 3));
}

// At D = 128: one wave per SIMD (the dK^T, dV^T accumulators and the K, V fragments take 192
// registers), so nothing hides LDS latency or fills the vector ALU but the schedule itself: the
// pipelined step described inside the kernel, with the query blocks arriving by direct global->LDS
// loads issued six blocks ahead into a seven-stage ring.
// At D = 64 the registers allow two workgroups per compute unit, i.e. two waves per SIMD that fill
// each other's gaps (the vector work per MFMA is twice that of D = 128 there), and the phases of a
// block run one after the other, every MFMA operand read one phase ahead of its use:
//     phase 1  S, dP MFMAs from row fragments already in registers; meanwhile the transposed
//              fragments (dO^T, Q^T) and the statistics of THIS block are read from LDS
//     phase 2  P, dS on the vector ALU
//     phase 3  dV^T, dK^T MFMAs from the transposed fragments; meanwhile the row fragments of the
//              NEXT block are read from LDS
// with the query blocks issued three blocks ahead into a four-stage ring.
//
// Nothing hides a workgroup's start-up and wind-down either, so the launch is persistent: the
// resident workgroups (one per compute unit, two at D = 64) walk the key tiles v = blockIdx.x, blockIdx.x + gridDim.x, ... and
// the query-block stream never stops: the loads issued during the last blocks of one key tile
// already fetch the first blocks of the next, and the next tile's K, V fragments are requested
// before the current tile's results are stored.
// Nq queries, Nk keys.  TAIL: the general case (Nq != Nk, or a length that is not a multiple of
// 128); the aligned square case compiles without any of the tail code.  Causal: query i sees keys
// j <= i + (Nk - Nq), Nq <= Nk.
//
// SPILL: every 32-key x 32-query block of dS is also written to DS as the wave holds it after the
// conversion to bf16: 2 KB per block, [2 halves][64 lanes][16 bytes], where lane (key k = lane % 32,
// h = lane / 32) holds in half s the queries 16s + 8g + 4h + t (g = 0..1, t = 0..3) of the block, at
// element 4g + t.  Block (query head, key tile kt, query block qb, wave w) sits at
// (((head * num_kv_tiles + kt) * n_qb + qb) * 4 + w) * 2048 bytes.  Masked pairs and padding rows hold 0.
template <int D, bool CAUSAL, bool TAIL, bool SPILL>
__global__ __launch_bounds__(256, D == 64 ? 2 : 1)
void attn_bwd_dkdv_kernel(const bf16* __restrict__ Q, const bf16* __restrict__ K, const bf16* __restrict__ V,
                          const bf16* __restrict__ dO, const float* __restrict__ LSE, const float* __restrict__ Delta,
                          bf16* __restrict__ dK, bf16* __restrict__ dV,
                          int Nq, int Nk, int num_kv_tiles, int total_units, float scale, int hq, int hkv,
                          char* __restrict__ DS, int n_qb)
{
    using S = DkdvShape<D>;
    __shared__ __attribute__((aligned(1024))) char ring[S::kStages * S::kStageBytes];
    __shared__ __attribute__((aligned(16))) char epi[S::kWaves * 32 * S::kEpiPitch];   // per-wave staging of the dK / dV tile

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int l32 = lane & 31;
    const int h = lane >> 5;
    const int j16 = lane & 15;
    const int ghalf = (lane >> 4) & 1;
    const float c = scale * kLog2e;

    // Work unit: one key tile, or, when causal, the pair (u, last - u): tile u loops over the
    // query blocks from its diagonal on, so the pairs carry (nearly) the same work and the static
    // schedule is balanced.  A "pass" is one key tile; (vu, half) names the pass `half` of unit vu.
    // Grouped-query attention: a key/value head is shared by `group` consecutive query heads, and a
    // pass streams the query blocks of all of them, one head after the other, into the same dK, dV
    // accumulators.  bh below counts key/value heads.
    const int group = hq / hkv;
    const int units = CAUSAL ? (num_kv_tiles + 1) / 2 : num_kv_tiles;
    auto q_head_row = [&](int bh) {         // first row of the first query head of key/value head bh
        return (size_t)((bh / hkv) * hq + (bh % hkv) * group) * Nq;
    };
    // The query blocks of a pass: blocks of 32 rows from pass_ibegin(kt) on, per query head of the
    // group; an even count (the loops below take two blocks per trip), of which the first
    // `n_masked` may touch the diagonal.  General case: the first query that sees a key of the tile
    // is j0 - off, rounded down to a block boundary; rows past Nq are padding.
    const int off = TAIL ? Nk - Nq : 0;
    auto pass_ibegin = [&](int kt) {
        if (!CAUSAL) return 0;
        if (!TAIL) return kt * S::kTileKV;
        const int first = kt * S::kTileKV - off;
        return first > 0 ? first & ~(S::kTileQ - 1) : 0;
    };
    auto pass_nblocks = [&](int ibegin) {
        return TAIL ? 2 * ((Nq - ibegin + 2 * S::kTileQ - 1) / (2 * S::kTileQ)) : (Nq - ibegin) / S::kTileQ;
    };
    auto pass_tile = [&](int vu, int half, int& bh, int& kt) {
        const int logical = xcd_remap(vu, total_units);
        bh = logical / units;
        const int unit = logical % units;
        kt = half == 0 ? unit : num_kv_tiles - 1 - unit;
    };
    // the pass after (vu, half) in this workgroup's walk; vu >= total_units means "none"
    auto next_pass = [&](int& vu, int& half) {
        if (CAUSAL && half == 0) {
            const int unit = xcd_remap(vu, total_units) % units;
            if (num_kv_tiles - 1 - unit != unit) { half = 1; return; }   // (odd tile count: the middle tile has no partner)
        }
        vu += gridDim.x;
        half = 0;
    };

    // ---- query-block prefetch: Q, dO rows (swizzled), LSE and Delta of 32 queries
    int q_src[S::kQLoads];
#pragma unroll
    for (int it = 0; it < S::kQLoads; it++) {
        int s = it * S::kThreads + tid;
        int row = s / S::kChunksPerRow, pc = s % S::kChunksPerRow;
        q_src[it] = row * D + ((pc ^ swz<D>(row)) * 8);
    }
    // Producer side of the ring: a cursor over the query blocks of this workgroup's passes, in the
    // order the passes consume them.  Every call issues the same number of loads in every wave (the
    // vmcnt waits below count them); once the walk is exhausted it fetches one block again and again
    // into stages nobody reads.
    // The lengths need not be multiples of the tile sizes: the kernel works on padded sequences.
    // Reads of rows past the end are redirected to the last row; a query row >= Nq gets LSE = +inf,
    // so its P and dS are exactly 0; key rows >= Nk are computed like any other and not stored.
    int p_vu = blockIdx.x, p_half = 0, p_nblocks = 0, p_g = 0, p_ibegin = 0;
    size_t p_head_row = 0;                  // first row of the group's first query head of the producer's pass
    size_t p_row = 0;                       // first row of the next block to fetch (rows of all heads counted through)
    int p_i0 = 0;                           // ... and its first query within its head
    int p_left = 0;                         // blocks left in the current head's run, this one included
    int p_advance = S::kTileQ;              // rows from one block to the next (0 once the walk is exhausted)
    int p_stage = 0;                        // byte offset of the ring stage the next block goes to
    auto next_stage = [&](int off) { return off + S::kStageBytes == S::kStages * S::kStageBytes ? 0 : off + S::kStageBytes; };
    auto producer_head = [&]() __attribute__((always_inline)) {            // the cursor at the first block of query head p_g of the pass
        p_row = p_head_row + (size_t)p_g * Nq + p_ibegin;
        p_i0 = p_ibegin;
        p_left = p_nblocks;
    };
    auto producer_open = [&]() __attribute__((always_inline)) {            // set the cursor to the first block of pass (p_vu, p_half)
        int bh, kt;
        pass_tile(p_vu, p_half, bh, kt);
        p_ibegin = pass_ibegin(kt);
        p_head_row = q_head_row(bh);
        p_nblocks = pass_nblocks(p_ibegin);
        p_g = 0;
        producer_head();
    };
    // the end of a head's run: rare, so that the steady state of prepare() below is straight-line scalar code
    auto producer_turn = [&]() __attribute__((always_inline)) {
        if (++p_g < group) { producer_head(); return; }
        next_pass(p_vu, p_half);
        if (p_vu < total_units) { producer_open(); return; }
        p_row -= p_advance;                 // exhausted: stay on the last block
        p_i0 -= p_advance;
        p_advance = 0;
        p_left = 0x7fffffff;
    };
    // A block's fetch is split into prepare() (the cursor: scalar work, one rare branch) and its loads,
    // emit(0 .. kLoadsPerBlock): the pipelined step spreads the loads over its matrix instructions, because
    // the compute unit's address unit takes one 16-byte-per-lane instruction every ~16 cycles and a wave
    // that issues several in a row stalls on it.
    size_t e_head_row = 0, e_row = 0;       // of the block being fetched: first row of its head; its own first row
    int e_i0 = 0, e_stage = 0;              // its first query within the head; byte offset of its ring stage
    auto prepare = [&]() __attribute__((always_inline)) {
        e_row = p_row;
        e_i0 = p_i0;
        e_head_row = p_row - p_i0;
        e_stage = p_stage;
        p_stage = next_stage(p_stage);
        p_row += p_advance;
        p_i0 += p_advance;
        --p_left;
    };
    // (kept apart from prepare(): the pipelined step calls prepare() in the middle of a long basic block,
    // which this branch would split)
    auto prepare_turn = [&]() __attribute__((always_inline)) {
        if (__builtin_expect(p_left == 0, 0)) producer_turn();
    };
    auto emit = [&](int which) {
        char* base = ring + e_stage;
        if (which < S::kLoadsPerBlock) {        // Q rows, then dO rows
            const int it = which % S::kQLoads;
            const bf16* block = (which < S::kQLoads ? Q : dO) + e_row * D;      // wave-uniform
            char* dst = base + (which < S::kQLoads ? 0 : S::kQTileBytes) + it * (S::kThreads * 16) + wave * 1024;
            if (TAIL) {
                // a block that runs past the last query: rows >= Nq fetch row Nq-1 instead
                const int r = e_i0 + (it * S::kThreads + tid) / S::kChunksPerRow;
                load_global_to_lds16_untracked(block + q_src[it] - (r < Nq ? 0 : r - (Nq - 1)) * D, dst);
            } else {
                load_global_to_lds16_sbase_untracked(block, (uint32_t)q_src[it] * 2, dst);
            }
        } else if (TAIL) {
            // The statistics: every wave fetches them, to the same place (the same bytes four times over cost
            // nothing; a branch on the wave number costs every wave a restart of its instruction stream, and
            // the waits would have to count differently per wave).
            // lanes 0..31 fetch LSE of the block's 32 queries, lanes 32..63 their Delta
            const int r = e_i0 + l32;
            const float* src = (lane < 32) ? (r < Nq ? LSE + e_head_row + r : g_lse_pad)
                                           : Delta + e_head_row + (r < Nq ? r : Nq - 1);
            load_global_to_lds4_untracked(src, base + 2 * S::kQTileBytes);
        } else {
            // 8 lanes fetch LSE[row..row+31], 8 lanes Delta[row..row+31], 16 bytes each; the other lanes are masked off
            const float* src = (lane < 8) ? (LSE + e_row + lane * 4) : (Delta + e_row + (lane - 8) * 4);
            load_global_to_lds16_lanes16_untracked(src, base + 2 * S::kQTileBytes);
        }
    };
    auto issue_next = [&]() {
        prepare();
#pragma unroll
        for (int which = 0; which <= S::kLoadsPerBlock; which++) emit(which);
        prepare_turn();
    };

    // ---- per-lane LDS offsets
    // row operand (A of S and dP): row l32, logical chunk 2*kb + h
    const int row_lane = l32 * S::kRowBytes + ((h ^ swz<D>(l32)) << 4);
    // transposed operand from a 32-row Q/dO block (A of dV^T, dK^T): rows 16*ks + 4h + j16/4 (+8)
    const int trq_row = 4 * h + (j16 >> 2);
    const int trq_lane = trq_row * S::kRowBytes + (((2 * ghalf + ((j16 & 3) >> 1)) ^ swz<D>(trq_row)) << 4) + ((j16 & 1) << 3);

    constexpr int kSteps = D / 16;          // MFMA steps of S / dP; also 2 * (D/32) steps of dV^T / dK^T
    bf16x8 kf[D / 16], vf[D / 16];          // K, V fragments of this wave's 32 keys (B operands of S = Q K^T and dP = dO V^T)
    auto load_kv = [&](int bh, int kt) {
        const int key = kt * S::kTileKV + wave * 32 + l32;
        const size_t row = (size_t)bh * Nk + ((!TAIL || key < Nk) ? key : Nk - 1);
#pragma unroll
        for (int kb = 0; kb < D / 16; kb++) {
            kf[kb] = *(const bf16x8*)(K + row * D + kb * 16 + h * 8);
            vf[kb] = *(const bf16x8*)(V + row * D + kb * 16 + h * 8);
        }
    };

    int c_vu = blockIdx.x, c_half = 0;      // consumer side: the pass being computed (the grid never exceeds the unit count)
    int c_stage = 0;                        // byte offset of the ring stage of the next block to consume ...
    int c_stage1 = S::kStageBytes, c_stage2 = 2 * S::kStageBytes;      // ... and of the two blocks after it (D = 128)
    {
        int bh, kt;
        pass_tile(c_vu, c_half, bh, kt);
        producer_open();
#pragma unroll
        for (int b = 0; b < S::kAhead; b++) issue_next();
        load_kv(bh, kt);
    }

#pragma unroll 1
    while (c_vu < total_units) {
    int bh, kt;
    pass_tile(c_vu, c_half, bh, kt);
    const size_t head = (size_t)bh * Nk * D;       // of the key/value head
    const int j0 = kt * S::kTileKV;
    const int jw0 = j0 + wave * 32;                // first key of this wave
    const int my_j = jw0 + l32;
    const int i_begin = pass_ibegin(kt);
    const int n_blocks = pass_nblocks(i_begin);           // per query head of the group
    // blocks that may hold a masked (query, key) pair: rows below j0 + 127 - off, i.e. four blocks
    // from i_begin when that is the tile's own first row, up to five when off is not a multiple of 32
    const int n_masked = !CAUSAL ? 0 : !TAIL ? 4 : (n_blocks < 6 ? n_blocks : 6);

    f32x16 dk_acc[D / 32], dv_acc[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; db++)
#pragma unroll
        for (int r = 0; r < 16; r++) { dk_acc[db][r] = 0.f; dv_acc[db][r] = 0.f; }

    // Every global load so far (this pass's K, V fragments, its first blocks, the previous pass's
    // stores) completes here.  The empty asm statements pin the fragment loads above this point (the
    // compiler would otherwise sink them to their first use inside the loop and wait for them there,
    // draining the prefetch every iteration): inside the loop the only waits on the vector memory
    // counter are the explicit ones, which leave the newest prefetches in flight.
#pragma unroll
    for (int kb = 0; kb < D / 16; kb++) {
        // (D = 128: into the accumulator half of the register file, from where the matrix instructions read
        // them just as well; that leaves the other half to the vector ALU's operands, the score blocks among them)
        if (S::kPipe) asm volatile("" : "+a"(kf[kb]), "+a"(vf[kb]));
        else asm volatile("" : "+v"(kf[kb]), "+v"(vf[kb]));
    }
    wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();           // the pass's first blocks landed and visible
    __builtin_amdgcn_sched_barrier(0);

    // register r of a score block <-> query i0 + 8*(r/4) + 4h + r%4, lane <-> key my_j
    const bool pad_key = TAIL && SPILL && my_j >= Nk;    // a padding key was computed from the last real row: its dS must not reach dQ
    auto q_head_of = [&](int g) { return (size_t)(bh / hkv) * hq + (size_t)(bh % hkv) * group + g; };

    if constexpr (S::kPipe) {
    // ------------------------------------------------------------------------------------------
    // D = 128: one wave per SIMD.  A wave issues in order, at most one instruction every four cycles,
    // and a matrix instruction holds the matrix pipe for 32: with matrix instructions back to back the
    // wave idles until the pipe frees, and the ~150 vector instructions of a block then run with the
    // pipe idle.  So every matrix instruction here is followed by the handful of other instructions
    // that fit in its shadow, and the work of three consecutive blocks is in flight at once:
    //     step n, first half    S, dP of block n+1 (16 MFMAs)  next to  P, dS of block n (vector ALU) and
    //                           the transposing LDS reads of block n's Q^T, dO^T fragments
    //     step n, second half   dV^T, dK^T of block n (16 MFMAs)  next to  the LDS reads of the statistics
    //                           of block n+1 and of the row fragments of block n+2, the dS stores and the prefetch
    // S and dP exist twice: the matrix pipe writes one copy (accumulator registers) in the first half, the
    // second half moves it, two registers per MFMA, to the copy the vector ALU reads in the next step.  The empty asm statements keep each group in program order: the compiler keeps them in
    // order with each other and with the scheduling barriers, and each one names a value that the
    // instructions of its group produce or consume.
    // ------------------------------------------------------------------------------------------
    bf16x8 rq[kSteps], rdo[kSteps];         // row fragments: operands of the next S, dP
    bf16x8 tq[kSteps], tdo[kSteps];         // transposed fragments [ks * (D/32) + db]: operands of the next dV^T, dK^T
    bf16x8 pb[2], dsb[2];                   // bf16 P, dS of the block in hand
    f32x4 lse4[4], dl4[4];                  // statistics of the block whose P, dS come next
    f32x16 s_acc, dp_acc;                   // S, dP as the matrix pipe leaves them
    float sc[16], dc[16];                   // ... and where the vector ALU reads them one step later

    auto read_rows = [&](const char* qs, int kb) {
        rq[kb] = lds_read_b128(qs, row_lane ^ ((2 * kb) << 4));
        rdo[kb] = lds_read_b128(qs + S::kQTileBytes, row_lane ^ ((2 * kb) << 4));
    };
    auto read_tq = [&](const char* qs, int idx) {
        const int ks = idx / (D / 32), db = idx % (D / 32);
        const int row_off = 16 * ks * S::kRowBytes;
        const int x0 = (4 * db) << 4, x1 = ((4 * db) ^ 2) << 4;
        tq[idx] = concat(lds_read_tr16(qs, (trq_lane ^ x0) + row_off),
                         lds_read_tr16(qs, (trq_lane ^ x1) + row_off + 8 * S::kRowBytes));
    };
    auto read_tdo = [&](const char* qs, int idx) {
        const int ks = idx / (D / 32), db = idx % (D / 32);
        const int row_off = 16 * ks * S::kRowBytes;
        const int x0 = (4 * db) << 4, x1 = ((4 * db) ^ 2) << 4;
        const char* dos = qs + S::kQTileBytes;
        tdo[idx] = concat(lds_read_tr16(dos, (trq_lane ^ x0) + row_off),
                          lds_read_tr16(dos, (trq_lane ^ x1) + row_off + 8 * S::kRowBytes));
    };
    // S, dP of the block whose row fragments are in rq / rdo; `between(kb, which)` runs after each MFMA
    auto scores = [&](f32x16& s_out, f32x16& dp_out, auto between) {
#pragma unroll
        for (int kb = 0; kb < kSteps; kb++) {
            if (kb == 0) {
                f32x16 zero;
#pragma unroll
                for (int r = 0; r < 16; r++) zero[r] = 0.f;
                asm volatile("" : "+v"(rq[0]));
                s_out = mfma32(rq[0], kf[0], zero);
                asm volatile("" : "+a"(s_out));
                between(kb, 0);
                __builtin_amdgcn_sched_barrier(0);
                asm volatile("" : "+v"(rdo[0]));
                dp_out = mfma32(rdo[0], vf[0], zero);
                asm volatile("" : "+a"(dp_out));
                between(kb, 1);
                __builtin_amdgcn_sched_barrier(0);
            } else {
                asm volatile("" : "+a"(s_out));
                s_out = mfma32(rq[kb], kf[kb], s_out);
                asm volatile("" : "+a"(s_out));
                between(kb, 0);
                __builtin_amdgcn_sched_barrier(0);
                asm volatile("" : "+a"(dp_out));
                dp_out = mfma32(rdo[kb], vf[kb], dp_out);
                asm volatile("" : "+a"(dp_out));
                between(kb, 1);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    // ---- start of the pass: S, dP of its first block; its statistics and the second block's row
    // fragments are read meanwhile.  (The previous pass computed scores for this block too, with its own
    // K and V: they are dropped.)
    {
        const char* q0s = ring + c_stage;
        const char* q1s = ring + c_stage1;
        const f32x4* stat0 = (const f32x4*)(q0s + 2 * S::kQTileBytes);
#pragma unroll
        for (int kb = 0; kb < kSteps; kb++) read_rows(q0s, kb);
        __builtin_amdgcn_sched_barrier(0);
        scores(s_acc, dp_acc, [&](int kb, int which) {
            if (kb < 4) {
                if (which == 0) lse4[kb] = stat0[2 * kb + h];
                else dl4[kb] = stat0[8 + 2 * kb + h];
            }
        });
#pragma unroll
        for (int kb = 0; kb < kSteps; kb++) read_rows(q1s, kb);
#pragma unroll
        for (int r = 0; r < 16; r++) { sc[r] = s_acc[r]; dc[r] = dp_acc[r]; }
        __builtin_amdgcn_sched_barrier(0);
    }

    auto step = [&](auto masked, int blk, char* ds_head) {
        const int i0 = i_begin + blk * S::kTileQ;
        const char* q0s = ring + c_stage;           // block n
        const char* q1s = ring + c_stage1;          // block n+1
        const char* q2s = ring + c_stage2;          // block n+2
        const f32x4* stat1 = (const f32x4*)(q1s + 2 * S::kQTileBytes);
        c_stage = c_stage1;
        c_stage1 = c_stage2;
        c_stage2 = next_stage(c_stage2);

        // ---- first half.  After each MFMA of the next block's S, dP: one element of P and dS - the
        // exponential of element r is started in one group and used in the next, so that nothing waits
        // for it - and the transposing reads of one operand of the second half.
        float pe[16], de[16], te[16];
        auto element_start = [&](int r) {
            const int g = r >> 2, t = r & 3;
            float sv = sc[r], dv = dc[r];
            asm volatile("" : "+v"(sv), "+v"(dv));
            if (decltype(masked)::value && i0 + 8 * g + 4 * h + t + off < my_j) sv = -INFINITY;
            if (pad_key) sv = -INFINITY;
            pe[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(sv, c, -lse4[g][t] * kLog2e));
            te[r] = dv - dl4[g][t];
            asm volatile("" : "+v"(pe[r]), "+v"(te[r]));
        };
        auto element_finish = [&](int r) {
            de[r] = pe[r] * te[r];
            asm volatile("" : "+v"(de[r]));
        };
        scores(s_acc, dp_acc, [&](int kb, int which) {
            const int r = 2 * kb + which;
            element_start(r);
            if (r > 0) element_finish(r - 1);
            if (which == 0) read_tdo(q0s, kb); else read_tq(q0s, kb);
            if (kb == kSteps / 2 + 1) {          // (elements 0..8 are done)
                if (which == 0) {
                    pb[0] = cvt8(pe[0], pe[1], pe[2], pe[3], pe[4], pe[5], pe[6], pe[7]);
                    asm volatile("" : "+v"(pb[0]));
                } else {
                    dsb[0] = cvt8(de[0], de[1], de[2], de[3], de[4], de[5], de[6], de[7]);
                    asm volatile("" : "+v"(dsb[0]));
                }
            }
        });

        // ---- second half: the products of this block, next to the reads of the next blocks' fragments
        element_finish(15);
        // group g of 16 moves two registers of the next block's scores: S first (its last MFMA was issued before dP's)
        auto move_scores = [&](int g) {
            const int r = 2 * (g & 7);
            float a = g < 8 ? s_acc[r] : dp_acc[r], b = g < 8 ? s_acc[r + 1] : dp_acc[r + 1];
            asm volatile("" : "+v"(a), "+v"(b));
            if (g < 8) { sc[r] = a; sc[r + 1] = b; } else { dc[r] = a; dc[r + 1] = b; }
        };
#pragma unroll
        for (int idx = 0; idx < kSteps; idx++) {
            const int ks = idx / (D / 32), db = idx % (D / 32);
            if (idx == 0) {                  // the second half of P, dS is not needed before idx = kSteps / 2
                pb[1] = cvt8(pe[8], pe[9], pe[10], pe[11], pe[12], pe[13], pe[14], pe[15]);
                dsb[1] = cvt8(de[8], de[9], de[10], de[11], de[12], de[13], de[14], de[15]);
            }
            asm volatile("" : "+a"(dv_acc[db]));
            dv_acc[db] = mfma32(tdo[idx], pb[ks], dv_acc[db]);
            asm volatile("" : "+a"(dv_acc[db]));
            rq[idx] = lds_read_b128(q2s, row_lane ^ ((2 * idx) << 4));
            if (idx < 4) lse4[idx] = stat1[2 * idx + h];
            if (idx == 0) asm volatile("" : "+v"(pb[1]), "+v"(dsb[1]));
            if (idx == 0) prepare();         // block n+6 goes into the stage of block n-1, which every wave has left
            if (idx == S::kLoadsPerBlock + 1) emit(S::kLoadsPerBlock);
            move_scores(2 * idx);
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("" : "+a"(dk_acc[db]));
            dk_acc[db] = mfma32(tq[idx], dsb[ks], dk_acc[db]);
            asm volatile("" : "+a"(dk_acc[db]));
            rdo[idx] = lds_read_b128(q2s + S::kQTileBytes, row_lane ^ ((2 * idx) << 4));
            if (idx < 4) dl4[idx] = stat1[8 + 2 * idx + h];
            if (idx >= 1 && idx <= S::kLoadsPerBlock) emit(idx - 1);
            if (SPILL && idx == kSteps / 2 + 2) {       // (both halves of dS exist; every step issues exactly these two stores)
                char* dst = ds_head + ((size_t)(i0 / S::kTileQ) * 4 + wave) * 2048 + lane * 16;
                *(bf16x8*)dst = dsb[0];
                *(bf16x8*)(dst + 1024) = dsb[1];
            }
            move_scores(2 * idx + 1);
            __builtin_amdgcn_sched_barrier(0);
        }

        // Block n+3 (issued three steps ago) must have landed before the next step reads it; the newer
        // prefetches stay in flight, and so do the dS stores issued since: the counter retires loads and stores in issue order, and the stores of the last
        // four steps are younger than the loads waited for.  The wave's own LDS reads must have
        // returned as well: after the barrier the next step's prefetch overwrites the stage of block n.
        constexpr int kStores = SPILL ? 8 : 0;
        prepare_turn();
        wait_vmcnt_lds_done<3 * (S::kLoadsPerBlock + 1) + kStores>();
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
    };

    // When causal, the first n_masked blocks of every query head are the ones that may touch the
    // diagonal.  The stream runs on across the heads of the group.
#pragma unroll 1
    for (int g = 0; g < group; g++) {
        // dS blocks of (this query head, this key tile); query block 0 = queries 0..31 of the head
        char* ds_head = SPILL ? DS + ((q_head_of(g) * num_kv_tiles + kt) * n_qb) * (size_t)8192 : nullptr;
        int blk = 0;
        if (CAUSAL) {
#pragma unroll 1
            for (; blk < n_masked; blk++) step(std::true_type{}, blk, ds_head);
        }
#pragma unroll 1
        for (; blk < n_blocks; blk++) step(std::false_type{}, blk, ds_head);
    }
    } else {
    // ------------------------------------------------------------------------------------------
    // D = 64: the registers allow two workgroups per compute unit, i.e. two waves per SIMD that fill
    // each other's gaps; the phases of a block run one after the other.
    // ------------------------------------------------------------------------------------------
    bf16x8 rq[kSteps], rdo[kSteps];         // row fragments of the block about to be computed
    bf16x8 tq[kSteps], tdo[kSteps], pb[2], dsb[2];      // transposed fragments [ks * (D/32) + db] and bf16 P / dS of a block
    f32x4 lse4[4], dl4[4];

    auto read_rows = [&](const char* qs, int kb) {
        rq[kb] = lds_read_b128(qs, row_lane ^ ((2 * kb) << 4));
        rdo[kb] = lds_read_b128(qs + S::kQTileBytes, row_lane ^ ((2 * kb) << 4));
    };
    auto read_transposed = [&](const char* qs, int idx) {
        const int ks = idx / (D / 32), db = idx % (D / 32);
        const int row_off = 16 * ks * S::kRowBytes;
        const int x0 = (4 * db) << 4, x1 = ((4 * db) ^ 2) << 4;
        const char* dos = qs + S::kQTileBytes;
        tdo[idx] = concat(lds_read_tr16(dos, (trq_lane ^ x0) + row_off),
                          lds_read_tr16(dos, (trq_lane ^ x1) + row_off + 8 * S::kRowBytes));
        tq[idx] = concat(lds_read_tr16(qs, (trq_lane ^ x0) + row_off),
                         lds_read_tr16(qs, (trq_lane ^ x1) + row_off + 8 * S::kRowBytes));
    };
#pragma unroll
    for (int kb = 0; kb < kSteps; kb++) read_rows(ring + c_stage, kb);

    auto step = [&](auto masked, int blk, char* ds_head) {
        const int i0 = i_begin + blk * S::kTileQ;
        const char* qs = ring + c_stage;
        c_stage = next_stage(c_stage);
        const char* qs_next = ring + c_stage;
        const f32x4* stat = (const f32x4*)(qs + 2 * S::kQTileBytes);

        issue_next();                       // into the stage of the previous block, which every wave has left
        __builtin_amdgcn_sched_barrier(0);

        // ---- phase 1: S = Q K^T, dP = dO V^T; read this block's transposed fragments and statistics
        f32x16 s, dp;
#pragma unroll
        for (int r = 0; r < 16; r++) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
        for (int kb = 0; kb < kSteps; kb++) {
            s = mfma32(rq[kb], kf[kb], s);
            dp = mfma32(rdo[kb], vf[kb], dp);
            read_transposed(qs, kb);
            if (kb < 4) { lse4[kb] = stat[2 * kb + h]; dl4[kb] = stat[8 + 2 * kb + h]; }
            __builtin_amdgcn_sched_barrier(0);
        }

        // ---- phase 2: P, dS.  Only the first blocks of a causal tile touch the diagonal: they run as a
        // loop of their own that pushes the masked scores to -inf (P = 2^-inf = 0), so that the main
        // loop carries no compare / select per element.
        if (decltype(masked)::value) {
#pragma unroll
            for (int r = 0; r < 16; r++)
                if (i0 + 8 * (r >> 2) + 4 * h + (r & 3) + off < my_j) s[r] = -INFINITY;
        }
        if (pad_key) {
#pragma unroll
            for (int r = 0; r < 16; r++) s[r] = -INFINITY;
        }
#pragma unroll
        for (int g = 0; g < 4; g++) {
#pragma unroll
            for (int t = 0; t < 4; t++) {
                const int r = 4 * g + t;
                const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], c, -lse4[g][t] * kLog2e));
                s[r] = p;
                dp[r] = p * (dp[r] - dl4[g][t]);
            }
        }
#pragma unroll
        for (int ks = 0; ks < 2; ks++) {
            const int r0 = 8 * ks;
            pb[ks] = cvt8(s[r0], s[r0 + 1], s[r0 + 2], s[r0 + 3], s[r0 + 4], s[r0 + 5], s[r0 + 6], s[r0 + 7]);
            dsb[ks] = cvt8(dp[r0], dp[r0 + 1], dp[r0 + 2], dp[r0 + 3], dp[r0 + 4], dp[r0 + 5], dp[r0 + 6], dp[r0 + 7]);
        }
        // SPILL: every step issues exactly these two stores - the waits below count them
        if (SPILL) {
            char* dst = ds_head + ((size_t)(i0 / S::kTileQ) * 4 + wave) * 2048 + lane * 16;
            *(bf16x8*)dst = dsb[0];
            *(bf16x8*)(dst + 1024) = dsb[1];
        }

        // ---- phase 3: dV^T += dO^T P, dK^T += Q^T dS, and the reads of the next block's row fragments
        // (that block landed before the barrier that ended the previous iteration; the next block in the
        // stream is the next pass's first one after this pass's last)
#pragma unroll
        for (int idx = 0; idx < kSteps; idx++) {
            const int ks = idx / (D / 32), db = idx % (D / 32);
            dv_acc[db] = mfma32(tdo[idx], pb[ks], dv_acc[db]);
            dk_acc[db] = mfma32(tq[idx], dsb[ks], dk_acc[db]);
            read_rows(qs_next, idx);
        }

        // the block two ahead in the stream (issued two iterations ago) must have landed before the
        // next iteration reads its rows; the newer prefetches may stay in flight.  The wave's own LDS reads of this block's stage must have returned as
        // well: after the barrier the next step's prefetch overwrites that stage.
        // (the counter retires loads and stores in issue order: the dS stores of this step and of the
        // previous one were issued after the loads waited for)
        constexpr int kStores = SPILL ? 4 : 0;
        wait_vmcnt_lds_done<(S::kAhead - 2) * (S::kLoadsPerBlock + 1) + kStores>();
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
    };

#pragma unroll 1
    for (int g = 0; g < group; g++) {
        char* ds_head = SPILL ? DS + ((q_head_of(g) * num_kv_tiles + kt) * n_qb) * (size_t)8192 : nullptr;
        int blk = 0;
        if (CAUSAL) {
#pragma unroll 1
            for (; blk < n_masked; blk++) step(std::true_type{}, blk, ds_head);
        }
#pragma unroll 1
        for (; blk < n_blocks; blk++) step(std::false_type{}, blk, ds_head);
    }
    }

    // The next pass's K, V fragments are requested now, so that they travel while this pass's last
    // products and its stores run (S and dP are done with the old fragments).
    next_pass(c_vu, c_half);
    if (c_vu < total_units) {
        int nbh, nkt;
        pass_tile(c_vu, c_half, nbh, nkt);
        load_kv(nbh, nkt);
    }
    // ---- epilogue.  In accumulator layout a lane holds 4 consecutive columns of ONE key row
    // (lane <-> key my_j, register r of block db <-> column 32db + 8*(r/4) + 4h + r%4), so storing
    // from there would touch 32 rows per instruction.  Each wave instead turns its 32 x D tile
    // around in a private LDS buffer and stores whole rows, 16 bytes per lane.
    char* my_epi = epi + wave * (32 * S::kEpiPitch);
    auto store_tile = [&](const f32x16 (&acc)[D / 32], float mul, bf16* dst) {   // dst: first row of this wave's tile
#pragma unroll
        for (int db = 0; db < D / 32; db++)
#pragma unroll
            for (int g = 0; g < 4; g++) {
                bf16x2 a = cvt2(acc[db][4 * g] * mul, acc[db][4 * g + 1] * mul);
                bf16x2 b = cvt2(acc[db][4 * g + 2] * mul, acc[db][4 * g + 3] * mul);
                *(bf16x4*)(my_epi + l32 * S::kEpiPitch + (32 * db + 8 * g + 4 * h) * 2) = __builtin_shufflevector(a, b, 0, 1, 2, 3);
            }
        constexpr int kLanesPerRow = D * 2 / 16;
        constexpr int kRowsPerStore = 64 / kLanesPerRow;
        const int sub_row = lane / kLanesPerRow, col16 = lane % kLanesPerRow;
#pragma unroll
        for (int i = 0; i < 32 / kRowsPerStore; i++) {
            const int row = i * kRowsPerStore + sub_row;
            const char* src = my_epi + row * S::kEpiPitch + col16 * 16;
            const bf16x4 lo = *(const bf16x4*)src, hi = *(const bf16x4*)(src + 8);
            if (!TAIL || jw0 + row < Nk) *(bf16x8*)(dst + (size_t)row * D + col16 * 8) = concat(lo, hi);
        }
    };
    store_tile(dk_acc, scale, dK + head + (size_t)jw0 * D);
    store_tile(dv_acc, 1.0f, dV + head + (size_t)jw0 * D);
    }   // pass
    wait_vmcnt<0>();      // the spare prefetches of the last blocks must not outlive the workgroup's LDS
}

template <int D, bool CAUSAL, bool TAIL, bool SPILL>
static hipError_t launch_dkdv_tt(const void* q, const void* k, const void* v, const void* d_o,
                                 const float* lse, const float* delta, void* dk, void* dv,
                                 int B, int H, int Hkv, int Nq, int Nk, float scale, hipStream_t stream, void* ds)
{
    using S = DkdvShape<D>;
    const int num_kv_tiles = (Nk + S::kTileKV - 1) / S::kTileKV;
    const int total_units = B * Hkv * (CAUSAL ? (num_kv_tiles + 1) / 2 : num_kv_tiles);
    int cus = 0;
    hipError_t e = compute_unit_count(&cus);
    if (e != hipSuccess) return e;
    const int resident = cus * (D == 64 ? 2 : 1);               // as many workgroups as fit at once
    const int grid = total_units < resident ? total_units : resident;
    hipLaunchKernelGGL((attn_bwd_dkdv_kernel<D, CAUSAL, TAIL, SPILL>), dim3(grid), dim3(S::kThreads), 0, stream,
                       (const bf16*)q, (const bf16*)k, (const bf16*)v, (const bf16*)d_o, lse, delta,
                       (bf16*)dk, (bf16*)dv, Nq, Nk, num_kv_tiles, total_units, scale, H, Hkv,
                       (char*)ds, ds_query_blocks(Nq));
    return hipGetLastError();
}

template <int D, bool CAUSAL>
static hipError_t launch_dkdv_t(const void* q, const void* k, const void* v, const void* d_o,
                                const float* lse, const float* delta, void* dk, void* dv,
                                int B, int H, int Hkv, int Nq, int Nk, float scale, hipStream_t stream, void* ds)
{
    using S = DkdvShape<D>;
    const bool tail = Nq != Nk || Nk % S::kTileKV;
    if (ds) return tail ? launch_dkdv_tt<D, CAUSAL, true, true>(q, k, v, d_o, lse, delta, dk, dv, B, H, Hkv, Nq, Nk, scale, stream, ds)
                        : launch_dkdv_tt<D, CAUSAL, false, true>(q, k, v, d_o, lse, delta, dk, dv, B, H, Hkv, Nq, Nk, scale, stream, ds);
    return tail ? launch_dkdv_tt<D, CAUSAL, true, false>(q, k, v, d_o, lse, delta, dk, dv, B, H, Hkv, Nq, Nk, scale, stream, ds)
                : launch_dkdv_tt<D, CAUSAL, false, false>(q, k, v, d_o, lse, delta, dk, dv, B, H, Hkv, Nq, Nk, scale, stream, ds);
}

// ds != nullptr: the kernel also stores its dS blocks there (ds_spill_bytes(...) bytes) for launch_attn_bwd_dq_from_ds
hipError_t launch_attn_bwd_dkdv(const void* q, const void* k, const void* v, const void* d_o,
                                const float* lse, const float* delta, void* dk, void* dv,
                                int B, int H, int Hkv, int Nq, int Nk, int D, int causal, float scale, hipStream_t stream,
                                void* ds)
{
    if (D == 128) return causal ? launch_dkdv_t<128, true>(q, k, v, d_o, lse, delta, dk, dv, B, H, Hkv, Nq, Nk, scale, stream, ds)
                                : launch_dkdv_t<128, false>(q, k, v, d_o, lse, delta, dk, dv, B, H, Hkv, Nq, Nk, scale, stream, ds);
    return causal ? launch_dkdv_t<64, true>(q, k, v, d_o, lse, delta, dk, dv, B, H, Hkv, Nq, Nk, scale, stream, ds)
                  : launch_dkdv_t<64, false>(q, k, v, d_o, lse, delta, dk, dv, B, H, Hkv, Nq, Nk, scale, stream, ds);
}

// ------------------------------------------------------------------------------------------
// kernel 3: dQ
// ------------------------------------------------------------------------------------------
template <int D>
struct DqShape {
    static constexpr int kWaves = 4;
    static constexpr int kThreads = 256;
    static constexpr int kTileQ = 128;                  // queries per workgroup (32 per wave)
    static constexpr int kTileKV = 64;                  // keys per LDS stage
    static constexpr int kRowBytes = D * 2;
    static constexpr int kChunksPerRow = D / 8;
    static constexpr int kTileBytes = kTileKV * kRowBytes;
    static constexpr int kStageBytes = 2 * kTileBytes;  // K tile then V tile
    static constexpr int kLoadsPerTile = kTileKV * kChunksPerRow / kThreads;   // per thread, per tensor
};

// FUSED: Delta is not an input: the kernel computes Delta_i = sum_d dO_id O_id for its own rows (a
// lane already holds its query's dO row), writes it to DeltaOut for the dK/dV kernel that follows,
// and uses it; the separate Delta pass over O and dO is then not needed.
template <int D, bool CAUSAL, bool TAIL, bool FUSED>
__global__ __launch_bounds__(256, 2)
void attn_bwd_dq_kernel(const bf16* __restrict__ Q, const bf16* __restrict__ K, const bf16* __restrict__ V,
                        const bf16* __restrict__ dO, const float* __restrict__ LSE, const float* __restrict__ Delta,
                        bf16* __restrict__ dQ, int Nq, int Nk, int num_q_tiles, int total_wg, float scale, int hq, int hkv,
                        const bf16* __restrict__ O, float* __restrict__ DeltaOut)
{
    using S = DqShape<D>;
    __shared__ __attribute__((aligned(1024))) char stage0[S::kStageBytes];
    __shared__ __attribute__((aligned(1024))) char stage1[S::kStageBytes];

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int l32 = lane & 31;
    const int h = lane >> 5;

    // Work unit: one query tile, or, when causal, the pair (last - u, u): tile t streams the keys up
    // to its diagonal, so the pairs carry (nearly) the same work and the launch is balanced.
    // Nq queries, Nk keys; TAIL and the causal alignment as in the kernels above.
    const int units = CAUSAL ? (num_q_tiles + 1) / 2 : num_q_tiles;
    const int logical = xcd_remap(blockIdx.x, total_wg);
    const int bh = logical / units;
    const int unit = logical % units;
    // grouped-query attention: query head h of a batch entry reads key/value head h / (hq / hkv)
    const size_t head = (size_t)bh * Nq * D;
    const size_t kv_head = (size_t)((bh / hq) * hkv + (bh % hq) / (hq / hkv)) * Nk * D;
    const int off = TAIL ? Nk - Nq : 0;          // causal: query i sees keys <= i + off
    const bf16* Kh = K + kv_head;
    const bf16* Vh = V + kv_head;
#pragma unroll 1
    for (int pass = 0; pass < (CAUSAL ? 2 : 1); pass++) {
    const int qt = pass == 0 ? num_q_tiles - 1 - unit : unit;
    if (pass == 1 && qt == num_q_tiles - 1 - unit) break;   // odd tile count: the middle tile has no partner
    const int q0 = qt * S::kTileQ + wave * 32;
    const int my_q = q0 + l32;
    // The lengths need not be multiples of the tile sizes: the kernel works on padded sequences,
    // reads of rows past the end are redirected to the last row, keys >= Nk are masked, query rows
    // >= Nq are not stored.
    const int my_q_ld = (!TAIL || my_q < Nq) ? my_q : Nq - 1;
    const float c = scale * kLog2e;

    // ---- Q_i, dO_i fragments (B operands of S^T = K Q^T and dP^T = V dO^T) and the row statistics
    bf16x8 qf[D / 16], dof[D / 16];
#pragma unroll
    for (int kb = 0; kb < D / 16; kb++) {
        qf[kb] = *(const bf16x8*)(Q + head + (size_t)my_q_ld * D + kb * 16 + h * 8);
        dof[kb] = *(const bf16x8*)(dO + head + (size_t)my_q_ld * D + kb * 16 + h * 8);
    }
    const float lse2 = LSE[(size_t)bh * Nq + my_q_ld] * kLog2e;
    float delta;
    if (FUSED) {
        float part = 0.f;       // this lane's half of the row (columns 16*kb + 8*h .. +7)
#pragma unroll
        for (int kb = 0; kb < D / 16; kb++) {
            const bf16x8 of = *(const bf16x8*)(O + head + (size_t)my_q_ld * D + kb * 16 + h * 8);
#pragma unroll
            for (int e = 0; e < 8; e++) part = __builtin_fmaf((float)of[e], (float)dof[kb][e], part);
        }
        delta = half_sum(part);
        if (h == 0 && (!TAIL || my_q < Nq)) DeltaOut[(size_t)bh * Nq + my_q] = delta;
    } else {
        delta = Delta[(size_t)bh * Nq + my_q_ld];
    }

    // ---- direct-to-LDS tile loads (same slot arithmetic as the forward kernel)
    int kv_src[S::kLoadsPerTile];
#pragma unroll
    for (int it = 0; it < S::kLoadsPerTile; it++) {
        int s = it * S::kThreads + tid;
        int row = s / S::kChunksPerRow, pc = s % S::kChunksPerRow;
        kv_src[it] = row * D + ((pc ^ swz<D>(row)) * 8);
    }
    auto issue_tile = [&](char* base, int tile) {
        const int j0 = tile * S::kTileKV;
        const bf16* kt = Kh + (size_t)j0 * D;
        const bf16* vt = Vh + (size_t)j0 * D;
        if (!TAIL || j0 + S::kTileKV <= Nk) {
#pragma unroll
            for (int it = 0; it < S::kLoadsPerTile; it++)
                load_global_to_lds16(kt + kv_src[it], base + wave * 1024 + it * (S::kThreads * 16));
#pragma unroll
            for (int it = 0; it < S::kLoadsPerTile; it++)
                load_global_to_lds16(vt + kv_src[it], base + S::kTileBytes + wave * 1024 + it * (S::kThreads * 16));
        } else {
            // the tile runs past the last key: rows >= Nk fetch row Nk-1 instead (they are masked later)
#pragma unroll
            for (int it = 0; it < S::kLoadsPerTile; it++) {
                const int row = j0 + (it * S::kThreads + tid) / S::kChunksPerRow;
                const int back = (row < Nk ? 0 : row - (Nk - 1)) * D;   // elements to step back
                load_global_to_lds16(kt + kv_src[it] - back, base + wave * 1024 + it * (S::kThreads * 16));
                load_global_to_lds16(vt + kv_src[it] - back, base + S::kTileBytes + wave * 1024 + it * (S::kThreads * 16));
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    // ---- per-lane LDS offsets
    // row operand (A of S^T and dP^T): row 32b + l32, logical chunk 2*kb + h
    const int row_lane = l32 * S::kRowBytes + ((h ^ swz<D>(l32)) << 4);
    // transposed operand from the K tile (A of dQ^T = K^T dS^T): rows 16*kk + 4h + j16/4 (+8)
    const int j16 = lane & 15;
    const int tr_row = 4 * h + (j16 >> 2);
    const int tr_lane = tr_row * S::kRowBytes + (((2 * ((lane >> 4) & 1) + ((j16 & 3) >> 1)) ^ swz<D>(tr_row)) << 4) + ((j16 & 1) << 3);

    f32x16 dq_acc[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; db++)
#pragma unroll
        for (int r = 0; r < 16; r++) dq_acc[db][r] = 0.f;

    auto compute_tile = [&](const char* ks, int tile) {
        const int j0 = tile * S::kTileKV;
        if (CAUSAL && j0 > q0 + 31 + off) return;    // every key of the tile is masked for this wave
        const char* vs = ks + S::kTileBytes;
        // the tile crosses this wave's diagonal, or runs past the last key
        const bool diag = (CAUSAL && (j0 + S::kTileKV - 1 > q0 + off)) || (TAIL && j0 + S::kTileKV > Nk);
        // The tile is processed in two halves of 32 keys, so that only one half's S^T / dP^T
        // accumulators are live at a time.
#pragma unroll
        for (int b = 0; b < 2; b++) {
            f32x16 s, dp;
#pragma unroll
            for (int r = 0; r < 16; r++) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
            for (int kb = 0; kb < D / 16; kb++) {
                const int off = (row_lane ^ ((2 * kb) << 4)) + b * 32 * S::kRowBytes;
                s = mfma32(lds_read_b128(ks, off), qf[kb], s);
                dp = mfma32(lds_read_b128(vs, off), dof[kb], dp);
            }
            // P^T and dS^T: lane <-> query my_q, register r <-> key j0 + 32b + 8*(r/4) + 4h + r%4.
            // Only a tile on the diagonal needs the mask: it pushes the masked scores to -inf in a
            // branch of its own (P = 2^-inf = 0), so the common case carries no compare / select.
            if (diag) {
#pragma unroll
                for (int r = 0; r < 16; r++) {
                    const int key = j0 + 32 * b + 8 * (r >> 2) + 4 * h + (r & 3);
                    if ((CAUSAL && key > my_q + off) || (TAIL && key >= Nk)) s[r] = -INFINITY;
                }
            }
#pragma unroll
            for (int r = 0; r < 16; r++) {
                const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], c, -lse2));
                s[r] = p * (dp[r] - delta);
            }
            // dQ^T += K^T dS^T, 16 keys per MFMA
#pragma unroll
            for (int k2 = 0; k2 < 2; k2++) {
                const int kk = 2 * b + k2, r0 = 8 * k2;
                bf16x8 dsb = cvt8(s[r0 + 0], s[r0 + 1], s[r0 + 2], s[r0 + 3],
                                  s[r0 + 4], s[r0 + 5], s[r0 + 6], s[r0 + 7]);
#pragma unroll
                for (int db = 0; db < D / 32; db++) {
                    const int row_off = 16 * kk * S::kRowBytes;
                    const int x0 = (4 * db) << 4, x1 = ((4 * db) ^ 2) << 4;
                    bf16x4 a0 = lds_read_tr16(ks, (tr_lane ^ x0) + row_off);
                    bf16x4 a1 = lds_read_tr16(ks, (tr_lane ^ x1) + row_off + 8 * S::kRowBytes);
                    dq_acc[db] = mfma32(concat(a0, a1), dsb, dq_acc[db]);
                }
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
    issue_tile(stage0, 0);
    wait_vmcnt<0>();
    __syncthreads();
    for (int t = 0; t < n_tiles; t += 2) {
        issue_tile(stage1, t + 1);
        compute_tile(stage0, t);
        wait_vmcnt<0>();
        __syncthreads();
        if (t + 2 < n_tiles) issue_tile(stage0, t + 2);
        compute_tile(stage1, t + 1);
        wait_vmcnt<0>();
        __syncthreads();
    }

    // ---- epilogue: dQ = scale * acc; lane <-> query, register r of block db <-> column 32db + 8*(r/4) + 4h + r%4
    if (!TAIL || my_q < Nq) {
        bf16* dQr = dQ + head + (size_t)my_q * D;
#pragma unroll
        for (int db = 0; db < D / 32; db++)
#pragma unroll
            for (int g = 0; g < 4; g++) {
                bf16x2 lo = cvt2(dq_acc[db][4 * g + 0] * scale, dq_acc[db][4 * g + 1] * scale);
                bf16x2 hi = cvt2(dq_acc[db][4 * g + 2] * scale, dq_acc[db][4 * g + 3] * scale);
                *(bf16x4*)(dQr + 32 * db + 8 * g + 4 * h) = __builtin_shufflevector(lo, hi, 0, 1, 2, 3);
            }
    }
    }   // pass (the loop above ends with a barrier, so both stages are free again)
}

template <int D, bool CAUSAL, bool TAIL, bool FUSED>
static hipError_t launch_dq_tt(const void* q, const void* k, const void* v, const void* d_o,
                               const float* lse, const float* delta, void* dq,
                               int B, int H, int Hkv, int Nq, int Nk, float scale, hipStream_t stream,
                               const void* o, float* delta_out)
{
    using S = DqShape<D>;
    const int num_q_tiles = (Nq + S::kTileQ - 1) / S::kTileQ;
    const int total = B * H * (CAUSAL ? (num_q_tiles + 1) / 2 : num_q_tiles);
    hipLaunchKernelGGL((attn_bwd_dq_kernel<D, CAUSAL, TAIL, FUSED>), dim3(total), dim3(S::kThreads), 0, stream,
                       (const bf16*)q, (const bf16*)k, (const bf16*)v, (const bf16*)d_o, lse, delta,
                       (bf16*)dq, Nq, Nk, num_q_tiles, total, scale, H, Hkv, (const bf16*)o, delta_out);
    return hipGetLastError();
}

template <int D, bool CAUSAL>
static hipError_t launch_dq_t(const void* q, const void* k, const void* v, const void* d_o,
                              const float* lse, const float* delta, void* dq,
                              int B, int H, int Hkv, int Nq, int Nk, float scale, hipStream_t stream,
                              const void* o, float* delta_out)
{
    using S = DqShape<D>;
    const bool tail = Nq != Nk || Nq % S::kTileQ;
    if (o) return tail ? launch_dq_tt<D, CAUSAL, true, true>(q, k, v, d_o, lse, delta, dq, B, H, Hkv, Nq, Nk, scale, stream, o, delta_out)
                       : launch_dq_tt<D, CAUSAL, false, true>(q, k, v, d_o, lse, delta, dq, B, H, Hkv, Nq, Nk, scale, stream, o, delta_out);
    return tail ? launch_dq_tt<D, CAUSAL, true, false>(q, k, v, d_o, lse, delta, dq, B, H, Hkv, Nq, Nk, scale, stream, o, delta_out)
                : launch_dq_tt<D, CAUSAL, false, false>(q, k, v, d_o, lse, delta, dq, B, H, Hkv, Nq, Nk, scale, stream, o, delta_out);
}

// o != nullptr: Delta is computed from o and d_o inside the kernel and written to delta_out (delta is not read).
hipError_t launch_attn_bwd_dq(const void* q, const void* k, const void* v, const void* d_o,
                              const float* lse, const float* delta, void* dq,
                              int B, int H, int Hkv, int Nq, int Nk, int D, int causal, float scale, hipStream_t stream,
                              const void* o, float* delta_out)
{
    if (D == 128) return causal ? launch_dq_t<128, true>(q, k, v, d_o, lse, delta, dq, B, H, Hkv, Nq, Nk, scale, stream, o, delta_out)
                                : launch_dq_t<128, false>(q, k, v, d_o, lse, delta, dq, B, H, Hkv, Nq, Nk, scale, stream, o, delta_out);
    return causal ? launch_dq_t<64, true>(q, k, v, d_o, lse, delta, dq, B, H, Hkv, Nq, Nk, scale, stream, o, delta_out)
                  : launch_dq_t<64, false>(q, k, v, d_o, lse, delta, dq, B, H, Hkv, Nq, Nk, scale, stream, o, delta_out);
}

// ------------------------------------------------------------------------------------------
// kernel 4: dQ from the dS blocks that kernel 2 stored
// ------------------------------------------------------------------------------------------
template <int D>
struct DqDsShape {
    static constexpr int kWaves = 8;
    static constexpr int kThreads = 512;
    static constexpr int kTileQ = 256;                  // queries per workgroup (32 per wave)
    static constexpr int kTileKV = 64;                  // keys per step
    static constexpr int kRowBytes = D * 2;
    static constexpr int kChunksPerRow = D / 8;
    static constexpr int kKTileBytes = kTileKV * kRowBytes;
    static constexpr int kKStages = 4;                  // ring of K tiles, filled three tiles ahead
    static constexpr int kDsTileBytes = 2 * 2048;       // the two 32-key blocks of one wave and one step
    static constexpr int kDsAhead = 4;                  // dS tiles held in registers ahead of their use
    static constexpr int kKLoads = kTileKV * kChunksPerRow / kThreads;   // per thread and tile
    static constexpr int kDsLoads = kDsTileBytes / 1024;                  // per lane and tile
    static constexpr int kLdsBytes = kKStages * kKTileBytes + kWaves * 2 * kDsTileBytes;
    // vector-memory operations a wave issues per step, and how many of them are younger than the K tile
    // that must have landed at the end of a step (see the loop)
    static constexpr int kOpsPerStep = kKLoads + kDsLoads;
    static constexpr int kWaitCount = kDsLoads + 2 * kOpsPerStep;
};

// 16 bytes per lane from global memory into registers, issued through inline assembly so that the
// compiler does not place a wait of its own before the first use: the data is only touched after the
// loop's own wait (wait_vmcnt<>) and a claim_loaded() on the registers.
__device__ __forceinline__ void load16_untracked(bf16x8& dst, const void* gptr) {
    asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(dst) : "v"(gptr) : "memory");
}
__device__ __forceinline__ void claim_loaded(bf16x8& r) { asm volatile("" : "+v"(r) : : "memory"); }

// dQ_i = scale * sum_j dS_ij K_j: one workgroup per 256-query tile (causal: balanced pairs of tiles), wave w
// owns queries 32w..32w+31 and keeps dQ^T in registers while the workgroup walks 64-key tiles.  The kernel is
// bound by reading dS (2 bytes per query-key pair) from HBM, so everything is arranged around keeping many
// bytes in flight: each wave loads its own dS blocks into registers four steps ahead (they are private to the
// wave: no barrier is involved), K tiles go to a four-stage LDS ring by direct loads three steps ahead, and
// the single wait per step is for a K tile that is older than three steps' worth of dS loads (the counter
// retires in issue order), so those stay in flight across the barrier.
// dQ^T += K^T dS^T needs dS^T with the QUERY on lanes, and the stored blocks have the KEY on lanes: a wave
// writes the block it is about to use into a private LDS buffer, the 16-byte piece of (key, half, h) at
// (key * 4 + half * 2 + h) * 16, and takes the operand out with transposing reads (4 keys x 4 query quads per
// 16 lanes: every bank once).  No mask code: kernel 2 stored zeros for masked pairs, padding queries and
// padding keys; a wave does not compute on tiles that lie wholly beyond its diagonal, which kernel 2 may not
// have written: its loads of such tiles are redirected to its last real tile.
template <int D, bool CAUSAL, bool TAIL>
__global__ __launch_bounds__(512, 1)
void attn_bwd_dq_from_ds_kernel(const bf16* __restrict__ K, const char* __restrict__ DS, bf16* __restrict__ dQ,
                                int Nq, int Nk, int num_q_tiles, int total_wg, float scale, int hq, int hkv,
                                int num_kv_tiles, int n_qb)
{
    using S = DqDsShape<D>;
    __shared__ __attribute__((aligned(1024))) char smem[S::kLdsBytes];
    char* const kring = smem;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int l32 = lane & 31;
    const int h = lane >> 5;
    char* const dsbuf = smem + S::kKStages * S::kKTileBytes + wave * (2 * S::kDsTileBytes);   // two buffers of this wave

    const int units = CAUSAL ? (num_q_tiles + 1) / 2 : num_q_tiles;
    const int logical = xcd_remap(blockIdx.x, total_wg);
    const int bh = logical / units;                  // query head
    const int unit = logical % units;
    const size_t head = (size_t)bh * Nq * D;
    const size_t kv_head = (size_t)((bh / hq) * hkv + (bh % hq) / (hq / hkv)) * Nk * D;
    const int off = TAIL ? Nk - Nq : 0;              // causal: query i sees keys <= i + off
    const bf16* Kh = K + kv_head;
    const char* DSh = DS + (size_t)bh * num_kv_tiles * n_qb * 8192;

    // K tile loads: slot arithmetic of the other kernels
    int k_src[S::kKLoads];
#pragma unroll
    for (int it = 0; it < S::kKLoads; it++) {
        int s = it * S::kThreads + tid;
        int row = s / S::kChunksPerRow, pc = s % S::kChunksPerRow;
        k_src[it] = row * D + ((pc ^ swz<D>(row)) * 8);
    }
    // where this lane's 16-byte piece of a stored half-block goes in the wave's LDS buffer (half s adds 32)
    const int piece_off = (l32 * 4 + h) * 16;
    // transposed operand from the K tile (A of dQ^T = K^T dS^T): rows 16*kk + 4h + j16/4 (+8)
    const int j16 = lane & 15;
    const int tr_row = 4 * h + (j16 >> 2);
    const int tr_lane = tr_row * S::kRowBytes + (((2 * ((lane >> 4) & 1) + ((j16 & 3) >> 1)) ^ swz<D>(tr_row)) << 4) + ((j16 & 1) << 3);
    // dS^T operand (B): 16-lane group G = lane / 16 covers queries 16 * (G % 2) .. + 15 (= half G % 2 of the
    // block) and keys 4 * (G / 2) + j16 / 4 (+ 8) of a 16-key step; lane j of the group points at the query
    // quad j % 4, i.e. (h = quad % 2, g = quad / 2) of the stored layout
    const int ds_lane = (4 * h + (j16 >> 2)) * 64 + ((lane >> 4) & 1) * 32 + (j16 & 1) * 16 + ((j16 & 3) >> 1) * 8;

#pragma unroll 1
    for (int pass = 0; pass < (CAUSAL ? 2 : 1); pass++) {
    const int qt = pass == 0 ? num_q_tiles - 1 - unit : unit;
    if (pass == 1 && qt == num_q_tiles - 1 - unit) break;   // odd tile count: the middle tile has no partner
    const int q0 = qt * S::kTileQ + wave * 32;
    const int my_q = q0 + l32;
    const int qb = qt * (S::kTileQ / 32) + wave;     // this wave's query block

    // 64-key tiles the workgroup walks (every key visible to its last query), rounded up to the unroll of the loop
    int n_tiles;
    if (!TAIL) {
        n_tiles = (CAUSAL ? qt * S::kTileQ + S::kTileQ : Nk) / S::kTileKV;
    } else {
        int n_keys = Nk;
        if (CAUSAL && qt * S::kTileQ + S::kTileQ + off < n_keys) n_keys = qt * S::kTileQ + S::kTileQ + off;
        n_tiles = 2 * ((n_keys + 2 * S::kTileKV - 1) / (2 * S::kTileKV));
    }
    const int n_steps = (n_tiles + 3) & ~3;
    // the last tile this wave computes on; -1: none (a wave of padding rows)
    int last_tile = n_tiles - 1;
    if (CAUSAL) { const int d = (q0 + 31 + off) / S::kTileKV; if (d < last_tile) last_tile = d; }
    if (TAIL && q0 >= Nq) last_tile = -1;
    // block (key tile 0, query block 0) of the head is always written: the stand-in for a wave without tiles
    const char* ds_row = last_tile >= 0 ? DSh + (size_t)qb * 8192 : DSh;

    auto issue_k = [&](int tile) {                   // into ring stage tile % 4
        char* base = kring + (tile & (S::kKStages - 1)) * S::kKTileBytes + wave * 1024;
        if (tile > n_tiles - 1) tile = n_tiles - 1;  // (beyond the walk: the last tile again, into a stage nobody reads any more)
        const int j0 = tile * S::kTileKV;
        const bf16* kt = Kh + (size_t)j0 * D;
#pragma unroll
        for (int it = 0; it < S::kKLoads; it++) {
            int back = 0;
            if (TAIL) {                              // rows >= Nk fetch row Nk-1 (their dS is 0)
                const int row = j0 + (it * S::kThreads + tid) / S::kChunksPerRow;
                back = (row < Nk ? 0 : row - (Nk - 1)) * D;
            }
            load_global_to_lds16_untracked(kt + k_src[it] - back, base + it * (S::kThreads * 16));
        }
    };
    // the two 32-key blocks of step `tile` for this wave's queries: blocks 2*(tile%2), +1 of key tile tile/2
    auto issue_ds = [&](bf16x8 (&r)[4], int tile) {
        if (tile > last_tile) tile = last_tile < 0 ? 0 : last_tile;
        const char* blk = ds_row + ((size_t)(tile >> 1) * n_qb * 4 + 2 * (tile & 1)) * 2048 + lane * 16;
#pragma unroll
        for (int n = 0; n < 4; n++) load16_untracked(r[n], blk + n * 1024);
    };

    f32x16 dq_acc[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; db++)
#pragma unroll
        for (int r = 0; r < 16; r++) dq_acc[db][r] = 0.f;

    auto compute_tile = [&](const char* ks, const char* dss) {
#pragma unroll
        for (int kk = 0; kk < 4; kk++) {             // 16 keys per step
            const int ds_off = (kk >> 1) * 2048 + (kk & 1) * 1024;
            bf16x4 b0 = lds_read_tr16(dss, ds_lane + ds_off);
            bf16x4 b1 = lds_read_tr16(dss, ds_lane + ds_off + 512);
            const bf16x8 dsb = concat(b0, b1);
#pragma unroll
            for (int db = 0; db < D / 32; db++) {
                const int row_off = 16 * kk * S::kRowBytes;
                const int x0 = (4 * db) << 4, x1 = ((4 * db) ^ 2) << 4;
                bf16x4 a0 = lds_read_tr16(ks, (tr_lane ^ x0) + row_off);
                bf16x4 a1 = lds_read_tr16(ks, (tr_lane ^ x1) + row_off + 8 * S::kRowBytes);
                dq_acc[db] = mfma32(concat(a0, a1), dsb, dq_acc[db]);
            }
        }
    };

    // One step.  Issue order inside a step: the K tile three steps ahead, then the dS tile four steps ahead.
    // At the end of step t the K tile of step t+1 must have landed; younger than it are the dS loads of its own
    // step and everything of the two steps since: kWaitCount operations, which stay in flight.
    bf16x8 set0[4], set1[4], set2[4], set3[4];
    auto step = [&](bf16x8 (&r)[4], int t) {
        char* dss = dsbuf + (t & 1) * S::kDsTileBytes;
#pragma unroll
        for (int n = 0; n < 4; n++) claim_loaded(r[n]);
        // piece (block c = n / 2, half s = n % 2) of this lane -> its transposable place
#pragma unroll
        for (int n = 0; n < 4; n++) *(bf16x8*)(dss + (n >> 1) * 2048 + (n & 1) * 32 + piece_off) = r[n];
        issue_k(t + 3);
        issue_ds(r, t + 4);
        __builtin_amdgcn_sched_barrier(0);
        if (t <= last_tile) compute_tile(kring + (t & (S::kKStages - 1)) * S::kKTileBytes, dss);
        __builtin_amdgcn_sched_barrier(0);
        wait_vmcnt_lds_done<S::kWaitCount>();
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
    };

    // prologue in the loop's own issue order (steps -4 .. -1 without their computation)
    issue_ds(set0, 0);
    issue_k(0); issue_ds(set1, 1);
    issue_k(1); issue_ds(set2, 2);
    issue_k(2); issue_ds(set3, 3);
    wait_vmcnt<S::kWaitCount>();
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll 1
    for (int t = 0; t < n_steps; t += 4) {
        step(set0, t);
        step(set1, t + 1);
        step(set2, t + 2);
        step(set3, t + 3);
    }
    wait_vmcnt<0>();          // the redirected loads of the last steps must not outlive this pass (LDS, registers)
    __builtin_amdgcn_s_barrier();

    if (!TAIL || my_q < Nq) {
        bf16* dQr = dQ + head + (size_t)my_q * D;
#pragma unroll
        for (int db = 0; db < D / 32; db++)
#pragma unroll
            for (int g = 0; g < 4; g++) {
                bf16x2 lo = cvt2(dq_acc[db][4 * g + 0] * scale, dq_acc[db][4 * g + 1] * scale);
                bf16x2 hi = cvt2(dq_acc[db][4 * g + 2] * scale, dq_acc[db][4 * g + 3] * scale);
                *(bf16x4*)(dQr + 32 * db + 8 * g + 4 * h) = __builtin_shufflevector(lo, hi, 0, 1, 2, 3);
            }
    }
    }   // pass
}

template <int D, bool CAUSAL, bool TAIL>
static hipError_t launch_dq_from_ds_tt(const void* k, const void* ds, void* dq,
                                       int B, int H, int Hkv, int Nq, int Nk, float scale, hipStream_t stream)
{
    using S = DqDsShape<D>;
    auto kern = attn_bwd_dq_from_ds_kernel<D, CAUSAL, TAIL>;
    const int num_q_tiles = (Nq + S::kTileQ - 1) / S::kTileQ;
    const int num_kv_tiles = (Nk + 127) / 128;
    const int total = B * H * (CAUSAL ? (num_q_tiles + 1) / 2 : num_q_tiles);
    hipLaunchKernelGGL(kern, dim3(total), dim3(S::kThreads), 0, stream,
                       (const bf16*)k, (const char*)ds, (bf16*)dq, Nq, Nk, num_q_tiles, total, scale, H, Hkv,
                       num_kv_tiles, ds_query_blocks(Nq));
    return hipGetLastError();
}

template <int D>
static hipError_t launch_dq_from_ds_t(const void* k, const void* ds, void* dq,
                                      int B, int H, int Hkv, int Nq, int Nk, int causal, float scale, hipStream_t stream)
{
    const bool tail = Nq != Nk || Nq % 256;
    if (causal) return tail ? launch_dq_from_ds_tt<D, true, true>(k, ds, dq, B, H, Hkv, Nq, Nk, scale, stream)
                            : launch_dq_from_ds_tt<D, true, false>(k, ds, dq, B, H, Hkv, Nq, Nk, scale, stream);
    return tail ? launch_dq_from_ds_tt<D, false, true>(k, ds, dq, B, H, Hkv, Nq, Nk, scale, stream)
                : launch_dq_from_ds_tt<D, false, false>(k, ds, dq, B, H, Hkv, Nq, Nk, scale, stream);
}

hipError_t launch_attn_bwd_dq_from_ds(const void* k, const void* ds, void* dq,
                                      int B, int H, int Hkv, int Nq, int Nk, int D, int causal, float scale, hipStream_t stream)
{
    return D == 128 ? launch_dq_from_ds_t<128>(k, ds, dq, B, H, Hkv, Nq, Nk, causal, scale, stream)
                    : launch_dq_from_ds_t<64>(k, ds, dq, B, H, Hkv, Nq, Nk, causal, scale, stream);
}

}  // namespace tk
