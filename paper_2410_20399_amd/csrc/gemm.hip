// bf16 matrix multiply C = A B (fp32 accumulation) for gfx950 (MI355X): the GEMM of the paper's
// appendix as a second workload, and the reference point for what a kernel made of MFMAs and LDS
// traffic alone sustains on this chip.
//
// One workgroup = 4 waves (one per SIMD) = a 256 x 256 tile of C; wave (wm, wn) owns the 128 x 128
// quadrant and keeps its 16 accumulator blocks (256 registers) for the whole K loop.  A and B are
// streamed in steps of 64 along K through a two-stage LDS ring filled by direct global->LDS loads:
//
//   A stage  256 rows x 64 k    (128-byte rows, chunk-swizzled for 16-row same-chunk b128 reads)
//   B stage  64 k x 256 columns, kept as two 128-column halves (256-byte rows, chunk-swizzled for
//            the transposing reads that turn k-major rows into "8 consecutive k per lane")
//
// The products are issued as D^T: v_mfma(B fragment, A fragment), so that a lane owns one ROW of C
// and stores 4 consecutive columns at a time.  Fragments of k-sub-step t+1 are read from LDS while
// the 16 MFMAs of sub-step t run; the barrier that frees a stage sits before the last sub-step of
// a step, whose MFMAs cover the first fragment reads of the next stage.
#include "tk_common.h"
#include "tk_launch.h"

namespace tk {

struct GemmShape {
    static constexpr int kThreads = 256;
    static constexpr int kTileM = 256, kTileN = 256, kTileK = 64;
    static constexpr int kARowBytes = kTileK * 2;                 // 128
    static constexpr int kBRowBytes = 128 * 2;                    // one 128-column half
    static constexpr int kABytes = kTileM * kARowBytes;           // 32 KB
    static constexpr int kBHalfBytes = kTileK * kBRowBytes;       // 16 KB
    static constexpr int kStageBytes = kABytes + 2 * kBHalfBytes; // 64 KB
    static constexpr int kALoads = kABytes / (kThreads * 16);     // 8 per thread
    static constexpr int kBLoads = kBHalfBytes / (kThreads * 16); // 4 per thread and half
    static constexpr int kLoadsPerStage = kALoads + 2 * kBLoads;  // 16
    static constexpr int kSuperM = 8;                             // tile rows walked together (L2 reuse of the B panels)
};

// sixteen zero bytes: the source of the A chunks that lie beyond K in an edge tile
__device__ __attribute__((aligned(16))) const bf16 g_gemm_zero[8] = {};

__device__ __forceinline__ int gemm_swz_a(int row) { return (row >> 1) & 7; }
__device__ __forceinline__ int gemm_swz_b(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }

// EDGE: the general case (M not a multiple of 256, N not of 256, or K not of 64; N and K multiples of 8
// so that every row starts on a 16-byte boundary).  The kernel still works on whole 256 x 256 x 64 tiles:
// rows of A past M fetch row M-1 and columns of B past N fetch the last 8 columns (their results are never
// stored), the chunks of A and the rows of B past K are fetched from a block of zeros so that they add
// nothing, and rows / columns past the end are not stored.  The aligned case compiles without any of this.
template <bool EDGE>
__global__ __launch_bounds__(256, 1)
void gemm_kernel(const bf16* __restrict__ A, const bf16* __restrict__ B, bf16* __restrict__ C,
                 int M, int N, int K, int tiles_m, int tiles_n)
{
    using S = GemmShape;
    __shared__ __attribute__((aligned(1024))) char ring[2 * S::kStageBytes];

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int l32 = lane & 31;
    const int h = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;

    // tile order: XCD-contiguous ids, then groups of kSuperM tile rows walked column by column, so
    // the workgroups resident on one XCD share a few A and B panels in its L2 (Section 3.3 of the
    // paper makes the same point about block order for its GEMM)
    const int total = tiles_m * tiles_n;
    const int logical = xcd_remap(blockIdx.x, total);
    const int super_rows = (tiles_m / S::kSuperM) * S::kSuperM;
    int tm, tn;
    if (logical < super_rows * tiles_n) {
        const int grp = logical / (S::kSuperM * tiles_n), in = logical % (S::kSuperM * tiles_n);
        tm = grp * S::kSuperM + in % S::kSuperM;
        tn = in / S::kSuperM;
    } else {
        const int rest = tiles_m - super_rows, in = logical - super_rows * tiles_n;
        tm = super_rows + in % rest;
        tn = in / rest;
    }
    const size_t m0 = (size_t)tm * S::kTileM, n0 = (size_t)tn * S::kTileN;

    // ---- per-thread source offsets (elements) of the direct-to-LDS loads of one stage
    // A: LDS position s = it*256 + tid holds (row = s / 8, physical chunk = s % 8)
    // B half t: position s holds (k row = s / 16, physical chunk = s % 16)
    size_t a_src[S::kALoads], b_src[S::kBLoads];
#pragma unroll
    for (int it = 0; it < S::kALoads; it++) {
        const int s = it * S::kThreads + tid, row = s >> 3, pc = s & 7;
        a_src[it] = (m0 + row) * K + ((pc ^ gemm_swz_a(row)) << 3);
    }
#pragma unroll
    for (int it = 0; it < S::kBLoads; it++) {
        const int s = it * S::kThreads + tid, row = s >> 4, pc = s & 15;
        b_src[it] = (size_t)row * N + n0 + ((pc ^ gemm_swz_b(row)) << 3);
    }
    auto issue_stage = [&](int step) {
        char* base = ring + (step & 1) * S::kStageBytes + wave * 1024;
        if (!EDGE) {
            const bf16* a = A + (size_t)step * S::kTileK;
            const bf16* b = B + (size_t)step * S::kTileK * N;
#pragma unroll
            for (int it = 0; it < S::kALoads; it++)
                load_global_to_lds16_untracked(a + a_src[it], base + it * (S::kThreads * 16));
#pragma unroll
            for (int t = 0; t < 2; t++)
#pragma unroll
                for (int it = 0; it < S::kBLoads; it++)
                    load_global_to_lds16_untracked(b + b_src[it] + 128 * t,
                                                   base + S::kABytes + t * S::kBHalfBytes + it * (S::kThreads * 16));
        } else {
            const int k0 = step * S::kTileK;
#pragma unroll
            for (int it = 0; it < S::kALoads; it++) {
                const int s = it * S::kThreads + tid, row = s >> 3, pc = s & 7;
                size_t r = m0 + row;
                if (r > (size_t)M - 1) r = (size_t)M - 1;
                const int k = k0 + ((pc ^ gemm_swz_a(row)) << 3);
                const bf16* src = k < K ? A + r * K + k : g_gemm_zero;
                load_global_to_lds16_untracked(src, base + it * (S::kThreads * 16));
            }
#pragma unroll
            for (int t = 0; t < 2; t++)
#pragma unroll
                for (int it = 0; it < S::kBLoads; it++) {
                    const int s = it * S::kThreads + tid, row = s >> 4, pc = s & 15;
                    const int k = k0 + row;
                    size_t col = n0 + 128 * t + ((pc ^ gemm_swz_b(row)) << 3);
                    if (col > (size_t)N - 8) col = (size_t)N - 8;
                    const bf16* src = k < K ? B + (size_t)k * N + col : g_gemm_zero;
                    load_global_to_lds16_untracked(src, base + S::kABytes + t * S::kBHalfBytes + it * (S::kThreads * 16));
                }
        }
    };

    // ---- per-lane LDS read offsets
    // A fragment (second MFMA operand: lane <-> row of A, 8 consecutive k): row 32a + l32 of the wave's
    // 128 rows, logical chunk 2*kb + h
    const int a_lane = (wm * 128 + l32) * S::kARowBytes + ((h ^ gemm_swz_a(l32)) << 4);
    // B fragment (first MFMA operand: lane <-> column of B, 8 consecutive k) through transposing
    // reads: 16-lane group G = lane/16 -> (column half = G%2, k half = G/2 = h); lane j of the group
    // addresses k row 8h + j/4 (second read: +4), columns 32b + 16*(G%2) + 4*(j%4)
    const int j16 = lane & 15;
    const int b_row = 8 * h + (j16 >> 2);
    const int b_lane = b_row * S::kBRowBytes + (((2 * ((lane >> 4) & 1) + ((j16 & 3) >> 1)) ^ gemm_swz_b(b_row)) << 4) + ((j16 & 1) << 3);

    f32x16 acc[4][4];      // [column block b][row block a]
#pragma unroll
    for (int b = 0; b < 4; b++)
#pragma unroll
        for (int a = 0; a < 4; a++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[b][a][r] = 0.f;

    bf16x8 af[2][4], bfr[2][4];     // two sets of fragments: one being multiplied, one being read
    auto read_frags = [&](int set, int step, int kb) {
        const char* as = ring + (step & 1) * S::kStageBytes;
        const char* bs = as + S::kABytes + wn * S::kBHalfBytes;
#pragma unroll
        for (int a = 0; a < 4; a++)
            af[set][a] = lds_read_b128(as, (a_lane ^ ((2 * kb) << 4)) + a * 32 * S::kARowBytes);
#pragma unroll
        for (int b = 0; b < 4; b++) {
            // k rows 16kb + 8h + (0..3) and +4: the +4 flips bit 0 of the swizzle's low field
            const int row_off = 16 * kb * S::kBRowBytes;
            const int x0 = (4 * b) << 4, x1 = ((4 * b) ^ 1) << 4;
            bfr[set][b] = concat(lds_read_tr16(bs, (b_lane ^ x0) + row_off),
                                 lds_read_tr16(bs, (b_lane ^ x1) + row_off + 4 * S::kBRowBytes));
        }
    };
    auto multiply = [&](int set) {
#pragma unroll
        for (int b = 0; b < 4; b++)
#pragma unroll
            for (int a = 0; a < 4; a++) acc[b][a] = mfma32(bfr[set][b], af[set][a], acc[b][a]);
    };

    // schedule of one sub-step: the 12 fragment reads go out one per MFMA, ahead of the remaining MFMAs
    auto interleave = [&]() {
#pragma unroll
        for (int i = 0; i < 12; i++) {
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // DS read
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // MFMA
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
        __builtin_amdgcn_sched_barrier(0);
    };

    const int n_steps = (K + S::kTileK - 1) / S::kTileK;
    issue_stage(0);
    if (n_steps > 1) issue_stage(1);
    if (n_steps > 1) wait_vmcnt<S::kLoadsPerStage>(); else wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    read_frags(0, 0, 0);

#pragma unroll 1
    for (int s = 0; s < n_steps; s++) {
        // sub-steps 0..2: multiply one set while the next sub-step's fragments are read into the other
        read_frags(1, s, 1);
        multiply(0);
        interleave();
        read_frags(0, s, 2);
        multiply(1);
        interleave();
        read_frags(1, s, 3);
        multiply(0);
        interleave();
        // Once every wave's last fragment reads of this stage have completed the stage can be refilled;
        // the next stage (issued one step ago) must have landed before its first fragments are read.
        __builtin_amdgcn_s_waitcnt(0x0070);      // vmcnt(0) and lgkmcnt(0)
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        if (s + 2 < n_steps) issue_stage(s + 2);
        __builtin_amdgcn_sched_barrier(0);
        if (s + 1 < n_steps) read_frags(0, s + 1, 0);
        multiply(1);
        interleave();
    }

    // ---- epilogue: lane <-> row of C; register r of block (b, a) <-> column 32b + 8*(r/4) + 4h + r%4
#pragma unroll
    for (int a = 0; a < 4; a++) {
        const size_t row = m0 + wm * 128 + 32 * a + l32;
        if (EDGE && row >= (size_t)M) continue;
        bf16* crow = C + row * N + n0 + wn * 128;
#pragma unroll
        for (int b = 0; b < 4; b++)
#pragma unroll
            for (int g = 0; g < 4; g++) {
                const int col = 32 * b + 8 * g + 4 * h;      // within the wave's 128 columns; N is a multiple of 8
                if (EDGE && n0 + wn * 128 + col >= (size_t)N) continue;
                bf16x2 lo = cvt2(acc[b][a][4 * g + 0], acc[b][a][4 * g + 1]);
                bf16x2 hi = cvt2(acc[b][a][4 * g + 2], acc[b][a][4 * g + 3]);
                *(bf16x4*)(crow + col) = __builtin_shufflevector(lo, hi, 0, 1, 2, 3);
            }
    }
}

hipError_t launch_gemm(const void* a, const void* b, void* c, int M, int N, int K, hipStream_t stream)
{
    using S = GemmShape;
    const int tiles_m = (M + S::kTileM - 1) / S::kTileM, tiles_n = (N + S::kTileN - 1) / S::kTileN;
    const bool edge = M % S::kTileM || N % S::kTileN || K % S::kTileK;
    if (edge)
        hipLaunchKernelGGL(gemm_kernel<true>, dim3(tiles_m * tiles_n), dim3(S::kThreads), 0, stream,
                           (const bf16*)a, (const bf16*)b, (bf16*)c, M, N, K, tiles_m, tiles_n);
    else
        hipLaunchKernelGGL(gemm_kernel<false>, dim3(tiles_m * tiles_n), dim3(S::kThreads), 0, stream,
                           (const bf16*)a, (const bf16*)b, (bf16*)c, M, N, K, tiles_m, tiles_n);
    return hipGetLastError();
}

}  // namespace tk
