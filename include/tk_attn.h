/*
 * tk_attn.h - C ABI of the MI355X (gfx950) fused exact softmax attention library.
 *
 * The operation is the attention of the PyTorch listing in the paper's
 * introduction (its listing figure: softmax(Q K^T) V, softmax in fp32,
 * probabilities cast to bf16 before the second product) with the 1/sqrt(D)
 * temperature that the Appendix B.3 listing folds into a base-2 exponent, an
 * optional causal mask, and the per-row log-sum-exp as a second output.  The
 * backward pass is its gradient; the paper reports only its speed (the plots
 * of Section 4.1 and the profile table of Section 4.2), so the algorithm is
 * the chain rule with P recomputed from the saved LSE.
 *
 * Conventions common to every entry point
 *   - Every tensor pointer is a DEVICE pointer owned by the caller, to
 *     contiguous row-major memory, 16-byte aligned.  Q, K, V, O, dO, dQ, dK,
 *     dV are bf16 [B, H, N, D]; LSE is fp32 [B, H, N].
 *   - D is 64 or 128.  B, H, N >= 1 (any sequence length: the kernels work on
 *     tiles of 128 rows and mask the tail) and B*H*ceil(N/128) must fit a 31-bit grid.
 *   - scale must be finite and > 0 (the running maximum is taken on raw
 *     scores, which is only the maximum of the scaled scores for scale > 0).
 *   - causal != 0 masks keys j > i (the diagonal is kept).
 *   - stream is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work: no allocation, no free, no host
 *     synchronisation.  The only state the library keeps is the compute-unit
 *     count of each device, queried once (hipGetDevice +
 *     hipDeviceGetAttribute on the first launch of a persistent kernel on
 *     that device) and cached.  Outputs are fully overwritten.
 *   - Inputs and outputs must not alias.
 *   - Return value: TK_OK (0) or a negative TK_ERR_* code.  Arguments are
 *     validated on the host before any HIP call is made, so every error
 *     except TK_ERR_LAUNCH is reported without touching the GPU.
 */
#ifndef TK_ATTN_H
#define TK_ATTN_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    TK_OK = 0,
    TK_ERR_NULL_PTR = -1,            /* a required pointer is NULL */
    TK_ERR_BAD_DIM = -2,             /* D not in {64,128}; B, H or N < 1; Hkv not dividing Hq; grid overflow */
    TK_ERR_MISALIGNED = -3,          /* a tensor pointer is not 16-byte aligned */
    TK_ERR_BAD_SCALE = -4,           /* scale is not finite or not > 0 */
    TK_ERR_WORKSPACE_TOO_SMALL = -5, /* workspace_bytes < tk_attn_bwd_workspace_bytes(...) */
    TK_ERR_LAUNCH = -6,              /* hipGetLastError() reported a failure after a launch */
    TK_ERR_SCRATCH_LIMIT = -7        /* tk_attn_bwd_noalloc: B*H*N exceeds tk_attn_bwd_noalloc_max_rows() */
};

/*
 * Forward pass (the introduction's PyTorch listing; Appendix B.3 listing for the streaming
 * form: running max and sum per query row, base-2 exponent with the folded
 * temperature, rescale of the output accumulator, normalisation at the end).
 *
 *   S_ij  = scale * sum_d Q_id K_jd          (keys j <= i only when causal)
 *   P_ij  = exp(S_ij - LSE_i),  LSE_i = ln sum_j exp(S_ij)
 *   O_id  = sum_j P_ij V_jd
 *
 * q, k, v : in,  bf16 [B,H,N,D]
 * o       : out, bf16 [B,H,N,D]  (fp32 accumulation, one round-to-nearest-even at the end)
 * lse     : out, fp32 [B,H,N]    (natural log, of the SCALED scores)
 */
int tk_attn_fwd(const void* q, const void* k, const void* v,
                void* o, float* lse,
                int B, int H, int N, int D, int causal, float scale,
                void* stream);

/*
 * Backward pass: gradients of L = sum(O * dO) with respect to Q, K, V.
 *
 *   Delta_i = sum_d dO_id O_id
 *   P_ij    = exp(scale * Q_i.K_j - LSE_i)   (recomputed, never stored)
 *   dV_jd   = sum_i P_ij dO_id
 *   dP_ij   = sum_d dO_id V_jd
 *   dS_ij   = P_ij (dP_ij - Delta_i)
 *   dQ_id   = scale * sum_j dS_ij K_jd
 *   dK_jd   = scale * sum_i dS_ij Q_id
 *
 * q, k, v, o, d_o : in, bf16 [B,H,N,D]; o and lse exactly as tk_attn_fwd wrote them
 * lse             : in, fp32 [B,H,N]
 * dq, dk, dv      : out, bf16 [B,H,N,D] (fp32 accumulation)
 * workspace       : device scratch of at least tk_attn_bwd_workspace_bytes(B,H,N,D) bytes,
 *                   16-byte aligned; holds Delta (fp32 [B,H,N]).  It need not be cleared;
 *                   contents after the call are unspecified.  Two calls that overlap in time
 *                   must not share a workspace.
 *                   The call runs in one of two forms, chosen by workspace_bytes alone:
 *                   >= tk_attn_bwd_spill_workspace_bytes(B,H,N,N,D): the dK/dV kernel also stores
 *                      its bf16 dS blocks (2 bytes per query-key pair of the padded problem) in the
 *                      workspace and dQ = scale * dS K is formed from them: 10*D flops per pair;
 *                   smaller: dS is recomputed by a dQ kernel of its own (14*D flops per pair).
 *                   Both are the formulas above with the same roundings of P and dS; they differ
 *                   in summation order only.  The stored dS costs the same bytes at every D, the
 *                   recomputation it replaces shrinks with D: on MI355X the storing form is the
 *                   faster one at D = 128 and the slower one at D = 64.
 * No atomics are used: for a given form dQ, dK and dV are bit-reproducible from run to run.
 */
int tk_attn_bwd(const void* q, const void* k, const void* v,
                const void* o, const void* d_o, const float* lse,
                void* dq, void* dk, void* dv,
                int B, int H, int N, int D, int causal, float scale,
                void* workspace, size_t workspace_bytes,
                void* stream);

/* Bytes of workspace tk_attn_bwd needs for this shape; 0 if the shape is invalid. */
size_t tk_attn_bwd_workspace_bytes(int B, int H, int N, int D);

/*
 * Bytes of workspace from which tk_attn_bwd / _gqa / _rect take the faster form that stores dS:
 * Delta plus one 2 KB block per (query head, 128-key tile, 32-query block, 32 keys), i.e. about
 * 2 * B * Hq * Nq * Nk bytes (8.6 GB for B*Hq = 256, Nq = Nk = 4096).  0 if the shape is invalid.
 */
size_t tk_attn_bwd_spill_workspace_bytes(int B, int Hq, int Nq, int Nk, int D);

/*
 * tk_attn_bwd for callers that cannot allocate device memory and have no workspace to hand over: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same inputs, outputs,
 * kernels and results (bit for bit) as tk_attn_bwd with a minimal workspace, but Delta lives in a scratch
 * array that is part of the library's device image: 4 MiB per GPU the library runs on, held until the
 * process ends.  The call allocates and frees nothing, on the host or on the device; its first use on a
 * device looks the array's address up (hipGetSymbolAddress) and keeps it.
 *   Limit: B*H*N <= tk_attn_bwd_noalloc_max_rows() (1,048,576), else TK_ERR_SCRATCH_LIMIT.
 *   Every call on a GPU shares that GPU's array: calls that overlap in time on one GPU (different
 *   streams, or different threads) race on it and must be serialised by the caller.  Nothing in it
 *   needs clearing between calls (the first kernel writes every Delta the second one reads).
 * Other errors as tk_attn_bwd.
 */
int tk_attn_bwd_noalloc(const void* q, const void* k, const void* v,
                        const void* o, const void* d_o, const float* lse,
                        void* dq, void* dk, void* dv,
                        int B, int H, int N, int D, int causal, float scale,
                        void* stream);

size_t tk_attn_bwd_noalloc_max_rows(void);

/*
 * The backward pass as three separate stages (Delta, dK/dV, dQ), so that each kernel's throughput
 * can be measured on its own.  This three-stage form is an equivalent measuring aid: tk_attn_bwd
 * itself launches tk_attn_bwd_dq_delta (dQ with Delta folded in) followed by tk_attn_bwd_dkdv, see
 * below.  Same pointer, shape and error conventions as above.
 *
 * Stage 1: Delta_i = sum_d dO_id O_id.
 *   o, d_o : in, bf16 [B,H,N,D];  delta : out, fp32 [B,H,N]
 */
int tk_attn_bwd_delta(const void* o, const void* d_o, float* delta,
                      int B, int H, int N, int D, void* stream);

/*
 * Stage 2: dK and dV (bf16 out), computed per tile of 128 keys by persistent workgroups.
 *   lse, delta : in, fp32 [B,H,N]
 */
int tk_attn_bwd_dkdv(const void* q, const void* k, const void* v, const void* d_o,
                     const float* lse, const float* delta,
                     void* dk, void* dv,
                     int B, int H, int N, int D, int causal, float scale, void* stream);

/*
 * Stage 3: dQ (bf16 out), one workgroup per tile of 128 queries; independent of stage 2.
 *   lse, delta : in, fp32 [B,H,N]
 */
int tk_attn_bwd_dq(const void* q, const void* k, const void* v, const void* d_o,
                   const float* lse, const float* delta,
                   void* dq,
                   int B, int H, int N, int D, int causal, float scale, void* stream);

/*
 * Grouped-query attention (Section 4.1 lists it among the supported variants; no formula is
 * printed, so the usual definition is taken): Hq query heads share Hkv key/value heads, Hkv
 * dividing Hq, and query head h of a batch entry attends with key/value head h / (Hq / Hkv),
 * i.e. consecutive query heads form a group.  Everything else is as in the calls above, which
 * are the Hkv == Hq case of these.
 *
 *   q, o, d_o, dq : bf16 [B, Hq, N, D]        k, v, dk, dv : bf16 [B, Hkv, N, D]
 *   lse, delta    : fp32 [B, Hq, N]
 *   dk, dv are summed over the query heads of each group (in fp32, inside one workgroup: no atomics).
 *   workspace for tk_attn_bwd_gqa: tk_attn_bwd_workspace_bytes(B, Hq, N, D) bytes.
 * TK_ERR_BAD_DIM also covers Hkv < 1, Hkv > Hq and Hq % Hkv != 0.
 */
int tk_attn_fwd_gqa(const void* q, const void* k, const void* v,
                    void* o, float* lse,
                    int B, int Hq, int Hkv, int N, int D, int causal, float scale,
                    void* stream);

int tk_attn_bwd_gqa(const void* q, const void* k, const void* v,
                    const void* o, const void* d_o, const float* lse,
                    void* dq, void* dk, void* dv,
                    int B, int Hq, int Hkv, int N, int D, int causal, float scale,
                    void* workspace, size_t workspace_bytes,
                    void* stream);

/*
 * The two stages tk_attn_bwd / _gqa / _rect actually run: the dQ kernel with Delta folded in, then the
 * dK/dV kernel.  A lane of the dQ kernel holds its query's dO row already, so it reads the matching O
 * row, forms Delta_i = sum_d dO_id O_id, uses it and writes it out; the separate pass over O and dO
 * (tk_attn_bwd_delta) is then not needed.  Hkv == Hq: plain multi-head.
 *   o     : in,  bf16 [B, Hq, N, D] (the forward's output)
 *   delta : out, fp32 [B, Hq, N]    (input of tk_attn_bwd_dkdv / _dkdv_gqa afterwards)
 *   dq    : out, bf16 [B, Hq, N, D]
 */
int tk_attn_bwd_dq_delta(const void* q, const void* k, const void* v, const void* o, const void* d_o,
                         const float* lse, float* delta, void* dq,
                         int B, int Hq, int Hkv, int N, int D, int causal, float scale, void* stream);

/*
 * The stages of the form of tk_attn_bwd that stores dS, after tk_attn_bwd_delta: dK/dV with the dS blocks
 * written to ds (tk_attn_bwd_ds_bytes(B, Hq, N, N, D) bytes, 16-byte aligned, need not be cleared), then
 * dQ = scale * dS K from those blocks (k: the same keys; the same B, Hq, Hkv, N, D, causal as the call
 * that wrote ds).  The block layout is private to the two kernels.
 */
size_t tk_attn_bwd_ds_bytes(int B, int Hq, int Nq, int Nk, int D);

int tk_attn_bwd_dkdv_ds(const void* q, const void* k, const void* v, const void* d_o,
                        const float* lse, const float* delta,
                        void* dk, void* dv, void* ds,
                        int B, int Hq, int Hkv, int N, int D, int causal, float scale, void* stream);

int tk_attn_bwd_dq_from_ds(const void* k, const void* ds, void* dq,
                           int B, int Hq, int Hkv, int N, int D, int causal, float scale, void* stream);

/* Stages 2 and 3 of the three-stage form (stage 1 is tk_attn_bwd_delta with H = Hq). */
int tk_attn_bwd_dkdv_gqa(const void* q, const void* k, const void* v, const void* d_o,
                         const float* lse, const float* delta,
                         void* dk, void* dv,
                         int B, int Hq, int Hkv, int N, int D, int causal, float scale, void* stream);

int tk_attn_bwd_dq_gqa(const void* q, const void* k, const void* v, const void* d_o,
                       const float* lse, const float* delta,
                       void* dq,
                       int B, int Hq, int Hkv, int N, int D, int causal, float scale, void* stream);

/*
 * Different numbers of queries and keys (cross attention, decoding against a longer key/value
 * history).  The paper's listings take one sequence length, and its Appendix B.3 kernel guards
 * only the query tail; the reading taken here: q has Nq rows per head, k and v have Nk rows, and
 * with the causal mask the two sequences are aligned at their ENDS: query i attends to keys
 * j <= i + (Nk - Nq), so the last query sees every key and Nq == Nk gives the calls above.
 *
 *   q, o, d_o, dq : bf16 [B, Hq, Nq, D]       k, v, dk, dv : bf16 [B, Hkv, Nk, D]
 *   lse           : fp32 [B, Hq, Nq]
 *   Nq, Nk >= 1, any values; heads grouped as in the _gqa calls (Hkv == Hq: plain multi-head).
 *   workspace for tk_attn_bwd_rect: tk_attn_bwd_workspace_bytes(B, Hq, Nq, D) bytes.
 * TK_ERR_BAD_DIM also covers causal != 0 with Nq > Nk (the first queries would see no key).
 * Everything else (pointers, alignment, scale, stream, errors) as in the calls above.
 */
int tk_attn_fwd_rect(const void* q, const void* k, const void* v,
                     void* o, float* lse,
                     int B, int Hq, int Hkv, int Nq, int Nk, int D, int causal, float scale,
                     void* stream);

int tk_attn_bwd_rect(const void* q, const void* k, const void* v,
                     const void* o, const void* d_o, const float* lse,
                     void* dq, void* dk, void* dv,
                     int B, int Hq, int Hkv, int Nq, int Nk, int D, int causal, float scale,
                     void* workspace, size_t workspace_bytes,
                     void* stream);

/*
 * Decode-shaped forward: ONE query per head against Nk keys (the Nq = 1 case of tk_attn_fwd_rect,
 * where the causal mask removes nothing), organised for the memory system rather than the matrix
 * pipe: the query heads that share a key/value head are processed together, so K and V are read
 * once per group, and the keys are split over enough workgroups to fill the chip, with a merge of
 * the partial (O, LSE) pairs behind it.  Results equal tk_attn_fwd_rect's up to fp32 rounding
 * order of the merge.
 *
 *   q, o : bf16 [B, Hq, 1, D]      k, v : bf16 [B, Hkv, Nk, D]      lse : fp32 [B, Hq, 1]
 *   workspace : device scratch of at least tk_attn_decode_workspace_bytes(B, Hq, Hkv, Nk, D)
 *               bytes, 16-byte aligned; contents on entry are ignored (partial results live there).
 * tk_attn_decode_workspace_bytes returns 0 for shapes the call would reject.
 * Errors as in the calls above, plus TK_ERR_WORKSPACE_TOO_SMALL.
 */
size_t tk_attn_decode_workspace_bytes(int B, int Hq, int Hkv, int Nk, int D);

int tk_attn_decode(const void* q, const void* k, const void* v,
                   void* o, float* lse,
                   int B, int Hq, int Hkv, int Nk, int D, float scale,
                   void* workspace, size_t workspace_bytes,
                   void* stream);

/*
 * How tk_attn_decode would lay a call out on a device with `compute_units` compute units (host
 * arithmetic only; for callers that want to know, and for tests):
 *   plan[0] heads as the kernel sees them (B*Hkv when a group's query heads are packed, else B*Hq)
 *   plan[1] query rows per such head (Hq/Hkv when packed, else 1)
 *   plan[2] splits over the keys        plan[3] 64-key tiles per split (even)
 *   plan[4] most splits any device could give this shape (what the workspace is sized for)
 * plan: host pointer to 5 ints.  Errors: TK_ERR_NULL_PTR, TK_ERR_BAD_DIM.
 */
int tk_attn_decode_plan(int B, int Hq, int Hkv, int Nk, int D, int compute_units, int* plan);

/*
 * bf16 matrix multiply (the GEMM of the paper's appendix, second workload): C = A B with fp32
 * accumulation and one rounding to bf16.
 *
 *   a : in,  bf16 [M, K] row-major        b : in, bf16 [K, N] row-major        c : out, bf16 [M, N] row-major
 * M >= 1; N and K positive multiples of 8, so that every row starts on a 16-byte boundary
 * (TK_ERR_BAD_DIM otherwise).  The kernel works on 256 x 256 x 64 tiles; shapes that are not multiples
 * of those run a variant that masks the edge tiles (rows and columns past the end are not stored, the
 * part of the last K step past K contributes zeros).
 * No workspace; the result is bit-reproducible (every element is one fixed-order accumulation).
 */
int tk_gemm(const void* a, const void* b, void* c, int M, int N, int K, void* stream);

/*
 * Rotary positional encoding (the rotary kernel of the paper's appendix; applied to Q and K ahead
 * of attention).  With x1 = x[..., :D/2] and x2 = x[..., D/2:]:
 *
 *   o[..., :D/2] = x1 * cos - x2 * sin          o[..., D/2:] = x2 * cos + x1 * sin
 *
 *   x              : in,  bf16 [B,H,N,D]
 *   sin_table,
 *   cos_table      : in,  bf16 [N, D/2] (one angle per position and column pair, shared by all heads)
 *   o              : out, bf16 [B,H,N,D]; may be the same buffer as x (in place), no other overlap
 * fp32 arithmetic, one rounding to bf16.  D is 64 or 128, any N >= 1.
 */
int tk_rotary(const void* x, const void* sin_table, const void* cos_table, void* o,
              int B, int H, int N, int D, void* stream);

/*
 * Measurement aid, not part of the attention path: a bare stream of the bf16 MFMA that the
 * attention kernels use, on caller-supplied operand values.  The benchmark times it to report the
 * matrix-pipe rate the chip sustains with the same kind of data (the clock it holds depends on
 * the operand values), next to the published peak.
 *
 *   operands   : in, device, 16 fragments x 256 lanes x 16 bytes = 65536 bytes of bf16
 *   sink       : out, device, workgroups * 256 floats (sums of the accumulators; keeps the work alive)
 *   workgroups : 1..65536 workgroups of 256 threads (one wave per SIMD); the compute-unit count fills the chip once
 *   iters      : >= 1; every wave issues 32 * iters MFMAs of 32*32*16*2 flops
 */
int tk_mfma_probe(const void* operands, float* sink, int workgroups, int iters, void* stream);

/* Human-readable name of a status code (static storage; never NULL). */
const char* tk_status_string(int status);

/* Library version as major*10000 + minor*100 + patch. */
int tk_attn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TK_ATTN_H */
