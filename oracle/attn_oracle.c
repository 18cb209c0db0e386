/*
 * fp64 CPU oracle for exact softmax attention, forward and backward.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the checker the HIP kernels are
 * compared against; nothing in the product path may call it.  It shares no
 * code, header, table or constant with the HIP library.
 *
 * What it computes is the plain definition, one query row (or one key row)
 * at a time, with no tiling, no online softmax and no reordering:
 *
 *   forward  (the PyTorch attention listing in the introduction's listing figure, with
 *             the 1/sqrt(D) temperature that the Appendix B.3 listing
 *             folds into its exponent, and an optional causal mask):
 *     S_ij   = scale * sum_d Q_id K_jd            (j <= i only, if causal)
 *     m_i    = max_j S_ij
 *     l_i    = sum_j exp(S_ij - m_i)
 *     P_ij   = exp(S_ij - m_i) / l_i
 *     O_id   = sum_j P_ij V_jd
 *     LSE_i  = m_i + ln l_i                       (natural log of sum_j exp S_ij)
 *
 *   backward (the paper prints no backward algorithm; this is the chain
 *             rule applied to the forward definition for L = sum O*dO):
 *     Delta_i = sum_d dO_id O_id
 *     dP_ij   = sum_d dO_id V_jd
 *     dS_ij   = P_ij (dP_ij - Delta_i)
 *     dQ_id   = scale * sum_j dS_ij K_jd
 *     dK_jd   = scale * sum_i dS_ij Q_id
 *     dV_jd   = sum_i P_ij dO_id
 *
 * All inputs and outputs are double, row-major [BH][N][D] (LSE: [BH][N]).
 * bf16 test inputs are widened exactly to double by the caller.
 *
 * Pins (tests/test_oracle_pins.py): brute-force exp(S)/sum exp(S) on tiny
 * shapes, rows of P summing to one, LSE against a naive log-sum-exp, closed
 * forms (Q = 0, N = 1, causal row 0, shift and permutation invariances),
 * central finite differences of L for dQ, dK, dV, sum_j dS_ij = 0.
 * The grouped-query functions at the end of the file are pinned to the
 * per-head ones (keys/values repeated per group, gradients summed over the
 * group), to a brute-force numpy softmax and to finite differences.
 * The functions for different query and key lengths (tests/test_oracle_rect_pins.py) are
 * pinned to a library softmax, to the last rows of the square causal problem they are cut
 * from, to closed forms for equal keys and one query, and to finite differences.
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC attn_oracle.c -o liboracle_attn.so -lm
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* number of keys query row i may attend to */
static long visible(long i, long N, int causal) { return causal ? i + 1 : N; }

/*
 * One query row of one head: scores, probabilities, output row, LSE.
 * s is caller scratch of length N; on return s[j] = P_ij for j < visible, 0 after.
 */
static void forward_row(const double* q_i, const double* k, const double* v,
                        long i, long N, long D, int causal, double scale,
                        double* s, double* o_i, double* lse_i)
{
    long nj = visible(i, N, causal);
    double m = -INFINITY;
    for (long j = 0; j < nj; j++) {
        double dot = 0.0;
        for (long d = 0; d < D; d++) dot += q_i[d] * k[j * D + d];
        s[j] = scale * dot;
        if (s[j] > m) m = s[j];
    }
    double l = 0.0;
    for (long j = 0; j < nj; j++) { s[j] = exp(s[j] - m); l += s[j]; }
    for (long j = 0; j < nj; j++) s[j] /= l;
    for (long j = nj; j < N; j++) s[j] = 0.0;
    for (long d = 0; d < D; d++) o_i[d] = 0.0;
    for (long j = 0; j < nj; j++)
        for (long d = 0; d < D; d++) o_i[d] += s[j] * v[j * D + d];
    *lse_i = m + log(l);
}

/* Forward for BH independent heads. p may be NULL; else receives P as [BH][N][N]. */
int oracle_attn_fwd(const double* q, const double* k, const double* v,
                    double* o, double* lse, double* p,
                    long BH, long N, long D, int causal, double scale)
{
    if (!q || !k || !v || !o || !lse || BH <= 0 || N <= 0 || D <= 0) return -1;
    int fail = 0;
#pragma omp parallel
    {
        double* s = (double*)malloc((size_t)N * sizeof(double));
        if (!s) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for collapse(2) schedule(dynamic, 16)
            for (long bh = 0; bh < BH; bh++)
                for (long i = 0; i < N; i++) {
                    const double* qh = q + bh * N * D;
                    const double* kh = k + bh * N * D;
                    const double* vh = v + bh * N * D;
                    forward_row(qh + i * D, kh, vh, i, N, D, causal, scale, s,
                                o + (bh * N + i) * D, lse + bh * N + i);
                    if (p) memcpy(p + (bh * N + i) * N, s, (size_t)N * sizeof(double));
                }
            free(s);
        }
    }
    return fail ? -2 : 0;
}

/*
 * Forward for selected query rows of ONE head: rows[r] in [0,N).
 * o: [nrows][D], lse: [nrows].  Lets a test check sampled rows of a large problem.
 */
int oracle_attn_fwd_rows(const double* q, const double* k, const double* v,
                         const long* rows, long nrows, double* o, double* lse,
                         long N, long D, int causal, double scale)
{
    if (!q || !k || !v || !rows || !o || !lse || nrows < 0 || N <= 0 || D <= 0) return -1;
    for (long r = 0; r < nrows; r++) if (rows[r] < 0 || rows[r] >= N) return -1;
    int fail = 0;
#pragma omp parallel
    {
        double* s = (double*)malloc((size_t)N * sizeof(double));
        if (!s) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for schedule(dynamic, 1)
            for (long r = 0; r < nrows; r++) {
                long i = rows[r];
                forward_row(q + i * D, k, v, i, N, D, causal, scale, s, o + r * D, lse + r);
            }
            free(s);
        }
    }
    return fail ? -2 : 0;
}

/*
 * Backward for BH independent heads.  Two plain sweeps per head:
 *   sweep over query rows i  -> Delta_i, LSE_i (kept), dQ_i
 *   sweep over key rows j    -> dK_j, dV_j, using P_ij = exp(S_ij - LSE_i)
 * delta_out, lse_out may be NULL; else [BH][N].
 */
int oracle_attn_bwd(const double* q, const double* k, const double* v, const double* d_o,
                    double* dq, double* dk, double* dv, double* delta_out, double* lse_out,
                    long BH, long N, long D, int causal, double scale)
{
    if (!q || !k || !v || !d_o || !dq || !dk || !dv || BH <= 0 || N <= 0 || D <= 0) return -1;
    double* delta = (double*)malloc((size_t)BH * N * sizeof(double));
    double* lse = (double*)malloc((size_t)BH * N * sizeof(double));
    if (!delta || !lse) { free(delta); free(lse); return -2; }
    int fail = 0;

    /* sweep 1: per query row */
#pragma omp parallel
    {
        double* s = (double*)malloc((size_t)N * sizeof(double));
        double* o_i = (double*)malloc((size_t)D * sizeof(double));
        if (!s || !o_i) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for collapse(2) schedule(dynamic, 16)
            for (long bh = 0; bh < BH; bh++)
                for (long i = 0; i < N; i++) {
                    const double* kh = k + bh * N * D;
                    const double* vh = v + bh * N * D;
                    const double* q_i = q + (bh * N + i) * D;
                    const double* do_i = d_o + (bh * N + i) * D;
                    double lse_i;
                    forward_row(q_i, kh, vh, i, N, D, causal, scale, s, o_i, &lse_i); /* s = P_i: */
                    double dl = 0.0;
                    for (long d = 0; d < D; d++) dl += do_i[d] * o_i[d];
                    delta[bh * N + i] = dl;
                    lse[bh * N + i] = lse_i;
                    double* dq_i = dq + (bh * N + i) * D;
                    for (long d = 0; d < D; d++) dq_i[d] = 0.0;
                    long nj = visible(i, N, causal);
                    for (long j = 0; j < nj; j++) {
                        double dp = 0.0;
                        for (long d = 0; d < D; d++) dp += do_i[d] * vh[j * D + d];
                        double ds = s[j] * (dp - dl);
                        for (long d = 0; d < D; d++) dq_i[d] += ds * kh[j * D + d];
                    }
                    for (long d = 0; d < D; d++) dq_i[d] *= scale;
                }
        }
        free(s); free(o_i);
    }

    /* sweep 2: per key row */
    if (!fail) {
#pragma omp parallel for collapse(2) schedule(dynamic, 16)
        for (long bh = 0; bh < BH; bh++)
            for (long j = 0; j < N; j++) {
                const double* qh = q + bh * N * D;
                const double* doh = d_o + bh * N * D;
                const double* k_j = k + (bh * N + j) * D;
                const double* v_j = v + (bh * N + j) * D;
                double* dk_j = dk + (bh * N + j) * D;
                double* dv_j = dv + (bh * N + j) * D;
                for (long d = 0; d < D; d++) { dk_j[d] = 0.0; dv_j[d] = 0.0; }
                long i0 = causal ? j : 0;   /* query rows that see key j */
                for (long i = i0; i < N; i++) {
                    double dot = 0.0, dp = 0.0;
                    for (long d = 0; d < D; d++) {
                        dot += qh[i * D + d] * k_j[d];
                        dp += doh[i * D + d] * v_j[d];
                    }
                    double p = exp(scale * dot - lse[bh * N + i]);
                    double ds = p * (dp - delta[bh * N + i]);
                    for (long d = 0; d < D; d++) {
                        dv_j[d] += p * doh[i * D + d];
                        dk_j[d] += ds * qh[i * D + d];
                    }
                }
                for (long d = 0; d < D; d++) dk_j[d] *= scale;
            }
    }
    if (delta_out) memcpy(delta_out, delta, (size_t)BH * N * sizeof(double));
    if (lse_out) memcpy(lse_out, lse, (size_t)BH * N * sizeof(double));
    free(delta); free(lse);
    return fail ? -2 : 0;
}

/* dS for BH heads as [BH][N][N] (tiny shapes only; used by invariant tests). */
int oracle_attn_ds(const double* q, const double* k, const double* v, const double* d_o,
                   double* ds, long BH, long N, long D, int causal, double scale)
{
    if (!q || !k || !v || !d_o || !ds || BH <= 0 || N <= 0 || D <= 0) return -1;
    double* s = (double*)malloc((size_t)N * sizeof(double));
    double* o_i = (double*)malloc((size_t)D * sizeof(double));
    if (!s || !o_i) { free(s); free(o_i); return -2; }
    for (long bh = 0; bh < BH; bh++)
        for (long i = 0; i < N; i++) {
            const double* vh = v + bh * N * D;
            const double* do_i = d_o + (bh * N + i) * D;
            double lse_i;
            forward_row(q + (bh * N + i) * D, k + bh * N * D, vh, i, N, D, causal, scale, s, o_i, &lse_i);
            double dl = 0.0;
            for (long d = 0; d < D; d++) dl += do_i[d] * o_i[d];
            for (long j = 0; j < N; j++) {
                double dp = 0.0;
                for (long d = 0; d < D; d++) dp += do_i[d] * vh[j * D + d];
                ds[(bh * N + i) * N + j] = s[j] * (dp - dl);
            }
        }
    free(s); free(o_i);
    return 0;
}

/*
 * Grouped-query attention (Section 4.1 names it as a supported variant and cites Ainslie et
 * al. 2023; no formula is printed).  Reading taken: Hq query heads, Hkv key/value heads,
 * G = Hq / Hkv; query head h attends with key/value head h / G (consecutive query heads form
 * a group), every head otherwise exactly as in the definition above.  The gradient of a shared
 * key/value head is the sum over its group's query heads.
 *   q, d_o, o, dq : [B][Hq][N][D]     k, v, dk, dv : [B][Hkv][N][D]     lse : [B][Hq][N]
 */
int oracle_gqa_fwd(const double* q, const double* k, const double* v, double* o, double* lse,
                   long B, long Hq, long Hkv, long N, long D, int causal, double scale)
{
    if (!q || !k || !v || !o || !lse || B <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv || N <= 0 || D <= 0) return -1;
    const long G = Hq / Hkv;
    int fail = 0;
#pragma omp parallel
    {
        double* s = (double*)malloc((size_t)N * sizeof(double));
        if (!s) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for collapse(2) schedule(dynamic, 16)
            for (long bh = 0; bh < B * Hq; bh++)
                for (long i = 0; i < N; i++) {
                    const long b = bh / Hq, h = bh % Hq;
                    const long kvh = b * Hkv + h / G;
                    forward_row(q + (bh * N + i) * D, k + kvh * N * D, v + kvh * N * D, i, N, D, causal, scale, s,
                                o + (bh * N + i) * D, lse + bh * N + i);
                }
            free(s);
        }
    }
    return fail ? -2 : 0;
}

int oracle_gqa_bwd(const double* q, const double* k, const double* v, const double* d_o,
                   double* dq, double* dk, double* dv,
                   long B, long Hq, long Hkv, long N, long D, int causal, double scale)
{
    if (!q || !k || !v || !d_o || !dq || !dk || !dv || B <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv || N <= 0 || D <= 0) return -1;
    const long G = Hq / Hkv;
    double* delta = (double*)malloc((size_t)B * Hq * N * sizeof(double));
    double* lse = (double*)malloc((size_t)B * Hq * N * sizeof(double));
    if (!delta || !lse) { free(delta); free(lse); return -2; }
    int fail = 0;

    /* sweep 1: per query row of every query head -> Delta_i, LSE_i, dQ_i */
#pragma omp parallel
    {
        double* s = (double*)malloc((size_t)N * sizeof(double));
        double* o_i = (double*)malloc((size_t)D * sizeof(double));
        if (!s || !o_i) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for collapse(2) schedule(dynamic, 16)
            for (long bh = 0; bh < B * Hq; bh++)
                for (long i = 0; i < N; i++) {
                    const long b = bh / Hq, h = bh % Hq;
                    const double* kh = k + (b * Hkv + h / G) * N * D;
                    const double* vh = v + (b * Hkv + h / G) * N * D;
                    const double* do_i = d_o + (bh * N + i) * D;
                    double lse_i;
                    forward_row(q + (bh * N + i) * D, kh, vh, i, N, D, causal, scale, s, o_i, &lse_i);
                    double dl = 0.0;
                    for (long d = 0; d < D; d++) dl += do_i[d] * o_i[d];
                    delta[bh * N + i] = dl;
                    lse[bh * N + i] = lse_i;
                    double* dq_i = dq + (bh * N + i) * D;
                    for (long d = 0; d < D; d++) dq_i[d] = 0.0;
                    long nj = visible(i, N, causal);
                    for (long j = 0; j < nj; j++) {
                        double dp = 0.0;
                        for (long d = 0; d < D; d++) dp += do_i[d] * vh[j * D + d];
                        double ds = s[j] * (dp - dl);
                        for (long d = 0; d < D; d++) dq_i[d] += ds * kh[j * D + d];
                    }
                    for (long d = 0; d < D; d++) dq_i[d] *= scale;
                }
        }
        free(s); free(o_i);
    }

    /* sweep 2: per key row of every key/value head, summing over the query heads of its group */
    if (!fail) {
#pragma omp parallel for collapse(2) schedule(dynamic, 16)
        for (long bk = 0; bk < B * Hkv; bk++)
            for (long j = 0; j < N; j++) {
                const long b = bk / Hkv, hk = bk % Hkv;
                const double* k_j = k + (bk * N + j) * D;
                const double* v_j = v + (bk * N + j) * D;
                double* dk_j = dk + (bk * N + j) * D;
                double* dv_j = dv + (bk * N + j) * D;
                for (long d = 0; d < D; d++) { dk_j[d] = 0.0; dv_j[d] = 0.0; }
                for (long g = 0; g < G; g++) {
                    const long bh = b * Hq + hk * G + g;
                    const double* qh = q + bh * N * D;
                    const double* doh = d_o + bh * N * D;
                    long i0 = causal ? j : 0;
                    for (long i = i0; i < N; i++) {
                        double dot = 0.0, dp = 0.0;
                        for (long d = 0; d < D; d++) {
                            dot += qh[i * D + d] * k_j[d];
                            dp += doh[i * D + d] * v_j[d];
                        }
                        double p = exp(scale * dot - lse[bh * N + i]);
                        double ds = p * (dp - delta[bh * N + i]);
                        for (long d = 0; d < D; d++) {
                            dv_j[d] += p * doh[i * D + d];
                            dk_j[d] += ds * qh[i * D + d];
                        }
                    }
                }
                for (long d = 0; d < D; d++) dk_j[d] *= scale;
            }
    }
    free(delta); free(lse);
    return fail ? -2 : 0;
}

/*
 * Attention with different numbers of queries and keys (cross attention, decoding against a
 * longer key/value history).  The paper's listings take one sequence length; its Appendix B.3
 * kernel guards only the query tail.  Reading taken: q has Nq rows, k and v have Nk rows, every
 * sum over keys runs over the Nk keys.  With the causal mask the two sequences are aligned at
 * their ENDS: query i is position i + (Nk - Nq) of the key sequence and attends to keys
 * j <= i + (Nk - Nq), so the last query sees every key and Nq = Nk gives the usual mask.  The
 * causal case needs Nq <= Nk (otherwise the first queries would see no key at all).
 * Heads may be grouped as above.
 *   q, d_o, o, dq : [B][Hq][Nq][D]     k, v, dk, dv : [B][Hkv][Nk][D]     lse : [B][Hq][Nq]
 */
static long visible_rect(long i, long Nq, long Nk, int causal) { return causal ? i + (Nk - Nq) + 1 : Nk; }

/* scores of query row q_i against keys 0..nj-1 -> p[j] = softmax probabilities, *lse_i = ln sum exp */
static void softmax_row_rect(const double* q_i, const double* k, long nj, long D, double scale, double* p, double* lse_i)
{
    double m = -INFINITY, l = 0.0;
    for (long j = 0; j < nj; j++) {
        double dot = 0.0;
        for (long d = 0; d < D; d++) dot += q_i[d] * k[j * D + d];
        p[j] = scale * dot;
        if (p[j] > m) m = p[j];
    }
    for (long j = 0; j < nj; j++) { p[j] = exp(p[j] - m); l += p[j]; }
    for (long j = 0; j < nj; j++) p[j] /= l;
    *lse_i = m + log(l);
}

static int rect_args_bad(long B, long Hq, long Hkv, long Nq, long Nk, long D, int causal)
{
    return B <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv || Nq <= 0 || Nk <= 0 || D <= 0 || (causal && Nq > Nk);
}

int oracle_rect_fwd(const double* q, const double* k, const double* v, double* o, double* lse,
                    long B, long Hq, long Hkv, long Nq, long Nk, long D, int causal, double scale)
{
    if (!q || !k || !v || !o || !lse || rect_args_bad(B, Hq, Hkv, Nq, Nk, D, causal)) return -1;
    const long G = Hq / Hkv;
    int fail = 0;
#pragma omp parallel
    {
        double* p = (double*)malloc((size_t)Nk * sizeof(double));
        if (!p) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for collapse(2) schedule(dynamic, 16)
            for (long bh = 0; bh < B * Hq; bh++)
                for (long i = 0; i < Nq; i++) {
                    const long kvh = (bh / Hq) * Hkv + (bh % Hq) / G;
                    const double* kh = k + kvh * Nk * D;
                    const double* vh = v + kvh * Nk * D;
                    const long nj = visible_rect(i, Nq, Nk, causal);
                    softmax_row_rect(q + (bh * Nq + i) * D, kh, nj, D, scale, p, lse + bh * Nq + i);
                    double* o_i = o + (bh * Nq + i) * D;
                    for (long d = 0; d < D; d++) o_i[d] = 0.0;
                    for (long j = 0; j < nj; j++)
                        for (long d = 0; d < D; d++) o_i[d] += p[j] * vh[j * D + d];
                }
            free(p);
        }
    }
    return fail ? -2 : 0;
}

int oracle_rect_bwd(const double* q, const double* k, const double* v, const double* d_o,
                    double* dq, double* dk, double* dv,
                    long B, long Hq, long Hkv, long Nq, long Nk, long D, int causal, double scale)
{
    if (!q || !k || !v || !d_o || !dq || !dk || !dv || rect_args_bad(B, Hq, Hkv, Nq, Nk, D, causal)) return -1;
    const long G = Hq / Hkv;
    double* delta = (double*)malloc((size_t)B * Hq * Nq * sizeof(double));
    double* lse = (double*)malloc((size_t)B * Hq * Nq * sizeof(double));
    if (!delta || !lse) { free(delta); free(lse); return -2; }
    int fail = 0;

    /* sweep 1: per query row -> LSE_i, O_i, Delta_i = dO_i . O_i, dQ_i = scale * sum_j dS_ij K_j */
#pragma omp parallel
    {
        double* p = (double*)malloc((size_t)Nk * sizeof(double));
        double* o_i = (double*)malloc((size_t)D * sizeof(double));
        if (!p || !o_i) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for collapse(2) schedule(dynamic, 16)
            for (long bh = 0; bh < B * Hq; bh++)
                for (long i = 0; i < Nq; i++) {
                    const long kvh = (bh / Hq) * Hkv + (bh % Hq) / G;
                    const double* kh = k + kvh * Nk * D;
                    const double* vh = v + kvh * Nk * D;
                    const double* do_i = d_o + (bh * Nq + i) * D;
                    const long nj = visible_rect(i, Nq, Nk, causal);
                    softmax_row_rect(q + (bh * Nq + i) * D, kh, nj, D, scale, p, lse + bh * Nq + i);
                    for (long d = 0; d < D; d++) o_i[d] = 0.0;
                    for (long j = 0; j < nj; j++)
                        for (long d = 0; d < D; d++) o_i[d] += p[j] * vh[j * D + d];
                    double dl = 0.0;
                    for (long d = 0; d < D; d++) dl += do_i[d] * o_i[d];
                    delta[bh * Nq + i] = dl;
                    double* dq_i = dq + (bh * Nq + i) * D;
                    for (long d = 0; d < D; d++) dq_i[d] = 0.0;
                    for (long j = 0; j < nj; j++) {
                        double dp = 0.0;
                        for (long d = 0; d < D; d++) dp += do_i[d] * vh[j * D + d];
                        const double ds = p[j] * (dp - dl);
                        for (long d = 0; d < D; d++) dq_i[d] += ds * kh[j * D + d];
                    }
                    for (long d = 0; d < D; d++) dq_i[d] *= scale;
                }
        }
        free(p); free(o_i);
    }

    /* sweep 2: per key row -> dV_j = sum_i P_ij dO_i, dK_j = scale * sum_i dS_ij Q_i over the
       queries that see key j (i + Nk - Nq >= j when causal) of every query head of the group */
    if (!fail) {
#pragma omp parallel for collapse(2) schedule(dynamic, 16)
        for (long bk = 0; bk < B * Hkv; bk++)
            for (long j = 0; j < Nk; j++) {
                const long b = bk / Hkv, hk = bk % Hkv;
                const double* k_j = k + (bk * Nk + j) * D;
                const double* v_j = v + (bk * Nk + j) * D;
                double* dk_j = dk + (bk * Nk + j) * D;
                double* dv_j = dv + (bk * Nk + j) * D;
                for (long d = 0; d < D; d++) { dk_j[d] = 0.0; dv_j[d] = 0.0; }
                long i0 = causal ? j - (Nk - Nq) : 0;
                if (i0 < 0) i0 = 0;
                for (long g = 0; g < G; g++) {
                    const long bh = b * Hq + hk * G + g;
                    const double* qh = q + bh * Nq * D;
                    const double* doh = d_o + bh * Nq * D;
                    for (long i = i0; i < Nq; i++) {
                        double dot = 0.0, dp = 0.0;
                        for (long d = 0; d < D; d++) {
                            dot += qh[i * D + d] * k_j[d];
                            dp += doh[i * D + d] * v_j[d];
                        }
                        const double pij = exp(scale * dot - lse[bh * Nq + i]);
                        const double ds = pij * (dp - delta[bh * Nq + i]);
                        for (long d = 0; d < D; d++) {
                            dv_j[d] += pij * doh[i * D + d];
                            dk_j[d] += ds * qh[i * D + d];
                        }
                    }
                }
                for (long d = 0; d < D; d++) dk_j[d] *= scale;
            }
    }
    free(delta); free(lse);
    return fail ? -2 : 0;
}

/*
 * Rotary positional encoding (the rotary kernel of the paper's appendix, head dimension D):
 * with x1 = x[..., :D/2], x2 = x[..., D/2:] and one (sin, cos) pair per position and column,
 *     o1 = x1 * cos - x2 * sin        o2 = x2 * cos + x1 * sin
 * i.e. every pair (x1_c, x2_c) is rotated by the angle whose sine and cosine are given.
 *   x, o : [BH][N][D]      sin, cos : [N][D/2]
 */
int oracle_rotary(const double* x, const double* sn, const double* cs, double* o, long BH, long N, long D)
{
    if (!x || !sn || !cs || !o || BH <= 0 || N <= 0 || D <= 0 || D % 2) return -1;
    const long half = D / 2;
#pragma omp parallel for collapse(2) schedule(static)
    for (long bh = 0; bh < BH; bh++)
        for (long i = 0; i < N; i++) {
            const double* xr = x + (bh * N + i) * D;
            double* orow = o + (bh * N + i) * D;
            for (long c = 0; c < half; c++) {
                const double x1 = xr[c], x2 = xr[half + c];
                orow[c] = x1 * cs[i * half + c] - x2 * sn[i * half + c];
                orow[half + c] = x2 * cs[i * half + c] + x1 * sn[i * half + c];
            }
        }
    return 0;
}

/*
 * Matrix multiply (the GEMM kernel of the paper's appendix): C = A B with A [M][K], B [K][N],
 * C [M][N], all row-major.  The plain definition, one dot product per output element.
 */
int oracle_gemm(const double* a, const double* b, double* c, long M, long N, long K)
{
    if (!a || !b || !c || M <= 0 || N <= 0 || K <= 0) return -1;
#pragma omp parallel for schedule(static)
    for (long i = 0; i < M; i++)
        for (long j = 0; j < N; j++) {
            double acc = 0.0;
            for (long k = 0; k < K; k++) acc += a[i * K + k] * b[k * N + j];
            c[i * N + j] = acc;
        }
    return 0;
}

/* Selected elements of C = A B: out[e] = sum_k A[rows[e]][k] B[k][cols[e]] (for sampled checks of large products). */
int oracle_gemm_elements(const double* a, const double* b, const long* rows, const long* cols, long n,
                         double* out, long M, long N, long K)
{
    if (!a || !b || !rows || !cols || !out || n < 0 || M <= 0 || N <= 0 || K <= 0) return -1;
    for (long e = 0; e < n; e++) if (rows[e] < 0 || rows[e] >= M || cols[e] < 0 || cols[e] >= N) return -1;
#pragma omp parallel for schedule(static)
    for (long e = 0; e < n; e++) {
        double acc = 0.0;
        for (long k = 0; k < K; k++) acc += a[rows[e] * K + k] * b[k * N + cols[e]];
        out[e] = acc;
    }
    return 0;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
