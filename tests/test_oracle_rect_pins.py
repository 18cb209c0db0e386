"""Pins for the oracle functions with different query and key lengths (CPU only).

The paper's listings take one sequence length (its Appendix B.3 kernel guards only the query
tail).  The reading pinned here: q has Nq rows, k and v have Nk rows; with the causal mask the
two sequences are aligned at their ends, i.e. query i attends to keys j <= i + (Nk - Nq).
Checks, none of which re-types the oracle's own loops:
  * scipy's softmax / logsumexp with the mask written as an explicit boolean matrix;
  * the causal case equals the LAST Nq rows of the square causal problem of length Nk (whose
    oracle is pinned separately), forward and backward (dO zero on the leading rows);
  * closed forms: all keys equal -> O = mean of the visible values, LSE = s + ln(#visible);
    one query (decode shape) -> a single softmax over all keys;
  * central finite differences of L = sum(O * dO) for dQ, dK, dV;
  * Nq = Nk reduces to the grouped-query functions; argument errors.
"""
import math

import numpy as np
import pytest
from scipy.special import logsumexp, softmax

from oracle import attn_oracle as orc

RNG = np.random.default_rng(1152)


def rand(*shape):
    return RNG.standard_normal(shape)


def mask_matrix(Nq, Nk, causal):
    """keep[i, j]: query i may attend to key j."""
    i = np.arange(Nq)[:, None]
    j = np.arange(Nk)[None, :]
    return (j <= i + (Nk - Nq)) if causal else np.ones((Nq, Nk), bool)


def library_forward(q, k, v, causal, scale):
    B, Hq, Nq, D = q.shape
    Hkv, Nk = k.shape[1], k.shape[2]
    G = Hq // Hkv
    keep = mask_matrix(Nq, Nk, causal)
    o = np.empty_like(q)
    lse = np.empty((B, Hq, Nq))
    for b in range(B):
        for h in range(Hq):
            s = scale * (q[b, h] @ k[b, h // G].T)
            s = np.where(keep, s, -np.inf)
            o[b, h] = softmax(s, axis=1) @ v[b, h // G]
            lse[b, h] = logsumexp(s, axis=1)
    return o, lse


SHAPES = [(1, 1, 1, 5, 9), (2, 4, 2, 7, 7), (1, 2, 1, 1, 11), (1, 3, 3, 6, 17), (2, 2, 1, 12, 5), (1, 1, 1, 1, 1)]
# B, Hq, Hkv, Nq, Nk


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("B,Hq,Hkv,Nq,Nk", SHAPES)
def test_forward_matches_library_softmax(B, Hq, Hkv, Nq, Nk, causal):
    if causal and Nq > Nk:
        pytest.skip("causal needs Nq <= Nk")
    D = 6
    q, k, v = rand(B, Hq, Nq, D), rand(B, Hkv, Nk, D), rand(B, Hkv, Nk, D)
    scale = 1 / math.sqrt(D)
    o, lse = orc.rect_fwd(q, k, v, causal, scale)
    lo, llse = library_forward(q, k, v, causal, scale)
    np.testing.assert_allclose(o, lo, rtol=0, atol=1e-12)
    np.testing.assert_allclose(lse, llse, rtol=0, atol=1e-12)


@pytest.mark.parametrize("Nq,Nk", [(1, 9), (4, 9), (8, 9), (9, 9), (5, 33)])
def test_causal_is_the_tail_of_the_square_problem(Nq, Nk):
    """Queries = last Nq rows of a length-Nk sequence: same outputs and gradients as the square oracle."""
    BH, D = 3, 5
    scale = 0.4
    q_full, k, v, do_full = rand(BH, Nk, D), rand(BH, Nk, D), rand(BH, Nk, D), rand(BH, Nk, D)
    do_full[:, : Nk - Nq] = 0.0            # the leading rows contribute nothing to L
    o_sq, lse_sq = orc.attn_fwd(q_full, k, v, True, scale)
    dq_sq, dk_sq, dv_sq = orc.attn_bwd(q_full, k, v, do_full, True, scale)
    q = q_full[:, Nk - Nq:][:, None]       # [BH, 1, Nq, D]: BH batch entries of one head
    d_o = do_full[:, Nk - Nq:][:, None]
    o, lse = orc.rect_fwd(q, k[:, None], v[:, None], True, scale)
    dq, dk, dv = orc.rect_bwd(q, k[:, None], v[:, None], d_o, True, scale)
    np.testing.assert_allclose(o[:, 0], o_sq[:, Nk - Nq:], rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse[:, 0], lse_sq[:, Nk - Nq:], rtol=0, atol=1e-13)
    np.testing.assert_allclose(dq[:, 0], dq_sq[:, Nk - Nq:], rtol=0, atol=1e-13)
    np.testing.assert_allclose(dk[:, 0], dk_sq, rtol=0, atol=1e-13)
    np.testing.assert_allclose(dv[:, 0], dv_sq, rtol=0, atol=1e-13)


@pytest.mark.parametrize("causal", [False, True])
def test_equal_keys_give_the_mean_of_the_visible_values(causal):
    B, Hq, Hkv, Nq, Nk, D = 1, 2, 1, 6, 10, 4
    q = rand(B, Hq, Nq, D)
    k = np.broadcast_to(rand(B, Hkv, 1, D), (B, Hkv, Nk, D)).copy()
    v = rand(B, Hkv, Nk, D)
    scale = 0.7
    o, lse = orc.rect_fwd(q, k, v, causal, scale)
    for h in range(Hq):
        for i in range(Nq):
            n_vis = i + (Nk - Nq) + 1 if causal else Nk
            np.testing.assert_allclose(o[0, h, i], v[0, 0, :n_vis].mean(axis=0), rtol=0, atol=1e-13)
            s = scale * float(q[0, h, i] @ k[0, 0, 0])
            assert abs(lse[0, h, i] - (s + math.log(n_vis))) < 1e-13


@pytest.mark.parametrize("causal", [False, True])
def test_one_query_sees_every_key(causal):
    """Decode shape: the single query is the last position, so the causal mask removes nothing."""
    D, Nk = 8, 23
    q, k, v = rand(1, 1, 1, D), rand(1, 1, Nk, D), rand(1, 1, Nk, D)
    o, lse = orc.rect_fwd(q, k, v, causal, 0.3)
    w = softmax(0.3 * (k[0, 0] @ q[0, 0, 0]))
    np.testing.assert_allclose(o[0, 0, 0], w @ v[0, 0], rtol=0, atol=1e-13)
    d_o = rand(1, 1, 1, D)
    dq, dk, dv = orc.rect_bwd(q, k, v, d_o, causal, 0.3)
    # dV_j = P_j dO; rows of dV are multiples of dO with the softmax weights as factors
    np.testing.assert_allclose(dv[0, 0], np.outer(w, d_o[0, 0, 0]), rtol=0, atol=1e-13)
    # sum_j dS_j = 0 -> dQ = scale * sum_j dS_j K_j is unchanged when every key is shifted by a constant vector
    shift = rand(D)
    dq2, _, _ = orc.rect_bwd(q, k + shift, v, d_o, causal, 0.3)
    np.testing.assert_allclose(dq2, dq, rtol=0, atol=1e-12)


def loss(q, k, v, d_o, causal, scale):
    o, _ = orc.rect_fwd(q, k, v, causal, scale)
    return float((o * d_o).sum())


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("B,Hq,Hkv,Nq,Nk", [(1, 2, 1, 3, 6), (2, 2, 2, 4, 5), (1, 1, 1, 1, 4)])
def test_gradients_match_finite_differences(B, Hq, Hkv, Nq, Nk, causal):
    D = 3
    q, k, v, d_o = rand(B, Hq, Nq, D), rand(B, Hkv, Nk, D), rand(B, Hkv, Nk, D), rand(B, Hq, Nq, D)
    scale = 0.6
    dq, dk, dv = orc.rect_bwd(q, k, v, d_o, causal, scale)
    eps = 1e-6
    for name, x, g in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        num = np.empty_like(x)
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            keep = x[idx]
            x[idx] = keep + eps
            up = loss(q, k, v, d_o, causal, scale)
            x[idx] = keep - eps
            dn = loss(q, k, v, d_o, causal, scale)
            x[idx] = keep
            num[idx] = (up - dn) / (2 * eps)
        np.testing.assert_allclose(g, num, rtol=0, atol=2e-8, err_msg=name)


@pytest.mark.parametrize("causal", [False, True])
def test_equal_lengths_reduce_to_the_grouped_functions(causal):
    B, Hq, Hkv, N, D = 2, 4, 2, 9, 5
    q, k, v, d_o = rand(B, Hq, N, D), rand(B, Hkv, N, D), rand(B, Hkv, N, D), rand(B, Hq, N, D)
    o, lse = orc.rect_fwd(q, k, v, causal, 0.45)
    go, glse = orc.gqa_fwd(q, k, v, causal, 0.45)
    np.testing.assert_allclose(o, go, rtol=0, atol=1e-14)
    np.testing.assert_allclose(lse, glse, rtol=0, atol=1e-14)
    for a, b in zip(orc.rect_bwd(q, k, v, d_o, causal, 0.45), orc.gqa_bwd(q, k, v, d_o, causal, 0.45)):
        np.testing.assert_allclose(a, b, rtol=0, atol=1e-13)


def test_non_causal_keys_can_be_permuted():
    """Without a mask the result does not depend on the order of the keys; dK, dV follow the permutation."""
    B, Hq, Hkv, Nq, Nk, D = 1, 2, 1, 5, 12, 4
    q, k, v, d_o = rand(B, Hq, Nq, D), rand(B, Hkv, Nk, D), rand(B, Hkv, Nk, D), rand(B, Hq, Nq, D)
    perm = RNG.permutation(Nk)
    o, lse = orc.rect_fwd(q, k, v, False, 0.5)
    o2, lse2 = orc.rect_fwd(q, k[:, :, perm], v[:, :, perm], False, 0.5)
    np.testing.assert_allclose(o2, o, rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse2, lse, rtol=0, atol=1e-13)
    dq, dk, dv = orc.rect_bwd(q, k, v, d_o, False, 0.5)
    dq2, dk2, dv2 = orc.rect_bwd(q, k[:, :, perm], v[:, :, perm], d_o, False, 0.5)
    np.testing.assert_allclose(dq2, dq, rtol=0, atol=1e-13)
    np.testing.assert_allclose(dk2, dk[:, :, perm], rtol=0, atol=1e-13)
    np.testing.assert_allclose(dv2, dv[:, :, perm], rtol=0, atol=1e-13)


def test_bad_arguments():
    q, k = rand(1, 2, 6, 4), rand(1, 1, 4, 4)
    with pytest.raises(ValueError):
        orc.rect_fwd(q, k, k, True, 0.5)                 # causal with Nq > Nk
    with pytest.raises(ValueError):
        orc.rect_fwd(rand(1, 3, 6, 4), rand(1, 2, 8, 4), rand(1, 2, 8, 4), False, 0.5)   # Hkv does not divide Hq
    with pytest.raises(ValueError):
        orc.rect_bwd(q, k, k, rand(1, 2, 5, 4), False, 0.5)   # dO shape
    orc.rect_fwd(q, k, k, False, 0.5)                    # Nq > Nk is fine without the mask


def test_the_pins_tell_end_alignment_from_start_alignment():
    """The other plausible reading of "causal" for Nq < Nk (query i sees keys j <= i, sequences aligned
    at their starts) gives different numbers on the same inputs: the tail-of-the-square pin above
    would reject an oracle that implemented it."""
    Nq, Nk, D = 4, 9, 5
    q, k, v = rand(1, 1, Nq, D), rand(1, 1, Nk, D), rand(1, 1, Nk, D)
    o, lse = orc.rect_fwd(q, k, v, True, 0.4)
    s = 0.4 * (q[0, 0] @ k[0, 0].T)
    start_aligned = np.where(np.arange(Nk)[None, :] <= np.arange(Nq)[:, None], s, -np.inf)
    o_start = softmax(start_aligned, axis=1) @ v[0, 0]
    assert np.abs(o[0, 0] - o_start).max() > 1e-2
    end_aligned = np.where(np.arange(Nk)[None, :] <= np.arange(Nq)[:, None] + (Nk - Nq), s, -np.inf)
    np.testing.assert_allclose(o[0, 0], softmax(end_aligned, axis=1) @ v[0, 0], rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse[0, 0], logsumexp(end_aligned, axis=1), rtol=0, atol=1e-13)
