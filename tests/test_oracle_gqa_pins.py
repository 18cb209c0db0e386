"""Pins for the grouped-query functions of the fp64 oracle (CPU only).

Section 4.1 of the paper names grouped-query attention as a supported variant without printing
a formula; the reading pinned here is: query head h attends with key/value head h // G,
G = Hq / Hkv, and a shared head's gradient is the sum over its group.  Checks: a brute-force
numpy softmax with the head mapping written as explicit loops, reduction to the per-head
functions (keys/values repeated per group), finite differences of L = sum(O * dO) with respect
to the SHARED keys and values, and the degenerate group sizes (G = 1: plain multi-head; Hkv = 1:
multi-query).
"""
import math

import numpy as np
import pytest

from oracle import attn_oracle as orc

RNG = np.random.default_rng(657)


def rand(*shape):
    return RNG.standard_normal(shape)


def brute_gqa_forward(q, k, v, causal, scale):
    """q [B,Hq,N,D], k, v [B,Hkv,N,D]; exp(S)/sum exp(S) without max subtraction, head by head."""
    B, Hq, N, D = q.shape
    G = Hq // k.shape[1]
    o = np.empty_like(q)
    lse = np.empty((B, Hq, N))
    for b in range(B):
        for h in range(Hq):
            hk = h // G
            e = np.exp(scale * (q[b, h] @ k[b, hk].T))
            if causal:
                e = e * np.tril(np.ones((N, N)))
            z = e.sum(axis=1)
            o[b, h] = (e / z[:, None]) @ v[b, hk]
            lse[b, h] = np.log(z)
    return o, lse


CASES = [(1, 1, 1), (1, 4, 4), (2, 4, 2), (2, 6, 2), (1, 8, 1), (3, 3, 1)]   # B, Hq, Hkv


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("B,Hq,Hkv", CASES)
def test_gqa_forward_matches_brute_force(B, Hq, Hkv, causal):
    N, D = 13, 6
    q, k, v = rand(B, Hq, N, D), rand(B, Hkv, N, D), rand(B, Hkv, N, D)
    scale = 1 / math.sqrt(D)
    o, lse = orc.gqa_fwd(q, k, v, causal, scale)
    bo, blse = brute_gqa_forward(q, k, v, causal, scale)
    np.testing.assert_allclose(o, bo, rtol=0, atol=1e-12)
    np.testing.assert_allclose(lse, blse, rtol=0, atol=1e-12)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("B,Hq,Hkv", CASES)
def test_gqa_reduces_to_per_head_functions(B, Hq, Hkv, causal):
    """Repeating each key/value head G times turns GQA into plain multi-head attention; the shared
    head's gradient is the sum of the repeated heads' gradients."""
    N, D = 17, 8
    G = Hq // Hkv
    q, k, v, d_o = rand(B, Hq, N, D), rand(B, Hkv, N, D), rand(B, Hkv, N, D), rand(B, Hq, N, D)
    scale = 0.4
    kr, vr = np.repeat(k, G, axis=1), np.repeat(v, G, axis=1)
    o, lse = orc.gqa_fwd(q, k, v, causal, scale)
    o2, lse2 = orc.attn_fwd(q, kr, vr, causal, scale)
    np.testing.assert_allclose(o, o2, rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse, lse2, rtol=0, atol=1e-13)
    dq, dk, dv = orc.gqa_bwd(q, k, v, d_o, causal, scale)
    dq2, dk2, dv2 = orc.attn_bwd(q, kr, vr, d_o, causal, scale)
    np.testing.assert_allclose(dq, dq2, rtol=0, atol=1e-12)
    np.testing.assert_allclose(dk, dk2.reshape(B, Hkv, G, N, D).sum(2), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dv, dv2.reshape(B, Hkv, G, N, D).sum(2), rtol=0, atol=1e-12)


def test_interleaved_grouping_would_be_caught():
    """h // G and h % Hkv give different answers as soon as 1 < Hkv < Hq."""
    B, Hq, Hkv, N, D = 1, 4, 2, 9, 4
    q, k, v = rand(B, Hq, N, D), rand(B, Hkv, N, D), rand(B, Hkv, N, D)
    o, _ = orc.gqa_fwd(q, k, v, False, 0.5)
    wrong = np.empty_like(o)
    for h in range(Hq):
        e = np.exp(0.5 * (q[0, h] @ k[0, h % Hkv].T))
        wrong[0, h] = (e / e.sum(1, keepdims=True)) @ v[0, h % Hkv]
    assert np.abs(o - wrong).max() > 1e-2


@pytest.mark.parametrize("causal", [False, True])
def test_gqa_gradients_match_finite_differences(causal):
    B, Hq, Hkv, N, D = 1, 4, 2, 7, 3
    q, k, v, d_o = rand(B, Hq, N, D), rand(B, Hkv, N, D), rand(B, Hkv, N, D), rand(B, Hq, N, D)
    scale = 0.7
    dq, dk, dv = orc.gqa_bwd(q, k, v, d_o, causal, scale)

    def loss(q_, k_, v_):
        return float((brute_gqa_forward(q_, k_, v_, causal, scale)[0] * d_o).sum())

    eps = 1e-6
    for name, x, g in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        num = np.empty_like(x)
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            xp, xm = x.copy(), x.copy()
            xp[idx] += eps
            xm[idx] -= eps
            args_p = {"q": (xp, k, v), "k": (q, xp, v), "v": (q, k, xp)}[name]
            args_m = {"q": (xm, k, v), "k": (q, xm, v), "v": (q, k, xm)}[name]
            num[idx] = (loss(*args_p) - loss(*args_m)) / (2 * eps)
        np.testing.assert_allclose(g, num, rtol=0, atol=2e-7, err_msg=name)


def test_gqa_rejects_bad_head_counts():
    q, k = rand(1, 4, 4, 2), rand(1, 3, 4, 2)
    with pytest.raises(ValueError):
        orc.gqa_fwd(q, k, k, False, 1.0)
