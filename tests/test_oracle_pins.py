"""Pins for the fp64 oracle (CPU only).

Every check compares oracle/attn_oracle.c with something that is not the
oracle: a brute-force numpy softmax without max subtraction, closed forms,
algebraic invariants of the definition (the PyTorch attention listing in the paper's introduction + the
temperature of the Appendix B.3 listing), constants the paper prints, and
central finite differences of a brute-force forward for the gradients.
"""
import math
import os

import numpy as np
import pytest

from oracle import attn_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
RNG = np.random.default_rng(20399)


# ---------------------------------------------------------------- brute force (independent of the oracle)
def brute_forward(q, k, v, causal, scale):
    """exp(S)/sum(exp(S)) with no max subtraction; q,k,v [N,D] float64 (tiny shapes only)."""
    N = q.shape[0]
    e = np.exp(scale * (q @ k.T))
    if causal:
        e = e * np.tril(np.ones((N, N)))
    z = e.sum(axis=1, keepdims=True)
    p = e / z
    return p @ v, np.log(z[:, 0]), p


def rand(*shape):
    return RNG.standard_normal(shape)


SHAPES = [(1, 1), (1, 4), (2, 1), (2, 8), (5, 4), (16, 8), (33, 5)]


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("N,D", SHAPES)
def test_forward_matches_brute_force(N, D, causal):
    q, k, v = rand(2, N, D), rand(2, N, D), rand(2, N, D)
    scale = 1.0 / math.sqrt(D)
    o, lse, p = orc.attn_fwd(q, k, v, causal, scale, return_p=True)
    for h in range(2):
        bo, blse, bp = brute_forward(q[h], k[h], v[h], causal, scale)
        np.testing.assert_allclose(o[h], bo, rtol=0, atol=1e-12)
        np.testing.assert_allclose(lse[h], blse, rtol=0, atol=1e-12)
        np.testing.assert_allclose(p[h], bp, rtol=0, atol=1e-13)


@pytest.mark.parametrize("causal", [False, True])
def test_probability_invariants(causal):
    N, D = 37, 16
    q, k, v = 3 * rand(3, N, D), rand(3, N, D), rand(3, N, D)
    scale = 0.3
    o, lse, p = orc.attn_fwd(q, k, v, causal, scale, return_p=True)
    np.testing.assert_allclose(p.sum(-1), 1.0, rtol=0, atol=1e-14)
    assert (p >= 0).all()
    s = scale * np.einsum("hid,hjd->hij", q, k)
    if causal:
        assert (np.triu(p, 1) == 0).all()
        s = np.where(np.tril(np.ones((N, N), bool)), s, -np.inf)
    naive_lse = np.log(np.exp(s).sum(-1))
    np.testing.assert_allclose(lse, naive_lse, rtol=0, atol=1e-12)
    np.testing.assert_allclose(p, np.exp(s - lse[..., None]), rtol=0, atol=1e-13)


def test_large_scores_do_not_overflow():
    # the brute force would overflow here; the definition with max subtraction must not
    N, D = 8, 4
    q, k, v = 200 * rand(1, N, D), 5 * rand(1, N, D), rand(1, N, D)
    o, lse, p = orc.attn_fwd(q, k, v, False, 1.0, return_p=True)
    assert np.isfinite(o).all() and np.isfinite(lse).all()
    np.testing.assert_allclose(p.sum(-1), 1.0, atol=1e-14)
    s = np.einsum("hid,hjd->hij", q, k)
    # LSE within [max, max + ln N]
    assert (lse >= s.max(-1) - 1e-9).all() and (lse <= s.max(-1) + math.log(N) + 1e-9).all()


# ---------------------------------------------------------------- values the paper prints
def _constants():
    out = {}
    with open(os.path.join(GOLDEN, "temperature_constants.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, val = line.split()
            out[name] = float(val)
    return out


def test_paper_constants():
    c = _constants()
    assert abs(c["inv_sqrt_128"] - 1 / math.sqrt(128)) < 1e-11
    assert c["inv_sqrt_64"] == 1 / math.sqrt(64)
    assert abs(c["log2_e"] - math.log2(math.e)) < 1e-11


@pytest.mark.parametrize("D,key", [(128, "inv_sqrt_128"), (64, "inv_sqrt_64")])
def test_base2_temperature_equals_natural_softmax(D, key):
    """P from the oracle (natural exp, scale 1/sqrt(D)) equals 2^((S_raw - max) * TEMPERATURE_SCALE)
    normalised, with TEMPERATURE_SCALE built from the constants the listing prints."""
    c = _constants()
    temp = c[key] * c["log2_e"]
    N = 24
    q, k, v = rand(1, N, D), rand(1, N, D), rand(1, N, D)
    o, lse, p = orc.attn_fwd(q, k, v, False, 1 / math.sqrt(D), return_p=True)
    raw = q[0] @ k[0].T
    e2 = np.exp2((raw - raw.max(1, keepdims=True)) * temp)
    p2 = e2 / e2.sum(1, keepdims=True)
    np.testing.assert_allclose(p[0], p2, rtol=0, atol=5e-10)  # constants are printed to ~1e-11
    np.testing.assert_allclose(o[0], p2 @ v[0], rtol=0, atol=5e-9)


def test_two_key_closed_form():
    """Golden fixture two_key_example.txt: logistic closed form for N=2, D=1."""
    a, b = math.log(2) / 2, math.log(3) / 2
    q = np.array([[[a], [b]]]); k = np.array([[[1.0], [-1.0]]]); v = np.array([[[3.0], [-3.0]]])
    o, lse, p = orc.attn_fwd(q, k, v, False, 1.0, return_p=True)
    rows = []
    with open(os.path.join(GOLDEN, "two_key_example.txt")) as f:
        for line in f:
            if line[0] in "01":
                parts = line.split()
                rows.append((float(parts[1]), float(parts[2]), float(parts[3])))
    for i, (p0, p1, oi) in enumerate(rows):
        assert abs(p[0, i, 0] - p0) < 1e-15 and abs(p[0, i, 1] - p1) < 1e-15
        assert abs(o[0, i, 0] - oi) < 1e-14
    assert abs(lse[0, 0] - math.log(math.sqrt(2) + 1 / math.sqrt(2))) < 1e-15
    assert abs(lse[0, 1] - math.log(math.sqrt(3) + 1 / math.sqrt(3))) < 1e-15
    oc, lsec = orc.attn_fwd(q, k, v, True, 1.0)
    assert oc[0, 0, 0] == 3.0 and abs(lsec[0, 0] - a) < 1e-16
    assert abs(oc[0, 1, 0] - 1.5) < 1e-14


# ---------------------------------------------------------------- closed forms and invariances
def test_zero_queries_give_running_means():
    N, D = 19, 6
    k, v = rand(1, N, D), rand(1, N, D)
    q = np.zeros((1, N, D))
    o, lse = orc.attn_fwd(q, k, v, False, 0.7)
    np.testing.assert_allclose(lse[0], math.log(N), atol=1e-14)
    np.testing.assert_allclose(o[0], np.broadcast_to(v[0].mean(0), (N, D)), atol=1e-14)
    o, lse = orc.attn_fwd(q, k, v, True, 0.7)
    np.testing.assert_allclose(lse[0], np.log(np.arange(1, N + 1)), atol=1e-14)
    np.testing.assert_allclose(o[0], np.cumsum(v[0], 0) / np.arange(1, N + 1)[:, None], atol=1e-14)


def test_single_token():
    D = 8
    q, k, v, d_o = rand(1, 1, D), rand(1, 1, D), rand(1, 1, D), rand(1, 1, D)
    for causal in (False, True):
        o, lse = orc.attn_fwd(q, k, v, causal, 0.5)
        np.testing.assert_array_equal(o, v)
        np.testing.assert_allclose(lse[0, 0], 0.5 * (q[0, 0] @ k[0, 0]), atol=1e-15)
        dq, dk, dv = orc.attn_bwd(q, k, v, d_o, causal, 0.5)
        np.testing.assert_allclose(dv, d_o, atol=1e-15)
        np.testing.assert_allclose(dq, 0, atol=1e-15)
        np.testing.assert_allclose(dk, 0, atol=1e-15)


def test_causal_first_row_and_prefix_property():
    N, D = 21, 8
    q, k, v = rand(1, N, D), rand(1, N, D), rand(1, N, D)
    oc, lsec = orc.attn_fwd(q, k, v, True, 0.4)
    np.testing.assert_array_equal(oc[0, 0], v[0, 0])
    for i in (0, 3, 11, N - 1):
        on, lsen = orc.attn_fwd(q[:, : i + 1], k[:, : i + 1], v[:, : i + 1], False, 0.4)
        np.testing.assert_allclose(oc[0, i], on[0, i], atol=1e-14)
        np.testing.assert_allclose(lsec[0, i], lsen[0, i], atol=1e-14)


def test_equal_keys_give_uniform_attention():
    N, D = 12, 4
    q, v = rand(1, N, D), rand(1, N, D)
    k = np.broadcast_to(rand(1, 1, D), (1, N, D)).copy()
    o, lse, p = orc.attn_fwd(q, k, v, False, 1.3, return_p=True)
    np.testing.assert_allclose(p, 1.0 / N, atol=1e-15)
    np.testing.assert_allclose(o[0], np.broadcast_to(v[0].mean(0), (N, D)), atol=1e-14)


def test_key_shift_and_joint_permutation():
    N, D = 17, 8
    q, k, v = rand(1, N, D), rand(1, N, D), rand(1, N, D)
    scale = 0.35
    o, lse = orc.attn_fwd(q, k, v, False, scale)
    t = rand(D)
    o2, lse2 = orc.attn_fwd(q, k + t, v, False, scale)
    np.testing.assert_allclose(o2, o, atol=1e-13)
    np.testing.assert_allclose(lse2 - lse, scale * (q @ t), atol=1e-13)
    perm = RNG.permutation(N)
    o3, lse3 = orc.attn_fwd(q, k[:, perm], v[:, perm], False, scale)
    np.testing.assert_allclose(o3, o, atol=1e-13)
    np.testing.assert_allclose(lse3, lse, atol=1e-13)


def test_transposed_operand_would_be_caught():
    """Asymmetric K: the score matrix must be Q K^T, not K Q^T (checked on one entry by hand)."""
    q = np.array([[[1.0, 0.0], [0.0, 1.0]]]); k = np.array([[[2.0, 0.0], [3.0, 0.0]]])
    v = np.array([[[1.0, 0.0], [0.0, 1.0]]])
    o, lse, p = orc.attn_fwd(q, k, v, False, 1.0, return_p=True)
    # row 0: scores [2, 3] -> p = softmax([2,3]); row 1: scores [0, 0] -> uniform
    e = math.exp(-1.0)
    np.testing.assert_allclose(p[0, 0], [e / (1 + e), 1 / (1 + e)], atol=1e-15)
    np.testing.assert_allclose(p[0, 1], [0.5, 0.5], atol=1e-15)


def test_rows_entry_point_matches_full():
    N, D = 40, 8
    q, k, v = rand(N, D), rand(N, D), rand(N, D)
    for causal in (False, True):
        o, lse = orc.attn_fwd(q, k, v, causal, 0.2)
        rows = [0, 1, 17, 39]
        o_r, lse_r = orc.attn_fwd_rows(q, k, v, rows, causal, 0.2)
        np.testing.assert_array_equal(o_r, o[rows])
        np.testing.assert_array_equal(lse_r, lse[rows])


# ---------------------------------------------------------------- online-softmax recurrence == definition
def online_softmax_blocked(q, k, v, scale, block):
    """The streaming recurrence in the step order of the Appendix B.3 listing's compute stage
    (running max on raw scores, temperature folded into a base-2 exponent, rescale of the
    running sum and output, normalisation at the end); numpy float64, one head."""
    N, D = q.shape
    temp = scale * math.log2(math.e)
    m = np.full(N, -np.inf); l = np.zeros(N); o = np.zeros((N, D))
    for j0 in range(0, k.shape[0], block):
        s = q @ k[j0:j0 + block].T
        m_last_scaled = m * temp
        m = np.maximum(m, s.max(1))
        m_scaled = m * temp
        p = np.exp2(s * temp - m_scaled[:, None])
        corr = np.exp2(m_last_scaled - m_scaled)
        l = l * corr + p.sum(1)
        o = o * corr[:, None] + p @ v[j0:j0 + block]
    return o / l[:, None], m * scale + np.log(l)


@pytest.mark.parametrize("block", [1, 7, 16, 64])
def test_online_softmax_recurrence_equals_definition(block):
    N, D = 50, 16
    q, k, v = 2 * rand(N, D), rand(N, D), rand(N, D)
    o, lse = orc.attn_fwd(q, k, v, False, 0.25)
    o2, lse2 = online_softmax_blocked(q, k, v, 0.25, block)
    np.testing.assert_allclose(o2, o, atol=1e-13)
    np.testing.assert_allclose(lse2, lse, atol=1e-13)


# ---------------------------------------------------------------- gradients
def loss_brute(q, k, v, d_o, causal, scale):
    return float((brute_forward(q, k, v, causal, scale)[0] * d_o).sum())


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("N,D", [(2, 1), (3, 4), (6, 8), (9, 3)])
def test_gradients_match_finite_differences(N, D, causal):
    q, k, v, d_o = rand(N, D), rand(N, D), rand(N, D), rand(N, D)
    scale = 0.6
    dq, dk, dv = orc.attn_bwd(q, k, v, d_o, causal, scale)
    h = 1e-5
    for name, x, g in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        fd = np.zeros_like(x)
        for idx in np.ndindex(*x.shape):
            old = x[idx]
            x[idx] = old + h; lp = loss_brute(q, k, v, d_o, causal, scale)
            x[idx] = old - h; lm = loss_brute(q, k, v, d_o, causal, scale)
            x[idx] = old
            fd[idx] = (lp - lm) / (2 * h)
        err = np.linalg.norm(fd - g) / max(np.linalg.norm(fd), 1e-30)
        assert err < 1e-7, (name, err)


@pytest.mark.parametrize("causal", [False, True])
def test_backward_invariants(causal):
    N, D = 23, 8
    q, k, v, d_o = rand(2, N, D), rand(2, N, D), rand(2, N, D), rand(2, N, D)
    scale = 0.45
    ds = orc.attn_ds(q, k, v, d_o, causal, scale)
    np.testing.assert_allclose(ds.sum(-1), 0.0, atol=1e-13)          # softmax Jacobian annihilates constants
    o, lse, p = orc.attn_fwd(q, k, v, causal, scale, return_p=True)
    dq, dk, dv, delta, lse_b = orc.attn_bwd(q, k, v, d_o, causal, scale, return_stats=True)
    dp = np.einsum("hid,hjd->hij", d_o, v)
    np.testing.assert_allclose(delta, (p * dp).sum(-1), atol=1e-13)   # Delta_i = sum_j P_ij dP_ij
    np.testing.assert_allclose(delta, (d_o * o).sum(-1), atol=1e-13)
    np.testing.assert_allclose(lse_b, lse, atol=1e-14)
    # matrix forms of the chain rule, written with numpy matmuls
    np.testing.assert_allclose(dv, np.einsum("hij,hid->hjd", p, d_o), atol=1e-13)
    np.testing.assert_allclose(dq, scale * np.einsum("hij,hjd->hid", ds, k), atol=1e-13)
    np.testing.assert_allclose(dk, scale * np.einsum("hij,hid->hjd", ds, q), atol=1e-13)
    if causal:
        assert (np.triu(ds, 1) == 0).all()


def test_dv_linear_in_do_and_dq_dk_too():
    N, D = 11, 4
    q, k, v = rand(1, N, D), rand(1, N, D), rand(1, N, D)
    a, b = rand(1, N, D), rand(1, N, D)
    ga = orc.attn_bwd(q, k, v, a, True, 0.5)
    gb = orc.attn_bwd(q, k, v, b, True, 0.5)
    gab = orc.attn_bwd(q, k, v, 2 * a - 3 * b, True, 0.5)
    for x, y, z in zip(ga, gb, gab):
        np.testing.assert_allclose(z, 2 * x - 3 * y, atol=1e-13)


def test_key_shift_leaves_dq_dv_unchanged():
    """O does not depend on a common shift of all keys, so dQ and dV keep their values and
    dK's column sums vanish (sum_j dK_j = scale * sum_i (sum_j dS_ij) Q_i = 0)."""
    N, D = 13, 4
    q, k, v, d_o = rand(1, N, D), rand(1, N, D), rand(1, N, D), rand(1, N, D)
    dq, dk, dv = orc.attn_bwd(q, k, v, d_o, False, 0.8)
    np.testing.assert_allclose(dk.sum(1), 0.0, atol=1e-13)
    t = rand(D)
    dq2, dk2, dv2 = orc.attn_bwd(q, k + t, v, d_o, False, 0.8)
    np.testing.assert_allclose(dv2, dv, atol=1e-13)
    np.testing.assert_allclose(dk2, dk, atol=1e-13)
    # dQ_i = scale * sum_j dS_ij (K_j + t) = old dQ_i + scale * t * sum_j dS_ij = old dQ_i
    np.testing.assert_allclose(dq2, dq, atol=1e-13)
