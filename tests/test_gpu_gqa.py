"""GPU parity for grouped-query attention: the HIP path through the C ABI against the fp64 oracle.

Same tolerances as the multi-head parity tests; dK, dV have the key/value head count.
"""
import math

import numpy as np
import pytest
import torch

from oracle import attn_oracle as orc
from grad_check import check_grad

pytestmark = pytest.mark.gpu

O_MAX, O_MEAN, LSE_MAX, GRAD_RELF = 2e-2, 2e-3, 1e-3, 3e-2


@pytest.fixture(scope="module")
def attn():
    from paper_2410_20399_amd import attn as a
    a.load_library()          # raises if the HIP library is missing: no fallback
    return a


def f64(t):
    return t.double().numpy()


def relf(a, b):
    return float(np.linalg.norm(a - b) / np.linalg.norm(b))


def make(seed, B, Hq, Hkv, N, D):
    g = torch.Generator().manual_seed(seed)
    q = torch.randn(B, Hq, N, D, generator=g).to(torch.bfloat16)
    k = torch.randn(B, Hkv, N, D, generator=g).to(torch.bfloat16)
    v = torch.randn(B, Hkv, N, D, generator=g).to(torch.bfloat16)
    d_o = torch.randn(B, Hq, N, D, generator=g).to(torch.bfloat16)
    return q, k, v, d_o


CASES = [
    # B, Hq, Hkv, N, D, causal     group sizes 1, 2, 4, 8 and multi-query; odd tile counts; more
    #                              key/value work units than compute units (persistent walk)
    (1, 4, 2, 256, 64, True), (1, 4, 2, 256, 128, False), (2, 8, 2, 384, 128, True), (1, 8, 1, 512, 64, True),
    (2, 6, 3, 640, 128, True), (1, 4, 4, 256, 128, True), (1, 16, 2, 384, 64, False), (2, 96, 48, 640, 128, True),
    (1, 128, 64, 512, 64, False),
]


@pytest.mark.parametrize("spill", [False, True], ids=["recompute", "spill"])
@pytest.mark.parametrize("B,Hq,Hkv,N,D,causal", CASES)
def test_gqa_forward_backward(attn, B, Hq, Hkv, N, D, causal, spill):
    q, k, v, d_o = make(20657 + Hq * 7 + N + D, B, Hq, Hkv, N, D)
    scale = 1 / math.sqrt(D)
    print(f"launch gqa fwd/bwd B{B} Hq{Hq} Hkv{Hkv} N{N} D{D} causal={causal}", flush=True)
    qd, kd, vd, dod = (t.cuda() for t in (q, k, v, d_o))
    o, lse = attn.gqa_fwd(qd, kd, vd, causal, scale)
    ws = attn.alloc_bwd_workspace(B, Hq, N, D, spill=spill)     # (spill: the form of the backward that stores dS)
    dq, dk, dv = attn.gqa_bwd(qd, kd, vd, o, dod, lse, causal, scale, workspace=ws)
    torch.cuda.synchronize()
    o_ref, lse_ref = orc.gqa_fwd(f64(q), f64(k), f64(v), causal, scale)
    eo = np.abs(f64(o.cpu()) - o_ref)
    assert np.isfinite(eo).all()
    assert eo.max() <= O_MAX and eo.mean() <= O_MEAN, (eo.max(), eo.mean())
    assert np.abs(f64(lse.cpu()) - lse_ref).max() <= LSE_MAX
    rq, rk, rv = orc.gqa_bwd(f64(q), f64(k), f64(v), f64(d_o), causal, scale)
    for name, g, r in (("dq", dq, rq), ("dk", dk, rk), ("dv", dv, rv)):
        g = f64(g.cpu())
        assert g.shape == r.shape, name
        assert relf(g, r) <= GRAD_RELF, (name, relf(g, r))
        check_grad(g, r, name)      # every head, every 32-row block, every element


def test_gqa_with_one_head_per_group_is_the_multi_head_call(attn):
    """Hkv == Hq must give the bits of the multi-head entry points (they are the same kernels)."""
    B, H, N, D = 1, 4, 384, 128
    q, k, v, d_o = make(31, B, H, H, N, D)
    qd, kd, vd, dod = (t.cuda() for t in (q, k, v, d_o))
    scale = 0.09
    o1, l1 = attn.attn_fwd(qd, kd, vd, True, scale)
    o2, l2 = attn.gqa_fwd(qd, kd, vd, True, scale)
    assert torch.equal(o1, o2) and torch.equal(l1, l2)
    g1 = attn.attn_bwd(qd, kd, vd, o1, dod, l1, True, scale)
    g2 = attn.gqa_bwd(qd, kd, vd, o1, dod, l1, True, scale)
    for a, b in zip(g1, g2):
        assert torch.equal(a, b)


def test_gqa_full_size_sampled(attn):
    """B=4, Hq=32, Hkv=8, N=4096, D=128 causal (the benchmark's grouped-query shape at a quarter of
    its batch): forward rows and the gradients of one key/value head and its group against the oracle."""
    B, Hq, Hkv, N, D, causal = 4, 32, 8, 4096, 128, True
    G = Hq // Hkv
    q, k, v, d_o = make(20665, B, Hq, Hkv, N, D)
    scale = 1 / math.sqrt(D)
    print("launch gqa full size", flush=True)
    qd, kd, vd, dod = (t.cuda() for t in (q, k, v, d_o))
    o, lse = attn.gqa_fwd(qd, kd, vd, causal, scale)
    dq, dk, dv = attn.gqa_bwd(qd, kd, vd, o, dod, lse, causal, scale)
    torch.cuda.synchronize()
    b, hk = 2, 5
    hs = slice(hk * G, (hk + 1) * G)
    qs, ks, vs, dos = f64(q[b:b + 1, hs]), f64(k[b:b + 1, hk:hk + 1]), f64(v[b:b + 1, hk:hk + 1]), f64(d_o[b:b + 1, hs])
    o_ref, lse_ref = orc.gqa_fwd(qs, ks, vs, causal, scale)
    eo = np.abs(f64(o[b:b + 1, hs].cpu()) - o_ref)
    assert eo.max() <= O_MAX and eo.mean() <= O_MEAN
    assert np.abs(f64(lse[b:b + 1, hs].cpu()) - lse_ref).max() <= LSE_MAX
    rq, rk, rv = orc.gqa_bwd(qs, ks, vs, dos, causal, scale)
    check_grad(f64(dq[b:b + 1, hs].cpu()), rq, "dq")
    check_grad(f64(dk[b:b + 1, hk:hk + 1].cpu()), rk, "dk")
    check_grad(f64(dv[b:b + 1, hk:hk + 1].cpu()), rv, "dv")
