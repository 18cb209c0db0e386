"""GPU parity for different numbers of queries and keys (tk_attn_fwd_rect / tk_attn_bwd_rect).

Decode shapes (one or a few queries against a long history), cross attention with more queries
than keys, lengths that are not multiples of any tile size, offsets Nk - Nq that are not multiples
of the 32-row block, grouped heads, and launches with more work units than compute units.  With
the causal mask query i sees keys j <= i + (Nk - Nq).  Checked element by element against the fp64
oracle; the bytes after the end of every output are checked to be untouched.
"""
import math

import numpy as np
import pytest
import torch

from oracle import attn_oracle as orc
from grad_check import check_grad

pytestmark = pytest.mark.gpu

O_MAX, O_MEAN, LSE_MAX, GRAD_RELF = 2e-2, 2e-3, 1e-3, 3e-2
GUARD = 1024      # elements of padding after each output, filled with a sentinel


@pytest.fixture(scope="module")
def attn():
    from paper_2410_20399_amd import attn as a
    a.load_library()          # raises if the HIP library is missing: no fallback
    return a


def f64(t):
    return t.double().numpy()


def relf(a, b):
    return float(np.linalg.norm(a - b) / np.linalg.norm(b))


def guarded(shape, dtype, sentinel):
    n = int(np.prod(shape))
    buf = torch.full((n + GUARD,), sentinel, dtype=dtype, device="cuda")
    return buf, buf[:n].view(shape)


CASES = [
    # B, Hq, Hkv, Nq, Nk, D, causal
    (2, 4, 2, 1, 1000, 128, True), (2, 4, 2, 1, 1000, 128, False), (1, 2, 2, 1, 129, 64, True),
    (1, 2, 2, 5, 64, 128, True), (1, 2, 2, 100, 300, 128, True), (1, 2, 1, 128, 256, 64, True),
    (1, 2, 2, 130, 1000, 128, True), (1, 3, 3, 257, 290, 64, True), (1, 2, 2, 96, 127, 128, True),
    (2, 2, 2, 64, 4096, 128, False), (1, 2, 2, 300, 100, 128, False), (1, 2, 2, 1000, 1, 64, False),
    (1, 4, 2, 513, 77, 128, False), (1, 2, 2, 256, 512, 128, True), (1, 2, 2, 512, 256, 64, False),
    (1, 2, 2, 200, 200, 64, True), (2, 160, 80, 70, 700, 128, True), (1, 300, 300, 40, 300, 64, False),
    (1, 2, 2, 2048, 4096, 128, True), (1, 2, 1, 1500, 1531, 64, True),
]


@pytest.mark.parametrize("spill", [False, True], ids=["recompute", "spill"])
@pytest.mark.parametrize("B,Hq,Hkv,Nq,Nk,D,causal", CASES)
def test_rect_forward_backward(attn, B, Hq, Hkv, Nq, Nk, D, causal, spill):
    g = torch.Generator().manual_seed(115200 + Nq * 7 + Nk * 3 + D + Hq)
    q = torch.randn(B, Hq, Nq, D, generator=g).to(torch.bfloat16)
    k = torch.randn(B, Hkv, Nk, D, generator=g).to(torch.bfloat16)
    v = torch.randn(B, Hkv, Nk, D, generator=g).to(torch.bfloat16)
    d_o = torch.randn(B, Hq, Nq, D, generator=g).to(torch.bfloat16)
    scale = 1 / math.sqrt(D)
    print(f"launch rect fwd/bwd B{B} Hq{Hq} Hkv{Hkv} Nq{Nq} Nk{Nk} D{D} causal={causal}", flush=True)
    qd, kd, vd, dod = (t.cuda() for t in (q, k, v, d_o))
    obuf, o = guarded((B, Hq, Nq, D), torch.bfloat16, 77.0)
    lbuf, lse = guarded((B, Hq, Nq), torch.float32, 77.0)
    dqbuf, dq = guarded((B, Hq, Nq, D), torch.bfloat16, 77.0)
    dkbuf, dk = guarded((B, Hkv, Nk, D), torch.bfloat16, 77.0)
    dvbuf, dv = guarded((B, Hkv, Nk, D), torch.bfloat16, 77.0)
    ws = attn.alloc_bwd_workspace(B, Hq, Nq, D, spill=spill, Nk=Nk)     # (spill: the form of the backward that stores dS)
    ws.fill_(0xFF)
    rc = attn.tk_attn_fwd_rect(qd, kd, vd, o, lse, B, Hq, Hkv, Nq, Nk, D, causal, scale)
    assert rc == attn.TK_OK
    rc = attn.tk_attn_bwd_rect(qd, kd, vd, o, dod, lse, dq, dk, dv, B, Hq, Hkv, Nq, Nk, D, causal, scale, ws, ws.numel())
    assert rc == attn.TK_OK
    torch.cuda.synchronize()
    for buf in (obuf, lbuf, dqbuf, dkbuf, dvbuf):
        assert bool((buf[-GUARD:] == 77.0).all()), "wrote past the end of an output"

    o_ref, lse_ref = orc.rect_fwd(f64(q), f64(k), f64(v), causal, scale)
    eo = np.abs(f64(o.cpu()) - o_ref)
    assert np.isfinite(eo).all()
    assert eo.max() <= O_MAX and eo.mean() <= O_MEAN, (eo.max(), eo.mean())
    assert np.abs(f64(lse.cpu()) - lse_ref).max() <= LSE_MAX
    rq, rk, rv = orc.rect_bwd(f64(q), f64(k), f64(v), f64(d_o), causal, scale)
    for name, gpu, ref in (("dq", dq, rq), ("dk", dk, rk), ("dv", dv, rv)):
        gpu = f64(gpu.cpu())
        assert np.isfinite(gpu).all(), name
        if np.abs(ref).max() <= 1e-12:        # one key: softmax of a single score, dQ = dK = 0
            assert np.abs(gpu).max() <= 1e-4, name
            continue
        assert relf(gpu, ref) <= GRAD_RELF, (name, relf(gpu, ref))
        check_grad(gpu, ref, name)      # every head, every 32-row block, every element


def test_rect_equal_lengths_match_the_square_entry_points(attn):
    """Nq == Nk through the _rect calls gives bit-identical results to the _gqa calls."""
    B, Hq, Hkv, N, D = 2, 4, 2, 384, 128
    g = torch.Generator().manual_seed(384128)
    q, d_o = (torch.randn(B, Hq, N, D, generator=g).to(torch.bfloat16).cuda() for _ in range(2))
    k, v = (torch.randn(B, Hkv, N, D, generator=g).to(torch.bfloat16).cuda() for _ in range(2))
    scale = 1 / math.sqrt(D)
    print("launch rect vs gqa, equal lengths", flush=True)
    for causal in (False, True):
        o1, l1 = attn.rect_fwd(q, k, v, causal, scale)
        o2, l2 = attn.gqa_fwd(q, k, v, causal, scale)
        g1 = attn.rect_bwd(q, k, v, o1, d_o, l1, causal, scale)
        g2 = attn.gqa_bwd(q, k, v, o2, d_o, l2, causal, scale)
        torch.cuda.synchronize()
        assert torch.equal(o1, o2) and torch.equal(l1, l2)
        for a, b in zip(g1, g2):
            assert torch.equal(a, b)


def test_rect_rejects_causal_with_more_queries_than_keys(attn):
    t = torch.zeros(1, 1, 256, 64, dtype=torch.bfloat16, device="cuda")
    kk = torch.zeros(1, 1, 128, 64, dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros(1, 1, 256, dtype=torch.float32, device="cuda")
    assert attn.tk_attn_fwd_rect(t, kk, kk, t, lse, 1, 1, 1, 256, 128, 64, True, 0.125) == attn.TK_ERR_BAD_DIM
    assert attn.tk_attn_fwd_rect(t, kk, kk, t, lse, 1, 1, 1, 256, 128, 64, False, 0.125) == attn.TK_OK
    torch.cuda.synchronize()
