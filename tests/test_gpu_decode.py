"""GPU parity for the decode-shaped forward (tk_attn_decode): one query per head, grouped heads packed
into one tile, keys split over workgroups and merged.  Compared element by element with the fp64
oracle for Nq = 1 (where the causal mask removes nothing), and with tk_attn_fwd_rect on the GPU.
"""
import math

import numpy as np
import pytest
import torch

from oracle import attn_oracle as orc

pytestmark = pytest.mark.gpu

O_MAX, O_MEAN, LSE_MAX = 2e-2, 2e-3, 1e-3
GUARD = 1024


@pytest.fixture(scope="module")
def attn():
    from paper_2410_20399_amd import attn as a
    a.load_library()          # raises if the HIP library is missing: no fallback
    return a


def f64(t):
    return t.double().numpy()


CASES = [
    # B, Hq, Hkv, Nk, D        one split .. many splits, packed groups of 1..128 heads, a group too large to pack
    (1, 1, 1, 1, 64), (2, 4, 4, 77, 64), (1, 8, 2, 300, 128), (16, 32, 8, 8192, 128), (1, 8, 1, 100000, 128),
    (3, 16, 2, 5000, 64), (1, 128, 1, 4097, 128), (1, 256, 1, 1000, 64), (2, 6, 3, 12345, 128), (40, 8, 8, 2048, 64),
]


@pytest.mark.parametrize("B,Hq,Hkv,Nk,D", CASES)
def test_decode_matches_oracle(attn, B, Hq, Hkv, Nk, D):
    g = torch.Generator().manual_seed(4242 + Nk + Hq * 3 + D)
    q = torch.randn(B, Hq, 1, D, generator=g).to(torch.bfloat16)
    k = torch.randn(B, Hkv, Nk, D, generator=g).to(torch.bfloat16)
    v = torch.randn(B, Hkv, Nk, D, generator=g).to(torch.bfloat16)
    scale = 1 / math.sqrt(D)
    print(f"launch decode B{B} Hq{Hq} Hkv{Hkv} Nk{Nk} D{D}", flush=True)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    n = B * Hq * D
    obuf = torch.full((n + GUARD,), 77.0, dtype=torch.bfloat16, device="cuda")
    lbuf = torch.full((B * Hq + GUARD,), 77.0, dtype=torch.float32, device="cuda")
    o, lse = obuf[:n].view(B, Hq, 1, D), lbuf[:B * Hq].view(B, Hq, 1)
    need = attn.tk_attn_decode_workspace_bytes(B, Hq, Hkv, Nk, D)
    assert need > 0
    ws = torch.full((need + GUARD,), 0xFF, dtype=torch.uint8, device="cuda")      # stale contents must not matter
    assert attn.tk_attn_decode(qd, kd, vd, o, lse, B, Hq, Hkv, Nk, D, scale, ws, need) == attn.TK_OK
    torch.cuda.synchronize()
    assert bool((obuf[-GUARD:] == 77.0).all()) and bool((lbuf[-GUARD:] == 77.0).all())
    assert bool((ws[-GUARD:] == 0xFF).all()), "wrote past the end of the workspace"

    o_ref, lse_ref = orc.rect_fwd(f64(q), f64(k), f64(v), True, scale)     # one query: the mask removes nothing
    eo = np.abs(f64(o.cpu()) - o_ref)
    assert np.isfinite(eo).all()
    assert eo.max() <= O_MAX and eo.mean() <= O_MEAN, (eo.max(), eo.mean())
    assert np.abs(f64(lse.cpu()) - lse_ref).max() <= LSE_MAX

    # and against the plain entry point on the GPU (same kernel arithmetic; the merge reorders fp32 sums)
    o2, lse2 = attn.rect_fwd(qd, kd, vd, False, scale)
    torch.cuda.synchronize()
    assert float((o.float() - o2.float()).abs().max()) <= 2.0 ** -7 * max(1.0, float(o2.float().abs().max()))
    assert float((lse - lse2).abs().max()) <= 1e-4


def test_decode_rejects_bad_arguments(attn):
    t = torch.zeros(1, 4, 1, 64, dtype=torch.bfloat16, device="cuda")
    kk = torch.zeros(1, 2, 256, 64, dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros(1, 4, 1, dtype=torch.float32, device="cuda")
    need = attn.tk_attn_decode_workspace_bytes(1, 4, 2, 256, 64)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    assert attn.tk_attn_decode(t, kk, kk, t, lse, 1, 4, 2, 256, 64, 0.125, ws, need - 1) == attn.TK_ERR_WORKSPACE_TOO_SMALL
    assert attn.tk_attn_decode(t, kk, kk, t, lse, 1, 4, 3, 256, 64, 0.125, ws, need) == attn.TK_ERR_BAD_DIM
    assert attn.tk_attn_decode(t, kk, kk, t, lse, 1, 4, 2, 256, 64, 0.0, ws, need) == attn.TK_ERR_BAD_SCALE
    assert attn.tk_attn_decode(t, kk, kk, t, lse, 1, 4, 2, 256, 64, 0.125, ws, need) == attn.TK_OK
    torch.cuda.synchronize()
