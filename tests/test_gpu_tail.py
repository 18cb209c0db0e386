"""GPU parity for sequence lengths that are not a multiple of the 128-row tile.

The kernels work on the padded sequence: reads past the end are redirected to the last row, keys
past the end are masked, padded query rows get P = 0 in the backward, and nothing past the end is
stored.  Checked element by element against the fp64 oracle, and the bytes after the end of every
output are checked to be untouched.
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
    """A CUDA tensor of `shape` carved from a buffer with a sentinel-filled guard after it."""
    n = int(np.prod(shape))
    buf = torch.full((n + GUARD,), sentinel, dtype=dtype, device="cuda")
    return buf, buf[:n].view(shape)


CASES = [
    # B, Hq, Hkv, N, D, causal
    (1, 1, 1, 1, 64, False), (1, 1, 1, 1, 128, True), (2, 2, 2, 17, 128, True), (1, 3, 3, 100, 64, False),
    (1, 2, 2, 127, 128, True), (1, 2, 2, 129, 64, True), (2, 2, 2, 200, 128, False), (1, 3, 3, 333, 128, True),
    (1, 2, 2, 1000, 64, False), (1, 2, 2, 1001, 128, True), (1, 4, 2, 250, 128, True), (1, 8, 2, 77, 64, False),
    (1, 70, 70, 300, 64, True), (2, 160, 80, 130, 128, False),
]


@pytest.mark.parametrize("spill", [False, True], ids=["recompute", "spill"])
@pytest.mark.parametrize("B,Hq,Hkv,N,D,causal", CASES)
def test_tail_forward_backward(attn, B, Hq, Hkv, N, D, causal, spill):
    g = torch.Generator().manual_seed(20700 + N * 3 + D + Hq)
    q = torch.randn(B, Hq, N, D, generator=g).to(torch.bfloat16)
    k = torch.randn(B, Hkv, N, D, generator=g).to(torch.bfloat16)
    v = torch.randn(B, Hkv, N, D, generator=g).to(torch.bfloat16)
    d_o = torch.randn(B, Hq, N, D, generator=g).to(torch.bfloat16)
    scale = 1 / math.sqrt(D)
    print(f"launch tail fwd/bwd B{B} Hq{Hq} Hkv{Hkv} N{N} D{D} causal={causal}", flush=True)
    qd, kd, vd, dod = (t.cuda() for t in (q, k, v, d_o))
    obuf, o = guarded((B, Hq, N, D), torch.bfloat16, 77.0)
    lbuf, lse = guarded((B, Hq, N), torch.float32, 77.0)
    dqbuf, dq = guarded((B, Hq, N, D), torch.bfloat16, 77.0)
    dkbuf, dk = guarded((B, Hkv, N, D), torch.bfloat16, 77.0)
    dvbuf, dv = guarded((B, Hkv, N, D), torch.bfloat16, 77.0)
    ws = attn.alloc_bwd_workspace(B, Hq, N, D, spill=spill)     # (spill: the form of the backward that stores dS)
    ws.fill_(0xFF)
    rc = attn.tk_attn_fwd_gqa(qd, kd, vd, o, lse, B, Hq, Hkv, N, D, causal, scale)
    assert rc == attn.TK_OK
    rc = attn.tk_attn_bwd_gqa(qd, kd, vd, o, dod, lse, dq, dk, dv, B, Hq, Hkv, N, D, causal, scale, ws, ws.numel())
    assert rc == attn.TK_OK
    torch.cuda.synchronize()
    for buf in (obuf, lbuf, dqbuf, dkbuf, dvbuf):
        assert bool((buf[-GUARD:] == 77.0).all()), "wrote past the end of an output"

    o_ref, lse_ref = orc.gqa_fwd(f64(q), f64(k), f64(v), causal, scale)
    eo = np.abs(f64(o.cpu()) - o_ref)
    assert np.isfinite(eo).all()
    assert eo.max() <= O_MAX and eo.mean() <= O_MEAN, (eo.max(), eo.mean())
    assert np.abs(f64(lse.cpu()) - lse_ref).max() <= LSE_MAX
    rq, rk, rv = orc.gqa_bwd(f64(q), f64(k), f64(v), f64(d_o), causal, scale)
    for name, gpu, ref in (("dq", dq, rq), ("dk", dk, rk), ("dv", dv, rv)):
        gpu = f64(gpu.cpu())
        assert np.isfinite(gpu).all(), name
        if np.linalg.norm(ref) == 0:          # N = 1: softmax of one key, dQ = dK = 0 exactly
            assert np.abs(gpu).max() <= 1e-4, name
            continue
        assert relf(gpu, ref) <= GRAD_RELF, (name, relf(gpu, ref))
        check_grad(gpu, ref, name)      # every head, every 32-row block (the ragged last one too), every element


def test_long_ragged_sequence_sampled_through_the_causal_structure(attn):
    """N = 100003 (781 full tiles and a 35-row tail), causal.  The whole-head oracle is out of reach
    at this length, but the causal mask makes parts of the result small problems of their own:
      * the last 200 queries see every key, and the last 200 keys are seen by those queries only:
        O, LSE, dQ of those queries and dK, dV of those keys = a 200-query x N-key problem;
      * the first 300 queries see the first 300 keys only: their O, LSE, dQ = the N = 300 problem.
    """
    B, H, N, D = 1, 2, 100003, 128
    T, P = 200, 300
    scale = 1 / math.sqrt(D)
    g = torch.Generator().manual_seed(100003)
    q, k, v, d_o = (torch.randn(B, H, N, D, generator=g).to(torch.bfloat16) for _ in range(4))
    print(f"launch long ragged sequence N{N}", flush=True)
    qd, kd, vd, dod = (t.cuda() for t in (q, k, v, d_o))
    obuf, o = guarded((B, H, N, D), torch.bfloat16, 77.0)
    lbuf, lse = guarded((B, H, N), torch.float32, 77.0)
    dqbuf, dq = guarded((B, H, N, D), torch.bfloat16, 77.0)
    dkbuf, dk = guarded((B, H, N, D), torch.bfloat16, 77.0)
    dvbuf, dv = guarded((B, H, N, D), torch.bfloat16, 77.0)
    ws = attn.alloc_bwd_workspace(B, H, N, D)
    assert attn.tk_attn_fwd(qd, kd, vd, o, lse, B, H, N, D, True, scale) == attn.TK_OK
    assert attn.tk_attn_bwd(qd, kd, vd, o, dod, lse, dq, dk, dv, B, H, N, D, True, scale, ws, ws.numel()) == attn.TK_OK
    torch.cuda.synchronize()
    for buf in (obuf, lbuf, dqbuf, dkbuf, dvbuf):
        assert bool((buf[-GUARD:] == 77.0).all()), "wrote past the end of an output"

    # the last T queries against all keys
    o_ref, lse_ref = orc.rect_fwd(f64(q[:, :, -T:]), f64(k), f64(v), True, scale)
    eo = np.abs(f64(o[:, :, -T:].cpu()) - o_ref)
    assert eo.max() <= O_MAX and eo.mean() <= O_MEAN, (eo.max(), eo.mean())
    assert np.abs(f64(lse[:, :, -T:].cpu()) - lse_ref).max() <= LSE_MAX
    rq, rk, rv = orc.rect_bwd(f64(q[:, :, -T:]), f64(k), f64(v), f64(d_o[:, :, -T:]), True, scale)
    check_grad(f64(dq[:, :, -T:].cpu()), rq, "dq tail")
    check_grad(f64(dk[:, :, -T:].cpu()), rk[:, :, -T:], "dk tail")
    check_grad(f64(dv[:, :, -T:].cpu()), rv[:, :, -T:], "dv tail")

    # the first P queries: the N = P problem
    o_ref, lse_ref = orc.attn_fwd(f64(q[:, :, :P]), f64(k[:, :, :P]), f64(v[:, :, :P]), True, scale)
    eo = np.abs(f64(o[:, :, :P].cpu()) - o_ref)
    assert eo.max() <= O_MAX and eo.mean() <= O_MEAN
    assert np.abs(f64(lse[:, :, :P].cpu()) - lse_ref).max() <= LSE_MAX
    rq, _, _ = orc.attn_bwd(f64(q[:, :, :P]), f64(k[:, :, :P]), f64(v[:, :, :P]), f64(d_o[:, :, :P]), True, scale)
    check_grad(f64(dq[:, :, :P].cpu()), rq, "dq head")
    # everything in between was written
    for t in (o, dq, dk, dv):
        assert bool((t[:, :, ::1009, :] != 77.0).any(dim=-1).all())
