"""The entry points under HIP graph capture: they allocate nothing, never synchronise and launch
only kernels, so a forward+backward step can be captured once and replayed.  Every replay (with
new inputs copied into the captured buffers, and ordinary eager work and synchronisation between
replays) must reproduce the eager results bit for bit.
"""
import math

import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def attn():
    from paper_2410_20399_amd import attn as a
    a.load_library()          # raises if the HIP library is missing: no fallback
    return a


@pytest.mark.parametrize("B,Hq,Hkv,Nq,Nk,D,causal", [(2, 4, 4, 512, 512, 128, True), (1, 4, 2, 200, 333, 64, True),
                                                      (2, 2, 2, 384, 384, 64, False)])
def test_captured_step_replays_bit_exact(attn, B, Hq, Hkv, Nq, Nk, D, causal):
    dev = "cuda:0"
    scale = 1 / math.sqrt(D)
    gen = torch.Generator().manual_seed(586 + Nq + Nk)

    def draw(*shape):
        return torch.randn(*shape, generator=gen).to(torch.bfloat16)

    q, d_o = torch.empty(B, Hq, Nq, D, dtype=torch.bfloat16, device=dev), torch.empty(B, Hq, Nq, D, dtype=torch.bfloat16, device=dev)
    k, v = torch.empty(B, Hkv, Nk, D, dtype=torch.bfloat16, device=dev), torch.empty(B, Hkv, Nk, D, dtype=torch.bfloat16, device=dev)
    o, dq = torch.empty_like(q), torch.empty_like(q)
    dk, dv = torch.empty_like(k), torch.empty_like(v)
    lse = torch.empty(B, Hq, Nq, dtype=torch.float32, device=dev)
    ws = attn.alloc_bwd_workspace(B, Hq, Nq, D, dev)

    def step(stream):
        assert attn.tk_attn_fwd_rect(q, k, v, o, lse, B, Hq, Hkv, Nq, Nk, D, causal, scale, stream) == attn.TK_OK
        assert attn.tk_attn_bwd_rect(q, k, v, o, d_o, lse, dq, dk, dv, B, Hq, Hkv, Nq, Nk, D, causal, scale,
                                     ws, ws.numel(), stream) == attn.TK_OK

    def load_inputs():
        for dst, shape in ((q, q.shape), (k, k.shape), (v, v.shape), (d_o, d_o.shape)):
            dst.copy_(draw(*shape))

    print(f"capture B{B} Hq{Hq} Hkv{Hkv} Nq{Nq} Nk{Nk} D{D} causal={causal}", flush=True)
    load_inputs()
    step(torch.cuda.current_stream())          # warm-up outside the capture (module load, first launch)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        step(torch.cuda.current_stream())      # the capturing stream
    torch.cuda.synchronize()

    for replay in range(3):
        load_inputs()
        step(torch.cuda.current_stream())      # eager
        torch.cuda.synchronize()
        want = [t.clone() for t in (o, lse, dq, dk, dv)]
        for t in (o, lse, dq, dk, dv):
            t.fill_(7.0)                       # eager work between replays; the graph must overwrite all of it
        ws.fill_(0xFF)
        torch.cuda.synchronize()
        print(f"replay {replay}", flush=True)
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip((o, lse, dq, dk, dv), want):
            assert torch.equal(got, ref), replay
