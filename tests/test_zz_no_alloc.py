"""The allocation-free backward entry point (tk_attn_bwd_noalloc) against tk_attn_bwd.

tk_attn_bwd with a Delta-only workspace runs the same kernels; only the home of Delta differs (a scratch
array inside the library's device image instead of the caller's workspace), so the results must agree bit
for bit.  Two calls in a row, the
second on a smaller problem: the scratch keeps the first call's contents, which must not matter.
"""
import math

import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def attn():
    from paper_2410_20399_amd import attn as a
    a.load_library()
    return a


def run_pair(attn, B, H, N, D, causal, seed):
    g = torch.Generator().manual_seed(seed)
    q, k, v, d_o = (torch.randn(B, H, N, D, generator=g).to(torch.bfloat16).cuda() for _ in range(4))
    scale = 1 / math.sqrt(D)
    o, lse = attn.attn_fwd(q, k, v, causal, scale)
    ws = attn.alloc_bwd_workspace(B, H, N, D, spill=False)     # the form of tk_attn_bwd that keeps only Delta
    ref = attn.attn_bwd(q, k, v, o, d_o, lse, causal, scale, workspace=ws)
    out = [torch.full_like(q, 77.0) for _ in range(3)]
    print(f"launch tk_attn_bwd_noalloc B{B} H{H} N{N} D{D} causal={causal}", flush=True)
    rc = attn.tk_attn_bwd_noalloc(q, k, v, o, d_o, lse, *out, B, H, N, D, causal, scale)
    assert rc == attn.TK_OK, attn.status_string(rc)
    torch.cuda.synchronize()
    for name, a, b in zip(("dq", "dk", "dv"), out, ref):
        assert torch.isfinite(a.float()).all(), name
        assert torch.equal(a, b), (name, (a.float() - b.float()).abs().max().item())


def test_noalloc_backward_matches_workspace_backward_twice(attn):
    run_pair(attn, 2, 6, 1000, 128, True, 71)      # ragged length, 12000 rows of Delta
    run_pair(attn, 1, 3, 384, 64, False, 72)       # smaller: the scratch still holds the first call's Delta
    run_pair(attn, 4, 16, 4096, 128, True, 73)     # 262144 rows, a quarter of the limit


def test_noalloc_backward_limit(attn):
    rows = attn.tk_attn_bwd_noalloc_max_rows()
    B, H, N, D = 1, 1, rows + 1, 64
    t = torch.empty(16, dtype=torch.bfloat16, device="cuda")       # never touched: the size check comes first
    l = torch.empty(16, dtype=torch.float32, device="cuda")
    assert attn.tk_attn_bwd_noalloc(t, t, t, t, t, l, t, t, t, B, H, N, D, True, 0.125) == attn.TK_ERR_SCRATCH_LIMIT
