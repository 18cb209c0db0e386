"""GPU parity for the rotary kernel against the fp64 oracle, element by element.

Tolerance: the kernel computes in fp32 and rounds once to bf16, so every element is within half a
bf16 ulp of the exact value (<= 2^-8 |ref|) plus the fp32 arithmetic error."""
import numpy as np
import pytest
import torch

from oracle import attn_oracle as orc

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def attn():
    from paper_2410_20399_amd import attn as a
    a.load_library()
    return a


def tables(N, D, seed):
    g = torch.Generator().manual_seed(seed)
    theta = (torch.rand(N, D // 2, generator=g) * 8 - 4)
    return torch.sin(theta).to(torch.bfloat16), torch.cos(theta).to(torch.bfloat16)


@pytest.mark.parametrize("B,H,N,D", [(1, 1, 1, 64), (2, 3, 100, 128), (1, 4, 257, 64), (2, 8, 1024, 128), (1, 2, 4096, 128)])
def test_rotary_matches_oracle(attn, B, H, N, D):
    g = torch.Generator().manual_seed(1207 + N + D)
    x = (2 * torch.randn(B, H, N, D, generator=g)).to(torch.bfloat16)
    sn, cs = tables(N, D, 77 + N)
    print(f"launch rotary B{B} H{H} N{N} D{D}", flush=True)
    o = attn.rotary(x.cuda(), sn.cuda(), cs.cuda())
    torch.cuda.synchronize()
    ref = orc.rotary(x.double().numpy(), sn.double().numpy(), cs.double().numpy())
    err = np.abs(o.cpu().double().numpy() - ref)
    assert (err <= 2.0 ** -8 * np.abs(ref) + 1e-5).all(), float((err - 2.0 ** -8 * np.abs(ref)).max())


def test_rotary_in_place_and_guard(attn):
    B, H, N, D = 2, 2, 333, 128
    g = torch.Generator().manual_seed(5)
    x = torch.randn(B, H, N, D, generator=g).to(torch.bfloat16)
    sn, cs = tables(N, D, 9)
    n = x.numel()
    buf = torch.full((n + 512,), 55.0, dtype=torch.bfloat16, device="cuda")
    xd = buf[:n].view(B, H, N, D)
    xd.copy_(x)
    sep = attn.rotary(xd.clone(), sn.cuda(), cs.cuda())
    attn.rotary(xd, sn.cuda(), cs.cuda(), out=xd)
    torch.cuda.synchronize()
    assert torch.equal(xd, sep)
    assert bool((buf[n:] == 55.0).all())
