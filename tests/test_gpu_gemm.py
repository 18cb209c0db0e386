"""GPU parity for the bf16 GEMM against the fp64 oracle.

Tolerance: fp32 accumulation of K bf16 products and one rounding to bf16.  Per element the error
is at most half a bf16 ulp of the result (2^-8 |ref|) plus the fp32 accumulation error, bounded
here by K * 2^-24 * sum_k |a_ik b_kj| <= K * 2^-24 * (a generous 4 * sqrt(K)) for unit-variance data."""
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


def make(M, N, K, seed):
    g = torch.Generator().manual_seed(seed)
    return torch.randn(M, K, generator=g).to(torch.bfloat16), torch.randn(K, N, generator=g).to(torch.bfloat16)


def tol(ref, K):
    return 2.0 ** -8 * np.abs(ref) + K * 2.0 ** -24 * 4 * np.sqrt(K) + 1e-6


@pytest.mark.parametrize("M,N,K", [(256, 256, 64), (256, 512, 128), (512, 256, 192), (768, 1280, 320), (256, 256, 2048)])
def test_gemm_small_full(attn, M, N, K):
    a, b = make(M, N, K, 840 + M + N + K)
    print(f"launch gemm M{M} N{N} K{K}", flush=True)
    c = attn.gemm(a.cuda(), b.cuda())
    torch.cuda.synchronize()
    ref = orc.gemm(a.double().numpy(), b.double().numpy())
    err = np.abs(c.cpu().double().numpy() - ref)
    assert (err <= tol(ref, K)).all(), float((err - tol(ref, K)).max())


@pytest.mark.parametrize("M,N,K", [(1, 8, 8), (5, 24, 40), (255, 264, 72), (257, 248, 200), (300, 520, 1000), (1000, 1000, 1000),
                                   (256, 256, 56), (513, 256, 64), (256, 776, 128)])
def test_gemm_edge_tiles(attn, M, N, K):
    """Shapes that are not multiples of the 256 x 256 x 64 tile: every element against the oracle, and the
    memory after C untouched (rows and columns past the end are masked, not clipped by luck)."""
    a, b = make(M, N, K, 1840 + M + N + K)
    print(f"launch gemm edge M{M} N{N} K{K}", flush=True)
    guard = 4096
    buf = torch.full((M * N + guard,), 77.0, dtype=torch.bfloat16, device="cuda")
    c = buf[:M * N].view(M, N)
    attn.gemm(a.cuda(), b.cuda(), out=c)
    torch.cuda.synchronize()
    assert bool((buf[M * N:] == 77.0).all()), "wrote past the end of C"
    ref = orc.gemm(a.double().numpy(), b.double().numpy())
    err = np.abs(c.cpu().double().numpy() - ref)
    assert np.isfinite(err).all()
    assert (err <= tol(ref, K)).all(), float((err - tol(ref, K)).max())


def test_gemm_full_size_sampled_and_reproducible(attn):
    M = N = K = 8192
    a, b = make(M, N, K, 8192)
    print("launch gemm 8192^3", flush=True)
    ad, bd = a.cuda(), b.cuda()
    c1 = attn.gemm(ad, bd)
    c2 = attn.gemm(ad, bd)
    torch.cuda.synchronize()
    assert torch.equal(c1, c2)
    rng = np.random.default_rng(7)
    rows = np.concatenate([rng.integers(0, M, 4000), [0, M - 1, 255, 256]])
    cols = np.concatenate([rng.integers(0, N, 4000), [0, N - 1, 256, 255]])
    ref = orc.gemm_elements(a.double().numpy(), b.double().numpy(), rows, cols)
    got = c1.cpu().double().numpy()[rows, cols]
    err = np.abs(got - ref)
    assert (err <= tol(ref, K)).all(), float((err - tol(ref, K)).max())
    # every 256 x 256 tile is touched: no tile left at its initial value
    c3 = torch.full((M, N), 12345.0, dtype=torch.bfloat16, device="cuda")
    attn.gemm(ad, bd, out=c3)
    torch.cuda.synchronize()
    assert torch.equal(c3, c1)
