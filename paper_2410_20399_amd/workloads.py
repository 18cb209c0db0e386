"""Seeded synthetic attention workloads (inputs only; none of the method's arithmetic).

Both the HIP path's tests/benchmark and the CPU oracle's tests draw their
inputs here, so the two sides see the same bf16 bit patterns.  The recipe:
one CPU ``torch.Generator`` seeded with ``20399 + index``; Q, K, V, dO drawn in
that order as float32 standard normals of shape [B, H, N, D] (K, V: [B, Hkv, N, D]) and rounded to
bf16 (round-to-nearest-even); for workloads with ``q_mul`` the rounded Q is
multiplied by that power of two (exact in bf16).
"""
from dataclasses import dataclass
import math

import torch


@dataclass(frozen=True)
class Workload:
    index: int
    name: str
    B: int
    H: int
    N: int
    D: int
    causal: bool
    backward: bool
    q_mul: float = 1.0
    Hkv: int = 0          # key/value heads (grouped-query attention); 0 = H, plain multi-head

    @property
    def kv_heads(self) -> int:
        return self.Hkv or self.H

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.D)

    @property
    def seed(self) -> int:
        return 20399 + self.index

    def fwd_flops(self) -> float:
        """4*B*H*N^2*D, halved when causal (the convention of the attention-kernel literature)."""
        f = 4.0 * self.B * self.H * self.N * self.N * self.D
        return f / 2 if self.causal else f

    def bwd_flops(self) -> float:
        """Five matmuls against the forward's two: 2.5x the forward count."""
        return 2.5 * self.fwd_flops()


# The five benchmark configurations, plus the shape the performance target is quoted on.
WORKLOADS = {
    1: Workload(1, "fwd_nc_b1_h1_n128_d64", 1, 1, 128, 64, False, False),
    2: Workload(2, "fwd_nc_b16_h16_n1024_d64", 16, 16, 1024, 64, False, False),
    3: Workload(3, "fwd_causal_b16_h16_n4096_d128_q4", 16, 16, 4096, 128, True, False, 4.0),
    4: Workload(4, "fwdbwd_causal_b16_h16_n4096_d64", 16, 16, 4096, 64, True, True),
    5: Workload(5, "fwdbwd_causal_b1_h16_n16384_d128", 1, 16, 16384, 128, True, True),
    6: Workload(6, "fwdbwd_causal_b16_h16_n4096_d128", 16, 16, 4096, 128, True, True),
    7: Workload(7, "fwdbwd_nc_b16_h16_n4096_d128", 16, 16, 4096, 128, False, True),
    # grouped-query variant of the target shape: same query-side work, 4 query heads per key/value head
    8: Workload(8, "fwdbwd_causal_gqa_b8_hq32_hkv8_n4096_d128", 8, 32, 4096, 128, True, True, 1.0, 8),
}


def make_inputs(w: Workload, need_do: bool = None):
    """Return (q, k, v, d_o) CPU bf16 tensors [B, H, N, D] (k, v: [B, Hkv, N, D]); d_o is None unless asked for."""
    if need_do is None:
        need_do = w.backward
    g = torch.Generator().manual_seed(w.seed)
    shape = (w.B, w.H, w.N, w.D)
    kv_shape = (w.B, w.kv_heads, w.N, w.D)
    q = torch.randn(shape, generator=g, dtype=torch.float32).to(torch.bfloat16)
    k = torch.randn(kv_shape, generator=g, dtype=torch.float32).to(torch.bfloat16)
    v = torch.randn(kv_shape, generator=g, dtype=torch.float32).to(torch.bfloat16)
    d_o = torch.randn(shape, generator=g, dtype=torch.float32).to(torch.bfloat16) if need_do else None
    if w.q_mul != 1.0:
        q = q * w.q_mul
    return q, k, v, d_o


def make_small(seed: int, B: int, H: int, N: int, D: int, q_mul: float = 1.0):
    """Ad-hoc shape with the same recipe (for parity cases outside the table)."""
    return make_inputs(Workload(seed - 20399, f"adhoc_{B}_{H}_{N}_{D}", B, H, N, D, False, True, q_mul), True)
