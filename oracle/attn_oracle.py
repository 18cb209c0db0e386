"""ctypes front end of the fp64 C oracle (oracle/attn_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
benchmark's cpu_baseline leg.  Arrays are numpy float64, row-major, shaped
[..., N, D]; leading axes are flattened into independent heads.  The
arithmetic lives in the C file, whose header states the definition it follows
(the PyTorch attention listing in the paper's introduction plus the temperature of the Appendix B.3 listing;
backward by the chain rule).
"""
import ctypes
import os

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        lib = ctypes.CDLL(path)
        dp = ctypes.POINTER(ctypes.c_double)
        lp = ctypes.POINTER(ctypes.c_long)
        L, I, F = ctypes.c_long, ctypes.c_int, ctypes.c_double
        lib.oracle_attn_fwd.argtypes = [dp, dp, dp, dp, dp, dp, L, L, L, I, F]
        lib.oracle_attn_fwd_rows.argtypes = [dp, dp, dp, lp, L, dp, dp, L, L, I, F]
        lib.oracle_attn_bwd.argtypes = [dp, dp, dp, dp, dp, dp, dp, dp, dp, L, L, L, I, F]
        lib.oracle_attn_ds.argtypes = [dp, dp, dp, dp, dp, L, L, L, I, F]
        lib.oracle_gqa_fwd.argtypes = [dp, dp, dp, dp, dp, L, L, L, L, L, I, F]
        lib.oracle_gqa_bwd.argtypes = [dp, dp, dp, dp, dp, dp, dp, L, L, L, L, L, I, F]
        lib.oracle_rect_fwd.argtypes = [dp, dp, dp, dp, dp, L, L, L, L, L, L, I, F]
        lib.oracle_rect_fwd.restype = ctypes.c_int
        lib.oracle_rect_bwd.argtypes = [dp, dp, dp, dp, dp, dp, dp, L, L, L, L, L, L, I, F]
        lib.oracle_rect_bwd.restype = ctypes.c_int
        lib.oracle_gemm.argtypes = [dp, dp, dp, L, L, L]
        lib.oracle_gemm.restype = ctypes.c_int
        lib.oracle_gemm_elements.argtypes = [dp, dp, lp, lp, L, dp, L, L, L]
        lib.oracle_gemm_elements.restype = ctypes.c_int
        lib.oracle_rotary.argtypes = [dp, dp, dp, dp, L, L, L]
        lib.oracle_rotary.restype = ctypes.c_int
        for f in (lib.oracle_attn_fwd, lib.oracle_attn_fwd_rows, lib.oracle_attn_bwd,
                  lib.oracle_attn_ds, lib.oracle_gqa_fwd, lib.oracle_gqa_bwd, lib.oracle_num_threads):
            f.restype = ctypes.c_int
        _lib = lib
    return _lib


def _c(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _heads(q, k, v):
    if q.shape != k.shape or q.shape != v.shape or q.ndim < 2:
        raise ValueError("q, k, v must share a shape [..., N, D]")
    N, D = q.shape[-2:]
    BH = int(np.prod(q.shape[:-2], dtype=np.int64)) if q.ndim > 2 else 1
    return BH, N, D


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def attn_fwd(q, k, v, causal: bool, scale: float, return_p: bool = False):
    """O [..., N, D], LSE [..., N] (and P [..., N, N] if return_p), all float64."""
    BH, N, D = _heads(q, k, v)
    q, qp = _c(q); k, kp = _c(k); v, vp = _c(v)
    o = np.empty(q.shape, np.float64)
    lse = np.empty(q.shape[:-1], np.float64)
    p = np.empty(q.shape[:-1] + (N,), np.float64) if return_p else None
    rc = _load().oracle_attn_fwd(qp, kp, vp, _c(o)[1], _c(lse)[1],
                                 _c(p)[1] if return_p else None, BH, N, D, int(causal), float(scale))
    if rc:
        raise RuntimeError(f"oracle_attn_fwd failed: {rc}")
    return (o, lse, p) if return_p else (o, lse)


def attn_fwd_rows(q, k, v, rows, causal: bool, scale: float):
    """Selected query rows of ONE head: q, k, v are [N, D]; returns O [len(rows), D], LSE [len(rows)]."""
    BH, N, D = _heads(q, k, v)
    if BH != 1:
        raise ValueError("attn_fwd_rows takes one head")
    q, qp = _c(q); k, kp = _c(k); v, vp = _c(v)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    o = np.empty((len(rows), D), np.float64)
    lse = np.empty((len(rows),), np.float64)
    rc = _load().oracle_attn_fwd_rows(qp, kp, vp, rows.ctypes.data_as(ctypes.POINTER(ctypes.c_long)),
                                      len(rows), _c(o)[1], _c(lse)[1], N, D, int(causal), float(scale))
    if rc:
        raise RuntimeError(f"oracle_attn_fwd_rows failed: {rc}")
    return o, lse


def attn_bwd(q, k, v, d_o, causal: bool, scale: float, return_stats: bool = False):
    """dQ, dK, dV [..., N, D] float64 (and Delta, LSE [..., N] if return_stats)."""
    BH, N, D = _heads(q, k, v)
    if d_o.shape != q.shape:
        raise ValueError("d_o must have q's shape")
    q, qp = _c(q); k, kp = _c(k); v, vp = _c(v); d_o, dop = _c(d_o)
    dq = np.empty(q.shape, np.float64)
    dk = np.empty(q.shape, np.float64)
    dv = np.empty(q.shape, np.float64)
    delta = np.empty(q.shape[:-1], np.float64)
    lse = np.empty(q.shape[:-1], np.float64)
    rc = _load().oracle_attn_bwd(qp, kp, vp, dop, _c(dq)[1], _c(dk)[1], _c(dv)[1],
                                 _c(delta)[1], _c(lse)[1], BH, N, D, int(causal), float(scale))
    if rc:
        raise RuntimeError(f"oracle_attn_bwd failed: {rc}")
    return (dq, dk, dv, delta, lse) if return_stats else (dq, dk, dv)


def attn_ds(q, k, v, d_o, causal: bool, scale: float):
    """dS [..., N, N] float64 (tiny shapes; for invariant tests)."""
    BH, N, D = _heads(q, k, v)
    q, qp = _c(q); k, kp = _c(k); v, vp = _c(v); d_o, dop = _c(d_o)
    ds = np.empty(q.shape[:-1] + (N,), np.float64)
    rc = _load().oracle_attn_ds(qp, kp, vp, dop, _c(ds)[1], BH, N, D, int(causal), float(scale))
    if rc:
        raise RuntimeError(f"oracle_attn_ds failed: {rc}")
    return ds


def _gqa_dims(q, k, v):
    if q.ndim != 4 or k.ndim != 4 or k.shape != v.shape:
        raise ValueError("q must be [B, Hq, N, D]; k, v [B, Hkv, N, D]")
    B, Hq, N, D = q.shape
    if k.shape[0] != B or k.shape[2:] != (N, D) or Hq % k.shape[1]:
        raise ValueError("k, v must be [B, Hkv, N, D] with Hkv dividing Hq")
    return B, Hq, k.shape[1], N, D


def gqa_fwd(q, k, v, causal: bool, scale: float):
    """Grouped-query attention: q [B,Hq,N,D], k, v [B,Hkv,N,D] -> O [B,Hq,N,D], LSE [B,Hq,N] (float64).

    Query head h uses key/value head h // (Hq // Hkv)."""
    B, Hq, Hkv, N, D = _gqa_dims(q, k, v)
    q, qp = _c(q); k, kp = _c(k); v, vp = _c(v)
    o = np.empty(q.shape, np.float64)
    lse = np.empty(q.shape[:-1], np.float64)
    rc = _load().oracle_gqa_fwd(qp, kp, vp, _c(o)[1], _c(lse)[1], B, Hq, Hkv, N, D, int(causal), float(scale))
    if rc:
        raise RuntimeError(f"oracle_gqa_fwd failed: {rc}")
    return o, lse


def gqa_bwd(q, k, v, d_o, causal: bool, scale: float):
    """dQ [B,Hq,N,D], dK, dV [B,Hkv,N,D] (float64): dK, dV summed over each group's query heads."""
    B, Hq, Hkv, N, D = _gqa_dims(q, k, v)
    if d_o.shape != q.shape:
        raise ValueError("d_o must have q's shape")
    q, qp = _c(q); k, kp = _c(k); v, vp = _c(v); d_o, dop = _c(d_o)
    dq = np.empty(q.shape, np.float64)
    dk = np.empty(k.shape, np.float64)
    dv = np.empty(k.shape, np.float64)
    rc = _load().oracle_gqa_bwd(qp, kp, vp, dop, _c(dq)[1], _c(dk)[1], _c(dv)[1],
                                B, Hq, Hkv, N, D, int(causal), float(scale))
    if rc:
        raise RuntimeError(f"oracle_gqa_bwd failed: {rc}")
    return dq, dk, dv


def _rect_dims(q, k, v, causal):
    if q.ndim != 4 or k.ndim != 4 or k.shape != v.shape:
        raise ValueError("q must be [B, Hq, Nq, D]; k, v [B, Hkv, Nk, D]")
    B, Hq, Nq, D = q.shape
    if k.shape[0] != B or k.shape[3] != D or Hq % k.shape[1]:
        raise ValueError("k, v must be [B, Hkv, Nk, D] with Hkv dividing Hq")
    if causal and Nq > k.shape[2]:
        raise ValueError("the causal mask needs Nq <= Nk")
    return B, Hq, k.shape[1], Nq, k.shape[2], D


def rect_fwd(q, k, v, causal: bool, scale: float):
    """Attention with Nq queries and Nk keys: q [B,Hq,Nq,D], k, v [B,Hkv,Nk,D] -> O [B,Hq,Nq,D],
    LSE [B,Hq,Nq] (float64).  Causal: query i attends to keys j <= i + (Nk - Nq) (sequences
    aligned at their ends; needs Nq <= Nk)."""
    B, Hq, Hkv, Nq, Nk, D = _rect_dims(q, k, v, causal)
    q, qp = _c(q); k, kp = _c(k); v, vp = _c(v)
    o = np.empty(q.shape, np.float64)
    lse = np.empty(q.shape[:-1], np.float64)
    rc = _load().oracle_rect_fwd(qp, kp, vp, _c(o)[1], _c(lse)[1], B, Hq, Hkv, Nq, Nk, D, int(causal), float(scale))
    if rc:
        raise RuntimeError(f"oracle_rect_fwd failed: {rc}")
    return o, lse


def rect_bwd(q, k, v, d_o, causal: bool, scale: float):
    """dQ [B,Hq,Nq,D], dK, dV [B,Hkv,Nk,D] (float64) of rect_fwd for L = sum O * dO."""
    B, Hq, Hkv, Nq, Nk, D = _rect_dims(q, k, v, causal)
    if d_o.shape != q.shape:
        raise ValueError("d_o must have q's shape")
    q, qp = _c(q); k, kp = _c(k); v, vp = _c(v); d_o, dop = _c(d_o)
    dq = np.empty(q.shape, np.float64)
    dk = np.empty(k.shape, np.float64)
    dv = np.empty(k.shape, np.float64)
    rc = _load().oracle_rect_bwd(qp, kp, vp, dop, _c(dq)[1], _c(dk)[1], _c(dv)[1],
                                 B, Hq, Hkv, Nq, Nk, D, int(causal), float(scale))
    if rc:
        raise RuntimeError(f"oracle_rect_bwd failed: {rc}")
    return dq, dk, dv


def rotary(x, sin, cos):
    """Rotary positional encoding: x [..., N, D], sin, cos [N, D/2] -> o [..., N, D] (float64).

    o[..., :D/2] = x1 cos - x2 sin, o[..., D/2:] = x2 cos + x1 sin with x1, x2 the two halves of x."""
    N, D = x.shape[-2:]
    if sin.shape != (N, D // 2) or cos.shape != (N, D // 2) or D % 2:
        raise ValueError("sin, cos must be [N, D/2]")
    BH = int(np.prod(x.shape[:-2], dtype=np.int64)) if x.ndim > 2 else 1
    x, xp = _c(x); sin, sp = _c(sin); cos, cp = _c(cos)
    o = np.empty(x.shape, np.float64)
    rc = _load().oracle_rotary(xp, sp, cp, _c(o)[1], BH, N, D)
    if rc:
        raise RuntimeError(f"oracle_rotary failed: {rc}")
    return o


def gemm(a, b):
    """C = A B for A [M, K], B [K, N] (float64)."""
    if a.ndim != 2 or b.ndim != 2 or a.shape[1] != b.shape[0]:
        raise ValueError("a must be [M, K], b [K, N]")
    M, K = a.shape
    N = b.shape[1]
    a, ap = _c(a); b, bp = _c(b)
    c = np.empty((M, N), np.float64)
    rc = _load().oracle_gemm(ap, bp, _c(c)[1], M, N, K)
    if rc:
        raise RuntimeError(f"oracle_gemm failed: {rc}")
    return c


def gemm_elements(a, b, rows, cols):
    """Selected elements C[rows[e], cols[e]] of A B (float64)."""
    if a.ndim != 2 or b.ndim != 2 or a.shape[1] != b.shape[0]:
        raise ValueError("a must be [M, K], b [K, N]")
    M, K = a.shape
    N = b.shape[1]
    a, ap = _c(a); b, bp = _c(b)
    rows = np.ascontiguousarray(rows, dtype=np.int64); cols = np.ascontiguousarray(cols, dtype=np.int64)
    out = np.empty((len(rows),), np.float64)
    lp = ctypes.POINTER(ctypes.c_long)
    rc = _load().oracle_gemm_elements(ap, bp, rows.ctypes.data_as(lp), cols.ctypes.data_as(lp), len(rows),
                                      _c(out)[1], M, N, K)
    if rc:
        raise RuntimeError(f"oracle_gemm_elements failed: {rc}")
    return out
