"""Thin Python binding of the C ABI in include/tk_attn.h (argument marshalling only).

The functions named ``tk_*`` take torch CUDA tensors (used purely as device
buffers) and forward pointers, sizes and the current HIP stream to the
shared library; every step of the computation runs in the HIP kernels.
There is no fallback: if the library is missing, loading raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtk_attn.so")

TK_OK = 0
TK_ERR_NULL_PTR = -1
TK_ERR_BAD_DIM = -2
TK_ERR_MISALIGNED = -3
TK_ERR_BAD_SCALE = -4
TK_ERR_WORKSPACE_TOO_SMALL = -5
TK_ERR_LAUNCH = -6
TK_ERR_SCRATCH_LIMIT = -7

EXPORTS = ("tk_attn_fwd", "tk_attn_bwd", "tk_attn_bwd_workspace_bytes", "tk_attn_bwd_delta",
           "tk_attn_bwd_dkdv", "tk_attn_bwd_dq", "tk_attn_fwd_gqa", "tk_attn_bwd_gqa", "tk_attn_bwd_dkdv_gqa",
           "tk_attn_bwd_dq_gqa", "tk_attn_bwd_dq_delta", "tk_attn_fwd_rect", "tk_attn_bwd_rect", "tk_attn_decode",
           "tk_attn_decode_workspace_bytes", "tk_attn_decode_plan", "tk_attn_bwd_noalloc", "tk_attn_bwd_noalloc_max_rows",
           "tk_attn_bwd_spill_workspace_bytes", "tk_attn_bwd_ds_bytes", "tk_attn_bwd_dkdv_ds", "tk_attn_bwd_dq_from_ds", "tk_rotary", "tk_gemm", "tk_mfma_probe", "tk_status_string", "tk_attn_version")

_lib = None


class TkAttnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


def load_library(path: str = LIB_PATH) -> ctypes.CDLL:
    """Load libtk_attn.so (built by paper_2410_20399_amd/build.py). Raises if it is absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(path):
        raise FileNotFoundError(
            f"{path} not found: build it with `python -m paper_2410_20399_amd.build` "
            "(there is no CPU fallback)")
    lib = ctypes.CDLL(path)
    vp, fp, i, f, sz = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
    lib.tk_attn_fwd.argtypes = [vp, vp, vp, vp, fp, i, i, i, i, i, f, vp]
    lib.tk_attn_fwd.restype = i
    lib.tk_attn_bwd.argtypes = [vp, vp, vp, vp, vp, fp, vp, vp, vp, i, i, i, i, i, f, vp, sz, vp]
    lib.tk_attn_bwd.restype = i
    lib.tk_attn_bwd_noalloc.argtypes = [vp, vp, vp, vp, vp, fp, vp, vp, vp, i, i, i, i, i, f, vp]
    lib.tk_attn_bwd_noalloc.restype = i
    lib.tk_attn_bwd_noalloc_max_rows.argtypes = []
    lib.tk_attn_bwd_noalloc_max_rows.restype = sz
    lib.tk_attn_bwd_spill_workspace_bytes.argtypes = [i, i, i, i, i]
    lib.tk_attn_bwd_spill_workspace_bytes.restype = sz
    lib.tk_attn_bwd_ds_bytes.argtypes = [i, i, i, i, i]
    lib.tk_attn_bwd_ds_bytes.restype = sz
    lib.tk_attn_bwd_dkdv_ds.argtypes = [vp, vp, vp, vp, fp, fp, vp, vp, vp, i, i, i, i, i, i, f, vp]
    lib.tk_attn_bwd_dkdv_ds.restype = i
    lib.tk_attn_bwd_dq_from_ds.argtypes = [vp, vp, vp, i, i, i, i, i, i, f, vp]
    lib.tk_attn_bwd_dq_from_ds.restype = i
    lib.tk_attn_bwd_workspace_bytes.argtypes = [i, i, i, i]
    lib.tk_attn_bwd_workspace_bytes.restype = sz
    lib.tk_attn_bwd_delta.argtypes = [vp, vp, fp, i, i, i, i, vp]
    lib.tk_attn_bwd_delta.restype = i
    lib.tk_attn_bwd_dkdv.argtypes = [vp, vp, vp, vp, fp, fp, vp, vp, i, i, i, i, i, f, vp]
    lib.tk_attn_bwd_dkdv.restype = i
    lib.tk_attn_bwd_dq.argtypes = [vp, vp, vp, vp, fp, fp, vp, i, i, i, i, i, f, vp]
    lib.tk_attn_bwd_dq.restype = i
    lib.tk_attn_fwd_gqa.argtypes = [vp, vp, vp, vp, fp, i, i, i, i, i, i, f, vp]
    lib.tk_attn_fwd_gqa.restype = i
    lib.tk_attn_bwd_gqa.argtypes = [vp, vp, vp, vp, vp, fp, vp, vp, vp, i, i, i, i, i, i, f, vp, sz, vp]
    lib.tk_attn_bwd_gqa.restype = i
    lib.tk_attn_bwd_dkdv_gqa.argtypes = [vp, vp, vp, vp, fp, fp, vp, vp, i, i, i, i, i, i, f, vp]
    lib.tk_attn_bwd_dkdv_gqa.restype = i
    lib.tk_attn_bwd_dq_gqa.argtypes = [vp, vp, vp, vp, fp, fp, vp, i, i, i, i, i, i, f, vp]
    lib.tk_attn_bwd_dq_gqa.restype = i
    lib.tk_attn_bwd_dq_delta.argtypes = [vp, vp, vp, vp, vp, fp, fp, vp, i, i, i, i, i, i, f, vp]
    lib.tk_attn_bwd_dq_delta.restype = i
    lib.tk_attn_fwd_rect.argtypes = [vp, vp, vp, vp, fp, i, i, i, i, i, i, i, f, vp]
    lib.tk_attn_fwd_rect.restype = i
    lib.tk_attn_bwd_rect.argtypes = [vp, vp, vp, vp, vp, fp, vp, vp, vp, i, i, i, i, i, i, i, f, vp, sz, vp]
    lib.tk_attn_bwd_rect.restype = i
    lib.tk_attn_decode.argtypes = [vp, vp, vp, vp, fp, i, i, i, i, i, f, vp, sz, vp]
    lib.tk_attn_decode.restype = i
    lib.tk_attn_decode_plan.argtypes = [i, i, i, i, i, i, ctypes.POINTER(ctypes.c_int)]
    lib.tk_attn_decode_plan.restype = i
    lib.tk_attn_decode_workspace_bytes.argtypes = [i, i, i, i, i]
    lib.tk_attn_decode_workspace_bytes.restype = sz
    lib.tk_gemm.argtypes = [vp, vp, vp, i, i, i, vp]
    lib.tk_gemm.restype = i
    lib.tk_rotary.argtypes = [vp, vp, vp, vp, i, i, i, i, vp]
    lib.tk_rotary.restype = i
    lib.tk_mfma_probe.argtypes = [vp, fp, i, i, vp]
    lib.tk_mfma_probe.restype = i
    lib.tk_status_string.argtypes = [i]
    lib.tk_status_string.restype = ctypes.c_char_p
    lib.tk_attn_version.argtypes = []
    lib.tk_attn_version.restype = i
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().tk_status_string(int(status)).decode()


def version() -> int:
    return int(load_library().tk_attn_version())


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _check_bf16(name, t, shape=None):
    if not (t.is_cuda and t.dtype == torch.bfloat16 and t.is_contiguous()):
        raise ValueError(f"{name} must be a contiguous CUDA bf16 tensor")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} has shape {tuple(t.shape)}, expected {tuple(shape)}")


def _check_f32(name, t, shape):
    if not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and tuple(t.shape) == tuple(shape)):
        raise ValueError(f"{name} must be a contiguous CUDA fp32 tensor of shape {tuple(shape)}")


# ------------------------------------------------------------------ the C ABI, same names
def tk_attn_fwd(q, k, v, o, lse, B, H, N, D, causal, scale, stream=None) -> int:
    return load_library().tk_attn_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse),
                                      B, H, N, D, int(bool(causal)), float(scale), _stream(stream))


def tk_attn_bwd(q, k, v, o, d_o, lse, dq, dk, dv, B, H, N, D, causal, scale,
                workspace, workspace_bytes, stream=None) -> int:
    return load_library().tk_attn_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(d_o), _ptr(lse),
                                      _ptr(dq), _ptr(dk), _ptr(dv), B, H, N, D, int(bool(causal)),
                                      float(scale), _ptr(workspace), int(workspace_bytes), _stream(stream))


def tk_attn_bwd_noalloc(q, k, v, o, d_o, lse, dq, dk, dv, B, H, N, D, causal, scale, stream=None) -> int:
    return load_library().tk_attn_bwd_noalloc(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(d_o), _ptr(lse),
                                              _ptr(dq), _ptr(dk), _ptr(dv), B, H, N, D, int(bool(causal)),
                                              float(scale), _stream(stream))


def tk_attn_bwd_noalloc_max_rows() -> int:
    return int(load_library().tk_attn_bwd_noalloc_max_rows())


def tk_attn_bwd_workspace_bytes(B, H, N, D) -> int:
    return int(load_library().tk_attn_bwd_workspace_bytes(B, H, N, D))


def tk_attn_bwd_spill_workspace_bytes(B, Hq, Nq, Nk, D) -> int:
    return int(load_library().tk_attn_bwd_spill_workspace_bytes(B, Hq, Nq, Nk, D))


def tk_attn_bwd_ds_bytes(B, Hq, Nq, Nk, D) -> int:
    return int(load_library().tk_attn_bwd_ds_bytes(B, Hq, Nq, Nk, D))


def tk_attn_bwd_dkdv_ds(q, k, v, d_o, lse, delta, dk, dv, ds, B, Hq, Hkv, N, D, causal, scale, stream=None) -> int:
    return load_library().tk_attn_bwd_dkdv_ds(_ptr(q), _ptr(k), _ptr(v), _ptr(d_o), _ptr(lse), _ptr(delta),
                                              _ptr(dk), _ptr(dv), _ptr(ds), B, Hq, Hkv, N, D, int(bool(causal)),
                                              float(scale), _stream(stream))


def tk_attn_bwd_dq_from_ds(k, ds, dq, B, Hq, Hkv, N, D, causal, scale, stream=None) -> int:
    return load_library().tk_attn_bwd_dq_from_ds(_ptr(k), _ptr(ds), _ptr(dq), B, Hq, Hkv, N, D, int(bool(causal)),
                                                 float(scale), _stream(stream))


def tk_attn_bwd_delta(o, d_o, delta, B, H, N, D, stream=None) -> int:
    return load_library().tk_attn_bwd_delta(_ptr(o), _ptr(d_o), _ptr(delta), B, H, N, D, _stream(stream))


def tk_attn_bwd_dkdv(q, k, v, d_o, lse, delta, dk, dv, B, H, N, D, causal, scale, stream=None) -> int:
    return load_library().tk_attn_bwd_dkdv(_ptr(q), _ptr(k), _ptr(v), _ptr(d_o), _ptr(lse), _ptr(delta),
                                           _ptr(dk), _ptr(dv), B, H, N, D, int(bool(causal)),
                                           float(scale), _stream(stream))


def tk_attn_bwd_dq(q, k, v, d_o, lse, delta, dq, B, H, N, D, causal, scale, stream=None) -> int:
    return load_library().tk_attn_bwd_dq(_ptr(q), _ptr(k), _ptr(v), _ptr(d_o), _ptr(lse), _ptr(delta),
                                         _ptr(dq), B, H, N, D, int(bool(causal)), float(scale), _stream(stream))


def tk_attn_fwd_gqa(q, k, v, o, lse, B, Hq, Hkv, N, D, causal, scale, stream=None) -> int:
    return load_library().tk_attn_fwd_gqa(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), B, Hq, Hkv, N, D,
                                          int(bool(causal)), float(scale), _stream(stream))


def tk_attn_bwd_gqa(q, k, v, o, d_o, lse, dq, dk, dv, B, Hq, Hkv, N, D, causal, scale, workspace, workspace_bytes,
                    stream=None) -> int:
    return load_library().tk_attn_bwd_gqa(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(d_o), _ptr(lse), _ptr(dq),
                                          _ptr(dk), _ptr(dv), B, Hq, Hkv, N, D, int(bool(causal)), float(scale),
                                          _ptr(workspace), int(workspace_bytes), _stream(stream))


def tk_attn_bwd_dq_delta(q, k, v, o, d_o, lse, delta, dq, B, Hq, Hkv, N, D, causal, scale, stream=None) -> int:
    return load_library().tk_attn_bwd_dq_delta(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(d_o), _ptr(lse), _ptr(delta),
                                               _ptr(dq), B, Hq, Hkv, N, D, int(bool(causal)), float(scale), _stream(stream))


def tk_attn_fwd_rect(q, k, v, o, lse, B, Hq, Hkv, Nq, Nk, D, causal, scale, stream=None) -> int:
    return load_library().tk_attn_fwd_rect(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), B, Hq, Hkv, Nq, Nk, D,
                                           int(bool(causal)), float(scale), _stream(stream))


def tk_attn_bwd_rect(q, k, v, o, d_o, lse, dq, dk, dv, B, Hq, Hkv, Nq, Nk, D, causal, scale, workspace,
                     workspace_bytes, stream=None) -> int:
    return load_library().tk_attn_bwd_rect(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(d_o), _ptr(lse), _ptr(dq),
                                           _ptr(dk), _ptr(dv), B, Hq, Hkv, Nq, Nk, D, int(bool(causal)), float(scale),
                                           _ptr(workspace), int(workspace_bytes), _stream(stream))


def tk_attn_decode_workspace_bytes(B, Hq, Hkv, Nk, D) -> int:
    return int(load_library().tk_attn_decode_workspace_bytes(B, Hq, Hkv, Nk, D))


def tk_attn_decode_plan(B, Hq, Hkv, Nk, D, compute_units):
    """(status, [heads, rows per head, splits, tiles per split, max splits]) - host arithmetic only."""
    plan = (ctypes.c_int * 5)()
    rc = load_library().tk_attn_decode_plan(B, Hq, Hkv, Nk, D, compute_units, plan)
    return rc, list(plan)


def tk_attn_decode(q, k, v, o, lse, B, Hq, Hkv, Nk, D, scale, workspace, workspace_bytes, stream=None) -> int:
    return load_library().tk_attn_decode(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), B, Hq, Hkv, Nk, D,
                                         float(scale), _ptr(workspace), int(workspace_bytes), _stream(stream))


def tk_attn_bwd_dkdv_gqa(q, k, v, d_o, lse, delta, dk, dv, B, Hq, Hkv, N, D, causal, scale, stream=None) -> int:
    return load_library().tk_attn_bwd_dkdv_gqa(_ptr(q), _ptr(k), _ptr(v), _ptr(d_o), _ptr(lse), _ptr(delta),
                                               _ptr(dk), _ptr(dv), B, Hq, Hkv, N, D, int(bool(causal)),
                                               float(scale), _stream(stream))


def tk_attn_bwd_dq_gqa(q, k, v, d_o, lse, delta, dq, B, Hq, Hkv, N, D, causal, scale, stream=None) -> int:
    return load_library().tk_attn_bwd_dq_gqa(_ptr(q), _ptr(k), _ptr(v), _ptr(d_o), _ptr(lse), _ptr(delta),
                                             _ptr(dq), B, Hq, Hkv, N, D, int(bool(causal)), float(scale),
                                             _stream(stream))


def tk_gemm(a, b, c, M, N, K, stream=None) -> int:
    return load_library().tk_gemm(_ptr(a), _ptr(b), _ptr(c), M, N, K, _stream(stream))


def tk_rotary(x, sin_table, cos_table, o, B, H, N, D, stream=None) -> int:
    return load_library().tk_rotary(_ptr(x), _ptr(sin_table), _ptr(cos_table), _ptr(o), B, H, N, D, _stream(stream))


def tk_mfma_probe(operands, sink, workgroups, iters, stream=None) -> int:
    return load_library().tk_mfma_probe(_ptr(operands), _ptr(sink), int(workgroups), int(iters), _stream(stream))


# ------------------------------------------------------------------ convenience: allocate outputs, raise on error
def attn_fwd(q, k, v, causal: bool, scale: float, out=None, stream=None):
    """q, k, v: CUDA bf16 [B,H,N,D]. Returns (o bf16 [B,H,N,D], lse fp32 [B,H,N])."""
    _check_bf16("q", q)
    B, H, N, D = q.shape
    _check_bf16("k", k, q.shape)
    _check_bf16("v", v, q.shape)
    if out is None:
        o = torch.empty_like(q)
        lse = torch.empty((B, H, N), dtype=torch.float32, device=q.device)
    else:
        o, lse = out
        _check_bf16("o", o, q.shape)
        _check_f32("lse", lse, (B, H, N))
    rc = tk_attn_fwd(q, k, v, o, lse, B, H, N, D, causal, scale, stream)
    if rc != TK_OK:
        raise TkAttnError(rc, "tk_attn_fwd")
    return o, lse


SPILL_WORKSPACE_LIMIT = 24 << 30     # largest dS workspace the convenience wrappers allocate by themselves


def alloc_bwd_workspace(B, H, N, D, device="cuda", spill=None, Nk=None):
    """Backward workspace.  spill=True: large enough for the form that stores dS (about 2*B*H*N*Nk bytes);
    spill=False: Delta only; spill=None: the large one where it pays - at D = 128 (the stored dS costs the same
    bytes at every D while the recomputation it replaces shrinks with D: at D = 64 the storing form measured 25 %
    slower than the recomputing one) - and if it stays under SPILL_WORKSPACE_LIMIT."""
    small = tk_attn_bwd_workspace_bytes(B, H, N, D)
    if small == 0:
        raise TkAttnError(TK_ERR_BAD_DIM, "tk_attn_bwd_workspace_bytes")
    big = tk_attn_bwd_spill_workspace_bytes(B, H, N, N if Nk is None else Nk, D)
    if spill is None:
        spill = D == 128 and 0 < big <= SPILL_WORKSPACE_LIMIT
    return torch.empty(big if spill else small, dtype=torch.uint8, device=device)


def attn_bwd(q, k, v, o, d_o, lse, causal: bool, scale: float, workspace=None, out=None, stream=None):
    """Returns (dq, dk, dv) bf16 [B,H,N,D]; o and lse must come from attn_fwd on the same inputs."""
    _check_bf16("q", q)
    B, H, N, D = q.shape
    for name, t in (("k", k), ("v", v), ("o", o), ("d_o", d_o)):
        _check_bf16(name, t, q.shape)
    _check_f32("lse", lse, (B, H, N))
    if workspace is None:
        workspace = alloc_bwd_workspace(B, H, N, D, q.device)
    if out is None:
        dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(q)
    else:
        dq, dk, dv = out
    rc = tk_attn_bwd(q, k, v, o, d_o, lse, dq, dk, dv, B, H, N, D, causal, scale,
                     workspace, workspace.numel() * workspace.element_size(), stream)
    if rc != TK_OK:
        raise TkAttnError(rc, "tk_attn_bwd")
    return dq, dk, dv


def attn_bwd_delta(o, d_o, stream=None):
    _check_bf16("o", o)
    _check_bf16("d_o", d_o, o.shape)
    B, H, N, D = o.shape
    delta = torch.empty((B, H, N), dtype=torch.float32, device=o.device)
    rc = tk_attn_bwd_delta(o, d_o, delta, B, H, N, D, stream)
    if rc != TK_OK:
        raise TkAttnError(rc, "tk_attn_bwd_delta")
    return delta


def gqa_fwd(q, k, v, causal: bool, scale: float, stream=None):
    """Grouped-query forward: q bf16 [B,Hq,N,D], k, v bf16 [B,Hkv,N,D]. Returns (o [B,Hq,N,D], lse [B,Hq,N])."""
    _check_bf16("q", q)
    B, Hq, N, D = q.shape
    Hkv = k.shape[1]
    _check_bf16("k", k, (B, Hkv, N, D))
    _check_bf16("v", v, (B, Hkv, N, D))
    o = torch.empty_like(q)
    lse = torch.empty((B, Hq, N), dtype=torch.float32, device=q.device)
    rc = tk_attn_fwd_gqa(q, k, v, o, lse, B, Hq, Hkv, N, D, causal, scale, stream)
    if rc != TK_OK:
        raise TkAttnError(rc, "tk_attn_fwd_gqa")
    return o, lse


def gqa_bwd(q, k, v, o, d_o, lse, causal: bool, scale: float, workspace=None, stream=None):
    """Grouped-query backward. Returns (dq [B,Hq,N,D], dk, dv [B,Hkv,N,D]) bf16."""
    _check_bf16("q", q)
    B, Hq, N, D = q.shape
    Hkv = k.shape[1]
    _check_bf16("k", k, (B, Hkv, N, D))
    _check_bf16("v", v, (B, Hkv, N, D))
    _check_bf16("o", o, q.shape)
    _check_bf16("d_o", d_o, q.shape)
    _check_f32("lse", lse, (B, Hq, N))
    if workspace is None:
        workspace = alloc_bwd_workspace(B, Hq, N, D, q.device)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    rc = tk_attn_bwd_gqa(q, k, v, o, d_o, lse, dq, dk, dv, B, Hq, Hkv, N, D, causal, scale,
                         workspace, workspace.numel() * workspace.element_size(), stream)
    if rc != TK_OK:
        raise TkAttnError(rc, "tk_attn_bwd_gqa")
    return dq, dk, dv


def rect_fwd(q, k, v, causal: bool, scale: float, stream=None):
    """Forward with Nq queries and Nk keys: q bf16 [B,Hq,Nq,D], k, v bf16 [B,Hkv,Nk,D].
    Returns (o [B,Hq,Nq,D], lse [B,Hq,Nq]).  Causal: query i sees keys j <= i + (Nk - Nq)."""
    _check_bf16("q", q)
    B, Hq, Nq, D = q.shape
    Hkv, Nk = k.shape[1], k.shape[2]
    _check_bf16("k", k, (B, Hkv, Nk, D))
    _check_bf16("v", v, (B, Hkv, Nk, D))
    o = torch.empty_like(q)
    lse = torch.empty((B, Hq, Nq), dtype=torch.float32, device=q.device)
    rc = tk_attn_fwd_rect(q, k, v, o, lse, B, Hq, Hkv, Nq, Nk, D, causal, scale, stream)
    if rc != TK_OK:
        raise TkAttnError(rc, "tk_attn_fwd_rect")
    return o, lse


def rect_bwd(q, k, v, o, d_o, lse, causal: bool, scale: float, workspace=None, stream=None):
    """Backward of rect_fwd. Returns (dq [B,Hq,Nq,D], dk, dv [B,Hkv,Nk,D]) bf16."""
    _check_bf16("q", q)
    B, Hq, Nq, D = q.shape
    Hkv, Nk = k.shape[1], k.shape[2]
    _check_bf16("k", k, (B, Hkv, Nk, D))
    _check_bf16("v", v, (B, Hkv, Nk, D))
    _check_bf16("o", o, q.shape)
    _check_bf16("d_o", d_o, q.shape)
    _check_f32("lse", lse, (B, Hq, Nq))
    if workspace is None:
        workspace = alloc_bwd_workspace(B, Hq, Nq, D, q.device, Nk=Nk)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    rc = tk_attn_bwd_rect(q, k, v, o, d_o, lse, dq, dk, dv, B, Hq, Hkv, Nq, Nk, D, causal, scale,
                          workspace, workspace.numel() * workspace.element_size(), stream)
    if rc != TK_OK:
        raise TkAttnError(rc, "tk_attn_bwd_rect")
    return dq, dk, dv


def decode(q, k, v, scale: float, workspace=None, stream=None):
    """One query per head: q bf16 [B,Hq,1,D], k, v bf16 [B,Hkv,Nk,D]. Returns (o [B,Hq,1,D], lse [B,Hq,1])."""
    _check_bf16("q", q)
    B, Hq, one, D = q.shape
    if one != 1:
        raise ValueError("decode takes exactly one query per head")
    Hkv, Nk = k.shape[1], k.shape[2]
    _check_bf16("k", k, (B, Hkv, Nk, D))
    _check_bf16("v", v, (B, Hkv, Nk, D))
    if workspace is None:
        workspace = torch.empty(max(tk_attn_decode_workspace_bytes(B, Hq, Hkv, Nk, D), 16), dtype=torch.uint8, device=q.device)
    o = torch.empty_like(q)
    lse = torch.empty((B, Hq, 1), dtype=torch.float32, device=q.device)
    rc = tk_attn_decode(q, k, v, o, lse, B, Hq, Hkv, Nk, D, scale, workspace, workspace.numel() * workspace.element_size(), stream)
    if rc != TK_OK:
        raise TkAttnError(rc, "tk_attn_decode")
    return o, lse


def rotary(x, sin_table, cos_table, out=None, stream=None):
    """Rotary positional encoding: x bf16 [B,H,N,D], sin/cos bf16 [N, D/2]. Returns o (out=x works in place)."""
    _check_bf16("x", x)
    B, H, N, D = x.shape
    _check_bf16("sin_table", sin_table, (N, D // 2))
    _check_bf16("cos_table", cos_table, (N, D // 2))
    o = torch.empty_like(x) if out is None else out
    _check_bf16("o", o, x.shape)
    rc = tk_rotary(x, sin_table, cos_table, o, B, H, N, D, stream)
    if rc != TK_OK:
        raise TkAttnError(rc, "tk_rotary")
    return o


def gemm(a, b, out=None, stream=None):
    """C = A B: a bf16 [M,K], b bf16 [K,N] -> c bf16 [M,N] (N and K multiples of 8)."""
    if a.dtype != torch.bfloat16 or b.dtype != torch.bfloat16 or a.dim() != 2 or b.dim() != 2:
        raise ValueError("a, b must be 2-D bf16 tensors")
    if not (a.is_cuda and b.is_cuda and a.is_contiguous() and b.is_contiguous()) or a.shape[1] != b.shape[0]:
        raise ValueError("a [M,K], b [K,N] must be contiguous CUDA tensors")
    M, K = a.shape
    N = b.shape[1]
    c = torch.empty((M, N), dtype=torch.bfloat16, device=a.device) if out is None else out
    rc = tk_gemm(a, b, c, M, N, K, stream)
    if rc != TK_OK:
        raise TkAttnError(rc, "tk_gemm")
    return c
