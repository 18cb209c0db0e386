"""Host-side checks of the C ABI (no GPU needed): the library loads, exports every symbol the
header declares, and rejects bad arguments before making any HIP call."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "tk_attn.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2410_20399_amd import attn, build
    if build.stale():
        build.build()
    return attn.load_library()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tk_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_expected_entry_points():
    names = declared_functions()
    for must in ("tk_attn_fwd", "tk_attn_bwd", "tk_attn_bwd_workspace_bytes", "tk_attn_bwd_delta",
                 "tk_attn_bwd_dkdv", "tk_attn_bwd_dq", "tk_status_string", "tk_attn_version"):
        assert must in names


def test_library_exports_every_declared_symbol(lib):
    from paper_2410_20399_amd import attn
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} declared in tk_attn.h but not exported"
    assert sorted(attn.EXPORTS) == declared_functions()


def test_version_and_status_strings(lib):
    from paper_2410_20399_amd import attn
    assert attn.version() >= 100
    seen = set()
    for code in range(0, -8, -1):
        s = attn.status_string(code)
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 8
    assert attn.status_string(-99) == "unknown status"


P = ctypes.c_void_p(0x10000)        # never dereferenced: validation fails first
ODD = ctypes.c_void_p(0x10008)      # 8-byte aligned only


def fwd(lib, q=P, k=P, v=P, o=P, lse=P, B=1, H=1, N=128, D=64, causal=0, scale=0.125):
    return lib.tk_attn_fwd(q, k, v, o, lse, B, H, N, D, causal, ctypes.c_float(scale), None)


def bwd(lib, ptrs=None, B=1, H=1, N=128, D=64, causal=0, scale=0.125, ws=P, ws_bytes=1 << 40):
    ptrs = ptrs or [P] * 9
    return lib.tk_attn_bwd(*ptrs, B, H, N, D, causal, ctypes.c_float(scale), ws, ctypes.c_size_t(ws_bytes), None)


def test_forward_rejects_bad_arguments(lib):
    from paper_2410_20399_amd import attn as a
    for name in ("q", "k", "v", "o", "lse"):
        assert fwd(lib, **{name: None}) == a.TK_ERR_NULL_PTR
    for bad in (dict(D=32), dict(D=96), dict(D=256), dict(N=0), dict(N=-128),
                dict(B=0), dict(H=0), dict(B=-1), dict(B=1 << 20, H=1 << 12, N=128)):
        assert fwd(lib, **bad) == a.TK_ERR_BAD_DIM, bad
    for name in ("q", "k", "v", "o", "lse"):
        assert fwd(lib, **{name: ODD}) == a.TK_ERR_MISALIGNED
    for s in (0.0, -0.125, float("inf"), float("nan")):
        assert fwd(lib, scale=s) == a.TK_ERR_BAD_SCALE


def test_backward_rejects_bad_arguments(lib):
    from paper_2410_20399_amd import attn as a
    for i in range(9):
        ptrs = [P] * 9
        ptrs[i] = None
        assert bwd(lib, ptrs) == a.TK_ERR_NULL_PTR
        ptrs[i] = ODD
        assert bwd(lib, ptrs) == a.TK_ERR_MISALIGNED
    assert bwd(lib, ws=None) == a.TK_ERR_NULL_PTR
    assert bwd(lib, ws=ODD) == a.TK_ERR_MISALIGNED
    assert bwd(lib, D=100) == a.TK_ERR_BAD_DIM
    assert bwd(lib, N=0) == a.TK_ERR_BAD_DIM
    assert bwd(lib, scale=-1.0) == a.TK_ERR_BAD_SCALE
    need = lib.tk_attn_bwd_workspace_bytes(1, 1, 128, 64)
    assert bwd(lib, ws_bytes=need - 1) == a.TK_ERR_WORKSPACE_TOO_SMALL
    assert bwd(lib, ws_bytes=0) == a.TK_ERR_WORKSPACE_TOO_SMALL


def test_workspace_size(lib):
    # fp32 Delta [B,H,N], padded to a multiple of 256 B
    assert lib.tk_attn_bwd_workspace_bytes(1, 1, 128, 64) == 128 * 4
    assert lib.tk_attn_bwd_workspace_bytes(1, 3, 128, 64) == 3 * 128 * 4
    assert lib.tk_attn_bwd_workspace_bytes(16, 16, 4096, 128) == 16 * 16 * 4096 * 4
    assert lib.tk_attn_bwd_workspace_bytes(1, 1, 100, 64) == 512      # 400 bytes of Delta, padded to 256
    assert lib.tk_attn_bwd_workspace_bytes(1, 1, 0, 64) == 0
    assert lib.tk_attn_bwd_workspace_bytes(1, 1, 128, 80) == 0


def test_delta_entry_rejects_bad_arguments(lib):
    from paper_2410_20399_amd import attn as a
    assert lib.tk_attn_bwd_delta(None, P, P, 1, 1, 128, 64, None) == a.TK_ERR_NULL_PTR
    assert lib.tk_attn_bwd_delta(P, P, ODD, 1, 1, 128, 64, None) == a.TK_ERR_MISALIGNED
    assert lib.tk_attn_bwd_delta(P, P, P, 1, 1, 128, 48, None) == a.TK_ERR_BAD_DIM


def test_stage_entries_reject_bad_arguments(lib):
    from paper_2410_20399_amd import attn as a
    f = ctypes.c_float
    for fn, nptr in ((lib.tk_attn_bwd_dkdv, 8), (lib.tk_attn_bwd_dq, 7)):
        for i in range(nptr):
            ptrs = [P] * nptr
            ptrs[i] = None
            assert fn(*ptrs, 1, 1, 128, 64, 0, f(0.125), None) == a.TK_ERR_NULL_PTR
            ptrs[i] = ODD
            assert fn(*ptrs, 1, 1, 128, 64, 0, f(0.125), None) == a.TK_ERR_MISALIGNED
        assert fn(*([P] * nptr), 1, 1, 128, 64, 0, f(0.0), None) == a.TK_ERR_BAD_SCALE
        assert fn(*([P] * nptr), 1, 1, 0, 64, 0, f(0.125), None) == a.TK_ERR_BAD_DIM
        assert fn(*([P] * nptr), 1, 1, 128, 96, 0, f(0.125), None) == a.TK_ERR_BAD_DIM


def test_dq_delta_entry_rejects_bad_arguments(lib):
    from paper_2410_20399_amd import attn as a
    f = ctypes.c_float
    for i in range(8):
        ptrs = [P] * 8
        ptrs[i] = None
        assert lib.tk_attn_bwd_dq_delta(*ptrs, 1, 4, 2, 128, 64, 1, f(0.125), None) == a.TK_ERR_NULL_PTR
        ptrs[i] = ODD
        assert lib.tk_attn_bwd_dq_delta(*ptrs, 1, 4, 2, 128, 64, 1, f(0.125), None) == a.TK_ERR_MISALIGNED
    assert lib.tk_attn_bwd_dq_delta(*([P] * 8), 1, 4, 3, 128, 64, 1, f(0.125), None) == a.TK_ERR_BAD_DIM
    assert lib.tk_attn_bwd_dq_delta(*([P] * 8), 1, 4, 2, 0, 64, 1, f(0.125), None) == a.TK_ERR_BAD_DIM
    assert lib.tk_attn_bwd_dq_delta(*([P] * 8), 1, 4, 2, 128, 64, 1, f(-1.0), None) == a.TK_ERR_BAD_SCALE


def test_gqa_entries_reject_bad_arguments(lib):
    from paper_2410_20399_amd import attn as a
    f = ctypes.c_float
    sz = ctypes.c_size_t
    # head counts: Hkv must be >= 1, <= Hq and divide Hq
    for hq, hkv in ((4, 0), (4, 3), (4, 8), (4, -1)):
        assert lib.tk_attn_fwd_gqa(P, P, P, P, P, 1, hq, hkv, 128, 64, 0, f(0.125), None) == a.TK_ERR_BAD_DIM
        assert lib.tk_attn_bwd_gqa(P, P, P, P, P, P, P, P, P, 1, hq, hkv, 128, 64, 0, f(0.125), P, sz(1 << 30), None) == a.TK_ERR_BAD_DIM
        assert lib.tk_attn_bwd_dkdv_gqa(P, P, P, P, P, P, P, P, 1, hq, hkv, 128, 64, 0, f(0.125), None) == a.TK_ERR_BAD_DIM
        assert lib.tk_attn_bwd_dq_gqa(P, P, P, P, P, P, P, 1, hq, hkv, 128, 64, 0, f(0.125), None) == a.TK_ERR_BAD_DIM
    assert lib.tk_attn_fwd_gqa(None, P, P, P, P, 1, 4, 2, 128, 64, 0, f(0.125), None) == a.TK_ERR_NULL_PTR
    assert lib.tk_attn_fwd_gqa(P, ODD, P, P, P, 1, 4, 2, 128, 64, 0, f(0.125), None) == a.TK_ERR_MISALIGNED
    assert lib.tk_attn_fwd_gqa(P, P, P, P, P, 1, 4, 2, 0, 64, 0, f(0.125), None) == a.TK_ERR_BAD_DIM
    assert lib.tk_attn_fwd_gqa(P, P, P, P, P, 1, 4, 2, 128, 64, 0, f(-1.0), None) == a.TK_ERR_BAD_SCALE
    need = lib.tk_attn_bwd_workspace_bytes(1, 4, 128, 64)
    assert lib.tk_attn_bwd_gqa(P, P, P, P, P, P, P, P, P, 1, 4, 2, 128, 64, 0, f(0.125), P, sz(need - 1), None) == a.TK_ERR_WORKSPACE_TOO_SMALL
    assert lib.tk_attn_bwd_gqa(P, P, P, P, P, P, P, P, None, 1, 4, 2, 128, 64, 0, f(0.125), P, sz(need), None) == a.TK_ERR_NULL_PTR


def test_rect_entries_reject_bad_arguments(lib):
    from paper_2410_20399_amd import attn as a
    f = ctypes.c_float
    sz = ctypes.c_size_t

    def fwd_rect(*, q=P, Hq=2, Hkv=1, Nq=5, Nk=300, D=64, causal=1, scale=0.125):
        return lib.tk_attn_fwd_rect(q, P, P, P, P, 1, Hq, Hkv, Nq, Nk, D, causal, f(scale), None)

    def bwd_rect(*, dk=P, Hq=2, Hkv=1, Nq=5, Nk=300, D=64, causal=1, scale=0.125, ws=P, ws_bytes=1 << 30):
        return lib.tk_attn_bwd_rect(P, P, P, P, P, P, P, dk, P, 1, Hq, Hkv, Nq, Nk, D, causal, f(scale), ws, sz(ws_bytes), None)

    for fn in (fwd_rect, bwd_rect):
        assert fn(Nq=0) == a.TK_ERR_BAD_DIM
        assert fn(Nk=0) == a.TK_ERR_BAD_DIM
        assert fn(Nq=301, Nk=300, causal=1) == a.TK_ERR_BAD_DIM      # causal needs Nq <= Nk
        assert fn(D=96) == a.TK_ERR_BAD_DIM
        assert fn(Hq=3, Hkv=2) == a.TK_ERR_BAD_DIM
        assert fn(scale=0.0) == a.TK_ERR_BAD_SCALE
    assert fwd_rect(q=None) == a.TK_ERR_NULL_PTR
    assert fwd_rect(q=ODD) == a.TK_ERR_MISALIGNED
    assert bwd_rect(dk=None) == a.TK_ERR_NULL_PTR
    assert bwd_rect(dk=ODD) == a.TK_ERR_MISALIGNED
    assert bwd_rect(ws=None) == a.TK_ERR_NULL_PTR
    need = lib.tk_attn_bwd_workspace_bytes(1, 2, 5, 64)       # sized by the QUERY length
    assert need == 256
    assert bwd_rect(ws_bytes=need - 1) == a.TK_ERR_WORKSPACE_TOO_SMALL


def test_decode_entry_rejects_bad_arguments(lib):
    from paper_2410_20399_amd import attn as a
    f = ctypes.c_float
    sz = ctypes.c_size_t

    def decode(*, q=P, lse=P, ws=P, Hq=8, Hkv=2, Nk=1000, D=128, scale=0.1, ws_bytes=1 << 40):
        return lib.tk_attn_decode(q, P, P, P, lse, 2, Hq, Hkv, Nk, D, f(scale), ws, sz(ws_bytes), None)

    assert decode(q=None) == a.TK_ERR_NULL_PTR
    assert decode(ws=None) == a.TK_ERR_NULL_PTR
    assert decode(lse=ODD) == a.TK_ERR_MISALIGNED
    assert decode(ws=ODD) == a.TK_ERR_MISALIGNED
    assert decode(Nk=0) == a.TK_ERR_BAD_DIM
    assert decode(D=32) == a.TK_ERR_BAD_DIM
    assert decode(Hq=8, Hkv=3) == a.TK_ERR_BAD_DIM
    assert decode(scale=float("nan")) == a.TK_ERR_BAD_SCALE
    need = lib.tk_attn_decode_workspace_bytes(2, 8, 2, 1000, 128)
    # B*Hkv = 4 packed heads -> at most 256 splits: fp32 partial O [256][B*Hq][D] and partial LSE [256][B*Hq]
    assert need == 256 * 16 * 128 * 4 + 256 * 16 * 4
    # 512 packed heads -> at most 2 splits
    assert lib.tk_attn_decode_workspace_bytes(64, 32, 8, 1000, 64) == 2 * 2048 * 64 * 4 + 2 * 2048 * 4
    assert need % 256 == 0
    assert decode(ws_bytes=need - 1) == a.TK_ERR_WORKSPACE_TOO_SMALL
    assert lib.tk_attn_decode_workspace_bytes(2, 8, 3, 1000, 128) == 0
    assert lib.tk_attn_decode_workspace_bytes(2, 8, 2, 0, 128) == 0
    # K and V are [B, Hkv, Nk, D]: a long grouped history is bounded by B*Hkv*Nk, not B*Hq*Nk
    assert lib.tk_attn_decode_workspace_bytes(700, 512, 8, 100000, 128) > 0
    assert a.tk_attn_decode_plan(700, 512, 8, 100000, 128, 256)[0] == a.TK_OK
    # ... and a key side that really is too large is still rejected
    assert lib.tk_attn_decode_workspace_bytes(700, 512, 512, 100000, 128) == 0


def test_decode_plan_invariants(lib):
    """Host arithmetic of the decode layout: no empty split, even tile counts, splits within the bound
    the workspace is sized for, grouped heads packed while they fit one tile."""
    from paper_2410_20399_amd import attn as a
    import itertools
    for B, (Hq, Hkv), Nk, D, cus in itertools.product(
            (1, 2, 16, 300), ((1, 1), (8, 8), (32, 8), (128, 1), (129, 1), (256, 2)),
            (1, 63, 64, 65, 255, 256, 1000, 8192, 100000, 1 << 20), (64, 128), (1, 64, 256, 304)):
        rc, (heads, rows, splits, per, max_splits) = a.tk_attn_decode_plan(B, Hq, Hkv, Nk, D, cus)
        if B * Hkv * Nk > 0x7fffffff * 16:                # beyond what any entry point accepts (K, V are [B,Hkv,Nk,D])
            assert rc == a.TK_ERR_BAD_DIM
            continue
        assert rc == a.TK_OK
        G = Hq // Hkv
        assert (heads, rows) == ((B * Hkv, G) if G <= 128 else (B * Hq, 1))
        tiles = (Nk + 63) // 64
        assert 1 <= splits <= max_splits <= 256
        assert per % 2 == 0 and per >= 2
        assert splits * per >= tiles                      # the splits cover every tile
        assert (splits - 1) * per * 64 < Nk               # and the last one still holds a key
        if splits > 1:
            assert per >= 4 and heads * (splits - 1) < 2 * cus + heads      # no more splits than fill two workgroups per unit
        need = lib.tk_attn_decode_workspace_bytes(B, Hq, Hkv, Nk, D)
        assert need >= splits * B * Hq * (D + 1) * 4
    assert a.tk_attn_decode_plan(1, 8, 3, 100, 64, 256)[0] == a.TK_ERR_BAD_DIM
    assert a.tk_attn_decode_plan(1, 8, 2, 100, 64, 0)[0] == a.TK_ERR_BAD_DIM
    assert lib.tk_attn_decode_plan(1, 8, 2, 100, 64, 256, None) == a.TK_ERR_NULL_PTR


def test_noalloc_backward_rejects_bad_arguments(lib):
    """Validation comes before the scratch lookup and every HIP call, so it runs without a GPU."""
    from paper_2410_20399_amd import attn as a
    f = ctypes.c_float

    def call(ptrs=None, B=1, H=1, N=128, D=64, causal=0, scale=0.125):
        ptrs = ptrs or [P] * 9
        return lib.tk_attn_bwd_noalloc(*ptrs, B, H, N, D, causal, f(scale), None)

    for i in range(9):
        ptrs = [P] * 9
        ptrs[i] = None
        assert call(ptrs) == a.TK_ERR_NULL_PTR
    ptrs = [P] * 9
    ptrs[6] = ODD
    assert call(ptrs) == a.TK_ERR_MISALIGNED
    assert call(D=96) == a.TK_ERR_BAD_DIM
    assert call(N=0) == a.TK_ERR_BAD_DIM
    assert call(scale=0.0) == a.TK_ERR_BAD_SCALE
    limit = a.tk_attn_bwd_noalloc_max_rows()
    assert limit == 1 << 20
    assert call(B=16, H=16, N=4097) == a.TK_ERR_SCRATCH_LIMIT          # one row per head too many
    assert call(B=1, H=1, N=limit + 1) == a.TK_ERR_SCRATCH_LIMIT
    assert "scratch" in a.status_string(a.TK_ERR_SCRATCH_LIMIT)


def test_gemm_rejects_bad_arguments(lib):
    from paper_2410_20399_amd import attn as a
    for i in range(3):
        ptrs = [P] * 3
        ptrs[i] = None
        assert lib.tk_gemm(*ptrs, 256, 256, 64, None) == a.TK_ERR_NULL_PTR
        ptrs[i] = ODD
        assert lib.tk_gemm(*ptrs, 256, 256, 64, None) == a.TK_ERR_MISALIGNED
    # M >= 1; N and K positive multiples of 8 (rows must start on 16 bytes)
    for M, N, K in ((0, 256, 64), (256, 300, 64), (256, 4, 64), (256, 256, 4), (256, 256, 100), (-256, 256, 64), (256, 0, 64)):
        assert lib.tk_gemm(P, P, P, M, N, K, None) == a.TK_ERR_BAD_DIM, (M, N, K)


def test_rotary_rejects_bad_arguments(lib):
    from paper_2410_20399_amd import attn as a
    for i in range(4):
        ptrs = [P] * 4
        ptrs[i] = None
        assert lib.tk_rotary(*ptrs, 1, 1, 128, 64, None) == a.TK_ERR_NULL_PTR
        ptrs[i] = ODD
        assert lib.tk_rotary(*ptrs, 1, 1, 128, 64, None) == a.TK_ERR_MISALIGNED
    assert lib.tk_rotary(P, P, P, P, 1, 1, 128, 96, None) == a.TK_ERR_BAD_DIM
    assert lib.tk_rotary(P, P, P, P, 1, 1, 0, 128, None) == a.TK_ERR_BAD_DIM


def test_mfma_probe_rejects_bad_arguments(lib):
    from paper_2410_20399_amd import attn as a
    assert lib.tk_mfma_probe(None, P, 1, 1, None) == a.TK_ERR_NULL_PTR
    assert lib.tk_mfma_probe(P, None, 1, 1, None) == a.TK_ERR_NULL_PTR
    assert lib.tk_mfma_probe(ODD, P, 1, 1, None) == a.TK_ERR_MISALIGNED
    assert lib.tk_mfma_probe(P, P, 0, 1, None) == a.TK_ERR_BAD_DIM
    assert lib.tk_mfma_probe(P, P, 70000, 1, None) == a.TK_ERR_BAD_DIM
    assert lib.tk_mfma_probe(P, P, 1, 0, None) == a.TK_ERR_BAD_DIM


def test_missing_library_fails_loudly(tmp_path):
    from paper_2410_20399_amd import attn
    saved = attn._lib
    attn._lib = None
    try:
        with pytest.raises(FileNotFoundError):
            attn.load_library(str(tmp_path / "libtk_attn.so"))
    finally:
        attn._lib = saved


def test_product_path_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2410_20399_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower() or f == "workloads.py", f
