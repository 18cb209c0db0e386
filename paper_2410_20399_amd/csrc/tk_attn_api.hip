// C ABI of the attention library: host-side validation and dispatch only.
#include "../../include/tk_attn.h"
#include "tk_launch.h"

#include <math.h>
#include <stdint.h>

#include <atomic>

// Scratch of tk_attn_bwd_noalloc: Delta (fp32, one value per query row) for callers that cannot hand over a
// workspace.  One copy per GPU, held until the process ends.  In host code this name is only a stand-in
// for the symbol; the device address comes from hipGetSymbolAddress (noalloc_scratch() below).
constexpr size_t kNoallocScratchFloats = (size_t)1 << 20;      // 4 MiB: B*H*N <= 1,048,576 query rows
static __device__ __align__(256) float g_noalloc_scratch[kNoallocScratchFloats];

namespace {

constexpr int kTileN = 128;      // rows per workgroup tile (sequences are padded to it inside the kernels)

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_shape(int B, int H, int N, int D)
{
    if (D != 64 && D != 128) return TK_ERR_BAD_DIM;
    if (B < 1 || H < 1 || N < 1) return TK_ERR_BAD_DIM;
    const long long tiles = (long long)B * H * (((long long)N + kTileN - 1) / kTileN);
    if (tiles > 0x7fffffffLL) return TK_ERR_BAD_DIM;
    if ((long long)B * H * N > 0x7fffffffLL * 16) return TK_ERR_BAD_DIM;   // row indices stay far inside 64 bits
    return TK_OK;
}

// Device address of g_noalloc_scratch on the current device, looked up once per device (with that device
// current, as it is here: the caller's stream belongs to it) and kept.  Every GPU holds its own copy of the
// array at its own address.  nullptr if the lookup fails.
float* noalloc_scratch()
{
    constexpr int kMaxDevices = 64;
    static std::atomic<float*> ptr[kMaxDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    float* p = ptr[dev].load(std::memory_order_acquire);
    if (p) return p;
    void* sym = nullptr;
    if (hipGetSymbolAddress(&sym, HIP_SYMBOL(g_noalloc_scratch)) != hipSuccess || !sym) return nullptr;
    p = (float*)sym;
    ptr[dev].store(p, std::memory_order_release);      // (two threads racing here store the same address)
    return p;
}

int check_scale(float scale)
{
    return (isfinite(scale) && scale > 0.0f) ? TK_OK : TK_ERR_BAD_SCALE;
}

size_t delta_bytes(int B, int H, int N)
{
    size_t b = (size_t)B * H * N * sizeof(float);
    return (b + 255) & ~(size_t)255;
}

int check_heads(int H, int Hkv)
{
    return (Hkv >= 1 && Hkv <= H && H % Hkv == 0) ? TK_OK : TK_ERR_BAD_DIM;
}

// Head counts and lengths of one call: the query side is [B, Hq, Nq, D], the key side [B, Hkv, Nk, D], and
// each is bounded by its own extent; the causal mask aligns the sequences at their ends and needs Nq <= Nk.
int check_lengths(int B, int Hq, int Hkv, int Nq, int Nk, int D, int causal)
{
    if (int rc = check_heads(Hq, Hkv)) return rc;
    if (int rc = check_shape(B, Hq, Nq, D)) return rc;
    if (int rc = check_shape(B, Hkv, Nk, D)) return rc;
    if (causal && Nq > Nk) return TK_ERR_BAD_DIM;
    return TK_OK;
}

// Decode-shaped calls: one query per head against Nk keys.
constexpr int kDecodeMaxSplits = 256;      // upper bound on the split over the keys
constexpr int kDecodeMaxWorkgroups = 1024; // no more splits than it takes to reach this many workgroups (sizes the workspace)
constexpr int kDecodeWgPerCu = 2;          // workgroups per compute unit the split aims at (measured best on long histories)
constexpr int kDecodeMinTiles = 4;         // a split holds at least this many 64-key tiles
constexpr int kDecodeMaxPackedRows = 128;  // query heads of one group packed into the rows of one tile

struct DecodePlan {
    int b, h, hkv, nq;       // the call as the forward kernel sees it
    int n_splits, tiles_per_split;
};

// most splits a call of this shape can get, whatever the device (the workspace is sized by it)
int decode_max_splits(int B, int Hq, int Hkv)
{
    const int G = Hq / Hkv;
    const long long base = G <= kDecodeMaxPackedRows ? (long long)B * Hkv : (long long)B * Hq;
    long long s = (kDecodeMaxWorkgroups + base - 1) / base;
    if (s > kDecodeMaxSplits) s = kDecodeMaxSplits;
    return s < 1 ? 1 : (int)s;
}

// The query heads that share a key/value head are contiguous [G, D] rows when every head has one query:
// they are handed to the kernel as ONE head of G queries (so K and V are streamed once per group, not once
// per query head).  The keys are split so that about two workgroups per compute unit are in flight.
DecodePlan plan_decode(int B, int Hq, int Hkv, int Nk, int compute_units)
{
    DecodePlan p;
    const int G = Hq / Hkv;
    if (G <= kDecodeMaxPackedRows) { p.b = B * Hkv; p.h = 1; p.hkv = 1; p.nq = G; }
    else                           { p.b = B; p.h = Hq; p.hkv = Hkv; p.nq = 1; }
    const long long base = (long long)p.b * p.h;
    const int tiles = (Nk + 63) / 64;
    long long want = ((long long)kDecodeWgPerCu * compute_units + base - 1) / base;
    const int by_tiles = tiles / kDecodeMinTiles;
    const int by_shape = decode_max_splits(B, Hq, Hkv);
    if (want > by_tiles) want = by_tiles;
    if (want > by_shape) want = by_shape;
    if (want < 1) want = 1;
    int per = (int)((tiles + want - 1) / want);
    per += per & 1;                                   // the kernel walks the tiles in pairs
    p.tiles_per_split = per;
    p.n_splits = (tiles + per - 1) / per;             // no split is empty
    return p;
}

}  // namespace

extern "C" {

int tk_attn_fwd_rect(const void* q, const void* k, const void* v, void* o, float* lse,
                     int B, int Hq, int Hkv, int Nq, int Nk, int D, int causal, float scale, void* stream)
{
    if (!q || !k || !v || !o || !lse) return TK_ERR_NULL_PTR;
    if (int rc = check_lengths(B, Hq, Hkv, Nq, Nk, D, causal)) return rc;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(lse)) return TK_ERR_MISALIGNED;
    if (int rc = check_scale(scale)) return rc;
    hipError_t e = tk::launch_attn_fwd(q, k, v, o, lse, B, Hq, Hkv, Nq, Nk, D, causal != 0, scale, (hipStream_t)stream);
    return e == hipSuccess ? TK_OK : TK_ERR_LAUNCH;
}

int tk_attn_fwd_gqa(const void* q, const void* k, const void* v, void* o, float* lse,
                    int B, int Hq, int Hkv, int N, int D, int causal, float scale, void* stream)
{
    return tk_attn_fwd_rect(q, k, v, o, lse, B, Hq, Hkv, N, N, D, causal, scale, stream);
}

int tk_attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse,
                int B, int H, int N, int D, int causal, float scale, void* stream)
{
    return tk_attn_fwd_gqa(q, k, v, o, lse, B, H, H, N, D, causal, scale, stream);
}

int tk_attn_decode_plan(int B, int Hq, int Hkv, int Nk, int D, int compute_units, int* plan)
{
    if (!plan) return TK_ERR_NULL_PTR;
    if (int rc = check_lengths(B, Hq, Hkv, 1, Nk, D, 0)) return rc;
    if (compute_units < 1) return TK_ERR_BAD_DIM;
    const DecodePlan p = plan_decode(B, Hq, Hkv, Nk, compute_units);
    plan[0] = p.b * p.h;
    plan[1] = p.nq;
    plan[2] = p.n_splits;
    plan[3] = p.tiles_per_split;
    plan[4] = decode_max_splits(B, Hq, Hkv);
    return TK_OK;
}

size_t tk_attn_decode_workspace_bytes(int B, int Hq, int Hkv, int Nk, int D)
{
    if (check_lengths(B, Hq, Hkv, 1, Nk, D, 0) != TK_OK) return 0;
    // partial O (fp32 [splits][B*Hq][D]) and partial LSE (fp32 [splits][B*Hq]), each padded to 256 bytes
    const size_t rows = (size_t)B * Hq, splits = (size_t)decode_max_splits(B, Hq, Hkv);
    const size_t o_bytes = (splits * rows * D * sizeof(float) + 255) & ~(size_t)255;
    const size_t l_bytes = (splits * rows * sizeof(float) + 255) & ~(size_t)255;
    return o_bytes + l_bytes;
}

int tk_attn_decode(const void* q, const void* k, const void* v, void* o, float* lse,
                   int B, int Hq, int Hkv, int Nk, int D, float scale,
                   void* workspace, size_t workspace_bytes, void* stream)
{
    if (!q || !k || !v || !o || !lse || !workspace) return TK_ERR_NULL_PTR;
    if (int rc = check_lengths(B, Hq, Hkv, 1, Nk, D, 0)) return rc;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(lse) || !aligned16(workspace))
        return TK_ERR_MISALIGNED;
    if (int rc = check_scale(scale)) return rc;
    if (workspace_bytes < tk_attn_decode_workspace_bytes(B, Hq, Hkv, Nk, D)) return TK_ERR_WORKSPACE_TOO_SMALL;

    int cus = 0;
    if (tk::compute_unit_count(&cus) != hipSuccess || cus < 1) return TK_ERR_LAUNCH;
    const DecodePlan p = plan_decode(B, Hq, Hkv, Nk, cus);
    hipError_t e;
    if (p.n_splits == 1) {
        e = tk::launch_attn_fwd(q, k, v, o, lse, p.b, p.h, p.hkv, p.nq, Nk, D, 0, scale, (hipStream_t)stream);
    } else {
        const size_t rows = (size_t)B * Hq;
        float* o_part = (float*)workspace;
        float* lse_part = (float*)((char*)workspace + (((size_t)decode_max_splits(B, Hq, Hkv) * rows * D * sizeof(float) + 255) & ~(size_t)255));
        e = tk::launch_attn_fwd_splitk(q, k, v, o, lse, o_part, lse_part, p.b, p.h, p.hkv, p.nq, Nk, D, scale,
                                       p.n_splits, p.tiles_per_split, (hipStream_t)stream);
    }
    return e == hipSuccess ? TK_OK : TK_ERR_LAUNCH;
}

size_t tk_attn_bwd_workspace_bytes(int B, int H, int N, int D)
{
    if (check_shape(B, H, N, D) != TK_OK) return 0;
    return delta_bytes(B, H, N);
}

size_t tk_attn_bwd_spill_workspace_bytes(int B, int Hq, int Nq, int Nk, int D)
{
    if (check_lengths(B, Hq, Hq, Nq, Nk, D, 0) != TK_OK) return 0;
    return delta_bytes(B, Hq, Nq) + tk::ds_spill_bytes(B, Hq, Nq, Nk);
}

size_t tk_attn_bwd_ds_bytes(int B, int Hq, int Nq, int Nk, int D)
{
    if (check_lengths(B, Hq, Hq, Nq, Nk, D, 0) != TK_OK) return 0;
    return tk::ds_spill_bytes(B, Hq, Nq, Nk);
}

int tk_attn_bwd_dkdv_ds(const void* q, const void* k, const void* v, const void* d_o,
                        const float* lse, const float* delta, void* dk, void* dv, void* ds,
                        int B, int Hq, int Hkv, int N, int D, int causal, float scale, void* stream)
{
    if (!q || !k || !v || !d_o || !lse || !delta || !dk || !dv || !ds) return TK_ERR_NULL_PTR;
    if (int rc = check_lengths(B, Hq, Hkv, N, N, D, causal)) return rc;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(d_o) || !aligned16(lse) ||
        !aligned16(delta) || !aligned16(dk) || !aligned16(dv) || !aligned16(ds))
        return TK_ERR_MISALIGNED;
    if (int rc = check_scale(scale)) return rc;
    hipError_t e = tk::launch_attn_bwd_dkdv(q, k, v, d_o, lse, delta, dk, dv, B, Hq, Hkv, N, N, D, causal != 0, scale,
                                            (hipStream_t)stream, ds);
    return e == hipSuccess ? TK_OK : TK_ERR_LAUNCH;
}

int tk_attn_bwd_dq_from_ds(const void* k, const void* ds, void* dq,
                           int B, int Hq, int Hkv, int N, int D, int causal, float scale, void* stream)
{
    if (!k || !ds || !dq) return TK_ERR_NULL_PTR;
    if (int rc = check_lengths(B, Hq, Hkv, N, N, D, causal)) return rc;
    if (!aligned16(k) || !aligned16(ds) || !aligned16(dq)) return TK_ERR_MISALIGNED;
    if (int rc = check_scale(scale)) return rc;
    hipError_t e = tk::launch_attn_bwd_dq_from_ds(k, ds, dq, B, Hq, Hkv, N, N, D, causal != 0, scale, (hipStream_t)stream);
    return e == hipSuccess ? TK_OK : TK_ERR_LAUNCH;
}

int tk_attn_bwd_delta(const void* o, const void* d_o, float* delta, int B, int H, int N, int D, void* stream)
{
    if (!o || !d_o || !delta) return TK_ERR_NULL_PTR;
    if (int rc = check_shape(B, H, N, D)) return rc;
    if (!aligned16(o) || !aligned16(d_o) || !aligned16(delta)) return TK_ERR_MISALIGNED;
    hipError_t e = tk::launch_attn_bwd_delta(o, d_o, delta, B, H, N, D, (hipStream_t)stream);
    return e == hipSuccess ? TK_OK : TK_ERR_LAUNCH;
}

int tk_attn_bwd_dkdv_gqa(const void* q, const void* k, const void* v, const void* d_o,
                         const float* lse, const float* delta, void* dk, void* dv,
                         int B, int Hq, int Hkv, int N, int D, int causal, float scale, void* stream)
{
    if (!q || !k || !v || !d_o || !lse || !delta || !dk || !dv) return TK_ERR_NULL_PTR;
    if (int rc = check_shape(B, Hq, N, D)) return rc;
    if (int rc = check_heads(Hq, Hkv)) return rc;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(d_o) || !aligned16(lse) ||
        !aligned16(delta) || !aligned16(dk) || !aligned16(dv))
        return TK_ERR_MISALIGNED;
    if (int rc = check_scale(scale)) return rc;
    hipError_t e = tk::launch_attn_bwd_dkdv(q, k, v, d_o, lse, delta, dk, dv, B, Hq, Hkv, N, N, D, causal != 0, scale,
                                            (hipStream_t)stream);
    return e == hipSuccess ? TK_OK : TK_ERR_LAUNCH;
}

int tk_attn_bwd_dkdv(const void* q, const void* k, const void* v, const void* d_o,
                     const float* lse, const float* delta, void* dk, void* dv,
                     int B, int H, int N, int D, int causal, float scale, void* stream)
{
    return tk_attn_bwd_dkdv_gqa(q, k, v, d_o, lse, delta, dk, dv, B, H, H, N, D, causal, scale, stream);
}

int tk_attn_bwd_dq_gqa(const void* q, const void* k, const void* v, const void* d_o,
                       const float* lse, const float* delta, void* dq,
                       int B, int Hq, int Hkv, int N, int D, int causal, float scale, void* stream)
{
    if (!q || !k || !v || !d_o || !lse || !delta || !dq) return TK_ERR_NULL_PTR;
    if (int rc = check_shape(B, Hq, N, D)) return rc;
    if (int rc = check_heads(Hq, Hkv)) return rc;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(d_o) || !aligned16(lse) ||
        !aligned16(delta) || !aligned16(dq))
        return TK_ERR_MISALIGNED;
    if (int rc = check_scale(scale)) return rc;
    hipError_t e = tk::launch_attn_bwd_dq(q, k, v, d_o, lse, delta, dq, B, Hq, Hkv, N, N, D, causal != 0, scale,
                                          (hipStream_t)stream);
    return e == hipSuccess ? TK_OK : TK_ERR_LAUNCH;
}

int tk_attn_bwd_dq_delta(const void* q, const void* k, const void* v, const void* o, const void* d_o,
                         const float* lse, float* delta, void* dq,
                         int B, int Hq, int Hkv, int N, int D, int causal, float scale, void* stream)
{
    if (!q || !k || !v || !o || !d_o || !lse || !delta || !dq) return TK_ERR_NULL_PTR;
    if (int rc = check_shape(B, Hq, N, D)) return rc;
    if (int rc = check_heads(Hq, Hkv)) return rc;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(d_o) || !aligned16(lse) ||
        !aligned16(delta) || !aligned16(dq))
        return TK_ERR_MISALIGNED;
    if (int rc = check_scale(scale)) return rc;
    hipError_t e = tk::launch_attn_bwd_dq(q, k, v, d_o, lse, nullptr, dq, B, Hq, Hkv, N, N, D, causal != 0, scale,
                                          (hipStream_t)stream, o, delta);
    return e == hipSuccess ? TK_OK : TK_ERR_LAUNCH;
}

int tk_attn_bwd_dq(const void* q, const void* k, const void* v, const void* d_o,
                   const float* lse, const float* delta, void* dq,
                   int B, int H, int N, int D, int causal, float scale, void* stream)
{
    return tk_attn_bwd_dq_gqa(q, k, v, d_o, lse, delta, dq, B, H, H, N, D, causal, scale, stream);
}

int tk_attn_bwd_rect(const void* q, const void* k, const void* v, const void* o, const void* d_o, const float* lse,
                     void* dq, void* dk, void* dv,
                     int B, int Hq, int Hkv, int Nq, int Nk, int D, int causal, float scale,
                     void* workspace, size_t workspace_bytes, void* stream)
{
    if (!q || !k || !v || !o || !d_o || !lse || !dq || !dk || !dv || !workspace) return TK_ERR_NULL_PTR;
    if (int rc = check_lengths(B, Hq, Hkv, Nq, Nk, D, causal)) return rc;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(d_o) || !aligned16(lse) ||
        !aligned16(dq) || !aligned16(dk) || !aligned16(dv) || !aligned16(workspace))
        return TK_ERR_MISALIGNED;
    if (int rc = check_scale(scale)) return rc;
    if (workspace_bytes < tk_attn_bwd_workspace_bytes(B, Hq, Nq, D)) return TK_ERR_WORKSPACE_TOO_SMALL;

    hipStream_t s = (hipStream_t)stream;
    float* delta = (float*)workspace;
    if (workspace_bytes >= tk_attn_bwd_spill_workspace_bytes(B, Hq, Nq, Nk, D)) {
        // Large workspace: 10*D flops per (query, key) pair instead of 14*D.  Delta on its own, then dK/dV,
        // which also leaves its bf16 dS blocks behind Delta in the workspace, then dQ = scale * dS K from them.
        void* ds = (char*)workspace + delta_bytes(B, Hq, Nq);
        if (tk::launch_attn_bwd_delta(o, d_o, delta, B, Hq, Nq, D, s) != hipSuccess) return TK_ERR_LAUNCH;
        if (tk::launch_attn_bwd_dkdv(q, k, v, d_o, lse, delta, dk, dv, B, Hq, Hkv, Nq, Nk, D, causal != 0, scale, s, ds) != hipSuccess)
            return TK_ERR_LAUNCH;
        if (tk::launch_attn_bwd_dq_from_ds(k, ds, dq, B, Hq, Hkv, Nq, Nk, D, causal != 0, scale, s) != hipSuccess)
            return TK_ERR_LAUNCH;
        return TK_OK;
    }
    // Small workspace (Delta only): dS is recomputed by a dQ kernel of its own.
    // 1. dQ per query tile; the kernel also forms Delta = rowsum(dO * O) for its rows (each lane holds its
    //    query's dO row anyway) and leaves it in the workspace, which saves a pass over O and dO
    if (tk::launch_attn_bwd_dq(q, k, v, d_o, lse, nullptr, dq, B, Hq, Hkv, Nq, Nk, D, causal != 0, scale, s, o, delta) != hipSuccess)
        return TK_ERR_LAUNCH;
    // 2. dK, dV per key tile of every key/value head, with that Delta
    if (tk::launch_attn_bwd_dkdv(q, k, v, d_o, lse, delta, dk, dv, B, Hq, Hkv, Nq, Nk, D, causal != 0, scale, s) != hipSuccess)
        return TK_ERR_LAUNCH;
    return TK_OK;
}

int tk_attn_bwd_gqa(const void* q, const void* k, const void* v, const void* o, const void* d_o, const float* lse,
                    void* dq, void* dk, void* dv,
                    int B, int Hq, int Hkv, int N, int D, int causal, float scale,
                    void* workspace, size_t workspace_bytes, void* stream)
{
    return tk_attn_bwd_rect(q, k, v, o, d_o, lse, dq, dk, dv, B, Hq, Hkv, N, N, D, causal, scale,
                            workspace, workspace_bytes, stream);
}

int tk_attn_bwd(const void* q, const void* k, const void* v, const void* o, const void* d_o, const float* lse,
                void* dq, void* dk, void* dv,
                int B, int H, int N, int D, int causal, float scale,
                void* workspace, size_t workspace_bytes, void* stream)
{
    return tk_attn_bwd_gqa(q, k, v, o, d_o, lse, dq, dk, dv, B, H, H, N, D, causal, scale,
                           workspace, workspace_bytes, stream);
}

int tk_attn_bwd_noalloc(const void* q, const void* k, const void* v, const void* o, const void* d_o, const float* lse,
                        void* dq, void* dk, void* dv,
                        int B, int H, int N, int D, int causal, float scale, void* stream)
{
    if (!q || !k || !v || !o || !d_o || !lse || !dq || !dk || !dv) return TK_ERR_NULL_PTR;
    if (int rc = check_lengths(B, H, H, N, N, D, causal)) return rc;
    if ((size_t)B * H * N > kNoallocScratchFloats) return TK_ERR_SCRATCH_LIMIT;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(d_o) || !aligned16(lse) ||
        !aligned16(dq) || !aligned16(dk) || !aligned16(dv))
        return TK_ERR_MISALIGNED;
    if (int rc = check_scale(scale)) return rc;
    float* delta = noalloc_scratch();       // a pointer, never the array's name: that is not a device address in host code
    if (!delta) return TK_ERR_LAUNCH;
    hipStream_t s = (hipStream_t)stream;
    // the same two kernels as tk_attn_bwd in its small-workspace form; Delta is written in full by the first
    // before the second reads it, so nothing in the scratch has to be cleared
    if (tk::launch_attn_bwd_dq(q, k, v, d_o, lse, nullptr, dq, B, H, H, N, N, D, causal != 0, scale, s, o, delta) != hipSuccess)
        return TK_ERR_LAUNCH;
    if (tk::launch_attn_bwd_dkdv(q, k, v, d_o, lse, delta, dk, dv, B, H, H, N, N, D, causal != 0, scale, s) != hipSuccess)
        return TK_ERR_LAUNCH;
    return TK_OK;
}

size_t tk_attn_bwd_noalloc_max_rows(void) { return kNoallocScratchFloats; }

int tk_gemm(const void* a, const void* b, void* c, int M, int N, int K, void* stream)
{
    if (!a || !b || !c) return TK_ERR_NULL_PTR;
    if (M < 1 || N < 8 || K < 8 || N % 8 || K % 8) return TK_ERR_BAD_DIM;     // every row of A, B and C starts on 16 bytes
    if ((long long)((M + 255) / 256) * ((N + 255) / 256) > 0x7fffffffLL) return TK_ERR_BAD_DIM;
    if (!aligned16(a) || !aligned16(b) || !aligned16(c)) return TK_ERR_MISALIGNED;
    hipError_t e = tk::launch_gemm(a, b, c, M, N, K, (hipStream_t)stream);
    return e == hipSuccess ? TK_OK : TK_ERR_LAUNCH;
}

int tk_rotary(const void* x, const void* sin_table, const void* cos_table, void* o,
              int B, int H, int N, int D, void* stream)
{
    if (!x || !sin_table || !cos_table || !o) return TK_ERR_NULL_PTR;
    if (int rc = check_shape(B, H, N, D)) return rc;
    if (!aligned16(x) || !aligned16(sin_table) || !aligned16(cos_table) || !aligned16(o)) return TK_ERR_MISALIGNED;
    hipError_t e = tk::launch_rotary(x, sin_table, cos_table, o, B, H, N, D, (hipStream_t)stream);
    return e == hipSuccess ? TK_OK : TK_ERR_LAUNCH;
}

int tk_mfma_probe(const void* operands, float* sink, int workgroups, int iters, void* stream)
{
    if (!operands || !sink) return TK_ERR_NULL_PTR;
    if (workgroups < 1 || workgroups > 65536 || iters < 1) return TK_ERR_BAD_DIM;
    if (!aligned16(operands) || !aligned16(sink)) return TK_ERR_MISALIGNED;
    hipError_t e = tk::launch_mfma_probe(operands, sink, workgroups, iters, (hipStream_t)stream);
    return e == hipSuccess ? TK_OK : TK_ERR_LAUNCH;
}

const char* tk_status_string(int status)
{
    switch (status) {
        case TK_OK: return "ok";
        case TK_ERR_NULL_PTR: return "null pointer";
        case TK_ERR_BAD_DIM: return "unsupported shape (D must be 64 or 128; B, H, N >= 1; Hkv must divide Hq; causal needs Nq <= Nk)";
        case TK_ERR_MISALIGNED: return "pointer not 16-byte aligned";
        case TK_ERR_BAD_SCALE: return "scale must be finite and > 0";
        case TK_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case TK_ERR_LAUNCH: return "kernel launch failed";
        case TK_ERR_SCRATCH_LIMIT: return "B*H*N exceeds the built-in scratch of tk_attn_bwd_noalloc (use tk_attn_bwd with a workspace)";
        default: return "unknown status";
    }
}

int tk_attn_version(void) { return 100; }

}  // extern "C"
