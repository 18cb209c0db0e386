#!/usr/bin/env python3
"""Benchmark of the fused attention hot path on one MI355X.

One step = one forward (tk_attn_fwd) plus one backward (tk_attn_bwd) over one synthetic batch
of the target shape B=16, H=16, N=4096, D=128, causal, bf16 - the shape the performance
target is quoted on.  Inputs are resident in HBM before the timed region.

Prints ONE JSON line.  `value` is the whole step's TFLOP/s under the usual convention
(forward 4*B*H*N^2*D, backward 2.5x that, halved when causal).  `roofline` describes the
dominant kernel (the backward dK/dV/dQ kernel) against the dense bf16 MFMA peak, timed
with HIP events on the launch stream; `cpu_baseline` is the fp64 oracle timed on the
host cores of the same box on a few heads of the same workload.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 (published: 2.5 PFLOP/s)

# HBM bytes per launch of each op's dominant kernel on its default workload, read from the committed
# counter runs (rocprofv3 --pmc FETCH_SIZE, then WRITE_SIZE, each scaled by what a plain 1 GiB copy
# reads in the same run; the files under profiles/ give the commands and the raw counters).  The
# live run cannot collect counters itself, so other workloads report null.
MEASURED_TRAFFIC = {
    "fwdbwd_causal_b16_h16_n4096_d128": {"kernel": "attn_bwd_dkdv_kernel", "bytes": 1.802e9 + 4.966e9,      # (the form that stores dS)
                                         "source": "profiles/bench_fwdbwd_causal_b16_h16_n4096_d128.txt"},
    "fwdbwd_causal_b16_h16_n4096_d64/recompute": {"kernel": "attn_bwd_dkdv_kernel", "bytes": 0.583e9 + 0.268e9,
                                                  "source": "profiles/bench_fwdbwd_causal_b16_h16_n4096_d64.txt"},
    "gemm_8192x8192x8192": {"kernel": "gemm_kernel", "bytes": 1.61e9 + 0.148e9, "source": "profiles/gemm_8192x8192x8192.txt"},
    "decode_b16_hq32_hkv8_nk8192_d128": {"kernel": "attn_fwd_kernel", "bytes": 537.2e6 + 0.54e6, "source": "profiles/decode_b16_hq32_hkv8_nk8192_d128.txt"},
    "rotary_fwdbwd_causal_b16_h16_n4096_d128": {"kernel": "rotary_kernel", "bytes": 0.270e9 + 0.268e9, "source": "profiles/rotary_b16_h16_n4096_d128.txt"},
}


def measured_traffic(key, kernel):
    t = MEASURED_TRAFFIC.get(key)
    if t is None or t["kernel"] != kernel:
        return {"traffic": None}
    return {"traffic": t["bytes"], "traffic_unit": "HBM bytes per launch", "traffic_source": t["source"]}

HBM_PEAK_GBS = 8000.0


def bench_gemm(args, attn, torch, dev, M=8192, N=8192, K=8192):
    """bf16 GEMM C = A B on normal data: a kernel of MFMAs and LDS traffic only (MFMA roofline)."""
    g = torch.Generator().manual_seed(20399 + 840)
    a = torch.randn(M, K, generator=g).to(torch.bfloat16)
    b = torch.randn(K, N, generator=g).to(torch.bfloat16)
    ad, bd = a.to(dev), b.to(dev)
    c = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
    stream = torch.cuda.current_stream()

    def step():
        rc = attn.tk_gemm(ad, bd, c, M, N, K, stream)
        if rc != attn.TK_OK:
            raise attn.TkAttnError(rc, "tk_gemm")

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record(stream)
    for _ in range(args.steps):
        step()
    e1.record(stream)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    kernel_ms = e0.elapsed_time(e1) / args.steps
    flops = 2.0 * M * N * K
    tflops = flops / (kernel_ms * 1e-3) / 1e12
    out = {"metric": f"bf16 GEMM TFLOPS (M=N=K={M})", "value": round(flops / (ms_per_step * 1e-3) / 1e12, 2), "unit": "TFLOP/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": f"gemm_{M}x{N}x{K}", "M": M, "N": N, "K": K},
           "roofline": {"kernel": "gemm_kernel", "bound": "mfma", "achieved": round(tflops, 2), "peak": MFMA_BF16_PEAK_TFLOPS,
                        "unit": "TFLOP/s", "frac": round(tflops / MFMA_BF16_PEAK_TFLOPS, 4),
                        **measured_traffic(f"gemm_{M}x{N}x{K}", "gemm_kernel"), "flops_per_launch": flops}}
    if not args.no_cpu_baseline:
        from oracle import attn_oracle as orc
        rows = min(M, 16)
        a64, b64 = a[:rows].double().numpy(), b.double().numpy()
        c0 = time.perf_counter()
        reps = 0
        while time.perf_counter() - c0 < min(args.cpu_seconds, 10.0):
            orc.gemm(a64, b64)
            reps += 1
        spent = time.perf_counter() - c0
        out["cpu_baseline"] = {"value": round(reps * 2.0 * rows * N * K / spent / 1e12, 6), "unit": "TFLOP/s",
                               "cores": orc.num_threads(), "kind": "oracle",
                               "sample": f"fp64 oracle on the first {rows} of {M} rows of C, {reps} passes, {spent:.1f} s"}
    print(json.dumps(out))


def bench_rotary(args, attn, torch, dev, w, x):
    """Rotary positional encoding on the workload's Q tensor: an HBM-bound stream (read x, write o)."""
    B, H, N, D = w.B, w.H, w.N, w.D
    g = torch.Generator().manual_seed(w.seed)
    theta = torch.rand(N, D // 2, generator=g) * 8 - 4
    sn, cs = torch.sin(theta).to(torch.bfloat16), torch.cos(theta).to(torch.bfloat16)
    xd, snd, csd = x.to(dev), sn.to(dev), cs.to(dev)
    o = torch.empty_like(xd)
    stream = torch.cuda.current_stream()

    def step():
        rc = attn.tk_rotary(xd, snd, csd, o, B, H, N, D, stream)
        if rc != attn.TK_OK:
            raise attn.TkAttnError(rc, "tk_rotary")

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record(stream)
    for _ in range(args.steps):
        step()
    e1.record(stream)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    kernel_ms = e0.elapsed_time(e1) / args.steps
    nbytes = 2 * B * H * N * D * 2 + 2 * N * (D // 2) * 2        # read x, write o, read both tables once
    gbps = nbytes / (kernel_ms * 1e-3) / 1e9
    out = {"metric": f"rotary GB/s (bf16, {w.name})", "value": round(nbytes / (ms_per_step * 1e-3) / 1e9, 1), "unit": "GB/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": "rotary_" + w.name, "B": B, "H": H, "N": N, "D": D},
           "roofline": {"kernel": "rotary_kernel", "bound": "hbm", "achieved": round(gbps, 1), "peak": HBM_PEAK_GBS,
                        "unit": "GB/s", "frac": round(gbps / HBM_PEAK_GBS, 4),
                        **measured_traffic("rotary_" + w.name, "rotary_kernel"), "bytes_per_launch": nbytes}}
    if not args.no_cpu_baseline:
        from oracle import attn_oracle as orc
        nh = min(B * H, 64)
        xs = x.reshape(B * H, N, D)[:nh].double().numpy()
        c0 = time.perf_counter()
        reps = 0
        while time.perf_counter() - c0 < min(args.cpu_seconds, 5.0):
            orc.rotary(xs, sn.double().numpy(), cs.double().numpy())
            reps += 1
        spent = time.perf_counter() - c0
        out["cpu_baseline"] = {"value": round(reps * nh * N * D * 2 * 2 / spent / 1e9, 2), "unit": "GB/s (of bf16-sized traffic)",
                               "cores": orc.num_threads(), "kind": "oracle",
                               "sample": f"fp64 oracle on {nh} of {B * H} heads, {reps} passes, {spent:.1f} s"}
    print(json.dumps(out))


def bench_decode(args, attn, torch, dev, B=16, Hq=32, Hkv=8, Nk=8192, D=128):
    """One query per head against a long key/value history: bound by reading K and V once (HBM roofline)."""
    g = torch.Generator().manual_seed(20399 + 1152)
    q = torch.randn(B, Hq, 1, D, generator=g).to(torch.bfloat16)
    k = torch.randn(B, Hkv, Nk, D, generator=g).to(torch.bfloat16)
    v = torch.randn(B, Hkv, Nk, D, generator=g).to(torch.bfloat16)
    qd, kd, vd = q.to(dev), k.to(dev), v.to(dev)
    o = torch.empty_like(qd)
    lse = torch.empty((B, Hq, 1), dtype=torch.float32, device=dev)
    need = attn.tk_attn_decode_workspace_bytes(B, Hq, Hkv, Nk, D)
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    scale = 1.0 / math.sqrt(D)
    stream = torch.cuda.current_stream()

    def step():
        rc = attn.tk_attn_decode(qd, kd, vd, o, lse, B, Hq, Hkv, Nk, D, scale, ws, need, stream)
        if rc != attn.TK_OK:
            raise attn.TkAttnError(rc, "tk_attn_decode")

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record(stream)
    for _ in range(args.steps):
        step()
    e1.record(stream)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    kernel_ms = e0.elapsed_time(e1) / args.steps              # the split forward and its merge kernel together
    nbytes = 2 * B * Hkv * Nk * D * 2 + 2 * B * Hq * D * 2 + B * Hq * 4      # K and V once; Q in, O and LSE out
    gbps = nbytes / (kernel_ms * 1e-3) / 1e9
    name = f"decode_b{B}_hq{Hq}_hkv{Hkv}_nk{Nk}_d{D}"
    out = {"metric": f"decode attention GB/s of K and V (bf16, {name})", "value": round(nbytes / (ms_per_step * 1e-3) / 1e9, 1),
           "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": name, "B": B, "Hq": Hq, "Hkv": Hkv, "Nq": 1, "Nk": Nk, "D": D},
           "roofline": {"kernel": "attn_fwd_kernel (keys split) + attn_fwd_combine_kernel", "bound": "hbm", "achieved": round(gbps, 1),
                        "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(gbps / HBM_PEAK_GBS, 4),
                        **measured_traffic(name, "attn_fwd_kernel"), "bytes_per_launch": nbytes}}
    # the same call through the plain entry point (one workgroup per query head streams the whole history)
    o2 = torch.empty_like(qd)
    for _ in range(2):
        attn.tk_attn_fwd_rect(qd, kd, vd, o2, lse, B, Hq, Hkv, 1, Nk, D, False, scale, stream)
    torch.cuda.synchronize()
    e0.record(stream)
    for _ in range(args.steps):
        attn.tk_attn_fwd_rect(qd, kd, vd, o2, lse, B, Hq, Hkv, 1, Nk, D, False, scale, stream)
    e1.record(stream)
    torch.cuda.synchronize()
    out["plain_entry_point_ms"] = round(e0.elapsed_time(e1) / args.steps, 4)
    out["decode_ms"] = round(kernel_ms, 4)
    if not args.no_cpu_baseline:
        from oracle import attn_oracle as orc
        nb = min(B, 4)
        c0 = time.perf_counter()
        reps = 0
        while time.perf_counter() - c0 < min(args.cpu_seconds, 5.0):
            orc.rect_fwd(q[:nb].double().numpy(), k[:nb].double().numpy(), v[:nb].double().numpy(), False, scale)
            reps += 1
        spent = time.perf_counter() - c0
        out["cpu_baseline"] = {"value": round(reps * nbytes * nb / B / spent / 1e9, 2), "unit": "GB/s (of bf16-sized traffic)",
                               "cores": orc.num_threads(), "kind": "oracle",
                               "sample": f"fp64 oracle on {nb} of {B} batch entries, {reps} passes, {spent:.1f} s"}
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", type=int, default=6, help="index into workloads.WORKLOADS (default: the target shape)")
    ap.add_argument("--op", choices=["attention", "rotary", "gemm", "decode"], default="attention",
                    help="attention (default: the headline fwd+bwd step), the rotary kernel on the same tensor shape, "
                         "the bf16 GEMM (8192^3), or the decode-shaped forward (one query per head, B16 Hq32 Hkv8 Nk8192 D128)")
    ap.add_argument("--bwd-form", choices=["auto", "spill", "recompute"], default="auto",
                    help="spill: tk_attn_bwd gets the large workspace, its dK/dV kernel stores dS and dQ is formed "
                         "from it (Delta, dK/dV, dQ-from-dS kernels); recompute: Delta-only workspace, dQ kernel recomputes dS; "
                         "auto (default): spill at D = 128, recompute at D = 64 (the faster form of each)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="budget for the oracle sample")
    ap.add_argument("--no-mfma-probe", action="store_true", help="skip the bare-MFMA ceiling measurement")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy a few times, so that a counter run of this same "
                         "command can scale FETCH_SIZE / WRITE_SIZE by what they read for a known transfer")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; heads are independent, so N GPUs would each run "
              "this same benchmark on B*H/N heads (no multi-GPU figure is produced).", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2410_20399_amd import attn, workloads

    attn.load_library()                       # raises if the HIP library is missing: no fallback
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    dev = torch.device("cuda:0")
    if args.op == "gemm":
        return bench_gemm(args, attn, torch, dev)
    if args.op == "decode":
        return bench_decode(args, attn, torch, dev)
    w = workloads.WORKLOADS[args.workload]
    q, k, v, d_o = workloads.make_inputs(w, need_do=True)
    qd, kd, vd, dod = (t.to(dev) for t in (q, k, v, d_o))
    B, H, N, D = w.B, w.H, w.N, w.D
    if args.op == "rotary":
        return bench_rotary(args, attn, torch, dev, w, q)
    Hkv = w.kv_heads                          # == H unless the workload is grouped-query
    o = torch.empty_like(qd)
    lse = torch.empty((B, H, N), dtype=torch.float32, device=dev)
    dq, dk, dv = torch.empty_like(qd), torch.empty_like(kd), torch.empty_like(vd)
    if args.bwd_form == "auto":
        args.bwd_form = "spill" if D == 128 else "recompute"
    spill = args.bwd_form == "spill"
    ws = attn.alloc_bwd_workspace(B, H, N, D, dev, spill=spill)     # allocated once, outside every timed region
    ws_bytes = ws.numel()
    delta = ws[:B * H * N * 4].view(torch.float32)      # the workspace starts with the Delta array
    delta_pad = (B * H * N * 4 + 255) & ~255
    ds = ws[delta_pad:] if spill else None              # ... followed by the dS blocks in the spill form
    stream = torch.cuda.current_stream()

    def check(rc, what):
        if rc != attn.TK_OK:
            raise attn.TkAttnError(rc, what)

    # multi-head workloads go through tk_attn_fwd / tk_attn_bwd and their stage entry points,
    # grouped-query ones through the *_gqa entry points (the same kernels)
    if Hkv == H:
        fwd_call = lambda: attn.tk_attn_fwd(qd, kd, vd, o, lse, B, H, N, D, w.causal, w.scale, stream)
        bwd_call = lambda: attn.tk_attn_bwd(qd, kd, vd, o, dod, lse, dq, dk, dv, B, H, N, D, w.causal, w.scale, ws, ws_bytes, stream)
        dkdv_call = lambda: attn.tk_attn_bwd_dkdv(qd, kd, vd, dod, lse, delta, dk, dv, B, H, N, D, w.causal, w.scale, stream)
        dq_call = lambda: attn.tk_attn_bwd_dq(qd, kd, vd, dod, lse, delta, dq, B, H, N, D, w.causal, w.scale, stream)
    else:
        fwd_call = lambda: attn.tk_attn_fwd_gqa(qd, kd, vd, o, lse, B, H, Hkv, N, D, w.causal, w.scale, stream)
        bwd_call = lambda: attn.tk_attn_bwd_gqa(qd, kd, vd, o, dod, lse, dq, dk, dv, B, H, Hkv, N, D, w.causal, w.scale, ws, ws_bytes, stream)
        dkdv_call = lambda: attn.tk_attn_bwd_dkdv_gqa(qd, kd, vd, dod, lse, delta, dk, dv, B, H, Hkv, N, D, w.causal, w.scale, stream)
        dq_call = lambda: attn.tk_attn_bwd_dq_gqa(qd, kd, vd, dod, lse, delta, dq, B, H, Hkv, N, D, w.causal, w.scale, stream)

    def step():
        check(fwd_call(), "tk_attn_fwd")
        if w.backward:
            check(bwd_call(), "tk_attn_bwd")

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    flops_fwd = w.fwd_flops()
    flops_bwd = w.bwd_flops() if w.backward else 0.0
    value = (flops_fwd + flops_bwd) / (ms_per_step * 1e-3) / 1e12

    # ---- per-kernel durations: the same kernels through the stage entry points, HIP events on the launch stream

    # recompute form: the backward runs two kernels: dQ with Delta folded in, then dK/dV; the stand-alone Delta
    # pass (tk_attn_bwd_delta, an HBM stream over O and dO) is timed too, as the HBM-bound reference point.
    # spill form: three kernels: Delta, dK/dV storing dS, dQ from the stored dS.
    dq_delta_call = lambda: attn.tk_attn_bwd_dq_delta(qd, kd, vd, o, dod, lse, delta, dq, B, H, Hkv, N, D, w.causal, w.scale, stream)
    delta_call = lambda: attn.tk_attn_bwd_delta(o, dod, delta, B, H, N, D, stream)
    stages = [("attn_fwd_kernel", lambda: check(fwd_call(), "fwd"))]
    if w.backward and spill:
        stages += [
            ("attn_bwd_delta_kernel", lambda: check(delta_call(), "delta")),
            ("attn_bwd_dkdv_kernel", lambda: check(attn.tk_attn_bwd_dkdv_ds(qd, kd, vd, dod, lse, delta, dk, dv, ds, B, H, Hkv, N, D,
                                                                            w.causal, w.scale, stream), "dkdv+ds")),
            ("attn_bwd_dq_from_ds_kernel", lambda: check(attn.tk_attn_bwd_dq_from_ds(kd, ds, dq, B, H, Hkv, N, D, w.causal, w.scale, stream), "dq from ds")),
        ]
    elif w.backward:
        stages += [
            ("attn_bwd_dq_kernel", lambda: check(dq_delta_call(), "dq+delta")),
            ("attn_bwd_dkdv_kernel", lambda: check(dkdv_call(), "dkdv")),
            ("attn_bwd_delta_kernel", lambda: check(delta_call(), "delta")),
        ]
    kernel_ms = {name: 0.0 for name, _ in stages}
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(len(stages) + 1)] for _ in range(args.steps)]
    for s in range(args.steps):
        evs[s][0].record(stream)
        for i, (_, fn) in enumerate(stages):
            fn()
            evs[s][i + 1].record(stream)
    torch.cuda.synchronize()
    for s in range(args.steps):
        for i, (name, _) in enumerate(stages):
            kernel_ms[name] += evs[s][i].elapsed_time(evs[s][i + 1]) / args.steps

    fwd_tflops = flops_fwd / (kernel_ms["attn_fwd_kernel"] * 1e-3) / 1e12
    out = {
        "metric": "attention fwd+bwd TFLOPS (bf16, causal, N=4096, D=128)" if args.workload == 6 else f"attention TFLOPS ({w.name})",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "B": B, "H": H, "Hkv": Hkv, "N": N, "D": D, "causal": w.causal,
                   "pass": "fwd+bwd" if w.backward else "fwd",
                   **({"bwd_form": args.bwd_form, "bwd_workspace_bytes": ws_bytes} if w.backward else {}),
                   "flop_convention": "fwd 4*B*H*N^2*D, bwd 2.5x fwd, halved when causal"},
        "frac_of_mfma_peak": round(value / MFMA_BF16_PEAK_TFLOPS, 4),
        "fwd": {"ms": round(kernel_ms["attn_fwd_kernel"], 4), "tflops": round(fwd_tflops, 2),
                "frac_of_mfma_peak": round(fwd_tflops / MFMA_BF16_PEAK_TFLOPS, 4)},
        "kernel_ms": {k_: round(v_, 4) for k_, v_ in kernel_ms.items()},
    }
    if w.backward:
        # what tk_attn_bwd launches in this form
        dq_name = "attn_bwd_dq_from_ds_kernel" if spill else "attn_bwd_dq_kernel"
        bwd_ms = kernel_ms[dq_name] + kernel_ms["attn_bwd_dkdv_kernel"] + (kernel_ms["attn_bwd_delta_kernel"] if spill else 0.0)
        bwd_tflops = flops_bwd / (bwd_ms * 1e-3) / 1e12
        # the dK/dV kernel executes four of the backward's five products (S, dP, dV, dK: 8*D flops per kept
        # query-key pair); the recomputing dQ kernel three (S, dP, dQ: 6*D), the dQ-from-dS kernel one (2*D)
        dkdv_flops = flops_bwd * 4.0 / 5.0
        main_tflops = dkdv_flops / (kernel_ms["attn_bwd_dkdv_kernel"] * 1e-3) / 1e12
        dq_tflops = flops_bwd * (1.0 if spill else 3.0) / 5.0 / (kernel_ms[dq_name] * 1e-3) / 1e12
        out["bwd"] = {"ms": round(bwd_ms, 4), "tflops": round(bwd_tflops, 2),
                      "frac_of_mfma_peak": round(bwd_tflops / MFMA_BF16_PEAK_TFLOPS, 4)}
        delta_bytes = 2 * B * H * N * D * 2 + B * H * N * 4       # read O, dO; write Delta
        out["delta_stage"] = {"ms": round(kernel_ms["attn_bwd_delta_kernel"], 4),
                              "algorithmic_GBps": round(delta_bytes / (kernel_ms["attn_bwd_delta_kernel"] * 1e-3) / 1e9, 1),
                              "hbm_peak_GBps": HBM_PEAK_GBS,
                              "frac_of_hbm_peak": round(delta_bytes / (kernel_ms["attn_bwd_delta_kernel"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        out["dq_kernel"] = {"name": dq_name, "ms": round(kernel_ms[dq_name], 4), "executed_tflops": round(dq_tflops, 2),
                            "frac_of_mfma_peak": round(dq_tflops / MFMA_BF16_PEAK_TFLOPS, 4)}
        if spill:
            # kept pairs -> bytes of dS the dQ-from-dS kernel reads back (2 bytes per pair; diagonal blocks are read whole)
            ds_read = flops_bwd / (10.0 * D) * 2.0
            out["dq_kernel"]["algorithmic_ds_GBps"] = round(ds_read / (kernel_ms[dq_name] * 1e-3) / 1e9, 1)
            out["dq_kernel"]["frac_of_hbm_peak"] = round(ds_read / (kernel_ms[dq_name] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
        out["roofline"] = {"kernel": "attn_bwd_dkdv_kernel", "bound": "mfma", "achieved": round(main_tflops, 2),
                           "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                           "frac": round(main_tflops / MFMA_BF16_PEAK_TFLOPS, 4),
                           **measured_traffic(w.name + ("" if spill else "/recompute"), "attn_bwd_dkdv_kernel"),
                           "flops_per_launch": dkdv_flops}
    else:
        out["roofline"] = {"kernel": "attn_fwd_kernel", "bound": "mfma", "achieved": round(fwd_tflops, 2),
                           "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                           "frac": round(fwd_tflops / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None}

    # ---- what the matrix pipe sustains on its own: a bare MFMA stream, one wave per SIMD, timed
    # with constant operands (few wires toggle, the chip holds a high clock) and with the
    # workload's own kind of data (normal bf16).  The second figure is the practical ceiling of any
    # kernel fed with such data; the roofline fractions above stay priced against the published peak.
    if not args.no_mfma_probe:
        cus = torch.cuda.get_device_properties(dev).multi_processor_count
        iters = 4000
        probe_flops = cus * 4 * iters * 32 * (32 * 32 * 16 * 2)
        sink = torch.empty(cus * 256, dtype=torch.float32, device=dev)
        res = {}
        gen = torch.Generator().manual_seed(20399)
        for kind in ("constant", "normal"):
            ops = (torch.ones(16 * 256 * 8) if kind == "constant" else torch.randn(16 * 256 * 8, generator=gen)).to(torch.bfloat16).to(dev)
            check(attn.tk_mfma_probe(ops, sink, cus, iters, stream), "probe")
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(5):
                check(attn.tk_mfma_probe(ops, sink, cus, iters, stream), "probe")
            e1.record(stream)
            torch.cuda.synchronize()
            res[kind] = round(probe_flops / (e0.elapsed_time(e1) / 5 * 1e-3) / 1e12, 1)
        out["mfma_only_tflops"] = {"constant_operands": res["constant"], "normal_operands": res["normal"],
                                   "note": "bare v_mfma_f32_32x32x16_bf16 stream, one wave per SIMD, whole chip"}

    if args.copy_calibration:
        src = torch.empty(1 << 29, dtype=torch.bfloat16, device=dev).fill_(1.0)   # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        out["copy_calibration"] = {"bytes_read": src.numel() * 2, "bytes_written": dst.numel() * 2, "launches": 3}
        del src, dst

    # ---- CPU baseline: the oracle as it stands, on a bounded sample of the same workload
    if not args.no_cpu_baseline:
        from oracle import attn_oracle as orc
        # one sample = one key/value head with the query heads of its group (one head when multi-head)
        G = H // Hkv
        heads, spent, cpu_flops = [], 0.0, 0.0
        per_group = (flops_fwd + flops_bwd) / (B * Hkv)
        n_max = min(64, B * Hkv)
        for idx in range(n_max):
            b, hk = divmod(idx * (B * Hkv // n_max), Hkv)
            qs = q[b:b + 1, hk * G:(hk + 1) * G].double().numpy()
            ks, vs = k[b:b + 1, hk:hk + 1].double().numpy(), v[b:b + 1, hk:hk + 1].double().numpy()
            c0 = time.perf_counter()
            if G == 1:
                orc.attn_fwd(qs, ks, vs, w.causal, w.scale)
            else:
                orc.gqa_fwd(qs, ks, vs, w.causal, w.scale)
            if w.backward:
                dos = d_o[b:b + 1, hk * G:(hk + 1) * G].double().numpy()
                if G == 1:
                    orc.attn_bwd(qs, ks, vs, dos, w.causal, w.scale)
                else:
                    orc.gqa_bwd(qs, ks, vs, dos, w.causal, w.scale)
            spent += time.perf_counter() - c0
            cpu_flops += per_group
            heads.append([b, hk])
            if spent >= args.cpu_seconds:
                break
        out["cpu_baseline"] = {"value": round(cpu_flops / spent / 1e12, 6), "unit": "TFLOP/s",
                               "cores": orc.num_threads(), "kind": "oracle",
                               "sample": f"fp64 oracle fwd{'+bwd' if w.backward else ''} on {len(heads)} of {B * Hkv} "
                                         f"{'heads' if G == 1 else f'key/value heads (each with its {G} query heads)'} "
                                         f"(b,h)={heads[0]}..{heads[-1]} in steps of {B * Hkv // n_max} flat heads, {spent:.1f} s, same FLOP convention"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
