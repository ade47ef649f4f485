#!/usr/bin/env python3
"""Benchmark of the implicit-im2col convolution on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--layer cfg2] [--no-cpu] [--no-layers]

A step is one iconv_fwd call (the whole hot path: tile decomposition, on-the-fly im2col gather,
MFMA contraction, epilogue) over one batch of seeded synthetic input already resident in device
memory.  The headline workload is the ResNet-style 3x3 layer `cfg2`; the other benchmark layers
are timed briefly and reported under "layers".  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_TFLOPS = 2516.6   # bf16/fp16 dense MFMA, MI355X datasheet (256 CU x 2.4 GHz x 4096 flop/clk)
PEAK_HBM_GBS = 8000.0       # HBM3E, MI355X datasheet


def time_launches(fn, steps, warmup, torch):
    """Average time of one call in ms: `steps` back-to-back launches between two events recorded
    on the stream the kernels are launched on (torch's current stream)."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--layer", default=None, help="headline layer (default cfg2)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing leg")
    ap.add_argument("--no-layers", action="store_true", help="skip the per-layer table")
    ap.add_argument("--variant", type=int, default=-1, help="force a tile variant (sweeps)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; sharding over the batch needs no exchange step "
              "and is described in DESIGN.md. Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads
    from paper_2110_03901_amd import binding as B

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    B.iconv_set_variant(args.variant)

    def prepare(L):
        code = B.DTYPE_CODES[L.dtype]
        x, w = workloads.make_inputs(L)
        xd, wd = B.to_device(x, code), B.to_device(w, code)
        y = B.empty_output(L.N, L.P, L.Q, L.K, code)
        sa = L.shape_args()
        return code, (x, w), (lambda: B.iconv_fwd(xd, wd, y, *sa, code)), (xd, wd, y)

    def explicit_runner(L, code, bufs):
        xd, wd, y = bufs
        sa = L.shape_args()
        nbytes = B.iconv_workspace_bytes(B.ALGO_EXPLICIT, *sa, code)
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
        full = lambda: B.iconv_fwd_explicit(xd, wd, y, ws, nbytes, *sa, code)
        low = lambda: B.iconv_im2col(xd, ws, nbytes, L.N, L.H, L.W, L.C, L.R, L.S, L.stride, L.pad, L.dilation, code)
        return nbytes, full, low

    head_name = args.layer or workloads.BENCH_LAYER
    L = workloads.LAYERS[head_name]
    code, host_in, run, bufs = prepare(L)

    # ---- headline: exactly `steps` timed launches after `warmup` untimed ones -----------------
    ms = time_launches(run, args.steps, args.warmup, torch)
    tflops = L.flops / (ms * 1e-3) / 1e12
    gbs = L.algorithmic_bytes(4) / (ms * 1e-3) / 1e9
    mfma_bound = (L.flops / PEAK_MFMA_TFLOPS / 1e12) >= (L.algorithmic_bytes(4) / PEAK_HBM_GBS / 1e9)
    if mfma_bound:
        roofline = {"bound": "mfma", "achieved": round(tflops, 2), "peak": PEAK_MFMA_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(tflops / PEAK_MFMA_TFLOPS, 4), "traffic": None}
    else:
        roofline = {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": round(gbs / PEAK_HBM_GBS, 4), "traffic": None}
    roofline["kernel"] = "igemm_kernel (implicit-GEMM MFMA)"
    roofline["mfma_frac"] = round(tflops / PEAK_MFMA_TFLOPS, 4)
    roofline["hbm_frac_algorithmic"] = round(gbs / PEAK_HBM_GBS, 4)

    out = {
        "metric": "effective conv TFLOP/s (2*N*P*Q*K*C*R*S / time), 1 MI355X",
        "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 6), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if L.dtype == "bf16" else L.dtype, "data": "synthetic",
        "config": {"workload": f"{head_name}: N={L.N} H=W={L.H} C={L.C} K={L.K} {L.R}x{L.S} "
                               f"stride={L.stride} pad={L.pad} dil={L.dilation}, {L.dtype} in / fp32 acc+out, NHWC/KRSC",
                   "im2col_workspace_bytes": 0},
        "roofline": roofline,
    }

    # ---- explicit im2col + GEMM on the headline layer (the comparison the paper argues against)
    ws_bytes, full, low = explicit_runner(L, code, bufs)
    n_exp = max(20, args.steps // 10)
    ms_full = time_launches(full, n_exp, 5, torch)
    ms_low = time_launches(low, n_exp, 5, torch)
    out["explicit"] = {"workspace_bytes": ws_bytes, "ms_total": round(ms_full, 5), "ms_im2col": round(ms_low, 5),
                       "slowdown_vs_implicit": round(ms_full / ms, 3)}

    # ---- all benchmark layers, briefly ---------------------------------------------------------
    if not args.no_layers:
        layers = {}
        for name, Li in workloads.LAYERS.items():
            ci, _, ri, _ = prepare(Li)
            n = max(20, args.steps // 5)
            mi = time_launches(ri, n, 10, torch)
            tf = Li.flops_real / (mi * 1e-3) / 1e12
            gb = Li.algorithmic_bytes(4) / (mi * 1e-3) / 1e9
            layers[name] = {"us": round(mi * 1e3, 3), "tflops": round(tf, 2),
                            "mfma_frac": round(tf / PEAK_MFMA_TFLOPS, 4),
                            "gbs_algorithmic": round(gb, 1), "hbm_frac": round(gb / PEAK_HBM_GBS, 4)}
            torch.cuda.empty_cache()
        out["layers"] = layers

    # ---- the CPU oracle on the same layer, on this machine's host cores ---------------------------
    if not args.no_cpu:
        from oracle.conv_ref import conv_ref, threads
        x, w = host_in
        conv_ref(x[:1], w, L.stride, L.pad, L.dilation)     # warm-up on one image
        reps, t0 = 0, time.perf_counter()
        while True:
            conv_ref(x, w, L.stride, L.pad, L.dilation)
            reps += 1
            el = time.perf_counter() - t0
            if el > 10.0 or reps >= 20:
                break
        cpu_tflops = L.flops * reps / el / 1e12
        out["cpu_baseline"] = {"value": round(cpu_tflops, 5), "unit": "TFLOP/s", "cores": threads(), "kind": "oracle",
                               "sample": f"{reps} full evaluation(s) of {head_name} ({L.flops / 2e9:.2f} GMAC each), "
                                         f"{el:.1f} s wall, fp64 7-loop C/OpenMP"}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
