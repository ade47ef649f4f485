#!/usr/bin/env python3
"""Benchmark of the implicit-im2col convolution on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--layer cfg2] [--eager]
                    [--no-cpu] [--no-layers] [--no-explicit] [--no-probes] [--no-cold] [--calibrate] [--study]

A step is one iconv_fwd call (the whole hot path: tile decomposition, on-the-fly im2col gather,
MFMA contraction, epilogue) over one batch of seeded synthetic input already resident in device
memory.  The headline workload is the ResNet-style 3x3 layer `cfg2`; the other benchmark layers
are timed briefly and reported under "layers".  Prints ONE JSON line.

Timing: W untimed warm-up steps, then exactly K steps between two events recorded on the stream
the kernels run on, with a device synchronisation on both sides.  By default the K launches are
captured once into a HIP graph and the graph is replayed between the events, so that the
figure is the GPU's time per step and not the host's launch rate (a launch costs the host about
7 us, more than some of these kernels run); --eager times K plain launches instead.
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

def measured_traffic_bytes():
    """HBM bytes per launch of each layer's kernel as the last committed rocprofv3 --pmc runs of this script
    measured them (FETCH_SIZE / WRITE_SIZE, scaled by the same counters' reading for the copy probe): the lines
    `traffic_bytes <layer> <bytes>` of profiles/bench_all_layers_pmc.txt.  Missing file or layer -> None."""
    out = {}
    try:
        with open(os.path.join(ROOT, "profiles", "bench_all_layers_pmc.txt")) as f:
            for line in f:
                parts = line.split()
                if len(parts) == 3 and parts[0] == "traffic_bytes":
                    out[parts[1]] = int(parts[2])
    except OSError:
        pass
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--layer", default=None, help="headline layer (default cfg2)")
    ap.add_argument("--eager", action="store_true", help="time plain launches instead of a graph replay")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing leg")
    ap.add_argument("--no-layers", action="store_true", help="skip the per-layer table")
    ap.add_argument("--no-explicit", action="store_true", help="skip the explicit im2col + GEMM comparison")
    ap.add_argument("--no-probes", action="store_true", help="skip the achievable-rate probes (MFMA loop, copy)")
    ap.add_argument("--no-cold", action="store_true", help="skip the cold-cache timing of the headline layer")
    ap.add_argument("--calibrate", action="store_true",
                    help="also launch the copy probe on 64 MiB (counter calibration for rocprofv3 --pmc runs)")
    ap.add_argument("--variant", type=int, default=-1, help="force a kernel-table entry (sweeps)")
    ap.add_argument("--study", action="store_true",
                    help="add the stride/dilation sensitivity table, the batch 8/64 sweep and the output-type table")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (a forward convolution shards over the batch with no exchange "
              "step, so more GPUs would only run copies of this). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads
    from paper_2110_03901_amd import binding as B

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)

    def time_steps(fn, steps, warmup, repeats=1, keep_busy=False):
        """ms per step over exactly `steps` steps after `warmup` untimed ones; with repeats > 1 the graph of
        `steps` launches is replayed that many times and the median replay is reported.  keep_busy (the short
        graphs of the per-layer, explicit and study tables): each timed replay directly follows untimed replays of
        the same graph worth about 5 ms, with no synchronisation in between -- after an idle moment the chip runs
        its first few milliseconds at lower clocks (cfg2: 15.5 us per launch in a graph of 20, 14.1 in one of 200,
        13.2 from 1000 on), which a short graph would otherwise be charged with.  The headline does not use it:
        its `steps` launches are bracketed by synchronisations on both sides, as the contract asks."""
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        if args.eager:
            e0.record()
            for _ in range(steps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / steps
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                for _ in range(steps):
                    fn()
        torch.cuda.synchronize()
        times = []
        n_busy = 0
        if keep_busy:
            e0.record()
            graph.replay()
            e1.record()
            torch.cuda.synchronize()
            n_busy = max(1, min(200, int(5.0 / max(e0.elapsed_time(e1), 1e-3)) + 1))
        for _ in range(max(1, repeats)):
            for _ in range(n_busy):
                graph.replay()
            e0.record()
            graph.replay()
            e1.record()
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1) / steps)
        times.sort()
        return times[len(times) // 2]

    def prepare(L):
        code = B.DTYPE_CODES[L.dtype]
        x, w = workloads.make_inputs(L)
        xd, wd = B.to_device(x, code), B.to_device(w, code)
        y = B.empty_output(L.N, L.P, L.Q, L.K, code)
        sa = L.shape_args()
        if args.variant >= 0:
            return code, (x, w), (lambda: B.iconv_fwd_ex(xd, wd, y, *sa, code, args.variant, 0)), (xd, wd, y)
        return code, (x, w), (lambda: B.iconv_fwd(xd, wd, y, *sa, code)), (xd, wd, y)

    def bound_of(L, ms):
        """Which roofline binds the layer (by its algorithmic traffic and flops) and the fractions."""
        tflops = L.flops / (ms * 1e-3) / 1e12
        gbs = L.algorithmic_bytes(4) / (ms * 1e-3) / 1e9
        t_mfma = L.flops / (PEAK_MFMA_TFLOPS * 1e12)
        t_hbm = L.algorithmic_bytes(4) / (PEAK_HBM_GBS * 1e9)
        return ("mfma" if t_mfma >= t_hbm else "hbm"), tflops, gbs

    head_name = args.layer or workloads.BENCH_LAYER
    L = workloads.LAYERS[head_name]
    code, host_in, run, bufs = prepare(L)

    # ---- headline ------------------------------------------------------------------------------
    # (the graph of exactly --steps launches is replayed five times; the median replay is reported)
    ms = time_steps(run, args.steps, args.warmup, repeats=1 if args.eager else 5)
    bound, tflops, gbs = bound_of(L, ms)
    traffic = measured_traffic_bytes().get(head_name)
    if bound == "mfma":
        roofline = {"bound": "mfma", "achieved": round(tflops, 2), "peak": PEAK_MFMA_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(tflops / PEAK_MFMA_TFLOPS, 4), "traffic": traffic}
    else:
        roofline = {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": round(gbs / PEAK_HBM_GBS, 4), "traffic": traffic}
    roofline["kernel"] = B.iconv_variant_name(args.variant) if args.variant >= 0 else "auto-selected iconv_fwd kernel"
    roofline["algorithmic_bytes"] = L.algorithmic_bytes(4)
    roofline["flops"] = L.flops
    roofline["mfma_frac"] = round(tflops / PEAK_MFMA_TFLOPS, 4)
    roofline["hbm_frac_algorithmic"] = round(gbs / PEAK_HBM_GBS, 4)
    roofline["note"] = ("warm replays: x, w and y of consecutive launches stay in the 256 MiB last-level cache, so `achieved` is "
                        "algorithmic bytes over time, not DRAM traffic; see `cold` for launches on rotating buffers")

    out = {
        "metric": "effective conv TFLOP/s (2*N*P*Q*K*C*R*S / time), 1 MI355X",
        "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 6), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": L.dtype, "data": "synthetic",
        "config": {"workload": f"{head_name}: N={L.N} H=W={L.H} C={L.C} K={L.K} {L.R}x{L.S} "
                               f"stride={L.stride} pad={L.pad} dil={L.dilation}, {L.dtype} in / fp32 acc+out, NHWC/KRSC",
                   "im2col_workspace_bytes": 0,
                   "timing": "eager launches" if args.eager else "HIP graph replay, median of 5 replays of the graph of `steps` launches"},
        "roofline": roofline,
    }

    # ---- the same layer with cold caches: every launch of the graph works on another (x, y) pair, enough
    # pairs that their bytes exceed the 256 MiB last-level cache several times between two uses of a pair
    if not args.no_cold:
        xd0, wd0, _ = bufs
        pair_bytes = xd0.numel() * xd0.element_size() + L.M * L.K * 4
        n_sets = max(4, min(64, int(1.5e9 // pair_bytes) + 1))
        sets = [(xd0.clone(), B.empty_output(L.N, L.P, L.Q, L.K, code)) for _ in range(n_sets)]
        sa0 = L.shape_args()
        turn = [0]

        def cold_step():
            xs, ys = sets[turn[0] % n_sets]
            turn[0] += 1
            B.iconv_fwd(xs, wd0, ys, *sa0, code)
        n_cold = max(n_sets * 4, min(args.steps, 400))
        ms_cold = time_steps(cold_step, n_cold, n_sets, keep_busy=True)
        out["cold"] = {"ms_per_step": round(ms_cold, 6), "tflops": round(L.flops / (ms_cold * 1e-3) / 1e12, 2),
                       "gbs_algorithmic": round(L.algorithmic_bytes(4) / (ms_cold * 1e-3) / 1e9, 1),
                       "buffer_sets": n_sets, "bytes_between_reuse": n_sets * pair_bytes, "steps": n_cold}
        del sets
        torch.cuda.empty_cache()

    # ---- explicit im2col + GEMM (the comparison the paper argues against): headline layer here, every layer below --
    def explicit_of(Li, code_i, xd, wd, y, ms_implicit, n_exp):
        sa = Li.shape_args()
        ws_bytes = B.iconv_workspace_bytes(B.ALGO_EXPLICIT, *sa, code_i)
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda:0")
        ms_full = time_steps(lambda: B.iconv_fwd_explicit(xd, wd, y, ws, ws_bytes, *sa, code_i), n_exp, 5, repeats=3, keep_busy=True)
        ms_low = time_steps(lambda: B.iconv_im2col(xd, ws, ws_bytes, Li.N, Li.H, Li.W, Li.C, Li.R, Li.S, Li.stride, Li.pad,
                                                   Li.dilation, code_i), n_exp, 5, repeats=3, keep_busy=True)
        del ws
        torch.cuda.empty_cache()
        x_bytes = Li.N * Li.H * Li.W * Li.C * Li.elt_bytes()
        return {"workspace_bytes": ws_bytes, "ms_total": round(ms_full, 5), "ms_im2col": round(ms_low, 5),
                "ms_gemm": round(ms_full - ms_low, 5),
                # the lowering kernel reads x once and writes the lowered matrix; the GEMM reads the matrix and writes y
                "im2col_gbs": round((x_bytes + ws_bytes) / (ms_low * 1e-3) / 1e9, 1),
                "gemm_gbs": round((ws_bytes + Li.M * Li.K * 4) / (max(ms_full - ms_low, 1e-6) * 1e-3) / 1e9, 1),
                "slowdown_vs_implicit": round(ms_full / ms_implicit, 3)}

    if not args.no_explicit:
        xd, wd, y = bufs
        out["explicit"] = explicit_of(L, code, xd, wd, y, ms, max(20, args.steps // 10))

    # ---- all benchmark layers, briefly -----------------------------------------------------------
    if not args.no_layers:
        layers = {}
        for name, Li in workloads.LAYERS.items():
            _, _, ri, keep = prepare(Li)
            n = max(50, args.steps // 10)
            mi = time_steps(ri, n, max(20, args.warmup // 4), repeats=5, keep_busy=True)   # median of five replays of n launches
            bi, tf, gb = bound_of(Li, mi)
            tf_real = Li.flops_real / (mi * 1e-3) / 1e12
            layers[name] = {"us": round(mi * 1e3, 3), "tflops": round(tf_real, 2), "bound": bi,
                            "kernel": B.iconv_kernel_for(*Li.shape_args(), B.DTYPE_CODES[Li.dtype]),
                            # fraction of the MFMA peak by the flops of the real channels (cfg5a: 3 of the 4 stored)
                            "mfma_frac": round(tf_real / PEAK_MFMA_TFLOPS, 4),
                            "gbs_algorithmic": round(gb, 1), "hbm_frac": round(gb / PEAK_HBM_GBS, 4)}
            if Li.flops_real != Li.flops:
                layers[name]["mfma_frac_with_padding_channels"] = round(tf / PEAK_MFMA_TFLOPS, 4)
            if not args.no_explicit and name != head_name:
                ci = B.DTYPE_CODES[Li.dtype]
                layers[name]["explicit"] = explicit_of(Li, ci, keep[0], keep[1], keep[2], mi, 20)
            elif not args.no_explicit:
                layers[name]["explicit"] = out["explicit"]
            del keep
            torch.cuda.empty_cache()
        out["layers"] = layers

    # ---- studies beyond the headline (off by default; each entry is timed like a layer above) ------
    if args.study:
        def quick(Li, code_override=None):
            c = code_override if code_override is not None else B.DTYPE_CODES[Li.dtype]
            x, w = workloads.make_inputs(Li)
            xd, wd = B.to_device(x, c), B.to_device(w, c)
            y = B.empty_output(Li.N, Li.P, Li.Q, Li.K, c)
            sa = Li.shape_args()
            t = time_steps(lambda: B.iconv_fwd(xd, wd, y, *sa, c), 100, 20, repeats=5, keep_busy=True)
            del xd, wd, y
            torch.cuda.empty_cache()
            return t
        def quick_channel_last(Li):
            """The channel-last comparison kernel on the same layer (NCHW input, KCRS filters)."""
            c = B.DTYPE_CODES[Li.dtype]
            x, w = workloads.make_inputs(Li)
            xd = B.to_device(x, c).permute(0, 3, 1, 2).contiguous()
            wd = B.to_device(w, c).permute(0, 3, 1, 2).contiguous()
            y = B.empty_output(Li.N, Li.P, Li.Q, Li.K, c)
            sa = Li.shape_args()
            t = time_steps(lambda: B.iconv_fwd_channel_last(xd, wd, y, *sa, c), 50, 10, keep_busy=True)
            del xd, wd, y
            torch.cuda.empty_cache()
            return t
        study = {"stride_dilation": {}, "batch": {}, "output_type": {}}
        # (1) stride / dilation sensitivity: the convolution against the plain GEMM of the same M x K_gemm x K
        # shape (a 1x1 convolution over a 1 x 1 x M image with K_gemm channels), as in the paper's stride figure
        for label, Ls in workloads.study_layers():
            t_conv = quick(Ls)
            Lg = workloads.ConvLayer("gemm_" + label, 1, 1, Ls.M, Ls.k_gemm, Ls.K, 1, 1, 1, 0, 1, Ls.dtype, Ls.seed_id + 1)
            t_gemm = quick(Lg)
            t_cl = quick_channel_last(Ls)
            study["stride_dilation"][label] = {"M": Ls.M, "us": round(t_conv * 1e3, 2), "tflops": round(Ls.flops / t_conv / 1e9, 1),
                                               "gemm_only_us": round(t_gemm * 1e3, 2),
                                               "conv_over_gemm_time": round(t_conv / t_gemm, 3),
                                               "channel_last_us": round(t_cl * 1e3, 2),
                                               "channel_last_over_gemm_time": round(t_cl / t_gemm, 3)}
        # (2) batch 8 and 64 for every benchmark layer
        for name, Li in workloads.LAYERS.items():
            if name == "cfg1":
                continue
            for n in (8, 64):
                Lb = workloads.with_batch(Li, n)
                tb = quick(Lb)
                study["batch"][f"{name}_n{n}"] = {"us": round(tb * 1e3, 2), "tflops": round(Lb.flops_real / tb / 1e9, 1)}
        # (3) input/output types on the headline layer
        for tname in ("bf16", "bf16_bf16", "f16", "f16_f16"):
            Lt = workloads.ConvLayer(L.name, L.N, L.H, L.W, L.C, L.K, L.R, L.S, L.stride, L.pad, L.dilation,
                                     "f16" if tname.startswith("f16") else "bf16", L.seed_id)
            tt = quick(Lt, B.DTYPE_CODES[tname])
            study["output_type"][tname] = {"us": round(tt * 1e3, 2), "tflops": round(L.flops / tt / 1e9, 1)}
        # ... and on the stem layer, whose time is the write of y
        L5 = workloads.LAYERS["cfg5a"]
        for tname in ("bf16", "bf16_bf16"):
            tt = quick(L5, B.DTYPE_CODES[tname])
            study["output_type"]["cfg5a_" + tname] = {"us": round(tt * 1e3, 2), "tflops": round(L5.flops_real / tt / 1e9, 1)}
        out["study"] = study

    # ---- achievable rates on this machine: register-only MFMA loop and a large device copy ----------
    if not args.no_probes:
        iters = 2000
        pout = torch.empty(B.MFMA_PROBE_GROUPS * 256, dtype=torch.float32, device="cuda:0")
        probe_flop = B.MFMA_PROBE_GROUPS * 4 * iters * 8 * 32768
        t_m = time_steps(lambda: B.iconv_probe_mfma(pout, pout.numel() * 4, iters), 20, 3, keep_busy=True)
        probe_tflops = probe_flop / (t_m * 1e-3) / 1e12
        t_r = time_steps(lambda: B.iconv_probe_mfma(pout, pout.numel() * 4, iters, True), 20, 3, keep_busy=True)
        probe_random = probe_flop / (t_r * 1e-3) / 1e12
        nb = 256 << 20
        a = torch.zeros(nb, dtype=torch.uint8, device="cuda:0")
        b = torch.empty(nb, dtype=torch.uint8, device="cuda:0")
        t_c = time_steps(lambda: B.iconv_probe_copy(b, a, nb), 20, 3, keep_busy=True)
        # the same copy with the epilogues' store instructions (whole lines, written through)
        t_cw = time_steps(lambda: B.iconv_probe_copy_wt(b, a, nb), 20, 3, keep_busy=True)
        # launch-to-launch period of graph nodes that do next to nothing (a 16-byte copy): the part of every
        # ms_per_step above that lies between kernels
        t_gap = time_steps(lambda: B.iconv_probe_copy(b, a, 16), 500, 20, keep_busy=True)
        # LDS instruction cost: cycles per instruction and compute unit at the nominal 2.4 GHz
        lds_iters = 2000
        lds_cost = {}
        for pi, pname in enumerate(B.LDS_PROBE_PATTERNS):
            t_l = time_steps(lambda: B.iconv_probe_lds(pout, pout.numel() * 4, lds_iters, pi), 10, 2, keep_busy=True)
            lds_cost[pname] = round(t_l * 1e-3 * 2.4e9 / (B.MFMA_PROBE_GROUPS / 256 * 4 * lds_iters * 8), 2)
        out["achievable"] = {"mfma_bf16_tflops": round(probe_tflops, 1),
                             "mfma_frac_of_datasheet": round(probe_tflops / PEAK_MFMA_TFLOPS, 4),
                             "mfma_bf16_tflops_random_operands": round(probe_random, 1),
                             "copy_gbs_read_plus_write": round(2 * nb / (t_c * 1e-3) / 1e9, 1),
                             "copy_gbs_write_through_stores": round(2 * nb / (t_cw * 1e-3) / 1e9, 1),
                             "value_frac_of_achievable_mfma": round(tflops / probe_tflops, 4),
                             "lds_cycles_per_b128_instruction_per_cu": lds_cost,
                             "graph_node_period_us_empty_kernel": round(t_gap * 1e3, 3),
                             "headline_kernel_us_without_that_period": round((ms - t_gap) * 1e3, 3)}
        del a, b, pout
        torch.cuda.empty_cache()

    if args.calibrate:
        n = 64 << 20
        a = torch.zeros(n, dtype=torch.uint8, device="cuda:0")
        b = torch.empty(n, dtype=torch.uint8, device="cuda:0")
        for _ in range(5):
            B.iconv_probe_copy(b, a, n)
        # the LDS patterns with known conflicts, for reading SQ_LDS_BANK_CONFLICT
        cal = torch.empty(B.MFMA_PROBE_GROUPS * 256, dtype=torch.float32, device="cuda:0")
        for pi in range(len(B.LDS_PROBE_PATTERNS)):
            for _ in range(3):
                B.iconv_probe_lds(cal, cal.numel() * 4, 500, pi)
        torch.cuda.synchronize()
        out["calibration"] = {"copy_bytes_each_way": n, "launches": 5}

    # ---- the CPU oracle on this machine's host cores: the headline layer repeatedly (about 10 s), then every other
    # benchmark layer once (a full evaluation each: 0.15 M ... 19 G multiply-accumulates, under a second apiece)
    if not args.no_cpu:
        from oracle.conv_ref import conv_ref, threads
        x, w = host_in
        conv_ref(x[:1], w, L.stride, L.pad, L.dilation)     # warm-up on one image
        reps, t0 = 0, time.perf_counter()
        while True:
            conv_ref(x, w, L.stride, L.pad, L.dilation)
            reps += 1
            el = time.perf_counter() - t0
            if el > 10.0 or reps >= 400:
                break
        cpu_tflops = L.flops * reps / el / 1e12
        out["cpu_baseline"] = {"value": round(cpu_tflops, 5), "unit": "TFLOP/s", "cores": threads(), "kind": "oracle",
                               "sample": f"{reps} full evaluation(s) of {head_name} ({L.flops / 2e9:.2f} GMAC each), "
                                         f"{el:.1f} s wall, fp64 7-loop C/OpenMP"}
        per_layer = {}
        for name, Li in workloads.LAYERS.items():
            if name == head_name:
                per_layer[name] = {"ms": round(el / reps * 1e3, 2), "tflops": round(cpu_tflops, 5), "evaluations": reps}
                continue
            xi, wi = workloads.make_inputs(Li)
            t1 = time.perf_counter()
            conv_ref(xi, wi, Li.stride, Li.pad, Li.dilation)
            dt = time.perf_counter() - t1
            per_layer[name] = {"ms": round(dt * 1e3, 2), "tflops": round(Li.flops_real / dt / 1e12, 5), "evaluations": 1}
        out["cpu_baseline"]["layers"] = per_layer
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
