#!/usr/bin/env python3
"""Benchmark of the E0M4 matmul hot path on one MI355X.

A "step" is one pass over the decode workload: the 28 x 4 weight matrices of a
ChatGLM2-6B-shaped layer stack (E0M4, group 128, distinct random weights per
layer so that nothing is served from cache), each multiplied with an M=1 fp16
activation vector through e0m4_matmul.  All inputs are resident in HBM before
the timed region.  The 112 launches of a step are captured once into a HIP
graph and replayed, so the Python binding is not in the timed path.

Reported on one JSON line: decode HBM GB/s (value), its roofline object, the
prefill GEMM figures for the same four shapes at M=1024, and the CPU oracle
timed on a bounded sample of the same workload.
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

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_F16_PEAK_TFLOPS = 2500.0   # MI355X published dense fp16 matrix peak
GROUP = 128
PREFILL_M = 1024
# HBM bytes per launch from hardware counters (rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE in separate runs of
# this script, each scaled by the same counter's reading for a plain 1 GiB copy: x2.000 and x1.000); the
# figures and the commands are in profiles/gemv_gemm_chatglm2_6b_hbm_traffic.txt.  They cannot be collected
# inside a timed run, so they are constants here and apply to the default workload only.
MEASURED_TRAFFIC_DECODE_LAUNCH = 27.30e6      # average GEMV launch of the 28 x 4 stack (algorithmic: 27.12e6)
MEASURED_TRAFFIC_PREFILL_GATE_UP = 272.2e6    # M=1024 FFN gate+up GEMM (algorithmic: 124.1e6)


def algorithmic_bytes(M, N, K, G):
    """codes + fp16 scale and bias per group + X once + Y once."""
    return N * K // 2 + 4 * N * (K // G) + 2 * M * K + 2 * M * N


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--layers", type=int, default=None, help="override the number of layers (debug)")
    ap.add_argument("--no-prefill", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-table1", action="store_true", help="skip the E0M4 / INT4 latency comparison")
    ap.add_argument("--no-small-batch", action="store_true", help="skip the 2 <= M <= 16 latencies")
    ap.add_argument("--no-fusion", action="store_true", help="skip the fused / unfused layer comparison")
    ap.add_argument("--no-library", action="store_true",
                    help="skip the platform library's fp16 GEMM on the same prefill shapes (context figure)")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--copy-probe", action="store_true",
                    help="first run three plain device copies of 1 GiB (calibration of HBM traffic counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is a single-GPU kernel library; run with --gpus 1 "
              "(no multi-GPU figure exists for it)", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2403_20041_amd as e0m4
    import synth_inputs

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    e0m4.lib()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    shapes = synth_inputs.CHATGLM2_6B
    n_layers = args.layers or synth_inputs.CHATGLM2_LAYERS

    if args.copy_probe:
        # a plain copy of known size: reads 2^30 bytes and writes 2^30 bytes per launch
        src = torch.ones(1 << 29, dtype=torch.float16, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---------------- set-up: quantise every layer's weights on the GPU (offline step, untimed)
    layers = []
    t_q = time.perf_counter()
    q_bytes = 0
    for layer in range(n_layers):
        mats = []
        for p, (name, N, K) in enumerate(shapes):
            W = synth_inputs.weights_device(N, K, synth_inputs.layer_seed(layer, p), dev)
            packed = e0m4.e0m4_quantize(W, GROUP)
            q_bytes += W.numel() * 2
            del W
            mats.append((name, N, K) + packed)
        layers.append(mats)
    torch.cuda.synchronize()
    t_q = time.perf_counter() - t_q

    xs = {K: synth_inputs.activations_device(1, K, 99 + K, dev) for _, _, K in shapes}
    ys = {(N, K): torch.empty((1, N), dtype=torch.float16, device=dev) for _, N, K in shapes}
    ws_bytes = max(e0m4.e0m4_workspace_bytes(1, N, K, GROUP) for _, N, K in shapes)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev)
    step_bytes = sum(algorithmic_bytes(1, N, K, GROUP) for _, N, K in shapes) * n_layers
    launches = len(shapes) * n_layers

    stream = torch.cuda.Stream(device=dev)

    def decode_step():
        for mats in layers:
            for name, N, K, codes, scales, bias in mats:
                e0m4.e0m4_matmul(xs[K], codes, scales, bias, N, K, GROUP, out=ys[(N, K)], workspace=ws, stream=stream)

    graph = None
    with torch.cuda.stream(stream):
        decode_step()                       # eager once: loads code objects
        stream.synchronize()
        if not args.no_graph:
            try:
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=stream):
                    decode_step()
                graph = g
            except Exception as exc:        # noqa: BLE001
                print("graph capture failed (%s); timing eager launches" % exc, file=sys.stderr)
                graph = None

    def run_step():
        if graph is not None:
            graph.replay()
        else:
            decode_step()

    with torch.cuda.stream(stream):
        for _ in range(args.warmup):
            run_step()
        stream.synchronize()
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        ev0.record(stream)
        for _ in range(args.steps):
            run_step()
        ev1.record(stream)
        stream.synchronize()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
    ev_ms = ev0.elapsed_time(ev1)
    ms_per_step = wall * 1e3 / args.steps
    decode_gbps = step_bytes / (wall / args.steps) / 1e9
    # dominant kernel: the M=1 GEMV.  One launch moves step_bytes / launches algorithmic bytes on average;
    # its average duration is the event time of the timed region divided by the number of launches.
    avg_launch_us = ev_ms * 1e3 / (args.steps * launches)
    achieved = (step_bytes / launches) / (avg_launch_us * 1e-6) / 1e9

    # per-shape decode rate, rotating over the layers' distinct weights (cold in cache)
    per_shape = {}
    with torch.cuda.stream(stream):
        for p, (name, N, K) in enumerate(shapes):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            reps = max(1, 200 // n_layers)

            def shape_pass():
                for mats in layers:
                    _, _, _, codes, scales, bias = mats[p]
                    e0m4.e0m4_matmul(xs[K], codes, scales, bias, N, K, GROUP, out=ys[(N, K)], workspace=ws,
                                     stream=stream)

            run_pass = shape_pass
            if graph is not None:
                try:
                    gs = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(gs, stream=stream):
                        shape_pass()
                    run_pass = gs.replay
                except Exception:           # noqa: BLE001
                    run_pass = shape_pass
            for timed in (False, True):
                if timed:
                    e0.record(stream)
                for _ in range(reps):
                    run_pass()
                if timed:
                    e1.record(stream)
                stream.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / (reps * n_layers)
            b = algorithmic_bytes(1, N, K, GROUP)
            per_shape[name] = {"N": N, "K": K, "us": round(us, 3), "GBps": round(b / us / 1e3, 1),
                               "frac_hbm": round(b / us / 1e3 / HBM_PEAK_GBPS, 4)}

    out = {
        "metric": "E0M4 matmul: decode GEMV HBM GB/s (% peak); prefill GEMM TFLOP/s (% MFMA)",
        "value": round(decode_gbps, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16 x e0m4 codes, f32 accumulate",
        "data": "synthetic",
        "config": {"workload": "ChatGLM2-6B-shaped decode layer stack, M=1, %d layers x 4 projections, E0M4 group %d"
                               % (n_layers, GROUP),
                   "launches_per_step": launches, "algorithmic_bytes_per_step": step_bytes,
                   "launch_mode": "hip_graph" if graph is not None else "eager"},
        "pct_of_hbm_peak": round(100.0 * decode_gbps / HBM_PEAK_GBPS, 2),
        "roofline": {"bound": "hbm", "kernel": "gemv_kernel<G=128,M=1>", "achieved": round(achieved, 2),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "avg_launch_us": round(avg_launch_us, 3),
                     "algorithmic_bytes_per_launch": round(step_bytes / launches),
                     "traffic": MEASURED_TRAFFIC_DECODE_LAUNCH if args.layers is None else None},
        "decode_per_shape": per_shape,
        "quantize": {"GBps_fp16_in": round(q_bytes / t_q / 1e9, 1), "note": "offline step incl. weight generation"},
    }

    # ---------------- small batches (2 <= M <= 16) on the same weights: latency per launch, rotating over the
    # layers' distinct weights (cold in cache); the weight stream is what a launch has to move
    if not args.no_small_batch:
        sb = {}
        with torch.cuda.stream(stream):
            for M in (2, 4, 8, 16):
                row = {}
                for p, (name, N, K) in enumerate(shapes):
                    xm = synth_inputs.activations_device(M, K, 7000 + M + K, dev)
                    ym = torch.empty((M, N), dtype=torch.float16, device=dev)
                    wsm = torch.empty(max(e0m4.e0m4_workspace_bytes(M, N, K, GROUP), 16), dtype=torch.uint8, device=dev)

                    def batch_pass():
                        for mats in layers:
                            _, _, _, codes, scales, bias = mats[p]
                            e0m4.e0m4_matmul(xm, codes, scales, bias, N, K, GROUP, out=ym, workspace=wsm, stream=stream)

                    batch_pass()
                    stream.synchronize()
                    run_pass = batch_pass
                    if graph is not None:
                        gm = torch.cuda.CUDAGraph()
                        with torch.cuda.graph(gm, stream=stream):
                            batch_pass()
                        run_pass = gm.replay
                    reps = max(1, 100 // n_layers)
                    best = None
                    for _ in range(3):
                        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                        e0.record(stream)
                        for _ in range(reps):
                            run_pass()
                        e1.record(stream)
                        stream.synchronize()
                        t = e0.elapsed_time(e1) * 1e3 / (reps * n_layers)
                        best = t if best is None else min(best, t)
                    row[name] = {"us": round(best, 3), "GBps": round(algorithmic_bytes(M, N, K, GROUP) / best / 1e3, 1)}
                    del xm, ym, wsm
                sb["M=%d" % M] = row
        out["small_batch"] = {"workload": "ChatGLM2-6B shapes, 2 <= M <= 16, group %d; latency per launch, cold weights"
                                          % GROUP, "per_M": sb}

    # ---------------- the paper's Table 1: E0M4 against the INT4 twin, M = 1, weight [K, N]
    # (same layout, launch shape and accumulation; the twin extracts integers and converts them to fp16).
    # Each shape rotates over distinct weight copies (cold in cache), replayed from a HIP graph.
    if not args.no_table1:
        t1 = {}
        with torch.cuda.stream(stream):
            for K, N in synth_inputs.TABLE1_SHAPES:
                W = synth_inputs.weights_device(N, K, 8000 + K + N, dev)
                ec, _, _ = e0m4.e0m4_quantize(W, GROUP, stream=stream)
                ic, _, _ = e0m4.e0m4_int4_quantize(W, GROUP, stream=stream)
                del W
                copies = max(2, min(24, int(1.5e9 // ec.numel())))
                ecs = [ec] + [ec.clone() for _ in range(copies - 1)]
                ics = [ic] + [ic.clone() for _ in range(copies - 1)]
                x = synth_inputs.activations_device(1, K, 8100 + K, dev)
                y = torch.empty((1, N), dtype=torch.float16, device=dev)
                us = {}
                for fmt, bufs in (("e0m4", ecs), ("int4", ics)):
                    def one_pass():
                        for c in bufs:
                            if fmt == "e0m4":
                                e0m4.e0m4_matmul(x, c, None, None, N, K, GROUP, out=y, stream=stream)
                            else:
                                e0m4.e0m4_int4_gemv(x, c, N, K, GROUP, out=y, stream=stream)
                    one_pass()
                    stream.synchronize()
                    run = one_pass
                    if graph is not None:
                        gt = torch.cuda.CUDAGraph()
                        with torch.cuda.graph(gt, stream=stream):
                            one_pass()
                        run = gt.replay
                    best = None
                    for _ in range(5):
                        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                        e0.record(stream)
                        for _ in range(4):
                            run()
                        e1.record(stream)
                        stream.synchronize()
                        t = e0.elapsed_time(e1) * 1e3 / (4 * copies)
                        best = t if best is None else min(best, t)
                    us[fmt] = best
                b = algorithmic_bytes(1, N, K, GROUP)
                t1["K%d_N%d" % (K, N)] = {"e0m4_us": round(us["e0m4"], 3), "int4_us": round(us["int4"], 3),
                                           "int4_over_e0m4": round(us["int4"] / us["e0m4"], 3),
                                           "e0m4_GBps": round(b / us["e0m4"] / 1e3, 1),
                                           "int4_GBps": round(b / us["int4"] / 1e3, 1)}
                del ecs, ics, ec, ic, x, y
        out["table1_e0m4_vs_int4"] = {"workload": "M=1, weight [K,N] of the paper's Table 1, group %d; latency per launch, "
                                                  "cold weights; ratio as the table's 'acceleration'" % GROUP,
                                      "shapes": t1}

    # ---------------- E0M8 (8-bit codes) decode: the ChatGLM2-6B shapes at M = 1, cold weights, HIP graph
    if not args.no_table1:
        e8 = {}
        with torch.cuda.stream(stream):
            for name, N, K in shapes:
                W = synth_inputs.weights_device(N, K, 8500 + N + K, dev)
                c8, _, _ = e0m4.e0m8_quantize(W, GROUP, stream=stream)
                del W
                copies = max(2, min(24, int(1.5e9 // c8.numel())))
                bufs = [c8] + [c8.clone() for _ in range(copies - 1)]
                x = synth_inputs.activations_device(1, K, 8600 + K, dev)
                y = torch.empty((1, N), dtype=torch.float16, device=dev)

                def one_pass():
                    for c in bufs:
                        e0m4.e0m8_matmul(x, c, N, K, GROUP, out=y, stream=stream)
                one_pass()
                stream.synchronize()
                run = one_pass
                if graph is not None:
                    g8 = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(g8, stream=stream):
                        one_pass()
                    run = g8.replay
                best = None
                for _ in range(5):
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record(stream)
                    for _ in range(4):
                        run()
                    e1.record(stream)
                    stream.synchronize()
                    t = e0.elapsed_time(e1) * 1e3 / (4 * copies)
                    best = t if best is None else min(best, t)
                b = N * K * (1.0 + 4.0 / 64) + 2 * K + 2 * N        # a byte per code, a (scale, bias) word per 64 weights
                e8[name] = {"N": N, "K": K, "us": round(best, 3), "GBps": round(b / best / 1e3, 1),
                            "frac_hbm": round(b / best / 1e3 / HBM_PEAK_GBPS, 4)}
                if not args.no_prefill:                 # the same weights at M = 1024 on the MFMA kernels
                    X = synth_inputs.activations_device(PREFILL_M, K, 8700 + K, dev, outlier_frac=0.01)
                    Y = torch.empty((PREFILL_M, N), dtype=torch.float16, device=dev)
                    ws8 = torch.empty(max(e0m4.e0m8_workspace_bytes(PREFILL_M, N, K, GROUP), 16), dtype=torch.uint8, device=dev)
                    for _ in range(3):
                        e0m4.e0m8_matmul(X, c8, N, K, GROUP, out=Y, workspace=ws8, stream=stream)
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record(stream)
                    for _ in range(20):
                        e0m4.e0m8_matmul(X, c8, N, K, GROUP, out=Y, workspace=ws8, stream=stream)
                    e1.record(stream)
                    stream.synchronize()
                    ms = e0.elapsed_time(e1) / 20
                    e8[name]["prefill_M%d_ms" % PREFILL_M] = round(ms, 4)
                    e8[name]["prefill_TFLOPs"] = round(2.0 * PREFILL_M * N * K / ms / 1e9, 1)
                    del X, Y, ws8
                del bufs, c8, x, y
        out["e0m8_decode"] = {"workload": "E0M8 (8-bit codes, group %d), M=1, ChatGLM2-6B shapes; latency per launch, "
                                          "cold weights; algorithmic bytes N*K*(1 + 4/64) + 2K + 2N" % GROUP,
                              "per_shape": e8}

    # ---------------- prefill: same four shapes at M=1024 (activation outliers, per-row weight scale)
    if not args.no_prefill:
        pre = {}
        tot_flops, tot_ms, lib_tot_ms = 0.0, 0.0, 0.0
        best = None
        with torch.cuda.stream(stream):
            for p, (name, N, K) in enumerate(shapes):
                W = synth_inputs.weights_device(N, K, 5000 + p, dev, row_std_range=(0.5, 2.0))
                codes, scales, bias = e0m4.e0m4_quantize(W, GROUP, stream=stream)
                del W
                X = synth_inputs.activations_device(PREFILL_M, K, 6000 + p, dev, outlier_frac=0.01)
                Y = torch.empty((PREFILL_M, N), dtype=torch.float16, device=dev)
                pws_bytes = e0m4.e0m4_workspace_bytes(PREFILL_M, N, K, GROUP)    # split-K partial sums, if any
                pws = torch.empty(max(pws_bytes, 16), dtype=torch.uint8, device=dev)
                for _ in range(3):
                    e0m4.e0m4_matmul(X, codes, scales, bias, N, K, GROUP, out=Y, workspace=pws, stream=stream)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                reps = 20
                e0.record(stream)
                for _ in range(reps):
                    e0m4.e0m4_matmul(X, codes, scales, bias, N, K, GROUP, out=Y, workspace=pws, stream=stream)
                e1.record(stream)
                stream.synchronize()
                ms = e0.elapsed_time(e1) / reps
                flops = 2.0 * PREFILL_M * N * K
                tf = flops / ms / 1e9
                pre[name] = {"N": N, "K": K, "ms": round(ms, 4), "TFLOPs": round(tf, 1),
                             "frac_mfma": round(tf / MFMA_F16_PEAK_TFLOPS, 4), "workspace_bytes": pws_bytes}
                if not args.no_library:
                    # context only: the platform library's plain fp16 GEMM (torch.matmul) on the dequantised
                    # weights, four times the weight bytes and no dequantisation in the kernel
                    Wd = e0m4.e0m4_dequant(codes, scales, bias, N, K, GROUP, stream=stream)
                    for _ in range(3):
                        torch.matmul(X, Wd.t(), out=Y)
                    e0.record(stream)
                    for _ in range(reps):
                        torch.matmul(X, Wd.t(), out=Y)
                    e1.record(stream)
                    stream.synchronize()
                    lib_ms = e0.elapsed_time(e1) / reps
                    pre[name]["library_fp16_gemm_TFLOPs"] = round(flops / lib_ms / 1e9, 1)
                    lib_tot_ms += lib_ms
                    # and its fp16 vector-matrix product at M = 1, three copies of the weights in turn (cold)
                    wds = [Wd, Wd.clone(), Wd.clone()]
                    x1, y1 = X[:1], Y[:1]
                    for wd in wds:
                        torch.matmul(x1, wd.t(), out=y1)
                    e0.record(stream)
                    for _ in range(4):
                        for wd in wds:
                            torch.matmul(x1, wd.t(), out=y1)
                    e1.record(stream)
                    stream.synchronize()
                    pre[name]["library_fp16_gemv_us"] = round(e0.elapsed_time(e1) * 1e3 / 12, 2)
                    del Wd, wds
                tot_flops += flops
                tot_ms += ms
                if best is None or flops > best[0]:
                    best = (flops, ms, name)
                del codes, scales, bias, X, Y, pws
        layer_tf = tot_flops / tot_ms / 1e9
        out["prefill"] = {"workload": "ChatGLM2-6B-shaped prefill layer, M=%d, 4 GEMMs" % PREFILL_M,
                          "value": round(layer_tf, 1), "unit": "TFLOP/s", "ms_per_layer": round(tot_ms, 4),
                          "pct_of_mfma_peak": round(100.0 * layer_tf / MFMA_F16_PEAK_TFLOPS, 2), "per_shape": pre}
        if lib_tot_ms > 0:
            out["prefill"]["library_fp16_gemm_layer_TFLOPs"] = round(tot_flops / lib_tot_ms / 1e9, 1)
        dom_tf = best[0] / best[1] / 1e9
        out["roofline_prefill"] = {"bound": "mfma", "kernel": "gemm_pipe_kernel<G=128> (%s)" % best[2],
                                   "achieved": round(dom_tf, 1), "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                   "frac": round(dom_tf / MFMA_F16_PEAK_TFLOPS, 4),
                                   "traffic": MEASURED_TRAFFIC_PREFILL_GATE_UP}

    # ---------------- operator fusion: a layer's four matmuls with their neighbours (rms-norm before qkv and
    # gate+up, SiLU-gated product after gate+up, residual add after attn-out and down), fused into
    # e0m4_matmul_fused against e0m4_matmul followed by torch's own operators; HIP graphs on both sides
    if not args.no_fusion:
        import torch.nn.functional as F

        fus = {}
        for M, n_l, reps in ((1, n_layers, 10), (PREFILL_M, 1, 10)):
            (qn, qN, qK), (an, aN, aK), (gn, gN, gK), (dn, dN, dK) = shapes
            xh = synth_inputs.activations_device(M, qK, 7000, dev)          # hidden state
            xa = synth_inputs.activations_device(M, aK, 7001, dev)          # attention output
            xd = synth_inputs.activations_device(M, dK, 7002, dev)          # input of down (unfused: product below)
            gamma = torch.ones(qK, dtype=torch.float16, device=dev)
            resid = synth_inputs.activations_device(M, aN, 7003, dev)
            y_qkv = torch.empty((M, qN), dtype=torch.float16, device=dev)
            y_h = torch.empty((M, aN), dtype=torch.float16, device=dev)
            y_gu = torch.empty((M, gN), dtype=torch.float16, device=dev)
            y_act = torch.empty((M, gN // 2), dtype=torch.float16, device=dev)
            fws_bytes = max([e0m4.e0m4_fused_workspace_bytes(M, N, K, GROUP, True, e0m4.E0M4_EPILOGUE_SWIGLU
                                                             if N == gN else e0m4.E0M4_EPILOGUE_NONE)
                             for _, N, K in shapes] + [e0m4.e0m4_workspace_bytes(M, N, K, GROUP) for _, N, K in shapes])
            fws = torch.empty(max(fws_bytes, 16), dtype=torch.uint8, device=dev)

            def fused_layer(mats):
                (_, _, _, cq, _, _), (_, _, _, ca, _, _), (_, _, _, cg, _, _), (_, _, _, cd, _, _) = mats
                e0m4.e0m4_matmul_fused(xh, cq, qN, qK, GROUP, rms_gamma=gamma, rms_eps=1e-5, out=y_qkv,
                                       workspace=fws, stream=stream)
                e0m4.e0m4_matmul_fused(xa, ca, aN, aK, GROUP, residual=resid, out=y_h, workspace=fws, stream=stream)
                e0m4.e0m4_matmul_fused(xh, cg, gN, gK, GROUP, rms_gamma=gamma, rms_eps=1e-5,
                                       epilogue=e0m4.E0M4_EPILOGUE_SWIGLU, out=y_act, workspace=fws, stream=stream)
                e0m4.e0m4_matmul_fused(xd, cd, dN, dK, GROUP, residual=resid, out=y_h, workspace=fws, stream=stream)

            def unfused_layer(mats):
                (_, _, _, cq, _, _), (_, _, _, ca, _, _), (_, _, _, cg, _, _), (_, _, _, cd, _, _) = mats
                xn = F.rms_norm(xh, (qK,), gamma, 1e-5)
                e0m4.e0m4_matmul(xn, cq, None, None, qN, qK, GROUP, out=y_qkv, workspace=fws, stream=stream)
                e0m4.e0m4_matmul(xa, ca, None, None, aN, aK, GROUP, out=y_h, workspace=fws, stream=stream)
                torch.add(y_h, resid, out=y_h)
                xn = F.rms_norm(xh, (gK,), gamma, 1e-5)
                e0m4.e0m4_matmul(xn, cg, None, None, gN, gK, GROUP, out=y_gu, workspace=fws, stream=stream)
                torch.mul(F.silu(y_gu[:, : gN // 2]), y_gu[:, gN // 2:], out=y_act)
                e0m4.e0m4_matmul(xd, cd, None, None, dN, dK, GROUP, out=y_h, workspace=fws, stream=stream)
                torch.add(y_h, resid, out=y_h)

            res = {}
            with torch.cuda.stream(stream):
                for label, fn in (("fused", fused_layer), ("unfused", unfused_layer)):
                    for mats in layers[:n_l]:
                        fn(mats)
                    stream.synchronize()
                    gf = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(gf, stream=stream):
                        for mats in layers[:n_l]:
                            fn(mats)
                    for _ in range(2):
                        gf.replay()
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record(stream)
                    for _ in range(reps):
                        gf.replay()
                    e1.record(stream)
                    stream.synchronize()
                    res[label] = e0.elapsed_time(e1) * 1e3 / (reps * n_l)
                    del gf
            fus["M%d" % M] = {"layers_in_graph": n_l, "fused_us_per_layer": round(res["fused"], 2),
                              "unfused_us_per_layer": round(res["unfused"], 2),
                              "unfused_over_fused": round(res["unfused"] / res["fused"], 3)}
            del xh, xa, xd, gamma, resid, y_qkv, y_h, y_gu, y_act, fws
        out["fusion"] = {"workload": "ChatGLM2-6B-shaped layer: rms-norm + qkv, attn-out + residual, rms-norm + gate+up + "
                                     "SiLU-gated product, down + residual; e0m4_matmul_fused against e0m4_matmul plus "
                                     "torch operators, HIP graphs",
                         "results": fus}

    # ---------------- KV-cache append in place against the concatenation it replaces (one layer's K and V rows
    # of a ChatGLM2-6B-shaped model, 2 x 2 heads x 128, taken from the QKV output; cache of 2048 positions)
    if not args.no_fusion:
        kv = {}
        max_seq, row = 2048, 512
        for label, n_new in (("decode_1_token", 1), ("prefill_1024_tokens", 1024)):
            have = max_seq - n_new
            cache = torch.zeros((max_seq, row), dtype=torch.float16, device=dev)
            qkv_out = synth_inputs.activations_device(n_new, 4608, 7200, dev)
            pos = torch.arange(have, have + n_new, dtype=torch.int64, device=dev)
            res = {}
            with torch.cuda.stream(stream):
                for what in ("append", "concat"):
                    def op():
                        if what == "append":
                            e0m4.e0m4_kv_append(cache, qkv_out[:, 4096:], pos, stream=stream)
                        else:
                            torch.cat([cache[:have], qkv_out[:, 4096:]], dim=0)
                    op()
                    stream.synchronize()
                    gk = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(gk, stream=stream):
                        for _ in range(20):
                            op()
                    gk.replay()
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record(stream)
                    for _ in range(5):
                        gk.replay()
                    e1.record(stream)
                    stream.synchronize()
                    res[what] = e0.elapsed_time(e1) * 1e3 / 100
                    del gk
            kv[label] = {"append_us": round(res["append"], 2), "concat_us": round(res["concat"], 2),
                         "bytes_moved_append": 2 * n_new * row * 2, "bytes_moved_concat": 2 * max_seq * row * 2}
            del cache, qkv_out, pos
        out["kv_append"] = {"workload": "cache [2048, 512] fp16, new rows = columns 4096..4607 of the QKV output; "
                                        "20 back-to-back launches in a HIP graph", "results": kv}

    # ---------------- CPU oracle on a bounded sample of the decode workload (one layer, repeated)
    if not args.no_cpu:
        import numpy as np

        import oracle

        cpu_layers = 1
        packed = []
        for p, (name, N, K) in enumerate(shapes):
            W = synth_inputs.weights(N, K, synth_inputs.layer_seed(0, p))
            packed.append((N, K) + oracle.quantize(W, GROUP))
            del W
        xcpu = {K: synth_inputs.activations(1, K, 99 + K) for _, _, K in shapes}
        reps, t_cpu = 0, 0.0
        while t_cpu < 12.0 and reps < 64:
            t0 = time.perf_counter()
            for N, K, codes, scales, bias in packed:
                What = oracle.dequant(codes, scales, bias, GROUP)
                oracle.matmul(xcpu[K], What, want_absdot=False)
            t_cpu += time.perf_counter() - t0
            reps += 1
        cpu_bytes = sum(algorithmic_bytes(1, N, K, GROUP) for _, N, K in shapes) * cpu_layers * reps
        out["cpu_baseline"] = {"value": round(cpu_bytes / t_cpu / 1e9, 3), "unit": "GB/s",
                               "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": "%d x (dequant + fp64 matmul, M=1) over the 4 projections of one layer "
                                         "(%.1f s of CPU time)" % (reps, t_cpu)}
        del np

    print(json.dumps(out))


if __name__ == "__main__":
    main()
