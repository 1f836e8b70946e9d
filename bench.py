#!/usr/bin/env python3
"""Benchmark of the E0M4 matmul hot path on one MI355X.

A "step" is one pass over the decode workload: the 28 x 4 weight matrices of a
ChatGLM2-6B-shaped layer stack (E0M4, group 128, distinct random weights per
layer so that nothing is served from cache), each multiplied with an M=1 fp16
activation vector through e0m4_matmul.  All inputs are resident in HBM before
the timed region.  The 112 launches of a step are captured once into a HIP
graph and replayed, so the Python binding is not in the timed path.

Reported on one JSON line: decode HBM GB/s of that stack (value) with its
roofline object; under "configs" one roofline object per workload of the
benchmark set (the single 4096 x 4096 GEMV over rotating weight copies, the
ChatGLM2-6B prefill GEMMs at M=1024, the Gemma-2B-shaped layers with the LM
head, the 14B-shaped layers at groups 64 and 128, M=1 and M=2048); side
sections (small batches, E0M4 against INT4, 8-bit codes, operator fusion,
KV append); and the CPU oracle timed on bounded samples of the same work.

Sections can be selected with --only / --skip (names: decode, shapes, cfg1,
prefill, gemma, d14b, small_batch, table1, e0m8, bf16, fusion, kv, cpu); the profiler
commands under profiles/ use that to keep their runs short.

`python bench.py --summarize DIR [--last N]` prints a summary of a rocprofv3
output directory (kernel trace or counter collection) instead of running.
"""
from __future__ import annotations

import argparse
import glob
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_F16_PEAK_TFLOPS = 2500.0   # MI355X published dense fp16 matrix peak
GROUP = 128
SECTIONS = ("decode", "shapes", "cfg1", "prefill", "gemma", "d14b", "small_batch", "table1", "e0m8", "bf16", "fusion",
            "kv", "dispatch", "cpu", "gemma_prefill", "d14b_prefill")


def algorithmic_bytes(M, N, K, G):
    """codes + fp16 scale and bias per group + X once + Y once."""
    return N * K // 2 + 4 * N * (K // G) + 2 * M * K + 2 * M * N


def profile_traffic(key):
    """HBM bytes per launch measured with hardware counters: rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE cannot run
    inside a timed run, so the figures live in the summaries under profiles/ (lines `traffic_bytes <key> <bytes>`,
    written from the counter runs whose commands those files give) and are looked up here; None if absent."""
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*hbm_traffic*.txt"))):
        for line in open(path):
            m = re.match(r"\s*traffic_bytes\s+(\S+)\s+([0-9.eE+]+)", line)
            if m and m.group(1) == key:
                return float(m.group(2))
    return None


# ---------------------------------------------------------------------------------------------------------------------
# rocprofv3 summaries

def _short_kernel_name(n):
    m = re.search(r"(gemv_kernel|gemv_mfma_kernel|gemv_dq_kernel|splitk_reduce_fused_kernel|gemm_pipe_kernel|gemm_kernel|quantize_kernel|"
                  r"dequant_kernel|unpack_kernel|splitk_reduce_kernel|zero_fill_kernel|rmsnorm_kernel|kv_append_kernel|"
                  r"quantize8_kernel)I((?:L[ib]\d+E)+)E", n)
    if m:
        return "%s<%s>" % (m.group(1), ",".join(re.findall(r"L[ib](\d+)", m.group(2))))
    n = re.sub(r"^void ", "", n)
    m = re.search(r"(Cijk_\w{0,40}|__amd_rocclr_\w+|\w+_kernel\w*)", n)
    return (m.group(1) if m else n)[:60]


OUR_KERNELS = (r"gemv_kernel|gemv_mfma_kernel|gemv_dq_kernel|gemm_pipe_kernel|gemm_kernel|splitk_reduce|rmsnorm_kernel|"
               r"quantize_kernel|dequant_kernel|kv_append_kernel|zero_u32_kernel")


def summarize(directory, last):
    """Summary of the newest rocprofv3 results database under `directory`, for this library's kernels (and the
    runtime's plain buffer copy, which calibrates the traffic counters).
    Kernel trace: per kernel and grid, dispatch count and duration statistics; with --last N only the last N
    dispatches of the matmul kernels are counted: in a run of `--only decode` those are the timed graph replays
    (steps x launches per step).
    Counter collection: one row per kernel, grid and group of dispatches with like readings (dispatches of one
    kernel and grid whose first counter differs by more than 3 % are different problem shapes), one column per
    counter, averaged over the group."""
    import collections
    import sqlite3
    import statistics

    dbs = glob.glob(os.path.join(directory, "**", "*_results.db"), recursive=True)
    if not dbs:
        sys.exit("no *_results.db under %s" % directory)
    con = sqlite3.connect(max(dbs, key=os.path.getmtime))
    tables = {r[0] for r in con.execute("select name from sqlite_master where type in ('table','view')")}
    if "counters_collection" in tables and con.execute("select count(*) from counters_collection").fetchone()[0]:
        cols = [r[1] for r in con.execute("pragma table_info(counters_collection)")]
        key = "dispatch_id" if "dispatch_id" in cols else "rowid"
        per = collections.OrderedDict()
        for did, name, gx, cn, val in con.execute(
                "select %s,kernel_name,grid_size_x,counter_name,value from counters_collection order by %s" % (key, key)):
            if not re.search(OUR_KERNELS + "|__amd_rocclr_copyBuffer", name):
                continue
            d = per.setdefault((did, _short_kernel_name(name), gx), {})
            d[cn] = d.get(cn, 0.0) + val            # a counter may come in several rows (one per hardware instance)
        counters = sorted({c for d in per.values() for c in d})
        groups = collections.defaultdict(list)
        for (did, kname, gx), d in per.items():
            groups[(kname, gx)].append([d.get(c, 0.0) for c in counters])
        print("%-42s %9s %6s " % ("kernel", "grid_x", "calls") + " ".join("%22s" % c[-22:] for c in counters))
        rows = []
        for (kname, gx), vs in groups.items():
            vs.sort()
            start = 0
            for i in range(1, len(vs) + 1):
                if i == len(vs) or vs[i][0] > 1.03 * vs[i - 1][0] + 1e-9:
                    grp = vs[start:i]
                    rows.append((kname, gx, len(grp), [sum(v[c] for v in grp) / len(grp) for c in range(len(counters))]))
                    start = i
        for kname, gx, n, avg in sorted(rows, key=lambda r: (r[0], r[1], r[3][0])):
            print("%-42s %9d %6d " % (kname, gx, n) + " ".join("%22.1f" % a for a in avg))
        return
    rows = [r for r in con.execute("select name,grid_x,workgroup_x,start,end from kernels order by start")
            if re.search(OUR_KERNELS, r[0])]
    if last:
        rows = [r for r in rows if re.search(r"gemv_kernel|gemv_mfma_kernel|gemv_dq_kernel|gemm_pipe_kernel|gemm_kernel|splitk_reduce", r[0])][-last:]
        print("last %d dispatches of the matmul kernels (the timed graph replays): %.3f ms of kernel time, "
              "%.3f ms from the first start to the last end" % (len(rows), sum(r[4] - r[3] for r in rows) / 1e6,
                                                                 (rows[-1][4] - rows[0][3]) / 1e6))
    agg = collections.defaultdict(list)
    for name, gx, wx, t0, t1 in rows:
        agg[(_short_kernel_name(name), gx, wx)].append(t1 - t0)
    print("%-44s %10s %5s %7s %10s %10s %10s %10s" % ("kernel", "grid_x", "wg", "calls", "total_ms", "avg_us", "min_us", "med_us"))
    for k, v in sorted(agg.items(), key=lambda kv: -sum(kv[1])):
        print("%-44s %10d %5d %7d %10.3f %10.2f %10.2f %10.2f" % (k[0], k[1], k[2], len(v), sum(v) / 1e6, sum(v) / len(v) / 1e3,
                                                                  min(v) / 1e3, statistics.median(v) / 1e3))


# ---------------------------------------------------------------------------------------------------------------------

def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--layers", type=int, default=None, help="override the number of layers of the decode stack (debug)")
    ap.add_argument("--only", default="", help="comma-separated sections to run (default: all)")
    ap.add_argument("--skip", default="", help="comma-separated sections to leave out")
    ap.add_argument("--no-library", action="store_true",
                    help="skip the platform library's fp16 GEMM on the same prefill shapes (context figure)")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--copy-probe", action="store_true",
                    help="first run three plain device copies of 1 GiB (calibration of HBM traffic counters)")
    ap.add_argument("--summarize", default=None, metavar="DIR", help="summarise a rocprofv3 output directory and exit")
    ap.add_argument("--last", type=int, default=0, help="with --summarize: only the last N matmul dispatches")
    args = ap.parse_args()
    if args.summarize:
        summarize(args.summarize, args.last)
        return
    if args.gpus != 1:
        print("bench.py: this build is a single-GPU kernel library; run with --gpus 1 "
              "(no multi-GPU figure exists for it)", file=sys.stderr)
        sys.exit(2)
    want = set(s for s in args.only.split(",") if s) or set(SECTIONS)
    want -= set(s for s in args.skip.split(",") if s)
    unknown = want - set(SECTIONS)
    if unknown:
        sys.exit("unknown section(s): %s" % ", ".join(sorted(unknown)))
    want.add("decode")                          # the headline value always runs
    for model in ("gemma", "d14b"):             # "<model>_prefill": that model with its prefill GEMMs, whatever "prefill" says
        if model + "_prefill" in want:
            want.add(model)
        elif "prefill" in want and model in want:
            want.add(model + "_prefill")

    import torch

    import paper_2403_20041_amd as e0m4
    import synth_inputs

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    e0m4.lib()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = torch.cuda.Stream(device=dev)
    use_graph = not args.no_graph

    if args.copy_probe:
        # a plain copy of known size: reads 2^30 bytes and writes 2^30 bytes per launch
        src = torch.ones(1 << 29, dtype=torch.float16, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    def ev_pair():
        return torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def capture(fn):
        """fn captured into a HIP graph (after one eager pass that loads the code objects), or fn itself."""
        with torch.cuda.stream(stream):
            fn()
            stream.synchronize()
            if not use_graph:
                return fn
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=stream):
                fn()
            return g.replay

    def time_us(run, reps, rounds=3, warm=1):
        """Best of `rounds` HIP-event timings (events recorded on the launch stream) of `reps` calls; us per call."""
        best = None
        with torch.cuda.stream(stream):
            for _ in range(warm):
                run()
            for _ in range(rounds):
                e0, e1 = ev_pair()
                e0.record(stream)
                for _ in range(reps):
                    run()
                e1.record(stream)
                stream.synchronize()
                t = e0.elapsed_time(e1) * 1e3 / reps
                best = t if best is None else min(best, t)
        return best

    def quantized_layers(shapes, n_layers, groups, seed_of):
        """{G: [[(name, N, K, codes) per projection] per layer]}; every weight matrix is drawn once and packed per group."""
        out = {G: [] for G in groups}
        for layer in range(n_layers):
            rows = {G: [] for G in groups}
            for p, (name, N, K) in enumerate(shapes):
                W = synth_inputs.weights_device(N, K, seed_of(layer, p), dev)
                for G in groups:
                    rows[G].append((name, N, K, e0m4.e0m4_quantize(W, G)[0]))
                del W
            for G in groups:
                out[G].append(rows[G])
        torch.cuda.synchronize()
        return out

    def hbm_roofline(kernel, bytes_per_launch, us_per_launch, traffic_key=None, **extra):
        gbps = bytes_per_launch / us_per_launch / 1e3
        r = {"bound": "hbm", "kernel": kernel, "achieved": round(gbps, 2), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
             "frac": round(gbps / HBM_PEAK_GBPS, 4), "avg_launch_us": round(us_per_launch, 3),
             "algorithmic_bytes_per_launch": int(round(bytes_per_launch)),
             "traffic": profile_traffic(traffic_key) if traffic_key else None}
        r.update(extra)
        return r

    def mfma_roofline(kernel, flops, us, traffic_key=None, **extra):
        tf = flops / us / 1e6
        r = {"bound": "mfma", "kernel": kernel, "achieved": round(tf, 1), "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
             "frac": round(tf / MFMA_F16_PEAK_TFLOPS, 4), "avg_launch_us": round(us, 2),
             "traffic": profile_traffic(traffic_key) if traffic_key else None}
        r.update(extra)
        return r

    def decode_stack(shapes, layers, G, reps):
        """One graph of all layers' M=1 matmuls; us per graph replay and the algorithmic bytes it moves."""
        xs = {K: synth_inputs.activations_device(1, K, 99 + K, dev) for _, _, K in shapes}
        ys = {(N, K): torch.empty((1, N), dtype=torch.float16, device=dev) for _, N, K in shapes}

        def step():
            for mats in layers:
                for name, N, K, codes in mats:
                    e0m4.e0m4_matmul(xs[K], codes, None, None, N, K, G, out=ys[(N, K)], stream=stream)

        us = time_us(capture(step), reps)
        nbytes = sum(algorithmic_bytes(1, N, K, G) for _, N, K in shapes) * len(layers)
        return us, nbytes, len(shapes) * len(layers)

    def decode_per_shape(shapes, layers, G, key_prefix=None):
        """Latency per launch of each projection, rotating over the layers' distinct weights (cold in cache)."""
        res = {}
        for p, (name, N, K) in enumerate(shapes):
            x = synth_inputs.activations_device(1, K, 99 + K, dev)
            y = torch.empty((1, N), dtype=torch.float16, device=dev)

            def one_pass():
                for mats in layers:
                    e0m4.e0m4_matmul(x, mats[p][3], None, None, N, K, G, out=y, stream=stream)

            us = time_us(capture(one_pass), max(1, 200 // len(layers))) / len(layers)
            b = algorithmic_bytes(1, N, K, G)
            res[name] = {"N": N, "K": K, "us": round(us, 3), "GBps": round(b / us / 1e3, 1),
                         "frac_hbm": round(b / us / 1e3 / HBM_PEAK_GBPS, 4), "t_hbm_peak_us": round(b / 8e6, 3)}
            if key_prefix:
                res[name]["traffic"] = profile_traffic("%s_%s" % (key_prefix, name))
        return res

    def prefill_shapes(shapes, M, G, seed0, library, traffic_prefix=None):
        """Each projection at M rows (activation outliers, per-row weight scale): 20 back-to-back launches."""
        pre, tot_flops, tot_us, lib_us = {}, 0.0, 0.0, 0.0
        for p, (name, N, K) in enumerate(shapes):
            W = synth_inputs.weights_device(N, K, seed0 + p, dev, row_std_range=(0.5, 2.0))
            codes = e0m4.e0m4_quantize(W, G, stream=stream)[0]
            del W
            X = synth_inputs.activations_device(M, K, seed0 + 1000 + p, dev, outlier_frac=0.01)
            Y = torch.empty((M, N), dtype=torch.float16, device=dev)
            ws_bytes = e0m4.e0m4_workspace_bytes(M, N, K, G)
            ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev)

            def call():
                e0m4.e0m4_matmul(X, codes, None, None, N, K, G, out=Y, workspace=ws, stream=stream)

            us = time_us(call, 20, rounds=2, warm=3)
            flops = 2.0 * M * N * K
            pre[name] = mfma_roofline("e0m4_matmul M=%d N=%d K=%d G=%d" % (M, N, K, G), flops, us,
                                      traffic_key="%s_%s" % (traffic_prefix, name) if traffic_prefix else None,
                                      workspace_bytes=ws_bytes, t_mfma_peak_us=round(flops / 2.5e9, 2))
            if library:
                # context only: the platform library's plain fp16 GEMM (torch.matmul) on the dequantised weights
                Wd = e0m4.e0m4_dequant(codes, None, None, N, K, G, stream=stream)
                lus = time_us(lambda: torch.matmul(X, Wd.t(), out=Y), 20, rounds=2, warm=3)
                pre[name]["library_fp16_gemm_TFLOPs"] = round(flops / lus / 1e6, 1)
                lib_us += lus
                del Wd
            tot_flops += flops
            tot_us += us
            del codes, X, Y, ws
        layer = mfma_roofline("layer of %d GEMMs, M=%d, G=%d" % (len(shapes), M, G), tot_flops, tot_us)
        if lib_us > 0:
            layer["library_fp16_gemm_layer_TFLOPs"] = round(tot_flops / lib_us / 1e6, 1)
        return pre, layer

    # ================= headline: ChatGLM2-6B-shaped decode stack (M=1, group 128) =====================================
    shapes = synth_inputs.CHATGLM2_6B
    n_layers = args.layers or synth_inputs.CHATGLM2_LAYERS
    t_q = time.perf_counter()
    layers = quantized_layers(shapes, n_layers, (GROUP,), synth_inputs.layer_seed)[GROUP]
    t_q = time.perf_counter() - t_q

    xs = {K: synth_inputs.activations_device(1, K, 99 + K, dev) for _, _, K in shapes}
    ys = {(N, K): torch.empty((1, N), dtype=torch.float16, device=dev) for _, N, K in shapes}
    step_bytes = sum(algorithmic_bytes(1, N, K, GROUP) for _, N, K in shapes) * n_layers
    launches = len(shapes) * n_layers

    def decode_step():
        for mats in layers:
            for name, N, K, codes in mats:
                e0m4.e0m4_matmul(xs[K], codes, None, None, N, K, GROUP, out=ys[(N, K)], stream=stream)

    run_step = capture(decode_step)
    with torch.cuda.stream(stream):
        for _ in range(args.warmup):
            run_step()
        stream.synchronize()
        torch.cuda.synchronize()
        ev0, ev1 = ev_pair()
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
    headline_roofline = hbm_roofline("gemv_kernel<G=128,M=1>", step_bytes / launches, avg_launch_us,
                                     traffic_key="chatglm2_decode_avg_launch" if args.layers is None else None)

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
                   "launch_mode": "hip_graph" if use_graph else "eager"},
        "pct_of_hbm_peak": round(100.0 * decode_gbps / HBM_PEAK_GBPS, 2),
        "roofline": headline_roofline,
        "quantize": {"s_for_stack_incl_weight_generation": round(t_q, 2)},
    }
    # the offline kernels on their own: the widest projection, timed with events (bytes: fp16 in or out + packed)
    name, N, K = max(shapes, key=lambda s_: s_[1] * s_[2])
    Wq = synth_inputs.weights_device(N, K, 4242, dev)
    bufs_q = e0m4.alloc_packed(N, K, GROUP, dev)
    Wd = torch.empty_like(Wq)
    q_us = time_us(lambda: e0m4.e0m4_quantize(Wq, GROUP, out=bufs_q, stream=stream), 5, rounds=2)
    d_us = time_us(lambda: e0m4.e0m4_dequant(bufs_q[0], None, None, N, K, GROUP, out=Wd, stream=stream), 5, rounds=2)
    io_bytes = 2 * N * K + bufs_q[0].numel()
    out["quantize"].update({"shape": [N, K], "quantize_us": round(q_us, 1), "quantize_GBps": round(io_bytes / q_us / 1e3, 1),
                            "dequant_us": round(d_us, 1), "dequant_GBps": round(io_bytes / d_us / 1e3, 1)})
    del Wq, Wd, bufs_q
    configs = {}
    out["configs"] = configs
    cfg2 = {"workload": out["config"]["workload"], "roofline": headline_roofline}
    configs["cfg2_chatglm2_decode"] = cfg2
    if "shapes" in want:
        cfg2["per_shape"] = decode_per_shape(shapes, layers, GROUP, "chatglm2_decode")
        out["decode_per_shape"] = cfg2["per_shape"]

    # ================= config 1: the single 4096 x 4096 GEMV, rotating over >= 64 weight copies (> 256 MB) ============
    if "cfg1" in want:
        N1 = K1 = 4096
        copies = 72                                    # 72 x 8.9 MB = 643 MB: beyond the 256 MB memory-side cache
        W = synth_inputs.weights_device(N1, K1, 0, dev)
        c0 = e0m4.e0m4_quantize(W, GROUP)[0]
        del W
        bufs = [c0] + [c0.clone() for _ in range(copies - 1)]
        x1 = synth_inputs.activations_device(1, K1, 0, dev)
        y1 = torch.empty((1, N1), dtype=torch.float16, device=dev)

        def cold_pass():
            for c in bufs:
                e0m4.e0m4_matmul(x1, c, None, None, N1, K1, GROUP, out=y1, stream=stream)

        def warm_pass():
            for _ in range(copies):
                e0m4.e0m4_matmul(x1, c0, None, None, N1, K1, GROUP, out=y1, stream=stream)

        b1 = algorithmic_bytes(1, N1, K1, GROUP)
        cold = time_us(capture(cold_pass), 4) / copies
        warm = time_us(capture(warm_pass), 4) / copies
        configs["cfg1_single_gemv"] = {
            "workload": "X [1,4096] x W [4096,4096] E0M4 group 128, seed 0; %d distinct weight copies in turn (%d MB)"
                        % (copies, copies * c0.numel() // 1000000),
            "roofline": hbm_roofline("gemv_kernel<G=128,M=1>", b1, cold, traffic_key="cfg1_single_gemv",
                                     t_hbm_peak_us=round(b1 / 8e6, 3)),
            "same_weights_every_launch_us": round(warm, 3)}
        del bufs, c0, x1, y1

    # ================= config 3: ChatGLM2-6B prefill GEMMs, M = 1024 =================================================
    if "prefill" in want:
        pre, layer = prefill_shapes(shapes, 1024, GROUP, 5000, not args.no_library, "chatglm2_prefill")
        configs["cfg3_chatglm2_prefill_M1024"] = {"workload": "ChatGLM2-6B-shaped prefill GEMMs, M=1024, group 128, "
                                                              "1 % outlier channels x20, per-row weight std U(0.5,2)",
                                                  "per_shape": pre, "layer": layer}
        big = max(pre.values(), key=lambda r: r["achieved"] * r["avg_launch_us"])
        out["roofline_prefill"] = big
        # context, not a result: the same launch (gate+up, same kernel, grid and instruction stream) on all-zero
        # activations and all-zero codes.  The chip holds a higher clock when the operands toggle no bits, so the
        # gap between this figure and the one above is the clock under load, not the kernel's structure.
        Ng, Kg = [(N, K) for name, N, K in shapes if name == "ffn_gate_up"][0]
        zc = torch.zeros(e0m4.e0m4_codes_bytes(Ng, Kg, GROUP), dtype=torch.uint8, device=dev)
        zx = torch.zeros((1024, Kg), dtype=torch.float16, device=dev)
        zy = torch.empty((1024, Ng), dtype=torch.float16, device=dev)
        zws = torch.empty(max(e0m4.e0m4_workspace_bytes(1024, Ng, Kg, GROUP), 16), dtype=torch.uint8, device=dev)
        zus = time_us(lambda: e0m4.e0m4_matmul(zx, zc, None, None, Ng, Kg, GROUP, out=zy, workspace=zws, stream=stream),
                      20, rounds=2, warm=3)
        out["roofline_prefill"]["same_launch_on_zero_operands"] = {
            "us": round(zus, 2), "TFLOPs": round(2.0 * 1024 * Ng * Kg / zus / 1e6, 1),
            "frac": round(2.0 * 1024 * Ng * Kg / zus / 1e6 / MFMA_F16_PEAK_TFLOPS, 4)}
        del zc, zx, zy, zws
        out["prefill"] = {"workload": "ChatGLM2-6B-shaped prefill layer, M=1024, 4 GEMMs", "value": layer["achieved"],
                          "unit": "TFLOP/s", "pct_of_mfma_peak": round(100 * layer["frac"], 2),
                          "ms_per_layer": round(layer["avg_launch_us"] / 1e3, 4)}

    # ================= side sections on the ChatGLM2-6B weights ========================================================
    if "small_batch" in want:
        sb = {}
        for M in (2, 4, 8, 16, 32, 64):
            row = {}
            for p, (name, N, K) in enumerate(shapes):
                xm = synth_inputs.activations_device(M, K, 7000 + M + K, dev)
                ym = torch.empty((M, N), dtype=torch.float16, device=dev)
                wsm = torch.empty(max(e0m4.e0m4_workspace_bytes(M, N, K, GROUP), 16), dtype=torch.uint8, device=dev)

                def batch_pass():
                    for mats in layers:
                        e0m4.e0m4_matmul(xm, mats[p][3], None, None, N, K, GROUP, out=ym, workspace=wsm, stream=stream)

                us = time_us(capture(batch_pass), max(1, 100 // n_layers)) / n_layers
                row[name] = {"us": round(us, 3), "GBps": round(algorithmic_bytes(M, N, K, GROUP) / us / 1e3, 1)}
                del xm, ym, wsm
            sb["M=%d" % M] = row
        out["small_batch"] = {"workload": "ChatGLM2-6B shapes, 2 <= M <= 64, group %d; latency per launch, cold weights"
                                          % GROUP, "per_M": sb}
        # groups of 64 on the 14B shapes (config 5's other group): each projection over six distinct weight copies
        sb64 = {}
        for p, (name, N, K) in enumerate(synth_inputs.DENSE_14B):
            copies = []
            for c in range(6):
                W = synth_inputs.weights_device(N, K, 7300 + 10 * p + c, dev)
                copies.append(e0m4.e0m4_quantize(W, 64, stream=stream)[0])
                del W
            for M in (1, 4, 16, 32):
                xm = synth_inputs.activations_device(M, K, 7400 + M + K, dev)
                ym = torch.empty((M, N), dtype=torch.float16, device=dev)
                wsm = torch.empty(max(e0m4.e0m4_workspace_bytes(M, N, K, 64), 16), dtype=torch.uint8, device=dev)

                def pass64():
                    for cc in copies:
                        e0m4.e0m4_matmul(xm, cc, None, None, N, K, 64, out=ym, workspace=wsm, stream=stream)

                us = time_us(capture(pass64), 20) / len(copies)
                sb64.setdefault("M=%d" % M, {})[name] = {"us": round(us, 3),
                                                         "GBps": round(algorithmic_bytes(M, N, K, 64) / us / 1e3, 1)}
                del xm, ym, wsm
            del copies
            torch.cuda.empty_cache()
        out["small_batch_g64"] = {"workload": "14B shapes, group 64, M = 1, 4, 16, 32; latency per launch over six weight "
                                              "copies in turn (185-470 MB)", "per_M": sb64}

    if "dispatch" in want:
        # The kernel and tile that e0m4_matmul picks by itself, against every forced alternative, on seeded shapes that
        # none of its rules was fitted on: three per range of M, N and K multiples of 128, groups 32, 64 and 128.
        import random

        rnd = random.Random(20240331)
        ranges = (("2..8", 2, 8, {"vector_kernel": {"gemv_mfma": 1}, "matrix_core_kernel": {"gemv_mfma": 6}}),
                  ("9..16", 9, 16, {"gemm_64x256": {"gemv_mfma": 1, "gemm_variant": 4},
                                    "gemm_128x128": {"gemv_mfma": 1, "gemm_variant": 3}}),
                  ("17..64", 17, 64, {"gemm_64x256": {"gemv_mfma": 1, "gemm_variant": 4},
                                      "gemm_128x128": {"gemv_mfma": 1, "gemm_variant": 3}}),
                  ("65..384", 65, 384, {"gemm_64x256": {"gemm_variant": 4}, "gemm_128x128": {"gemm_variant": 3},
                                        "gemm_128x256": {"gemm_variant": 5}, "gemm_256x256": {"gemm_variant": 2}}),
                  ("385..4096", 385, 4096, {"gemm_64x256": {"gemm_variant": 4}, "gemm_128x256": {"gemm_variant": 5},
                                            "gemm_256x256": {"gemm_variant": 2},
                                            "even_scheduling_always": {"gemm_sk": 1}, "even_scheduling_never": {"gemm_sk": 2}}))
        knob_names = ("gemv_mfma", "gemm_variant", "gemm_sk")
        rows, ratios = [], []
        for label, m_lo, m_hi, forced in ranges:
            for _ in range(3):
                M = rnd.randint(m_lo, m_hi)
                N, K = 128 * rnd.randint(8, 128), 128 * rnd.randint(8, 96)
                G = rnd.choice((128, 128, 64, 32))
                W = synth_inputs.weights_device(N, K, 9100 + len(rows), dev)
                first = e0m4.e0m4_quantize(W, G, stream=stream)[0]
                del W
                copies = [first] + [first.clone() for _ in range(max(1, min(40, int(4e8 // first.numel()))) - 1)]
                xm = synth_inputs.activations_device(M, K, 9200 + len(rows), dev)
                ym = torch.empty((M, N), dtype=torch.float16, device=dev)
                times = {}
                try:
                    for name, knobs in [("default", {})] + sorted(forced.items()):
                        for k in knob_names:
                            e0m4.e0m4_set_knob(k, knobs.get(k, 0))
                        wsm = torch.empty(max(e0m4.e0m4_workspace_bytes(M, N, K, G), 16), dtype=torch.uint8, device=dev)

                        def variant_pass():
                            for cc in copies:
                                e0m4.e0m4_matmul(xm, cc, None, None, N, K, G, out=ym, workspace=wsm, stream=stream)

                        times[name] = time_us(capture(variant_pass), max(1, 400 // len(copies)), rounds=2) / len(copies)
                        del wsm
                finally:
                    for k in knob_names:
                        e0m4.e0m4_set_knob(k, 0)
                best = min(times, key=times.get)
                ratios.append(times["default"] / times[best])
                rows.append({"M": M, "N": N, "K": K, "G": G, "range": label, "default_us": round(times["default"], 2),
                             "best": best, "best_us": round(times[best], 2), "default_over_best": round(ratios[-1], 3),
                             "forced_us": {k: round(v, 2) for k, v in times.items() if k != "default"}})
                del copies, first, xm, ym
                torch.cuda.empty_cache()
        geo = 1.0
        for r in ratios:
            geo *= r
        out["dispatch"] = {"workload": "15 seeded shapes (N, K multiples of 128 up to 16384 x 12288; groups 32/64/128): the "
                                       "default choice of kernel and tile against every forced one, us per launch over "
                                       "rotating weight copies",
                           "worst_default_over_best": round(max(ratios), 3),
                           "geomean_default_over_best": round(geo ** (1.0 / len(ratios)), 4), "shapes": rows}

    if "table1" in want:
        # the paper's Table 1: E0M4 against the INT4 twin, M = 1, weight [K, N] (same layout, launch shape and
        # accumulation; the twin extracts integers and converts them to fp16); distinct weight copies in turn
        t1 = {}
        for K, N in synth_inputs.TABLE1_SHAPES:
            W = synth_inputs.weights_device(N, K, 8000 + K + N, dev)
            ec = e0m4.e0m4_quantize(W, GROUP, stream=stream)[0]
            ic = e0m4.e0m4_int4_quantize(W, GROUP, stream=stream)[0]
            del W
            copies = max(2, min(32, int(7e8 // ec.numel())))
            ecs = [ec] + [ec.clone() for _ in range(copies - 1)]
            ics = [ic] + [ic.clone() for _ in range(copies - 1)]
            x = synth_inputs.activations_device(1, K, 8100 + K, dev)
            y = torch.empty((1, N), dtype=torch.float16, device=dev)

            def e_pass():
                for c in ecs:
                    e0m4.e0m4_matmul(x, c, None, None, N, K, GROUP, out=y, stream=stream)

            def i_pass():
                for c in ics:
                    e0m4.e0m4_int4_gemv(x, c, N, K, GROUP, out=y, stream=stream)

            ue = time_us(capture(e_pass), 4, rounds=5) / copies
            ui = time_us(capture(i_pass), 4, rounds=5) / copies
            b = algorithmic_bytes(1, N, K, GROUP)
            t1["K%d_N%d" % (K, N)] = {"e0m4_us": round(ue, 3), "int4_us": round(ui, 3), "int4_over_e0m4": round(ui / ue, 3),
                                       "e0m4_GBps": round(b / ue / 1e3, 1), "int4_GBps": round(b / ui / 1e3, 1)}
            del ecs, ics, ec, ic, x, y
        out["table1_e0m4_vs_int4"] = {"workload": "M=1, weight [K,N] of the paper's Table 1, group %d; latency per launch, "
                                                  "cold weights; ratio as the table's 'acceleration'" % GROUP,
                                      "shapes": t1}

    if "e0m8" in want:
        e8 = {}
        for name, N, K in shapes:
            W = synth_inputs.weights_device(N, K, 8500 + N + K, dev)
            c8 = e0m4.e0m8_quantize(W, GROUP, stream=stream)[0]
            del W
            copies = max(2, min(24, int(1.5e9 // c8.numel())))
            bufs = [c8] + [c8.clone() for _ in range(copies - 1)]
            x = synth_inputs.activations_device(1, K, 8600 + K, dev)
            y = torch.empty((1, N), dtype=torch.float16, device=dev)

            def one_pass():
                for c in bufs:
                    e0m4.e0m8_matmul(x, c, N, K, GROUP, out=y, stream=stream)

            us = time_us(capture(one_pass), 4, rounds=5) / copies
            b = N * K * (1.0 + 4.0 / 64) + 2 * K + 2 * N        # a byte per code, a (scale, bias) word per 64 weights
            e8[name] = {"N": N, "K": K, "us": round(us, 3), "GBps": round(b / us / 1e3, 1),
                        "frac_hbm": round(b / us / 1e3 / HBM_PEAK_GBPS, 4)}
            if "prefill" in want:                   # the same weights at M = 1024 on the MFMA kernels
                X = synth_inputs.activations_device(1024, K, 8700 + K, dev, outlier_frac=0.01)
                Y = torch.empty((1024, N), dtype=torch.float16, device=dev)
                ws8 = torch.empty(max(e0m4.e0m8_workspace_bytes(1024, N, K, GROUP), 16), dtype=torch.uint8, device=dev)
                pus = time_us(lambda: e0m4.e0m8_matmul(X, c8, N, K, GROUP, out=Y, workspace=ws8, stream=stream), 20,
                              rounds=2, warm=3)
                e8[name]["prefill_M1024_us"] = round(pus, 2)
                e8[name]["prefill_TFLOPs"] = round(2.0 * 1024 * N * K / pus / 1e6, 1)
                del X, Y, ws8
            del bufs, c8, x, y
        out["e0m8_decode"] = {"workload": "E0M8 (8-bit codes, group %d), M=1, ChatGLM2-6B shapes; latency per launch, "
                                          "cold weights; algorithmic bytes N*K*(1 + 4/64) + 2K + 2N" % GROUP,
                              "per_shape": e8}

    if "bf16" in want:
        # E0M4 on bfloat16 (same packed codes, bfloat16 activations, parameters and outputs): M = 1 and M = 1024
        bf = {}
        for name, N, K in shapes:
            W = synth_inputs.weights_device(N, K, 8800 + N + K, dev).to(torch.bfloat16)
            cb = e0m4.e0m4_bf16_quantize(W, GROUP, stream=stream)[0]
            del W
            copies = max(2, min(32, int(7e8 // cb.numel())))
            bufs = [cb] + [cb.clone() for _ in range(copies - 1)]
            x = synth_inputs.activations_device(1, K, 8900 + K, dev).to(torch.bfloat16)
            y = torch.empty((1, N), dtype=torch.bfloat16, device=dev)

            def one_pass():
                for c in bufs:
                    e0m4.e0m4_bf16_matmul(x, c, N, K, GROUP, out=y, stream=stream)

            us = time_us(capture(one_pass), 4, rounds=5) / copies
            b = algorithmic_bytes(1, N, K, GROUP)
            bf[name] = {"N": N, "K": K, "us": round(us, 3), "GBps": round(b / us / 1e3, 1),
                        "frac_hbm": round(b / us / 1e3 / HBM_PEAK_GBPS, 4)}
            if "prefill" in want:
                X = synth_inputs.activations_device(1024, K, 8950 + K, dev, outlier_frac=0.01).to(torch.bfloat16)
                Y = torch.empty((1024, N), dtype=torch.bfloat16, device=dev)
                pus = time_us(lambda: e0m4.e0m4_bf16_matmul(X, cb, N, K, GROUP, out=Y, stream=stream), 20, rounds=2, warm=3)
                bf[name]["prefill_M1024_us"] = round(pus, 2)
                bf[name]["prefill_TFLOPs"] = round(2.0 * 1024 * N * K / pus / 1e6, 1)
                del X, Y
            del bufs, cb, x, y
        out["e0m4_bf16"] = {"workload": "E0M4 on bfloat16 (group %d), ChatGLM2-6B shapes: M=1 latency per launch over cold "
                                        "weights, M=1024 on the pipelined MFMA kernel in whole tiles (no workspace)" % GROUP, "per_shape": bf}

    if "fusion" in want:
        import torch.nn.functional as F

        fus = {}
        for M, n_l, reps in ((1, n_layers, 10), (1024, 1, 10)):
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
                cq, ca, cg, cd = (m[3] for m in mats)
                e0m4.e0m4_matmul_fused(xh, cq, qN, qK, GROUP, rms_gamma=gamma, rms_eps=1e-5, out=y_qkv,
                                       workspace=fws, stream=stream)
                e0m4.e0m4_matmul_fused(xa, ca, aN, aK, GROUP, residual=resid, out=y_h, workspace=fws, stream=stream)
                e0m4.e0m4_matmul_fused(xh, cg, gN, gK, GROUP, rms_gamma=gamma, rms_eps=1e-5,
                                       epilogue=e0m4.E0M4_EPILOGUE_SWIGLU, out=y_act, workspace=fws, stream=stream)
                e0m4.e0m4_matmul_fused(xd, cd, dN, dK, GROUP, residual=resid, out=y_h, workspace=fws, stream=stream)

            def unfused_layer(mats):
                cq, ca, cg, cd = (m[3] for m in mats)
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
            for label, fn in (("fused", fused_layer), ("unfused", unfused_layer)):
                def all_layers():
                    for mats in layers[:n_l]:
                        fn(mats)
                res[label] = time_us(capture(all_layers), reps, rounds=2, warm=2) / n_l
            fus["M%d" % M] = {"layers_in_graph": n_l, "fused_us_per_layer": round(res["fused"], 2),
                              "unfused_us_per_layer": round(res["unfused"], 2),
                              "unfused_over_fused": round(res["unfused"] / res["fused"], 3)}
            del xh, xa, xd, gamma, resid, y_qkv, y_h, y_gu, y_act, fws
        out["fusion"] = {"workload": "ChatGLM2-6B-shaped layer: rms-norm + qkv, attn-out + residual, rms-norm + gate+up + "
                                     "SiLU-gated product, down + residual; e0m4_matmul_fused against e0m4_matmul plus "
                                     "torch operators, HIP graphs",
                         "results": fus}

    if "kv" in want:
        # KV-cache append in place against the concatenation it replaces (one layer's K and V rows of a
        # ChatGLM2-6B-shaped model, 2 x 2 heads x 128, taken from the QKV output; cache of 2048 positions)
        kv = {}
        max_seq, row = 2048, 512
        for label, n_new in (("decode_1_token", 1), ("prefill_1024_tokens", 1024)):
            have = max_seq - n_new
            cache = torch.zeros((max_seq, row), dtype=torch.float16, device=dev)
            qkv_out = synth_inputs.activations_device(n_new, 4608, 7200, dev)
            pos = torch.arange(have, have + n_new, dtype=torch.int64, device=dev)

            def append20():
                for _ in range(20):
                    e0m4.e0m4_kv_append(cache, qkv_out[:, 4096:], pos, stream=stream)

            def concat20():
                for _ in range(20):
                    torch.cat([cache[:have], qkv_out[:, 4096:]], dim=0)

            ua = time_us(capture(append20), 5, rounds=2) / 20
            uc = time_us(capture(concat20), 5, rounds=2) / 20
            kv[label] = {"append_us": round(ua, 2), "concat_us": round(uc, 2),
                         "bytes_moved_append": 2 * n_new * row * 2, "bytes_moved_concat": 2 * max_seq * row * 2}
            del cache, qkv_out, pos
        out["kv_append"] = {"workload": "cache [2048, 512] fp16, new rows = columns 4096..4607 of the QKV output; "
                                        "20 back-to-back launches in a HIP graph", "results": kv}
    del layers, xs, ys
    torch.cuda.empty_cache()

    # ================= config 4: Gemma-2B-shaped layers and the LM head ================================================
    if "gemma" in want:
        gshapes = synth_inputs.GEMMA_2B
        glayers = quantized_layers(gshapes, synth_inputs.GEMMA_2B_LAYERS, (GROUP,), lambda l, p: 20000 + 4 * l + p)[GROUP]
        us, nb, nl = decode_stack(gshapes, glayers, GROUP, 20)
        cfg4 = {"workload": "Gemma-2B-shaped: decode M=1 over %d layers x 4 projections, LM head 256000 x 2048 at M=1, "
                            "prefill M=512; group 128" % len(glayers),
                "decode_stack": hbm_roofline("gemv_kernel<G=128,M=1>", nb / nl, us / nl, launches_per_step=nl),
                "decode_per_shape": decode_per_shape(gshapes, glayers, GROUP)}
        del glayers
        name, N, K = synth_inputs.GEMMA_2B_LM_HEAD
        W = synth_inputs.weights_device(N, K, 20900, dev)
        c0 = e0m4.e0m4_quantize(W, GROUP)[0]
        del W
        heads = [c0, c0.clone(), c0.clone(), c0.clone()]      # 4 x 279 MB in turn
        x = synth_inputs.activations_device(1, K, 20901, dev)
        y = torch.empty((1, N), dtype=torch.float16, device=dev)

        def head_pass():
            for c in heads:
                e0m4.e0m4_matmul(x, c, None, None, N, K, GROUP, out=y, stream=stream)

        hus = time_us(capture(head_pass), 10) / len(heads)
        cfg4["lm_head"] = hbm_roofline("gemv_kernel<G=128,M=1>", algorithmic_bytes(1, N, K, GROUP), hus,
                                       traffic_key="gemma_lm_head", N=N, K=K)
        del heads, c0, x, y
        if "gemma_prefill" in want:
            pre, layer = prefill_shapes(gshapes, 512, GROUP, 21000, not args.no_library)
            cfg4["prefill_M512"] = {"per_shape": pre, "layer": layer}
        configs["cfg4_gemma2b"] = cfg4
        torch.cuda.empty_cache()

    # ================= config 5: 14B-shaped layers, groups 64 and 128, M = 1 and M = 2048 ==============================
    if "d14b" in want:
        dshapes = synth_inputs.DENSE_14B
        n14 = synth_inputs.DENSE_14B_LAYERS
        both = quantized_layers(dshapes, n14, (64, 128), lambda l, p: 30000 + 4 * l + p)
        cfg5 = {"workload": "14B-shaped (hidden 5120, intermediate 13696): decode M=1 over %d layers x 4 projections, "
                            "prefill M=2048; groups 64 and 128" % n14}
        for G in (64, 128):
            us, nb, nl = decode_stack(dshapes, both[G], G, 10)
            entry = {"decode_stack": hbm_roofline("gemv_kernel<G=%d,M=1>" % G, nb / nl, us / nl, launches_per_step=nl),
                     "decode_per_shape": decode_per_shape(dshapes, both[G], G)}
            del both[G]
            torch.cuda.empty_cache()
            if "d14b_prefill" in want:
                pre, layer = prefill_shapes(dshapes, 2048, G, 31000 + G, not args.no_library and G == 128,
                                            "d14b_prefill_g%d" % G)
                entry["prefill_M2048"] = {"per_shape": pre, "layer": layer}
            cfg5["group_%d" % G] = entry
        configs["cfg5_dense14b"] = cfg5
        torch.cuda.empty_cache()

    # ================= CPU oracle on bounded samples of the same work =================================================
    if "cpu" in want:
        import oracle

        packed = []
        for p, (name, N, K) in enumerate(shapes):
            W = synth_inputs.weights(N, K, synth_inputs.layer_seed(0, p))
            packed.append((N, K) + oracle.quantize(W, GROUP))
            del W
        xcpu = {K: synth_inputs.activations(1, K, 99 + K) for _, _, K in shapes}
        layer_bytes = sum(algorithmic_bytes(1, N, K, GROUP) for _, N, K in shapes)

        def layer_pass():
            for N, K, codes, scales, bias in packed:
                What = oracle.dequant(codes, scales, bias, GROUP)
                oracle.matmul(xcpu[K], What, want_absdot=False)

        reps, t_cpu = 0, 0.0
        while t_cpu < 10.0 and reps < 64:
            t0 = time.perf_counter()
            layer_pass()
            t_cpu += time.perf_counter() - t0
            reps += 1
        cores = oracle.num_threads()
        out["cpu_baseline"] = {"value": round(layer_bytes * reps / t_cpu / 1e9, 3), "unit": "GB/s", "cores": cores,
                               "kind": "oracle",
                               "sample": "%d x (dequant + fp64 matmul, M=1) over the 4 projections of one ChatGLM2-6B-shaped "
                                         "layer, %.1f s wall on %d threads" % (reps, t_cpu, cores)}
        # one thread, the 4096 x 4096 projection only (the single-GEMV workload)
        N, K, codes, scales, bias = packed[1]
        if oracle.set_num_threads(1):
            t0 = time.perf_counter()
            r1 = 0
            while time.perf_counter() - t0 < 4.0:
                oracle.matmul(xcpu[K], oracle.dequant(codes, scales, bias, GROUP), want_absdot=False)
                r1 += 1
            t1 = time.perf_counter() - t0
            oracle.set_num_threads(cores)
            out["cpu_baseline"]["one_thread"] = {"value": round(algorithmic_bytes(1, N, K, GROUP) * r1 / t1 / 1e9, 4),
                                                 "unit": "GB/s", "cores": 1,
                                                 "sample": "%d x (dequant + fp64 matmul, M=1) of 4096 x 4096, %.1f s" % (r1, t1)}
        # prefill: an M = 16 slice of the M = 1024 problem on the true N x K, scaled linearly to 1024 rows
        X16 = {K: synth_inputs.activations(16, K, 6000 + K, outlier_frac=0.01) for _, _, K in shapes}
        t0 = time.perf_counter()
        flops16 = 0.0
        for N, K, codes, scales, bias in packed:
            What = oracle.dequant(codes, scales, bias, GROUP)
            oracle.matmul(X16[K], What, want_absdot=False)
            flops16 += 2.0 * 16 * N * K
        t16 = time.perf_counter() - t0
        out["cpu_baseline"]["prefill_extrapolated"] = {
            "value": round(flops16 / t16 / 1e12, 5), "unit": "TFLOP/s", "cores": cores,
            "sample": "dequant + fp64 matmul of an M=16 slice of the four M=1024 GEMMs (%.1f s); a full layer at this "
                      "rate would take %.0f s (extrapolated x64)" % (t16, t16 * 64)}

    print(json.dumps(out))


if __name__ == "__main__":
    main()
