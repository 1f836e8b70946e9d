"""Re-fit the constants of the prefill GEMM's launch-time estimate (csrc/e0m4_gemm_pipe.hip: kFlatCost, kHalfCost,
kBigCost, kReduceUs, kReduceUsPerMB, kSkUs, kSkUsPerSharer) on the GPU at hand.

    python -m paper_2403_20041_amd.tune_gemm_estimate time  timings.txt [--problems 120] [--seed 7]
    python -m paper_2403_20041_amd.tune_gemm_estimate fit   timings.txt [more.txt ...]

`time` draws seeded problems (M = 65 .. 8192, N and K multiples of 128, plus the layer shapes of synth_inputs) and
times e0m4_matmul on each with every tile forced (knob gemm_variant 4, 5, 2), one to eight K splits (gemm_splits)
and, where the large tile leaves a partly filled last round of at least 128 tiles, even scheduling (gemm_sk 1): us
per launch in a HIP graph over rotating weight copies, so that the weights come from HBM.  `fit` minimises the squared
logarithm of estimate / measurement over all timings, prints the constants in the order of the C++ initialisers and
says how much slower than the measured best the estimate's choice is (geometric mean over the problems).  The knobs
are diagnostic and belong to the calling thread; nothing here changes the library's defaults: paste the constants
into the source and rebuild.
"""
from __future__ import annotations

import argparse
import math
import random
import re
import sys

CU = 256
TILES = {"f": (64, 256, 2 * CU, 0), "h": (128, 256, 2 * CU, 1), "b": (256, 256, CU, 2)}   # rows, columns, items per round
VARIANT = {"f": 4, "h": 5, "b": 2}
NP = 8                                                      # constants per tile: four low knots, three high, b
START = [0.8, 1.2, 1.3, 1.45, 1.6, 2.0, 2.0, 4.4, 1.4, 1.5, 1.6, 1.9, 2.6, 3.1, 3.4, 5.9,
         2.0, 2.3, 2.45, 2.5, 2.45, 2.9, 3.5, 9.3, 4.9, 0.18, 35.0, 0.7]


def interp(x, xs, ys):
    for i in range(len(xs) - 1):
        if x <= xs[i + 1]:
            return ys[i] + (ys[i + 1] - ys[i]) * (x - xs[i]) / (xs[i + 1] - xs[i])
    return ys[-1]


def estimate(p, M, N, K, tile, splits):
    """The launch time in us as rounds_us / split_launch_us / sk_launch_us compute it; splits = 'sk': even scheduling."""
    bm, bn, cap, i = TILES[tile]
    lo, hi, b = p[NP * i:NP * i + 4], p[NP * i + 4:NP * i + 7], p[NP * i + 7]
    r0, r1, c0, c1 = p[3 * NP:3 * NP + 4]
    tiles, pairs = -(-M // bm) * -(-N // bn), K // 128
    if splits == "sk":
        full, rem = divmod(tiles, CU)
        return full * (pairs * hi[2] + b) + rem * pairs / CU * hi[2] + b + c0 + c1 * min(CU / rem + 1, pairs)
    full, rem = divmod(tiles * splits, cap)
    kp = pairs / splits
    t = full * (kp * hi[2] + b)
    if rem:
        fill = rem / cap
        a = interp(fill, [0, 0.125, 0.25, 0.5], lo) if fill <= 0.5 else interp(fill, [0.5, 0.75, 1.0], hi)
        t += kp * a + b
    if splits > 1:
        t += r0 + r1 * splits * M * N * 4 / 1e6
    return t


def read_timings(paths):
    """lines 'M N K tile splits us' -> {(M, N, K): [(tile, splits, us), ...]}"""
    groups = {}
    for path in paths:
        for line in open(path):
            m = re.match(r"(\d+) (\d+) (\d+) ([fhb]) (\d+|sk) ([0-9.]+)\s*$", line)
            if m:
                M, N, K = int(m.group(1)), int(m.group(2)), int(m.group(3))
                s = m.group(5) if m.group(5) == "sk" else int(m.group(5))
                groups.setdefault((M, N, K), []).append((m.group(4), s, float(m.group(6))))
    return groups


def fit(paths):
    import numpy as np
    from scipy.optimize import least_squares

    groups = read_timings(paths)
    pts = [(M, N, K, t, s, us) for (M, N, K), c in groups.items() for t, s, us in c]
    lo = ([0.01] * 7 + [0.0]) * 3 + [0.0] * 4
    hi = ([8.0] * 7 + [40.0]) * 3 + [50.0, 5.0, 100.0, 10.0]

    def resid(p):
        return [math.log(estimate(p, M, N, K, t, s) / us) for M, N, K, t, s, us in pts]

    p = least_squares(resid, START, bounds=(lo, hi)).x
    r = np.array(resid(p))
    regret = [min(c, key=lambda x: estimate(p, M, N, K, x[0], x[1]))[2] / min(x[2] for x in c)
              for (M, N, K), c in groups.items()]
    print("%d timings of %d problems; rms of log(estimate / measured) %.3f" % (len(pts), len(groups), r.std()))
    print("choice by the estimate over the measured best: geometric mean %.4f, worst %.3f"
          % (math.exp(sum(math.log(x) for x in regret) / len(regret)), max(regret)))
    for name, i in (("kFlatCost", 0), ("kHalfCost", 1), ("kBigCost", 2)):
        q = p[NP * i:NP * i + NP]
        print("%s{{%.3f, %.3f, %.3f, %.3f}, {%.3f, %.3f, %.3f}, %.2f, ...}" % ((name,) + tuple(q)))
    print("kReduceUs = %.2f, kReduceUsPerMB = %.3f, kSkUs = %.1f, kSkUsPerSharer = %.2f" % tuple(p[3 * NP:3 * NP + 4]))


def time_problems(out_path, n_problems, seed):
    import torch

    import paper_2403_20041_amd as e0m4
    import synth_inputs

    dev = torch.device("cuda:0")
    stream = torch.cuda.Stream()
    rnd = random.Random(seed)
    problems = []
    for lo_m, hi_m, share in ((65, 384, 0.35), (385, 1024, 0.3), (1025, 2560, 0.25), (2561, 8192, 0.1)):
        for _ in range(int(n_problems * share)):
            problems.append((rnd.randint(lo_m, hi_m), 128 * rnd.randint(8, 160), 128 * rnd.randint(8, 112)))
    for shapes in (synth_inputs.CHATGLM2_6B, synth_inputs.DENSE_14B):
        for M in (256, 512, 1024, 2048):
            problems += [(M, N, K) for _, N, K in shapes]
    knobs = ("gemm_variant", "gemm_splits", "gemm_sk")
    with open(out_path, "a") as out:
        for M, N, K in problems:
            W = synth_inputs.weights_device(N, K, 1, dev)
            first = e0m4.e0m4_quantize(W, 128)[0]
            del W
            copies = [first] + [first.clone() for _ in range(max(2, min(40, int(4e8 // first.numel()))) - 1)]
            x = synth_inputs.activations_device(M, K, 2, dev)
            y = torch.empty((M, N), dtype=torch.float16, device=dev)
            pairs = K // 128
            cands = []
            for tile, (bm, bn, cap, _) in TILES.items():
                tiles = -(-M // bm) * -(-N // bn)
                for s in ((1,) if tiles >= CU else [s for s in (1, 2, 3, 4, 6, 8) if s == 1 or pairs // s >= 4]):
                    cands.append((tile, s))
            big = -(-M // 256) * -(-N // 256)
            if big >= 128 and big % CU:
                cands.append(("b", "sk"))
            try:
                for tile, s in cands:
                    e0m4.e0m4_set_knob("gemm_variant", VARIANT[tile])
                    e0m4.e0m4_set_knob("gemm_splits", 1 if s == "sk" else s)
                    e0m4.e0m4_set_knob("gemm_sk", 1 if s == "sk" else 2)
                    ws = torch.empty(max(16, e0m4.e0m4_workspace_bytes(M, N, K, 128)), dtype=torch.uint8, device=dev)
                    with torch.cuda.stream(stream):
                        for c in copies[:2]:
                            e0m4.e0m4_matmul(x, c, None, None, N, K, 128, out=y, workspace=ws, stream=stream)
                        stream.synchronize()
                        g = torch.cuda.CUDAGraph()
                        with torch.cuda.graph(g, stream=stream):
                            for c in copies:
                                e0m4.e0m4_matmul(x, c, None, None, N, K, 128, out=y, workspace=ws, stream=stream)
                        best = None
                        for _ in range(3):
                            g.replay()
                            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                            e0.record(stream)
                            g.replay()
                            g.replay()
                            e1.record(stream)
                            stream.synchronize()
                            us = e0.elapsed_time(e1) * 1e3 / (2 * len(copies))
                            best = us if best is None else min(best, us)
                        del g
                    out.write("%d %d %d %s %s %.2f\n" % (M, N, K, tile, s, best))
                    out.flush()
            finally:
                for k in knobs:
                    e0m4.e0m4_set_knob(k, 0)
            print("timed M=%d N=%d K=%d (%d launch shapes)" % (M, N, K, len(cands)), flush=True)
            del copies, first, x, y
            torch.cuda.empty_cache()


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("mode", choices=("time", "fit"))
    ap.add_argument("files", nargs="+")
    ap.add_argument("--problems", type=int, default=120)
    ap.add_argument("--seed", type=int, default=7)
    args = ap.parse_args()
    if args.mode == "time":
        time_problems(args.files[0], args.problems, args.seed)
    else:
        fit(args.files)


if __name__ == "__main__":
    sys.exit(main())
