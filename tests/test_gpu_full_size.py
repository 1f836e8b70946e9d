"""Parity at the full sizes of the benchmark workloads, in the launch
configuration the benchmark times (default knobs): linear layers shaped like
ChatGLM2-6B, Gemma-2B and a 14B decoder.  Codes/scales/bias/dequantised weights
are compared in full (bit-exact).  The decode output (M=1) is compared in full;
the prefill output on sampled rows (all N) and sampled columns (all M), which
the oracle can compute one by one."""
import numpy as np
import pytest

import synth_inputs
from test_gpu_parity import DEV, assert_quantize_exact, bits, check_matmul, e0m4, to_dev, torch  # noqa: F401

pytestmark = pytest.mark.gpu

CASES = [
    # (name, N, K, G, prefill M or None, seed or None)
    ("cfg1_square_seed0", 4096, 4096, 128, None, 0),        # the single decode GEMV of the first workload, its own seed
    ("cfg1_square", 4096, 4096, 128, None, None),
    ("chatglm2_qkv", 4608, 4096, 128, 1024, None),
    ("chatglm2_attn_out", 4096, 4096, 128, 1024, None),
    ("chatglm2_gate_up", 27392, 4096, 128, 1024, None),
    ("chatglm2_down", 4096, 13696, 128, 1024, None),
    ("gemma_qkv", 2560, 2048, 128, 512, None),
    ("gemma_attn_out", 2048, 2048, 128, 512, None),
    ("gemma_gate_up", 32768, 2048, 128, 512, None),
    ("gemma_down", 2048, 16384, 128, 512, None),
    ("gemma_lm_head", 256000, 2048, 128, None, None),
]
# the 14B-shaped layer: every projection with groups of 64 and of 128, decode in full and prefill at M = 2048
CASES += [("d14b_%s_g%d" % (name, G), N, K, G, 2048, None)
          for name, N, K in (("qkv", 15360, 5120), ("attn_out", 5120, 5120), ("gate_up", 27392, 5120),
                             ("down", 5120, 13696))
          for G in (64, 128)]


def sample_indices(count, total, tile, rng):
    fixed = {0, total - 1, tile - 1, tile, total // 2, max(total - tile, 0), max(total - tile - 1, 0)}
    fixed = {i for i in fixed if 0 <= i < total}
    extra = set(int(i) for i in rng.integers(0, total, max(count - len(fixed), 0)))
    return np.array(sorted(fixed | extra), dtype=np.int64)


@pytest.mark.parametrize("name,N,K,G,Mp,seed", CASES, ids=[c[0] for c in CASES])
def test_full_size_layer(e0m4, oracle, name, N, K, G, Mp, seed):
    if seed is None:
        seed = abs(hash((N, K, G))) % 10007
    prefill = Mp is not None
    W = synth_inputs.weights(N, K, seed=seed, row_std_range=(0.5, 2.0) if prefill else None)
    (codes, scales, bias), What = assert_quantize_exact(e0m4, oracle, W, G)
    del W
    # decode: whole output
    X1 = synth_inputs.activations(1, K, seed=seed)
    Y1 = e0m4.e0m4_matmul(to_dev(X1), codes, scales, bias, N, K, G)
    Yref, absdot = oracle.matmul(X1, What)
    check_matmul(Y1, Yref, absdot, name + " decode")
    if not prefill:
        return
    # prefill: sampled rows over all N, sampled columns over all M
    X = synth_inputs.activations(Mp, K, seed=seed + 1, outlier_frac=0.01)
    Y = e0m4.e0m4_matmul(to_dev(X), codes, scales, bias, N, K, G).cpu().numpy()
    rng = np.random.default_rng(seed)
    ms = sample_indices(16, Mp, 128, rng)
    Yr, ad = oracle.matmul(X[ms], What)
    check_matmul(torch.from_numpy(Y[ms]), Yr, ad, name + " prefill rows")
    ns = sample_indices(64, N, 128, rng)
    Yc, adc = oracle.matmul(X, What[ns])
    check_matmul(torch.from_numpy(np.ascontiguousarray(Y[:, ns])), Yc, adc, name + " prefill cols")


def test_decode_layer_in_a_hip_graph_matches_eager(e0m4):
    """The benchmark replays a captured HIP graph of e0m4_matmul launches: several replays, with eager
    work and synchronisation in between, must reproduce the eager results bit for bit."""
    G = 128
    stream = torch.cuda.Stream()
    mats = []
    for p, (name, N, K) in enumerate(synth_inputs.CHATGLM2_6B):
        W = synth_inputs.weights_device(N, K, 7000 + p, DEV)
        codes, scales, bias = e0m4.e0m4_quantize(W, G)
        del W
        x = synth_inputs.activations_device(1, K, 7100 + p, DEV)
        y = torch.empty((1, N), dtype=torch.float16, device=DEV)
        mats.append((N, K, codes, scales, bias, x, y))
    torch.cuda.synchronize()
    eager = [e0m4.e0m4_matmul(x, codes, scales, bias, N, K, G).clone() for N, K, codes, scales, bias, x, y in mats]
    torch.cuda.synchronize()
    with torch.cuda.stream(stream):
        for N, K, codes, scales, bias, x, y in mats:           # loads the code objects before capture
            e0m4.e0m4_matmul(x, codes, scales, bias, N, K, G, out=y, stream=stream)
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            for N, K, codes, scales, bias, x, y in mats:
                e0m4.e0m4_matmul(x, codes, scales, bias, N, K, G, out=y, stream=stream)
    for replay in range(3):
        for m in mats:
            m[6].fill_(float("nan"))                           # eager work between replays
        torch.cuda.synchronize()
        with torch.cuda.stream(stream):
            graph.replay()
        stream.synchronize()
        for want, m in zip(eager, mats):
            assert np.array_equal(bits(m[6]), bits(want)), "replay %d" % replay
