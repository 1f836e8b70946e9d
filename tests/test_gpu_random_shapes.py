"""Parity of e0m4_matmul and e0m4_matmul_fused with the CPU oracle on seeded random shapes: every dispatch rule
(decode kernel with its wavefront counts and staging modes, small-batch kernel, GEMM tiles and K splits) is met by
shapes nobody chose by hand.  Same tolerances as the hand-picked cases."""
import numpy as np
import pytest

import synth_inputs
from test_gpu_fused import check_fused

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

DEV = "cuda:0"
KNOBS = ("gemv_waves", "gemv_workgroups", "gemv_mfma", "gemv_xreg", "gemm_variant", "gemm_splits", "gemm_sk", "gemm_panel", "gemm_split_order")


@pytest.fixture(scope="module")
def e0m4():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (run with -m 'not gpu' elsewhere)")
    import paper_2403_20041_amd as pkg

    pkg.lib()
    for k in KNOBS:
        pkg.e0m4_set_knob(k, 0)
    return pkg


def to_dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def random_cases(count, seed):
    rng = np.random.default_rng(seed)
    ms = [1, 1, 1, 2, 3, 4, 5, 6, 7, 8, 9, 12, 16, 17, 33, 64, 65, 100, 129, 200, 257, 385, 400, 520]
    cases = []
    for i in range(count):
        G = int(rng.choice([32, 64, 128]))
        M = int(rng.choice(ms))
        # K: a multiple of the group (and of 32); mostly whole blocks of 128, sometimes ragged, sometimes long
        kind = rng.integers(0, 10)
        if kind < 6:
            K = 128 * int(rng.integers(1, 65))
        elif kind < 8:
            K = max(G, 32) * int(rng.integers(1, 100))
        else:
            K = 512 * int(rng.choice([8, 10, 12, 14, 16, 27]))
        K = (K // max(G, 32)) * max(G, 32)
        N = int(rng.choice([int(rng.integers(1, 400)), 64 * int(rng.integers(1, 40)), int(rng.integers(400, 6000))]))
        # keep the oracle's work (M * N * K multiply-adds in fp64) within a second or two
        while M * N * K > 6e8:
            N = max(16, N // 2)
        fused = bool(rng.integers(0, 2))
        norm, swiglu, res = (bool(rng.integers(0, 2)) for _ in range(3)) if fused else (False, False, False)
        if swiglu:
            N = max(64, (N // 64) * 64)
        cases.append((i, M, N, K, G, fused, norm, swiglu, res))
    return cases


CASES = random_cases(72, seed=20240327)


@pytest.mark.parametrize("case", CASES, ids=["%d-M%d-N%d-K%d-G%d-%s" % (c[0], c[1], c[2], c[3], c[4],
                                                                       ("f%d%d%d" % c[6:9]) if c[5] else "plain")
                                             for c in CASES])
def test_random_shape(e0m4, oracle, case):
    i, M, N, K, G, fused, norm, swiglu, res = case
    W = synth_inputs.weights(N, K, seed=9000 + i, row_std_range=(0.5, 2.0) if i % 3 == 0 else None)
    X = synth_inputs.activations(M, K, seed=9100 + i, outlier_frac=0.01 if i % 2 else 0.0)
    codes, scales, bias = e0m4.e0m4_quantize(to_dev(W), G)
    oc, os_, ob = oracle.quantize(W, G)
    assert np.array_equal(e0m4.e0m4_unpack_codes(codes, N, K, G).cpu().numpy(), oc)
    What = oracle.dequant(oc, os_, ob, G)
    if not fused:
        Y = e0m4.e0m4_matmul(to_dev(X), codes, scales, bias, N, K, G).cpu().numpy()
        Yref, absdot = oracle.matmul(X, What)
        err = np.abs(Y.astype(np.float64) - Yref.astype(np.float64))
        assert (err <= 1e-2 * np.maximum(1.0, absdot)).all(), "case %s" % (case,)
        assert (err <= 2.0 ** -9 * absdot + 2.0 ** -10 * np.abs(Yref.astype(np.float64)) + 1e-6).all(), "quality, case %s" % (case,)
        return
    gamma = synth_inputs.norm_weight(K, 9200 + i) if norm else None
    n_out = N // 2 if swiglu else N
    R = synth_inputs.residual(M, n_out, 9300 + i) if res else None
    Y = e0m4.e0m4_matmul_fused(to_dev(X), codes, N, K, G, rms_gamma=to_dev(gamma), rms_eps=1e-5,
                               epilogue=e0m4.E0M4_EPILOGUE_SWIGLU if swiglu else e0m4.E0M4_EPILOGUE_NONE,
                               residual=to_dev(R))
    Yref, info = oracle.matmul_fused(X, What, gamma=gamma, eps=1e-5, swiglu=swiglu, residual=R)
    torch.cuda.synchronize()
    check_fused(Y, Yref, info, swiglu, norm, "case %s" % (case,))


CASES8 = [c for c in random_cases(60, seed=20240328) if c[4] != 32][:30]


@pytest.mark.parametrize("case", CASES8, ids=["%d-M%d-N%d-K%d-G%d-%s" % (c[0], c[1], c[2], c[3], c[4],
                                                                        ("f%d%d%d" % c[6:9]) if c[5] else "plain")
                                              for c in CASES8])
def test_random_shape_8bit(e0m4, oracle, case):
    i, M, N, K, G, fused, norm, swiglu, res = case
    if M > 8 and N % 8 != 0:
        N += 8 - N % 8                  # larger M with K not a multiple of 128 runs in row chunks: Y rows 16-byte aligned
    if fused and M > 8 and K % 128 != 0:
        K += 128 - K % 128              # the fused 8-bit GEMM needs whole slices of 128
    W = synth_inputs.weights(N, K, seed=9500 + i)
    X = synth_inputs.activations(M, K, seed=9600 + i, outlier_frac=0.01 if i % 2 else 0.0)
    codes, _, _ = e0m4.e0m8_quantize(to_dev(W), G)
    oc, os_, ob = oracle.quantize_k(W, G, 8)
    assert np.array_equal(e0m4.e0m8_unpack_codes(codes, N, K, G).cpu().numpy(), oc)
    What = oracle.dequant_k(oc, os_, ob, G, 8)
    if not fused:
        Y = e0m4.e0m8_matmul(to_dev(X), codes, N, K, G).cpu().numpy()
        Yref, absdot = oracle.matmul(X, What)
        err = np.abs(Y.astype(np.float64) - Yref.astype(np.float64))
        assert (err <= 1e-2 * np.maximum(1.0, absdot)).all(), "case %s" % (case,)
        assert (err <= 2.0 ** -9 * absdot + 2.0 ** -10 * np.abs(Yref.astype(np.float64)) + 1e-6).all(), "quality, case %s" % (case,)
        return
    gamma = synth_inputs.norm_weight(K, 9700 + i) if norm else None
    n_out = N // 2 if swiglu else N
    R = synth_inputs.residual(M, n_out, 9800 + i) if res else None
    Y = e0m4.e0m8_matmul_fused(to_dev(X), codes, N, K, G, rms_gamma=to_dev(gamma), rms_eps=1e-5,
                               epilogue=e0m4.E0M4_EPILOGUE_SWIGLU if swiglu else e0m4.E0M4_EPILOGUE_NONE,
                               residual=to_dev(R))
    Yref, info = oracle.matmul_fused(X, What, gamma=gamma, eps=1e-5, swiglu=swiglu, residual=R)
    torch.cuda.synchronize()
    check_fused(Y, Yref, info, swiglu, norm, "8-bit case %s" % (case,))


def wide_cases(count, seed):
    """Shapes of the paths the list above does not reach: 17 to 64 rows (row chunks in one launch) and GEMMs of many
    tiles (whole rounds, the even scheduling of a partly filled last round, also forced on arbitrary shapes)."""
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(count):
        G = int(rng.choice([32, 64, 128]))
        mode = i % 3
        if mode == 0:
            M, K = int(rng.choice([18, 24, 31, 40, 47, 48, 49, 63])), 128 * int(rng.integers(1, 40))
            N = int(rng.choice([int(rng.integers(16, 400)), 64 * int(rng.integers(1, 80)), int(rng.integers(400, 12000))]))
        elif mode == 1:
            M, K = int(rng.choice([1024, 1100, 1536, 2048, 2304])), 128 * int(rng.integers(1, 12))
            N = 256 * int(rng.integers(20, 60)) + int(rng.integers(0, 256))
        else:
            M, K, N = int(rng.integers(257, 1500)), 128 * int(rng.integers(1, 24)), int(rng.integers(100, 5000))
        cases.append((i, M, N, K, G, mode == 2))
    return cases


WIDE = wide_cases(24, seed=20240329)


@pytest.mark.parametrize("case", WIDE, ids=["%d-M%d-N%d-K%d-G%d%s" % (c[0], c[1], c[2], c[3], c[4], "-even" if c[5] else "")
                                            for c in WIDE])
def test_random_shape_wide(e0m4, oracle, case):
    i, M, N, K, G, forced = case
    rng = np.random.default_rng(i)
    W = synth_inputs.weights(N, K, seed=9900 + i, row_std_range=(0.5, 2.0) if i % 2 else None)
    X = synth_inputs.activations(M, K, seed=9950 + i, outlier_frac=0.01)
    codes, scales, bias = e0m4.e0m4_quantize(to_dev(W), G)
    What = oracle.dequant(*oracle.quantize(W, G), G)
    rows = np.arange(M) if M * N * K <= 4e8 else np.unique(np.concatenate(
        [np.arange(0, M, 256), np.arange(255, M, 256), [M - 1], rng.integers(0, M, size=10)]))
    if forced:
        e0m4.e0m4_set_knob("gemm_variant", 2)
        e0m4.e0m4_set_knob("gemm_sk", 1)
    try:
        Y = e0m4.e0m4_matmul(to_dev(X), codes, scales, bias, N, K, G)
    finally:
        e0m4.e0m4_set_knob("gemm_variant", 0)
        e0m4.e0m4_set_knob("gemm_sk", 0)
    got = Y[torch.from_numpy(rows).to(DEV)].cpu().numpy().astype(np.float64)
    Yref, absdot = oracle.matmul(X[rows], What)
    err = np.abs(got - Yref.astype(np.float64))
    assert (err <= 1e-2 * np.maximum(1.0, absdot)).all(), "case %s" % (case,)
    assert (err <= 2.0 ** -9 * absdot + 2.0 ** -10 * np.abs(Yref.astype(np.float64)) + 1e-6).all(), "quality, case %s" % (case,)
