"""Parity of the INT4 twin (paper: section "Evaluation of FP4 quantization") with the CPU oracle:
codes, scales, zero points and dequantised weights bit-exact; the M = 1 product within the same
tolerance as the E0M4 matmul; and the three weight shapes of the paper's Table 1 at full size."""
import numpy as np
import pytest

import synth_inputs
from test_gpu_parity import DEV, bits, check_matmul, e0m4, to_dev, torch  # noqa: F401

pytestmark = pytest.mark.gpu


def assert_int4_quantize_exact(e0m4, oracle, W, G):
    N, K = W.shape
    codes, scales, zeros = e0m4.e0m4_int4_quantize(to_dev(W), G)
    oc, os_, oz = oracle.int4_quantize(W, G)
    torch.cuda.synchronize()
    assert np.array_equal(bits(scales), os_.view(np.uint16)), "scales differ"
    assert np.array_equal(bits(zeros), oz.view(np.uint16)), "zero points differ"
    assert np.array_equal(bits(e0m4.e0m4_unpack_codes(codes, N, K, G)), oc), "codes differ"
    want = oracle.int4_dequant(oc, os_, oz, G)
    assert np.array_equal(bits(e0m4.e0m4_int4_dequant(codes, N, K, G)), want.view(np.uint16)), "dequantised weights differ"
    return codes, want


@pytest.mark.parametrize("N,K,G", [(N, K, G) for N, K in [(64, 128), (200, 384), (1, 128), (65, 256), (130, 1024), (70, 416)]
                                   for G in (32, 64, 128) if K % G == 0])
def test_int4_quantize_dequant_bit_exact(e0m4, oracle, N, K, G):
    assert_int4_quantize_exact(e0m4, oracle, synth_inputs.weights(N, K, seed=2000 + N + K + G), G)


def test_int4_quantize_value_distributions(e0m4, oracle):
    rng = np.random.default_rng(17)
    N, K = 96, 512
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float16)
    W[0:8] = 0.0
    W[8:16] = np.float16(0.5)
    W[16:24] = np.abs(W[16:24])
    W[24:32] = -np.abs(W[24:32])
    W[32:40] = (rng.standard_normal((8, K)) * 3e-6).astype(np.float16)
    W[40:48] = np.clip(rng.standard_normal((8, K)) * 2e4, -6e4, 6e4).astype(np.float16)
    W[48, ::2] = np.float16(65504.0)
    W[48, 1::2] = np.float16(-65504.0)
    W[56:64] = rng.integers(-3, 4, (8, K)).astype(np.float16) * np.float16(2.0 ** -14)
    W[64:72] = (rng.integers(-7, 9, (8, K)) * 0.5).astype(np.float16)       # values on rounding ties
    with np.errstate(over="ignore"):
        for G in (32, 128):
            assert_int4_quantize_exact(e0m4, oracle, W, G)


def run_int4_gemv_case(e0m4, oracle, N, K, G, seed):
    W = synth_inputs.weights(N, K, seed=seed)
    X = synth_inputs.activations(1, K, seed=seed)
    codes, What = assert_int4_quantize_exact(e0m4, oracle, W, G)
    Y = e0m4.e0m4_int4_gemv(to_dev(X), codes, N, K, G)
    Yref, absdot = oracle.matmul(X, What)
    torch.cuda.synchronize()
    check_matmul(Y, Yref, absdot, "int4 N=%d K=%d G=%d" % (N, K, G))
    return codes, X, Y


@pytest.mark.parametrize("N,K,G", [(200, 1152, 128), (64, 128, 128), (1, 32, 32), (333, 1024, 32), (700, 3968, 64),
                                    (203, 1664, 128), (48, 512, 64)])
def test_int4_gemv_small(e0m4, oracle, N, K, G):
    run_int4_gemv_case(e0m4, oracle, N, K, G, seed=N + K)


@pytest.mark.parametrize("waves", [4, 8, 16])
def test_int4_gemv_forced_waves(e0m4, oracle, waves):
    e0m4.e0m4_set_knob("gemv_waves", waves)
    try:
        run_int4_gemv_case(e0m4, oracle, 300, 2304, 128, seed=3)
    finally:
        e0m4.e0m4_set_knob("gemv_waves", 0)


def test_int4_one_hot_reproduces_weights_and_is_deterministic(e0m4, oracle):
    N, K, G = 200, 512, 128
    W = synth_inputs.weights(N, K, seed=60)
    codes, What = assert_int4_quantize_exact(e0m4, oracle, W, G)
    for k in (0, 77, K - 1):
        X = np.zeros((1, K), dtype=np.float16)
        X[0, k] = 1.0
        Y = bits(e0m4.e0m4_int4_gemv(to_dev(X), codes, N, K, G))
        assert np.array_equal(Y[0], What.view(np.uint16)[:, k])
    X = to_dev(synth_inputs.activations(1, K, seed=61))
    assert np.array_equal(bits(e0m4.e0m4_int4_gemv(X, codes, N, K, G)), bits(e0m4.e0m4_int4_gemv(X, codes, N, K, G)))


def test_int4_data_through_the_e0m4_path(e0m4, oracle):
    """An INT4 group with integer zero point is an E0M4 group with scale 8 s and bias 2 + z/8: encoding the
    INT4 codes with those parameters makes e0m4_dequant and e0m4_matmul reproduce the INT4 results."""
    N, K, G = 256, 1024, 128
    W = synth_inputs.weights(N, K, seed=70)
    oc, os_, oz = oracle.int4_quantize(W, G)
    What = oracle.int4_dequant(oc, os_, oz, G)
    s8 = (os_.astype(np.float32) * 8).astype(np.float16)
    assert np.array_equal(s8.astype(np.float32), os_.astype(np.float32) * 8)         # exact
    bias = (0x4000 | (oz.astype(np.uint16) << 6)).astype(np.uint16).view(np.float16)
    assert np.array_equal(oracle.encode(What, s8, bias, G), oc)          # the E0M4 encoder finds the same codes
    codes = e0m4.e0m4_encode(to_dev(What), to_dev(s8), to_dev(bias), G)
    assert np.array_equal(bits(e0m4.e0m4_unpack_codes(codes, N, K, G)), oc)
    assert np.array_equal(bits(e0m4.e0m4_dequant(codes, None, None, N, K, G)), What.view(np.uint16))
    X = synth_inputs.activations(1, K, seed=71)
    Yref, absdot = oracle.matmul(X, What)
    check_matmul(e0m4.e0m4_matmul(to_dev(X), codes, None, None, N, K, G), Yref, absdot)


def test_int4_error_codes(e0m4):
    L = e0m4.lib()
    assert L.e0m4_int4_gemv(0x1000, 0x1000, 64, 100, 128, 0x1000, None) == -2
    assert L.e0m4_int4_gemv(None, 0x1000, 64, 128, 128, 0x1000, None) == -1
    assert L.e0m4_int4_quantize(0x1000, 64, 128, 16, 0x1000, 0x1000, 0x1000, None) == -3
    assert L.e0m4_int4_dequant(0x1008, 64, 128, 128, 0x1000, None) == -4
    assert L.e0m4_int4_gemv(None, None, 0, 128, 128, None, None) == 0


# The three weight shapes of the paper's Table 1 (weight [K, N], activation [1, K]), at full size.
@pytest.mark.parametrize("K,N", [(4096, 4096), (4096, 11008), (11008, 4096)])
def test_table1_shapes_full_size(e0m4, oracle, K, N):
    G = 128
    codes, X, Y = run_int4_gemv_case(e0m4, oracle, N, K, G, seed=K + N)
    # and the E0M4 kernel on the same weights
    W = synth_inputs.weights(N, K, seed=K + N)
    ec, es, eb = e0m4.e0m4_quantize(to_dev(W), G)
    oc, os_, ob = oracle.quantize(W, G)
    Yref, absdot = oracle.matmul(X, oracle.dequant(oc, os_, ob, G))
    check_matmul(e0m4.e0m4_matmul(to_dev(X), ec, es, eb, N, K, G), Yref, absdot, "e0m4")
