"""Parity of the two further members of the format family with the CPU oracle, through the C ABI:
E0M4 on bfloat16 (codes, parameters and dequantised weights bit-exact; matmul within the matmul bar) and E0M3
(3-bit codes stored in 4-bit slots: quantiser bit-exact, then the E0M4 kernels on the same buffer)."""
import numpy as np
import pytest

import synth_inputs
from test_gpu_parity import DEV, bits, check_matmul, e0m4, to_dev, torch  # noqa: F401

pytestmark = pytest.mark.gpu


def bf_dev(bits_u16: np.ndarray):
    return torch.from_numpy(np.ascontiguousarray(bits_u16).view(np.int16)).to(DEV).view(torch.bfloat16)


def bf_bits(t) -> np.ndarray:
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def assert_bf16_quantize_exact(e0m4, oracle, W: np.ndarray, G: int):
    N, K = W.shape
    codes, scales, bias = e0m4.e0m4_bf16_quantize(bf_dev(W), G)
    oc, os_, ob = oracle.bf16_quantize(W, G)
    torch.cuda.synchronize()
    assert np.array_equal(bf_bits(scales), os_), "scales differ"
    assert np.array_equal(bf_bits(bias), ob), "bias differ"
    assert np.array_equal(bits(e0m4.e0m4_unpack_codes(codes, N, K, G)), oc), "codes differ"
    want = oracle.bf16_dequant(oc, os_, ob, G)
    assert np.array_equal(bf_bits(e0m4.e0m4_bf16_dequant(codes, N, K, G)), want), "dequantised weights differ"
    return codes, want, (oc, os_, ob)


def check_bf16_matmul(oracle, y_gpu, y_ref_bits, absdot, what):
    got = oracle.bf16_to_float64(bf_bits(y_gpu))
    ref = oracle.bf16_to_float64(y_ref_bits)
    err = np.abs(got - ref)
    tol = 1e-2 * np.maximum(1.0, absdot)
    assert (err <= tol).all(), "%s: %g" % (what, (err / tol).max())
    # quality bound well inside the bar: bfloat16 rounding of y (2^-9) and of the weights (2^-9), fp32 accumulation
    tight = 2.0 ** -8 * absdot + 2.0 ** -8 * np.abs(ref) + 1e-7
    assert (err <= tight).all(), "%s: quality bound: %g" % (what, (err / tight).max())


@pytest.mark.parametrize("N,K,G", [(N, K, G) for N, K in [(64, 128), (200, 384), (1, 128), (63, 256), (130, 1024), (256, 4096),
                                                         (70, 416)] for G in (32, 64, 128) if K % G == 0])
def test_bf16_quantize_dequant_bit_exact(e0m4, oracle, N, K, G):
    assert_bf16_quantize_exact(e0m4, oracle, synth_inputs.weights_bf16(N, K, seed=3000 + N + K + G), G)


def test_bf16_quantize_value_distributions(e0m4, oracle):
    rng = np.random.default_rng(19)
    N, K = 96, 512
    W = rng.standard_normal((N, K)).astype(np.float32) * np.float32(0.02)
    W[0:8] = 0.0
    W[8:16] = 0.5
    W[16:24] = np.abs(W[16:24])
    W[24:32] = -np.abs(W[24:32])
    W[32:40] = rng.standard_normal((8, K)).astype(np.float32) * np.float32(1e-30)     # tiny, still normal numbers
    W[40:48] = rng.standard_normal((8, K)).astype(np.float32) * np.float32(1e30)      # huge
    W[48, ::2], W[48, 1::2] = 3.0e38, -3.0e38                                           # range overflows fp32
    W[56:64] = (rng.integers(-7, 9, (8, K)) * 0.5).astype(np.float32)                   # values on rounding ties
    W[64:72] = rng.standard_normal((8, K)).astype(np.float32) * np.float32(1e-38)     # scale at its floor
    Wb = synth_inputs.to_bf16_bits(W)
    with np.errstate(over="ignore", invalid="ignore"):
        for G in (32, 128):
            assert_bf16_quantize_exact(e0m4, oracle, Wb, G)


def test_bf16_encode_with_given_parameters(e0m4, oracle):
    N, K, G = 80, 512, 64
    W = synth_inputs.weights_bf16(N, K, seed=3100)
    _, scales, bias = oracle.bf16_quantize(W, G)
    scales = np.roll(scales, 1, axis=0)                         # somebody else's parameters: clamping gets exercised
    codes = e0m4.e0m4_bf16_encode(bf_dev(W), bf_dev(scales), bf_dev(bias), G)
    assert np.array_equal(bits(e0m4.e0m4_unpack_codes(codes, N, K, G)), oracle.bf16_encode(W, scales, bias, G))


@pytest.mark.parametrize("G", [32, 64, 128])
@pytest.mark.parametrize("M", [1, 2, 3, 4, 5, 6, 7, 8])
def test_bf16_decode_matmul(e0m4, oracle, M, G):
    N, K = 203, 1664
    codes, What, _ = assert_bf16_quantize_exact(e0m4, oracle, synth_inputs.weights_bf16(N, K, seed=3200 + G), G)
    X = synth_inputs.activations_bf16(M, K, seed=3300 + M)
    Y = e0m4.e0m4_bf16_matmul(bf_dev(X), codes, N, K, G)
    Yref, absdot = oracle.bf16_matmul(X, What)
    check_bf16_matmul(oracle, Y, Yref, absdot, "bf16 decode M=%d G=%d" % (M, G))


@pytest.mark.parametrize("N,K,G", [(4096, 4096, 128), (1040, 2048, 64), (64, 128, 128), (1, 32, 32), (530, 13696, 128),
                                   (4608, 5120, 64)])
@pytest.mark.parametrize("waves", [0, 4, 16])
def test_bf16_decode_shapes_and_wavefront_counts(e0m4, oracle, N, K, G, waves):
    codes, What, _ = assert_bf16_quantize_exact(e0m4, oracle, synth_inputs.weights_bf16(N, K, seed=3400 + N), G)
    X = synth_inputs.activations_bf16(1, K, seed=3500 + K)
    e0m4.e0m4_set_knob("gemv_waves", waves)
    try:
        Y = e0m4.e0m4_bf16_matmul(bf_dev(X), codes, N, K, G)
        Y2 = e0m4.e0m4_bf16_matmul(bf_dev(X), codes, N, K, G)
    finally:
        e0m4.e0m4_set_knob("gemv_waves", 0)
    Yref, absdot = oracle.bf16_matmul(X, What)
    check_bf16_matmul(oracle, Y, Yref, absdot, "bf16 decode N=%d K=%d" % (N, K))
    assert torch.equal(Y.view(torch.int16), Y2.view(torch.int16))           # deterministic


@pytest.mark.parametrize("M,N,K,G", [(9, 203, 1664, 128), (64, 256, 512, 32), (200, 520, 1024, 64), (300, 1040, 2080, 32),
                                     (1024, 1280, 4096, 128), (130, 64, 128, 128), (17, 4608, 416, 32)])
def test_bf16_gemm(e0m4, oracle, M, N, K, G):
    codes, What, _ = assert_bf16_quantize_exact(e0m4, oracle, synth_inputs.weights_bf16(N, K, seed=3600 + N + K), G)
    X = synth_inputs.activations_bf16(M, K, seed=3700 + M)
    Y = e0m4.e0m4_bf16_matmul(bf_dev(X), codes, N, K, G)
    Yref, absdot = oracle.bf16_matmul(X, What)
    check_bf16_matmul(oracle, Y, Yref, absdot, "bf16 gemm M=%d N=%d K=%d" % (M, N, K))


@pytest.mark.parametrize("variant", [1, 2, 3, 4, 5])
@pytest.mark.parametrize("M,N,K,G", [(300, 600, 1024, 128), (513, 272, 384, 32), (70, 1040, 2048, 64), (256, 256, 128, 64)])
def test_bf16_gemm_every_kernel_and_tile(e0m4, oracle, variant, M, N, K, G):
    # gemm_variant 1: the 128 x 128-tile kernel with both operands through LDS; 2, 3, 4: the pipelined kernel (weights
    # dequantised in registers, in whole tiles) with its 256 x 256, 128 x 128 and 64 x 256 tile; 5: its 128 x 256 tile
    codes, What, _ = assert_bf16_quantize_exact(e0m4, oracle, synth_inputs.weights_bf16(N, K, seed=3650 + N + K), G)
    X = synth_inputs.activations_bf16(M, K, seed=3750 + M)
    e0m4.e0m4_set_knob("gemm_variant", variant)
    try:
        Y = e0m4.e0m4_bf16_matmul(bf_dev(X), codes, N, K, G)
        Y2 = e0m4.e0m4_bf16_matmul(bf_dev(X), codes, N, K, G)
    finally:
        e0m4.e0m4_set_knob("gemm_variant", 0)
    Yref, absdot = oracle.bf16_matmul(X, What)
    check_bf16_matmul(oracle, Y, Yref, absdot, "bf16 gemm variant %d M=%d N=%d K=%d" % (variant, M, N, K))
    assert torch.equal(Y.view(torch.int16), Y2.view(torch.int16))


def test_bf16_gemm_default_choice_with_many_tiles(e0m4, oracle):
    # 5 x 26 tiles of 64 x 256: enough to fill the chip in whole tiles, so the pipelined kernel is the default;
    # all of N on sampled rows, and one-hot rows that must reproduce the weights through the MFMA path
    M, N, K, G = 300, 6656, 512, 128
    codes, What, _ = assert_bf16_quantize_exact(e0m4, oracle, synth_inputs.weights_bf16(N, K, seed=3660), G)
    X = synth_inputs.activations_bf16(M, K, seed=3760)
    hot = {5: 17, 64: 300, 299: 511}
    for m, k in hot.items():
        X[m] = 0
        X[m, k] = 0x3F80
    Y = e0m4.e0m4_bf16_matmul(bf_dev(X), codes, N, K, G)
    rows = np.array([0, 5, 63, 64, 65, 127, 128, 200, 255, 256, 299])
    Yref, absdot = oracle.bf16_matmul(X[rows], What)
    check_bf16_matmul(oracle, Y[torch.from_numpy(rows).to(DEV)], Yref, absdot, "bf16 gemm, pipelined by default")
    Yb = bf_bits(Y)
    for m, k in hot.items():
        nz = (What[:, k] & 0x7FFF) != 0
        assert np.array_equal(Yb[m][nz], What[:, k][nz])
        assert not (Yb[m][~nz] & 0x7FFF).any()


@pytest.mark.parametrize("M", [1, 4, 40])
def test_bf16_one_hot_activations_reproduce_the_weights(e0m4, oracle, M):
    N, K, G = 96, 256, 64
    codes, What, _ = assert_bf16_quantize_exact(e0m4, oracle, synth_inputs.weights_bf16(N, K, seed=3800), G)
    ks = [(37 * m + 5) % K for m in range(M)]
    X = np.zeros((M, K), dtype=np.uint16)
    for m, k in enumerate(ks):
        X[m, k] = 0x3F80
    Y = bf_bits(e0m4.e0m4_bf16_matmul(bf_dev(X), codes, N, K, G))
    for m, k in enumerate(ks):
        assert np.array_equal(Y[m] & 0x7FFF, What[:, k] & 0x7FFF)          # bit-exact up to the sign of zero
        nz = (What[:, k] & 0x7FFF) != 0
        assert np.array_equal(Y[m][nz], What[:, k][nz])


def test_bf16_empty_problems(e0m4):
    x = torch.zeros((2, 0), dtype=torch.bfloat16, device=DEV)
    y = torch.full((2, 64), 3.0, dtype=torch.bfloat16, device=DEV)
    e0m4.e0m4_bf16_matmul(x, torch.empty(16, dtype=torch.uint8, device=DEV), 64, 0, 128, out=y)
    assert not y.view(torch.int16).any()


# ------------------------------------------------------------------ E0M3

@pytest.mark.parametrize("N,K,G", [(N, K, G) for N, K in [(64, 128), (200, 384), (1, 128), (130, 1024), (256, 4096)]
                                   for G in (32, 64, 128) if K % G == 0])
def test_e0m3_quantize_bit_exact_and_the_e0m4_kernels_read_it(e0m4, oracle, N, K, G):
    W = synth_inputs.weights(N, K, seed=3900 + N + K + G)
    codes, scales, bias = e0m4.e0m3_quantize(to_dev(W), G)
    oc, os_, ob = oracle.quantize_k(W, G, 3)
    assert oc.max() <= 7
    assert np.array_equal(bits(scales), os_.view(np.uint16)) and np.array_equal(bits(bias), ob.view(np.uint16))
    assert np.array_equal(bits(e0m4.e0m3_unpack_codes(codes, N, K, G)), oc)
    assert np.array_equal(bits(e0m4.e0m4_unpack_codes(codes, N, K, G)), 2 * oc)      # stored as the E0M4 code of the same value
    What = oracle.dequant_k(oc, os_, ob, G, 3)
    assert np.array_equal(bits(e0m4.e0m4_dequant(codes, None, None, N, K, G)), What.view(np.uint16))
    for M in (1, 5, 16, 200):
        X = synth_inputs.activations(M, K, seed=3950 + M)
        Y = e0m4.e0m4_matmul(to_dev(X), codes, None, None, N, K, G)
        Yref, absdot = oracle.matmul(X, What)
        check_matmul(Y, Yref, absdot, "e0m3 M=%d" % M)


def test_e0m3_value_distributions(e0m4, oracle):
    rng = np.random.default_rng(23)
    N, K = 64, 512
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float16)
    W[0:8] = 0.0
    W[8:16] = np.float16(0.5)
    W[16:24] = np.abs(W[16:24])
    W[24:32] = -np.abs(W[24:32])
    W[32:40] = (rng.standard_normal((8, K)) * 3e-6).astype(np.float16)
    W[40:48] = np.clip(rng.standard_normal((8, K)) * 2e4, -6e4, 6e4).astype(np.float16)
    W[48:56] = (rng.integers(-7, 9, (8, K)) * 0.5).astype(np.float16)
    for G in (32, 128):
        codes, scales, bias = e0m4.e0m3_quantize(to_dev(W), G)
        with np.errstate(over="ignore"):
            oc, os_, ob = oracle.quantize_k(W, G, 3)
        assert np.array_equal(bits(scales), os_.view(np.uint16)) and np.array_equal(bits(bias), ob.view(np.uint16))
        assert np.array_equal(bits(e0m4.e0m3_unpack_codes(codes, N, K, G)), oc)
