"""Parity of the 8-bit format E0M8 (paper: closing remark of the section "E0M4 FP4 quantization") with the
CPU oracle, through the C ABI: codes, scales, bias and dequantised weights bit for bit; matmul outputs within
    |y_gpu - y_ref| <= 1e-2 * max(1, sum_k |x_k * w_k|)
and within the tighter quality bound of the other matmul tests."""
import numpy as np
import pytest

import synth_inputs

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

DEV = "cuda:0"
KNOBS = ("gemv_waves", "gemv_workgroups", "gemv_mfma", "gemv_xreg", "gemm_variant", "gemm_splits", "gemm_sk", "gemm_panel", "gemm_split_order")


@pytest.fixture(scope="module")
def e0m4():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (run with -m 'not gpu' elsewhere)")
    import paper_2403_20041_amd as pkg

    pkg.lib()                                   # raises if the HIP library is not built
    for k in KNOBS:
        pkg.e0m4_set_knob(k, 0)
    return pkg


def to_dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def bits(t):
    a = t.detach().cpu().numpy()
    return a.view(np.uint16) if a.dtype == np.float16 else a


def assert_quantize_exact(e0m4, oracle, W, G):
    N, K = W.shape
    codes, scales, bias = e0m4.e0m8_quantize(to_dev(W), G)
    oc, os_, ob = oracle.quantize_k(W, G, 8)
    torch.cuda.synchronize()
    assert np.array_equal(bits(scales), os_.view(np.uint16)), "scales differ"
    assert np.array_equal(bits(bias), ob.view(np.uint16)), "bias differ"
    assert np.array_equal(bits(e0m4.e0m8_unpack_codes(codes, N, K, G)), oc), "codes differ"
    want = oracle.dequant_k(oc, os_, ob, G, 8)
    assert np.array_equal(bits(e0m4.e0m8_dequant(codes, N, K, G)), want.view(np.uint16)), "dequantised weights differ"
    return codes, want


@pytest.mark.parametrize("G", [64, 128])
@pytest.mark.parametrize("N,K", [(64, 128), (200, 384), (1, 128), (63, 256), (65, 1152), (130, 1024), (256, 4096)])
def test_quantize_dequant_bit_exact(e0m4, oracle, N, K, G):
    assert_quantize_exact(e0m4, oracle, synth_inputs.weights(N, K, seed=2000 + N + K + G), G)


def test_quantize_ragged_block_pair(e0m4, oracle):
    # K = 17 and 3 blocks of 64: the last pair of blocks holds one block only
    assert_quantize_exact(e0m4, oracle, synth_inputs.weights(70, 1088, seed=5), 64)
    assert_quantize_exact(e0m4, oracle, synth_inputs.weights(33, 192, seed=6), 64)


@pytest.mark.parametrize("G", [64, 128])
def test_quantize_value_distributions(e0m4, oracle, G):
    rng = np.random.default_rng(17 + G)
    N, K = 96, 512
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float16)
    W[0:8] = 0.0
    W[8:16] = np.float16(0.5)
    W[16:24] = np.abs(W[16:24])
    W[24:32] = -np.abs(W[24:32])
    W[32:40] = (rng.standard_normal((8, K)) * 3e-6).astype(np.float16)          # floor on the scale
    W[40:48] = np.clip(rng.standard_normal((8, K)) * 2e4, -6e4, 6e4).astype(np.float16)
    W[48, ::2] = np.float16(65504.0)
    W[48, 1::2] = np.float16(-65504.0)                                            # scale saturates
    W[56:64, ::7] = 0.0
    W[64:72, ::5] = np.float16(-0.0)
    W[72:80] = rng.integers(-3, 4, (8, K)).astype(np.float16) * np.float16(2.0 ** -14)
    assert_quantize_exact(e0m4, oracle, W, G)


def check_matmul(y_gpu, y_ref, absdot, what):
    got = y_gpu.detach().cpu().numpy().astype(np.float64)
    ref = y_ref.astype(np.float64)
    err = np.abs(got - ref)
    tol = 1e-2 * np.maximum(1.0, absdot)
    worst = np.unravel_index(np.argmax(err / tol), err.shape)
    assert (err <= tol).all(), "%s: worst at %s err %g tol %g" % (what, worst, err[worst], tol[worst])
    tight = 2.0 ** -9 * absdot + 2.0 ** -10 * np.abs(ref) + 1e-7
    assert (err <= tight).all(), "%s: quality bound: %g" % (what, (err / tight).max())


def run_matmul_case(e0m4, oracle, M, N, K, G, seed, outliers=False):
    W = synth_inputs.weights(N, K, seed=seed)
    X = synth_inputs.activations(M, K, seed=seed, outlier_frac=0.01 if outliers else 0.0)
    codes, What = assert_quantize_exact(e0m4, oracle, W, G)
    Y = e0m4.e0m8_matmul(to_dev(X), codes, N, K, G)
    Yref, absdot = oracle.matmul(X, What)
    torch.cuda.synchronize()
    check_matmul(Y, Yref, absdot, "M=%d N=%d K=%d G=%d" % (M, N, K, G))


@pytest.mark.parametrize("G", [64, 128])
@pytest.mark.parametrize("M", [1, 2, 3, 4, 5, 6, 7, 8])
def test_decode_small(e0m4, oracle, M, G):
    run_matmul_case(e0m4, oracle, M, 200, 1152, G, seed=700 + M)


@pytest.mark.parametrize("N,K,G", [(64, 128, 128), (1, 64, 64), (4096, 4096, 128), (1000, 6848, 64), (203, 832, 64),
                                    (77, 1088, 64), (8192, 1024, 128)])
def test_decode_shapes_m1(e0m4, oracle, N, K, G):
    run_matmul_case(e0m4, oracle, 1, N, K, G, seed=N + K, outliers=True)


@pytest.mark.parametrize("waves", [4, 8, 16])
@pytest.mark.parametrize("target", [0, 7, 100000])
def test_decode_forced_shapes(e0m4, oracle, waves, target):
    e0m4.e0m4_set_knob("gemv_waves", waves)
    e0m4.e0m4_set_knob("gemv_workgroups", target)
    try:
        run_matmul_case(e0m4, oracle, 1, 300, 576, 64, seed=710 + waves)        # 9 blocks
        run_matmul_case(e0m4, oracle, 3, 1000, 2048, 128, seed=711 + waves)
    finally:
        e0m4.e0m4_set_knob("gemv_waves", 0)
        e0m4.e0m4_set_knob("gemv_workgroups", 0)


@pytest.mark.parametrize("M", [2, 3, 5, 8, 9, 13, 16])
def test_small_batch_matrix_core_kernel(e0m4, oracle, M):
    run_matmul_case(e0m4, oracle, M, 200, 1152, 64, seed=770 + M)                   # 18 blocks: ragged last work item
    run_matmul_case(e0m4, oracle, M, 333, 4096, 128, seed=771 + M, outliers=True)   # 16 work items per row block
    run_matmul_case(e0m4, oracle, M, 40, 64, 64, seed=772 + M)                      # a single block
    run_matmul_case(e0m4, oracle, M, 1000, 2048, 128, seed=773 + M)                 # 8 work items: activations in registers


@pytest.mark.parametrize("waves", [4, 8, 16])
@pytest.mark.parametrize("mode", [0, 2])                # 2: activations always from LDS
def test_small_batch_matrix_core_kernel_forced_shapes(e0m4, oracle, waves, mode):
    e0m4.e0m4_set_knob("gemv_waves", waves)
    e0m4.e0m4_set_knob("gemv_workgroups", 3)
    e0m4.e0m4_set_knob("gemv_mfma", mode)
    try:
        run_matmul_case(e0m4, oracle, 6, 300, 1024, 128, seed=780 + waves)
        run_matmul_case(e0m4, oracle, 16, 130, 2048, 64, seed=781 + waves)
    finally:
        e0m4.e0m4_set_knob("gemv_waves", 0)
        e0m4.e0m4_set_knob("gemv_workgroups", 0)
        e0m4.e0m4_set_knob("gemv_mfma", 0)


@pytest.mark.parametrize("M", [2, 8, 12])
def test_small_batch_other_kernels_when_the_matrix_core_kernel_is_off(e0m4, oracle, M):
    e0m4.e0m4_set_knob("gemv_mfma", 1)
    try:
        run_matmul_case(e0m4, oracle, M, 200, 1152, 64, seed=790 + M)
        run_matmul_case(e0m4, oracle, M, 336, 4096, 128, seed=791 + M)
    finally:
        e0m4.e0m4_set_knob("gemv_mfma", 0)


@pytest.mark.parametrize("variant", [2, 3, 4, 5])     # pipelined kernel with tiles of 2: 256 x 256, 3: 128 x 128, 4: 64 x 256, 5: 128 x 256
@pytest.mark.parametrize("splits", [0, 2, 3])
def test_gemm_kernels(e0m4, oracle, variant, splits):
    e0m4.e0m4_set_knob("gemm_variant", variant)
    e0m4.e0m4_set_knob("gemm_splits", splits)
    try:
        run_matmul_case(e0m4, oracle, 300, 600, 1024, 128, seed=740 + variant, outliers=True)    # ragged in M and N
        run_matmul_case(e0m4, oracle, 9, 200, 384, 64, seed=741 + variant)
        run_matmul_case(e0m4, oracle, 257, 1040, 512, 64, seed=742 + variant)
    finally:
        e0m4.e0m4_set_knob("gemm_variant", 0)
        e0m4.e0m4_set_knob("gemm_splits", 0)


@pytest.mark.parametrize("M", [16, 64, 200, 1024])
def test_gemm_default_choice(e0m4, oracle, M):
    run_matmul_case(e0m4, oracle, M, 1152, 2048, 128, seed=750 + M, outliers=True)


def test_decode_long_rows_and_row_chunks(e0m4, oracle):
    run_matmul_case(e0m4, oracle, 8, 40, 16384, 128, seed=720)      # activations staged in several segments
    run_matmul_case(e0m4, oracle, 37, 136, 1088, 64, seed=721)      # K = 8.5 x 128: launches of 8 + 8 + 8 + 8 + 5 rows
    run_matmul_case(e0m4, oracle, 16, 64, 256, 128, seed=722)


@pytest.mark.parametrize("M", [17, 21, 32])
def test_small_batch_chunks_of_rows(e0m4, oracle, M):
    # 17 <= M <= 32 on small weights: the small-batch kernel on two equal chunks of rows in one launch; no workspace
    for N, K, G, seed in ((333, 1152, 128, 770), (1000, 2048, 64, 771), (68, 192, 64, 772)):
        assert e0m4.e0m8_workspace_bytes(M, N, K, G) == 0
        run_matmul_case(e0m4, oracle, M, N, K, G, seed=seed + M, outliers=True)
    run_matmul_case(e0m4, oracle, 33, 336, 1152, 128, seed=773)         # beyond 32 rows: the GEMM


@pytest.mark.parametrize("M", [1, 20])
def test_longest_rows(e0m4, oracle, M):
    run_matmul_case(e0m4, oracle, M, 24, 1 << 19, 128, seed=760 + M)   # K at its limit


def test_one_hot_activations_reproduce_weights_bit_exactly(e0m4, oracle):
    N, K, G = 100, 256, 64
    W = synth_inputs.weights(N, K, seed=730)
    codes, What = assert_quantize_exact(e0m4, oracle, W, G)
    for k in (0, 15, 16, 63, 64, 127, 200, 255):
        X = np.zeros((1, K), np.float16)
        X[0, k] = 1.0
        Y = e0m4.e0m8_matmul(to_dev(X), codes, N, K, G).cpu().numpy()
        assert np.array_equal(Y[0].view(np.uint16), What[:, k].view(np.uint16)), k


def test_argument_errors(e0m4):
    x = torch.zeros((1, 128), dtype=torch.float16, device=DEV)
    w = torch.zeros((64, 128), dtype=torch.float16, device=DEV)
    with pytest.raises(ValueError):
        e0m4.e0m8_quantize(w, 32)                       # group 32 is not offered for the 8-bit format
    codes, _, _ = e0m4.e0m8_quantize(w, 64)
    with pytest.raises(e0m4.E0M4Error):
        e0m4.e0m8_matmul(x, codes, 64, 128, 48)
    assert e0m4.e0m8_codes_bytes(64, 128, 64) == 4 * 2 * (1024 + 64)
    assert e0m4.e0m8_codes_bytes(64, 100, 64) == 0


def test_full_size_layer_shapes(e0m4, oracle):
    """The benchmark's configuration: ChatGLM2-6B shapes, decode output in full, prefill on sampled rows."""
    for name, N, K in (("gate_up", 27392, 4096), ("down", 4096, 13696)):
        W = synth_inputs.weights(N, K, seed=760 + N % 13, row_std_range=(0.5, 2.0))
        codes, What = assert_quantize_exact(e0m4, oracle, W, 128)
        del W
        X1 = synth_inputs.activations(1, K, seed=761)
        Yref, absdot = oracle.matmul(X1, What)
        check_matmul(e0m4.e0m8_matmul(to_dev(X1), codes, N, K, 128), Yref, absdot, name + " decode")
        X = synth_inputs.activations(1024, K, seed=762, outlier_frac=0.01)
        Y = e0m4.e0m8_matmul(to_dev(X), codes, N, K, 128).cpu().numpy()
        rows = np.array([0, 1, 127, 128, 255, 256, 511, 640, 1023])
        Yr, ad = oracle.matmul(X[rows], What)
        check_matmul(torch.from_numpy(Y[rows]), Yr, ad, name + " prefill rows")
        cols = np.array([0, 15, 16, 255, 256, N // 2, N - 257, N - 1])
        Yc, adc = oracle.matmul(X, What[cols])
        check_matmul(torch.from_numpy(np.ascontiguousarray(Y[:, cols])), Yc, adc, name + " prefill cols")
