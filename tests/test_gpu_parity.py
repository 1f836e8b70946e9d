"""Parity of the HIP path with the CPU oracle, element by element, through the
C ABI (ctypes binding).  Codes, scales, bias and dequantised weights must be
bit-exact; matmul outputs must satisfy
    |y_gpu - y_ref| <= 1e-2 * max(1, sum_k |x_k * w_k|)
per element (fp32 accumulation on the GPU, fp64 in the oracle)."""
import numpy as np
import pytest

import synth_inputs

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def e0m4():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (run with -m 'not gpu' elsewhere)")
    import paper_2403_20041_amd as pkg

    pkg.lib()                                   # raises if the HIP library is not built
    for k in ("gemv_waves", "gemv_workgroups", "gemv_mfma", "gemv_xreg", "gemm_variant", "gemm_splits", "gemm_sk", "gemm_panel", "gemm_split_order"):
        pkg.e0m4_set_knob(k, 0)
    return pkg


DEV = "cuda:0"


def to_dev(a: np.ndarray):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def bits(t) -> np.ndarray:
    a = t.detach().cpu().numpy()
    return a.view(np.uint16) if a.dtype == np.float16 else a


def gpu_quantize(e0m4, W: np.ndarray, G: int):
    N, K = W.shape
    codes, scales, bias = e0m4.e0m4_quantize(to_dev(W), G)
    return codes, scales, bias


def assert_quantize_exact(e0m4, oracle, W: np.ndarray, G: int):
    N, K = W.shape
    codes, scales, bias = gpu_quantize(e0m4, W, G)
    oc, os_, ob = oracle.quantize(W, G)
    torch.cuda.synchronize()
    assert np.array_equal(bits(scales), os_.view(np.uint16)), "scales differ"
    assert np.array_equal(bits(bias), ob.view(np.uint16)), "bias differ"
    got_codes = bits(e0m4.e0m4_unpack_codes(codes, N, K, G))
    assert np.array_equal(got_codes, oc), "codes differ"
    got_w = bits(e0m4.e0m4_dequant(codes, scales, bias, N, K, G))
    want_w = oracle.dequant(oc, os_, ob, G)
    assert np.array_equal(got_w, want_w.view(np.uint16)), "dequantised weights differ"
    return (codes, scales, bias), want_w


def check_matmul(y_gpu, y_ref: np.ndarray, absdot: np.ndarray, what=""):
    got = y_gpu.detach().cpu().numpy().astype(np.float64)
    ref = y_ref.astype(np.float64)
    err = np.abs(got - ref)
    tol = 1e-2 * np.maximum(1.0, absdot)
    worst = np.unravel_index(np.argmax(err / tol), err.shape)
    assert (err <= tol).all(), "%s: worst at %s err %g tol %g" % (what, worst, err[worst], tol[worst])
    # quality bound well inside the acceptance bar: fp16 rounding of y and of the weights, fp32 accumulation
    tight = 2.0 ** -9 * absdot + 2.0 ** -10 * np.abs(ref) + 1e-7
    assert (err <= tight).all(), "%s: quality bound: %g" % (what, (err / tight).max())


# ------------------------------------------------------------------ quantise / dequant / unpack

SMALL_SHAPES = [
    (64, 128), (200, 384), (1, 128), (63, 256), (65, 256), (130, 1024), (256, 4096),
]


@pytest.mark.parametrize("G", [32, 64, 128])
@pytest.mark.parametrize("N,K", SMALL_SHAPES)
def test_quantize_dequant_bit_exact(e0m4, oracle, N, K, G):
    W = synth_inputs.weights(N, K, seed=1000 + N + K + G)
    assert_quantize_exact(e0m4, oracle, W, G)


def test_quantize_ragged_k_tile(e0m4, oracle):
    # K = 416 = 13 chunks: the last 128-wide tile holds one chunk only
    assert_quantize_exact(e0m4, oracle, synth_inputs.weights(70, 416, seed=3), 32)
    assert_quantize_exact(e0m4, oracle, synth_inputs.weights(70, 448, seed=4), 64)


@pytest.mark.parametrize("G", [32, 64, 128])
def test_quantize_value_distributions(e0m4, oracle, G):
    rng = np.random.default_rng(7 + G)
    N, K = 192, 512
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float16)
    W[0:8] = 0.0                                              # all-zero groups
    W[8:16] = np.float16(0.5)                                 # constant groups
    W[16:24] = np.abs(W[16:24])                               # one-signed groups
    W[24:32] = -np.abs(W[24:32])
    W[32:40] = (rng.standard_normal((8, K)) * 3e-6).astype(np.float16)      # subnormal weights, floor on the scale
    W[40:48] = np.clip(rng.standard_normal((8, K)) * 2e4, -6e4, 6e4).astype(np.float16)   # large weights
    W[48, ::2] = np.float16(65504.0)
    W[48, 1::2] = np.float16(-65504.0)                        # scale saturates
    W[49:56] = (rng.standard_normal((7, K)) * 1e-4).astype(np.float16)
    W[56:64, ::7] = 0.0
    W[64:72, ::5] = np.float16(-0.0)
    W[72:80] *= np.float16(50.0)
    W[80:88] = rng.integers(-3, 4, (8, K)).astype(np.float16) * np.float16(2.0 ** -14)
    with np.errstate(over="ignore"):
        assert_quantize_exact(e0m4, oracle, W, G)


def test_quantize_exhaustive_fp16_values(e0m4, oracle):
    # every finite fp16 value appears; groups of mixed magnitudes
    vals = np.arange(65536, dtype=np.uint32).astype(np.uint16).view(np.float16)
    vals = vals[np.isfinite(vals)]
    rng = np.random.default_rng(11)
    W = rng.permutation(np.resize(vals, 64 * 1024)).reshape(64, 1024)
    with np.errstate(over="ignore"):
        assert_quantize_exact(e0m4, oracle, W, 32)
    Ws = np.sort(np.resize(vals, 64 * 1024)).reshape(64, 1024)    # neighbours in value share a group
    with np.errstate(over="ignore"):
        assert_quantize_exact(e0m4, oracle, Ws, 128)


@pytest.mark.parametrize("G", [32, 128])
def test_encode_with_given_parameters(e0m4, oracle, G):
    rng = np.random.default_rng(21 + G)
    N, K = 130, 512
    W = synth_inputs.weights(N, K, seed=22)
    sc = (np.abs(rng.standard_normal((N, K // G))) * 0.02 + 1e-3).astype(np.float16)
    z = rng.integers(0, 16, (N, K // G)).astype(np.uint16)
    bi = (0x4000 | (z << 6)).astype(np.uint16).view(np.float16)
    want = oracle.encode(W, sc, bi, G)
    codes = e0m4.e0m4_encode(to_dev(W), to_dev(sc), to_dev(bi), G)
    got = bits(e0m4.e0m4_unpack_codes(codes, N, K, G))
    assert np.array_equal(got, want)
    got_w = bits(e0m4.e0m4_dequant(codes, to_dev(sc), to_dev(bi), N, K, G))
    assert np.array_equal(got_w, oracle.dequant(want, sc, bi, G).view(np.uint16))


def test_dequant_all_codes_all_biases_many_scales(e0m4, oracle):
    """Drive e0m4_dequant over every (code, bias) pair for a sweep of scales, including
    scales whose products are subnormal or overflow."""
    G, K = 32, 32
    sb = np.concatenate([np.arange(0x0400, 0x7C00, 13, dtype=np.uint16), np.array([0x0400, 0x7BFF], np.uint16)])
    N = sb.size * 16
    scales = np.repeat(sb, 16)[:, None]
    zz = np.tile(np.arange(16, dtype=np.uint16), sb.size)
    bias = (0x4000 | (zz << 6)).astype(np.uint16)[:, None]
    codes_np = np.tile(np.concatenate([np.arange(16), np.arange(15, -1, -1)]).astype(np.uint8), (N, 1))
    # build W whose codes under these parameters are exactly codes_np (fixed-parameter round trip)
    with np.errstate(over="ignore"):
        W = oracle.dequant(codes_np, scales, bias, G)
    ok_rows = np.isfinite(W).all(axis=1)
    W, scales, bias, codes_np = W[ok_rows], scales[ok_rows], bias[ok_rows], codes_np[ok_rows]
    N = W.shape[0]
    sd, bd = to_dev(scales.view(np.float16)), to_dev(bias.view(np.float16))
    codes = e0m4.e0m4_encode(to_dev(W), sd, bd, G)
    assert np.array_equal(bits(e0m4.e0m4_unpack_codes(codes, N, K, G)), codes_np)
    assert np.array_equal(bits(e0m4.e0m4_dequant(codes, sd, bd, N, K, G)), W.view(np.uint16))


# ------------------------------------------------------------------ matmul, small-M path

def run_matmul_case(e0m4, oracle, M, N, K, G, seed, outliers=False, row_std=None):
    W = synth_inputs.weights(N, K, seed=seed, row_std_range=row_std)
    X = synth_inputs.activations(M, K, seed=seed, outlier_frac=0.01 if outliers else 0.0)
    (codes, scales, bias), What = assert_quantize_exact(e0m4, oracle, W, G)
    Y = e0m4.e0m4_matmul(to_dev(X), codes, scales, bias, N, K, G)
    Yref, absdot = oracle.matmul(X, What)
    torch.cuda.synchronize()
    check_matmul(Y, Yref, absdot, "M=%d N=%d K=%d G=%d" % (M, N, K, G))
    return Y


@pytest.mark.parametrize("G", [32, 64, 128])
@pytest.mark.parametrize("M", [1, 2, 3, 4, 5, 6, 7, 8])
def test_gemv_small(e0m4, oracle, M, G):
    run_matmul_case(e0m4, oracle, M, 200, 1152, G, seed=30 + M)
    if M >= 2:                                          # and on the vector kernel where a matrix-core kernel is the default
        e0m4.e0m4_set_knob("gemv_mfma", 1)
        try:
            run_matmul_case(e0m4, oracle, M, 200, 1152, G, seed=30 + M)
        finally:
            e0m4.e0m4_set_knob("gemv_mfma", 0)


@pytest.mark.parametrize("N,K,G", [(64, 128, 128), (1, 32, 32), (4096, 4096, 128), (1000, 13696, 128),
                                    (5120, 5120, 64), (8192, 2048, 32), (130, 13696, 64)])
def test_gemv_shapes_m1(e0m4, oracle, N, K, G):
    run_matmul_case(e0m4, oracle, 1, N, K, G, seed=N + K)


@pytest.mark.parametrize("waves", [4, 8, 16])
def test_gemv_forced_waves_per_workgroup(e0m4, oracle, waves):
    e0m4.e0m4_set_knob("gemv_waves", waves)
    try:
        run_matmul_case(e0m4, oracle, 1, 300, 1152, 128, seed=50)      # 9 k blocks
        run_matmul_case(e0m4, oracle, 3, 300, 1152, 64, seed=51)
        run_matmul_case(e0m4, oracle, 8, 40, 16384, 128, seed=52)      # activations staged in several segments
    finally:
        e0m4.e0m4_set_knob("gemv_waves", 0)


@pytest.mark.parametrize("N,K,G", [(4096, 4096, 128), (8192, 2048, 64), (333, 1024, 32), (48, 512, 128),
                                    (700, 3968, 128)])
def test_gemv_forced_workgroup_counts(e0m4, oracle, N, K, G):
    # few workgroups: many row blocks each, dealt unevenly; many: one row block each
    for target in (0, 7, 100000):
        e0m4.e0m4_set_knob("gemv_workgroups", target)
        try:
            run_matmul_case(e0m4, oracle, 1, N, K, G, seed=N + K + 1)
        finally:
            e0m4.e0m4_set_knob("gemv_workgroups", 0)


@pytest.mark.parametrize("xreg", [0, 2])              # 0: activations in registers wherever possible, 2: never
@pytest.mark.parametrize("waves", [0, 4, 8, 16])
def test_gemv_activations_in_registers(e0m4, oracle, waves, xreg):
    e0m4.e0m4_set_knob("gemv_waves", waves)
    e0m4.e0m4_set_knob("gemv_xreg", xreg)
    try:
        run_matmul_case(e0m4, oracle, 1, 333, 4096, 128, seed=60 + waves, outliers=True)     # 8 work items per row block
        run_matmul_case(e0m4, oracle, 1, 200, 2048, 64, seed=61 + waves)                     # 4
        run_matmul_case(e0m4, oracle, 1, 100, 8192, 32, seed=62 + waves)                     # 16
        run_matmul_case(e0m4, oracle, 1, 40, 512, 128, seed=63 + waves)                      # 1
    finally:
        e0m4.e0m4_set_knob("gemv_waves", 0)
        e0m4.e0m4_set_knob("gemv_xreg", 0)


@pytest.mark.parametrize("K,G", [(5120, 128), (6144, 64), (7168, 32), (5120, 64)])
def test_gemv_one_wavefront_per_work_item(e0m4, oracle, K, G):
    # 10, 12 or 14 work items per row block: as many wavefronts, activations in registers; and the same shapes without
    run_matmul_case(e0m4, oracle, 1, 333, K, G, seed=70 + K // 1024, outliers=True)
    run_matmul_case(e0m4, oracle, 1, 12300, K, G, seed=71 + K // 1024)         # four row blocks per workgroup (10 and 14
                                                                               # wavefronts are used from three on)
    e0m4.e0m4_set_knob("gemv_xreg", 2)
    try:
        run_matmul_case(e0m4, oracle, 1, 333, K, G, seed=72 + K // 1024)
    finally:
        e0m4.e0m4_set_knob("gemv_xreg", 0)


@pytest.mark.parametrize("M", [1, 2, 5, 8])
def test_gemv_ragged_last_work_item(e0m4, oracle, M):
    # K = 13 and 14 blocks of 128: the last group of four k blocks holds one or two; N ends inside a row block
    run_matmul_case(e0m4, oracle, M, 203, 1664, 128, seed=80 + M)
    run_matmul_case(e0m4, oracle, M, 77, 1760, 32, seed=90 + M)     # K = 13.75 blocks: ragged inside the last block


# ------------------------------------------------------------------ matmul, small batch on the matrix cores

@pytest.mark.parametrize("M", [2, 3, 4, 5, 7, 8, 9, 12, 15, 16])
def test_small_batch_matrix_core_kernel(e0m4, oracle, M):
    # group 128 and 2 <= M <= 16: the MFMA small-batch kernel
    run_matmul_case(e0m4, oracle, M, 200, 1152, 128, seed=130 + M)              # 9 k blocks: ragged last work item
    run_matmul_case(e0m4, oracle, M, 333, 4096, 128, seed=140 + M, outliers=True)
    run_matmul_case(e0m4, oracle, M, 40, 128, 128, seed=150 + M)                # a single block
    run_matmul_case(e0m4, oracle, M, 1000, 1664, 128, seed=160 + M, row_std=(0.5, 2.0))   # 13 k blocks, N ends inside a row block


@pytest.mark.parametrize("waves", [4, 8, 16])
@pytest.mark.parametrize("target", [0, 3])
def test_small_batch_matrix_core_kernel_forced_shapes(e0m4, oracle, waves, target):
    e0m4.e0m4_set_knob("gemv_waves", waves)
    e0m4.e0m4_set_knob("gemv_workgroups", target)       # 3 workgroups: many row blocks each
    try:
        run_matmul_case(e0m4, oracle, 6, 300, 2304, 128, seed=170 + waves)
        run_matmul_case(e0m4, oracle, 16, 130, 4096, 128, seed=171 + waves)
    finally:
        e0m4.e0m4_set_knob("gemv_waves", 0)
        e0m4.e0m4_set_knob("gemv_workgroups", 0)


@pytest.mark.parametrize("M", [2, 5, 16])
def test_small_batch_matrix_core_kernel_reduction_per_row_block(e0m4, oracle, M):
    # knob value 3: the wavefront sums are reduced after every row block even where all of them fit the LDS
    e0m4.e0m4_set_knob("gemv_mfma", 3)
    try:
        run_matmul_case(e0m4, oracle, M, 1000, 2048, 128, seed=172 + M)
        run_matmul_case(e0m4, oracle, M, 200, 1152, 128, seed=173 + M)
    finally:
        e0m4.e0m4_set_knob("gemv_mfma", 0)


@pytest.mark.parametrize("M", [3, 16])
def test_small_batch_matrix_core_kernel_activations_from_lds(e0m4, oracle, M):
    # K = 4096 with 8 wavefronts would keep the activations in registers; knob value 2 reads them from LDS
    e0m4.e0m4_set_knob("gemv_mfma", 2)
    try:
        run_matmul_case(e0m4, oracle, M, 333, 4096, 128, seed=175 + M, outliers=True)
    finally:
        e0m4.e0m4_set_knob("gemv_mfma", 0)


@pytest.mark.parametrize("M", [2, 5, 8])
def test_small_batch_vector_kernel_when_the_matrix_core_kernel_is_off(e0m4, oracle, M):
    e0m4.e0m4_set_knob("gemv_mfma", 1)
    try:
        run_matmul_case(e0m4, oracle, M, 200, 1152, 128, seed=180 + M)
        run_matmul_case(e0m4, oracle, M, 333, 4096, 128, seed=190 + M, outliers=True)
    finally:
        e0m4.e0m4_set_knob("gemv_mfma", 0)


@pytest.mark.parametrize("M,N,K", [(16, 130, 16384), (8, 130, 16384), (16, 1000, 5248), (11, 333, 8192),
                                   (6, 1100, 13696), (2, 40, 1 << 18)])
def test_small_batch_rows_longer_than_the_lds(e0m4, oracle, M, N, K):
    # M rows of X need more than the 160 KiB of LDS: the kernel walks K in phases (K = 5248: a last phase that is
    # shorter and ends inside a work item)
    run_matmul_case(e0m4, oracle, M, N, K, 128, seed=200 + M)


@pytest.mark.parametrize("waves", [8, 16])
@pytest.mark.parametrize("target", [0, 3])
def test_small_batch_rows_longer_than_the_lds_forced_shapes(e0m4, oracle, waves, target):
    e0m4.e0m4_set_knob("gemv_waves", waves)
    e0m4.e0m4_set_knob("gemv_workgroups", target)       # 3 workgroups asked for: more are used, as many as the sums in LDS need
    try:
        run_matmul_case(e0m4, oracle, 16, 1000, 5248, 128, seed=210 + waves)
        run_matmul_case(e0m4, oracle, 5, 300, 1 << 16, 128, seed=211 + waves)
    finally:
        e0m4.e0m4_set_knob("gemv_waves", 0)
        e0m4.e0m4_set_knob("gemv_workgroups", 0)


@pytest.mark.parametrize("M", [17, 18, 25, 32, 33, 47, 48, 49, 64])
def test_small_batch_chunks_of_rows(e0m4, oracle, M):
    # 17 <= M <= 64, group 128, small weights: equal chunks of at most 16 rows of X, one per y index of a single
    # launch of the small-batch kernel (M = 17: 9 + 8 rows, M = 49: 13 + 13 + 13 + 10), instead of the GEMM; no workspace
    for N, K, seed in ((333, 1152, 220), (1000, 4096, 221), (40, 128, 222)):
        assert e0m4.e0m4_workspace_bytes(M, N, K, 128) == 0
        run_matmul_case(e0m4, oracle, M, N, K, 128, seed=seed + M, outliers=True)
    # not beyond 64 rows, not when a chunk of X needs phases along K
    run_matmul_case(e0m4, oracle, 65, 333, 1152, 128, seed=223)
    run_matmul_case(e0m4, oracle, M, 130, 8192, 128, seed=224 + M)


def test_small_batch_long_rows_without_the_late_reduction_take_another_kernel(e0m4, oracle):
    # knob value 3 (reduction per row block) rules the phases out: the GEMM serves the case
    e0m4.e0m4_set_knob("gemv_mfma", 3)
    try:
        run_matmul_case(e0m4, oracle, 16, 130, 16384, 128, seed=215)
    finally:
        e0m4.e0m4_set_knob("gemv_mfma", 0)


# ------------------------------------------------------------------ matmul, MFMA path

@pytest.mark.parametrize("M,N,K,G", [
    (9, 64, 128, 128), (128, 128, 128, 128), (200, 328, 384, 128), (257, 200, 448, 64), (130, 70, 416, 32),
    (512, 512, 1024, 128), (300, 1000, 2048, 64), (1024, 256, 4096, 128),
])
def test_gemm_small(e0m4, oracle, M, N, K, G):
    run_matmul_case(e0m4, oracle, M, N, K, G, seed=M + N + K, outliers=True, row_std=(0.5, 2.0))


# 1: small-tile kernel; pipelined kernel with tiles of 2: 256 x 256, 3: 128 x 128, 4: 64 x 256, 5: 128 x 256
@pytest.mark.parametrize("variant", [1, 2, 3, 4, 5])
@pytest.mark.parametrize("M,N,K,G", [
    (300, 600, 1024, 128),      # ragged in M and N against every tile size, several tiles each way
    (513, 272, 416, 32),        # ragged K slice (416 = 6.5 x 64), N ends inside a 16-row block run
    (256, 256, 192, 64),        # exactly one large tile
    (40, 1040, 2048, 128),      # fewer rows than any tile
])
def test_gemm_both_kernels(e0m4, oracle, variant, M, N, K, G):
    e0m4.e0m4_set_knob("gemm_variant", variant)
    try:
        run_matmul_case(e0m4, oracle, M, N, K, G, seed=variant + M + N, outliers=True, row_std=(0.5, 2.0))
    finally:
        e0m4.e0m4_set_knob("gemm_variant", 0)


@pytest.mark.parametrize("variant", [2, 3, 4, 5])
@pytest.mark.parametrize("splits", [2, 3, 8])
@pytest.mark.parametrize("M,N,K,G", [
    (300, 600, 1024, 128),      # 6 tiles, 8 slice pairs: 3 splits get 2, 3 and 3 pairs; 8 splits one each
    (513, 272, 384, 32),        # 3 slice pairs: fewer pairs than the 8 splits asked for
    (256, 256, 128, 64),        # one tile, one slice pair: cannot split
    (1024, 1040, 2048, 128),    # 20 tiles, ragged last column of tiles
])
def test_gemm_split_k(e0m4, oracle, variant, splits, M, N, K, G):
    e0m4.e0m4_set_knob("gemm_variant", variant)
    e0m4.e0m4_set_knob("gemm_splits", splits)
    try:
        run_matmul_case(e0m4, oracle, M, N, K, G, seed=splits + M + N, outliers=True, row_std=(0.5, 2.0))
    finally:
        e0m4.e0m4_set_knob("gemm_variant", 0)
        e0m4.e0m4_set_knob("gemm_splits", 0)


# Tile numbering in panels of row tiles (gemm_panel: height in tiles, -1 whole columns, 0 the default of 4 tiles, 2 for
# the 256 x 256 tile).  700 rows are 11, 6 or 3 row tiles of 64, 128 or 256: panels of unequal height at the end, a
# height of one, a height above the number of row tiles; 600 columns are 3 tiles with a ragged last one.  Every
# numbering must visit every tile exactly once: Y starts as NaN.
@pytest.mark.parametrize("panel", [0, 1, 3, 5, 16, -1])
@pytest.mark.parametrize("variant", [2, 3, 4, 5])
def test_gemm_panelled_tile_numbering(e0m4, oracle, variant, panel):
    M, N, K, G = 700, 600, 256, 128
    W = synth_inputs.weights(N, K, seed=910)
    X = synth_inputs.activations(M, K, seed=911)
    (codes, scales, bias), What = assert_quantize_exact(e0m4, oracle, W, G)
    Yref, absdot = oracle.matmul(X, What)
    e0m4.e0m4_set_knob("gemm_variant", variant)
    e0m4.e0m4_set_knob("gemm_panel", panel)
    try:
        # (gemm_split_order: the work items of a K split by tile first, 1, or by split first, 2)
        for splits, order in ((1, 0), (2, 1), (2, 2)):
            e0m4.e0m4_set_knob("gemm_splits", splits)
            e0m4.e0m4_set_knob("gemm_split_order", order)
            ws = torch.empty(max(16, e0m4.e0m4_workspace_bytes(M, N, K, G)), dtype=torch.uint8, device=DEV)
            Y = torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV)
            e0m4.e0m4_matmul(to_dev(X), codes, scales, bias, N, K, G, out=Y, workspace=ws)
            torch.cuda.synchronize()
            check_matmul(Y, Yref, absdot, "variant %d panel %d splits %d order %d" % (variant, panel, splits, order))
    finally:
        for k in ("gemm_variant", "gemm_panel", "gemm_splits", "gemm_split_order"):
            e0m4.e0m4_set_knob(k, 0)


def test_gemm_split_k_default_choice_and_reused_workspace(e0m4, oracle):
    # 1024 x 2304 outputs are few tiles of any size and K is long: the default plan splits K; two calls share one
    # workspace, the second with other activations
    M, N, K, G = 1024, 2304, 4096, 128
    need = e0m4.e0m4_workspace_bytes(M, N, K, G)
    assert need > 0
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    W = synth_inputs.weights(N, K, seed=70)
    codes, scales, bias = e0m4.e0m4_quantize(to_dev(W), G)
    What = oracle.dequant(*oracle.quantize(W, G), G)
    rows = np.array([0, 1, 255, 256, 511, 777, 1023])
    for seed in (71, 72):
        X = synth_inputs.activations(M, K, seed=seed)
        Xd = to_dev(X)
        Y = e0m4.e0m4_matmul(Xd, codes, scales, bias, N, K, G, workspace=ws)
        y_ref, absdot = oracle.matmul(X[rows], What)
        check_matmul(Y[torch.from_numpy(rows).to(DEV)], y_ref, absdot, "seed %d" % seed)
    # a workspace that is too small is refused before anything is launched
    rc = e0m4.lib().e0m4_matmul(Xd.data_ptr(), M, codes.data_ptr(), None, None, N, K, G, Y.data_ptr(), ws.data_ptr(),
                               need - 256, None)
    assert rc == -5


# Groups of 64 and 32 on the group-128 small-batch kernel: every row of X staged once per group of a block, masked to
# that group's k (gemv_mfma 6 sends every shape it can run to it: M <= 8 at group 64, M <= 4 at group 32).
@pytest.mark.parametrize("M,N,K,G", [
    (2, 200, 1152, 64), (5, 200, 1152, 64), (8, 200, 1152, 64), (8, 333, 4096, 64), (3, 1000, 2048, 64),
    (8, 130, 8192, 64), (6, 64, 16384, 64),             # 16 staged rows longer than the LDS: K in phases
    (2, 200, 1152, 32), (4, 200, 1152, 32), (3, 333, 4096, 32), (4, 130, 8192, 32), (4, 48, 16384, 32),
    (7, 5000, 640, 64), (4, 5000, 640, 32),             # many row blocks per workgroup, ragged last k block
])
def test_small_batch_groups_of_64_and_32_on_the_group_128_kernel(e0m4, oracle, M, N, K, G):
    e0m4.e0m4_set_knob("gemv_mfma", 6)
    try:
        assert e0m4.e0m4_workspace_bytes(M, N, K, G) == 0
        run_matmul_case(e0m4, oracle, M, N, K, G, seed=600 + M + N // 7 + K // 128 + G, outliers=True, row_std=(0.5, 2.0))
    finally:
        e0m4.e0m4_set_knob("gemv_mfma", 0)


@pytest.mark.parametrize("waves,target", [(4, 0), (8, 3), (16, 0), (16, 3)])
@pytest.mark.parametrize("G,M", [(64, 7), (32, 4)])
def test_small_batch_groups_forced_shapes(e0m4, oracle, G, M, waves, target):
    e0m4.e0m4_set_knob("gemv_mfma", 6)
    e0m4.e0m4_set_knob("gemv_waves", waves)
    e0m4.e0m4_set_knob("gemv_workgroups", target)
    try:
        run_matmul_case(e0m4, oracle, M, 1000, 2432, G, seed=620 + waves + target + G)
        run_matmul_case(e0m4, oracle, M, 160, 8192, G, seed=630 + waves + target + G)      # phases
    finally:
        e0m4.e0m4_set_knob("gemv_mfma", 0)
        e0m4.e0m4_set_knob("gemv_waves", 0)
        e0m4.e0m4_set_knob("gemv_workgroups", 0)


@pytest.mark.parametrize("G,M", [(64, 8), (64, 3), (32, 4)])
def test_small_batch_groups_one_hot_rows_reproduce_the_weights(e0m4, oracle, G, M):
    # one-hot rows of X at k in different groups of one block: each must return that column of the dequantised
    # weights bit for bit -- a row staged under the wrong group's mask, or folded with the wrong group's
    # parameters, cannot
    N, K = 300, 1024
    W = synth_inputs.weights(N, K, seed=640 + G, row_std_range=(0.5, 2.0))
    codes, scales, bias = e0m4.e0m4_quantize(to_dev(W), G)
    What = oracle.dequant(*oracle.quantize(W, G), G)
    ks = [(m * 37 + 5 + 128 * m + (G // 2) * (m % (128 // G))) % K for m in range(M)]
    X = np.zeros((M, K), dtype=np.float16)
    for m, k in enumerate(ks):
        X[m, k] = 1.0
    e0m4.e0m4_set_knob("gemv_mfma", 6)
    try:
        Y = bits(e0m4.e0m4_matmul(to_dev(X), codes, scales, bias, N, K, G))
    finally:
        e0m4.e0m4_set_knob("gemv_mfma", 0)
    for m, k in enumerate(ks):
        want = What[:, k].view(np.uint16)
        nz = (want & 0x7FFF) != 0
        assert np.array_equal(Y[m][nz], want[nz]), "row %d, k %d" % (m, k)
        assert not (Y[m][~nz] & 0x7FFF).any()


# Even scheduling of the large-tile GEMM: the tiles beyond whole rounds of 256 are shared out by K ranges
# among all workgroups, each writes fp32 sums to a slab of the workspace, and the last to arrive adds a
# tile's slabs in K order.  Forced here on small problems (gemm_variant 2: the 256 x 256 tile; gemm_sk 1).
@pytest.mark.parametrize("M,N,K,G", [
    (300, 600, 1024, 128),      # 6 tiles x 8 slice pairs = 48 units on 256 workgroups: most have none, 8 sharers a tile
    (513, 272, 384, 32),        # 6 tiles x 3 pairs
    (256, 256, 128, 64),        # one tile, one pair: a single owner, written directly
    (1024, 1040, 2048, 128),    # 20 tiles x 16 pairs = 320 units: ranges that end in one tile and begin in the next
    (1000, 1300, 8192, 64),     # 24 tiles x 64 pairs: six pairs a workgroup, tiles shared by 10 or 11
    (2304, 7680, 512, 128),     # 270 tiles: one whole tile each, then 14 tiles x 4 pairs shared out
    (4096, 4112, 256, 128),     # 272 tiles (ragged last column), 16 tiles x 2 pairs shared out
])
def test_gemm_even_scheduling(e0m4, oracle, M, N, K, G):
    W = synth_inputs.weights(N, K, seed=M + N, row_std_range=(0.5, 2.0))
    X = synth_inputs.activations(M, K, seed=M + N + 1, outlier_frac=0.01)
    codes, scales, bias = e0m4.e0m4_quantize(to_dev(W), G)
    What = oracle.dequant(*oracle.quantize(W, G), G)
    rng = np.random.default_rng(M)
    rows = np.unique(np.concatenate([np.arange(0, M, 256), np.arange(255, M, 256), [M - 1],
                                     rng.integers(0, M, size=24)]))
    e0m4.e0m4_set_knob("gemm_variant", 2)
    e0m4.e0m4_set_knob("gemm_sk", 1)
    try:
        need = e0m4.e0m4_workspace_bytes(M, N, K, G)
        tiles = -(-M // 256) * -(-N // 256)
        if tiles % 256 and tiles > 1:
            assert need == 1024 + (256 + tiles % 256) * 256 * 256 * 4
        ws = torch.full((max(need, 16),), 0xFF, dtype=torch.uint8, device=DEV)       # NaNs wherever a slab is read unwritten
        Xd = to_dev(X)
        Y1 = e0m4.e0m4_matmul(Xd, codes, scales, bias, N, K, G, workspace=ws).clone()
        Y2 = e0m4.e0m4_matmul(Xd, codes, scales, bias, N, K, G, workspace=ws)       # counters and slabs left by the first call
        torch.cuda.synchronize()
        assert torch.equal(Y1.view(torch.int16), Y2.view(torch.int16)), "two runs differ"
        # other activations through the same workspace: no slab of the calls before may be read in place of a new one
        X3 = synth_inputs.activations(M, K, seed=M + N + 2, outlier_frac=0.01)
        Y3 = e0m4.e0m4_matmul(to_dev(X3), codes, scales, bias, N, K, G, workspace=ws)
        y3_ref, absdot3 = oracle.matmul(X3[rows], What)
        check_matmul(Y3[torch.from_numpy(rows).to(DEV)], y3_ref, absdot3, "even scheduling, reused workspace")
        y_ref, absdot = oracle.matmul(X[rows], What)
        check_matmul(Y1[torch.from_numpy(rows).to(DEV)], y_ref, absdot, "even scheduling M=%d N=%d K=%d" % (M, N, K))
        if need > 1024:
            rc = e0m4.lib().e0m4_matmul(Xd.data_ptr(), M, codes.data_ptr(), None, None, N, K, G, Y2.data_ptr(),
                                       ws.data_ptr(), need - 256, None)
            assert rc == -5
        # the rows not sampled: against the whole-tile kernel, whose sums differ by fp32 rounding order only
        e0m4.e0m4_set_knob("gemm_sk", 2)
        Y0 = e0m4.e0m4_matmul(Xd, codes, scales, bias, N, K, G)
        torch.cuda.synchronize()
        d = (Y1.float() - Y0.float()).abs()
        bound = 2.0 ** -9 * Y0.float().abs() + 2.0 ** -6
        assert bool((d <= bound).all()), "differs from the whole-tile kernel: %g" % float((d - bound).max())
    finally:
        e0m4.e0m4_set_knob("gemm_variant", 0)
        e0m4.e0m4_set_knob("gemm_sk", 0)


# ------------------------------------------------------------------ special inputs through both paths

@pytest.mark.parametrize("M", [4, 160])
def test_one_hot_activations_reproduce_weights_bit_exactly(e0m4, oracle, M):
    N, K, G = 200, 512, 128
    W = synth_inputs.weights(N, K, seed=60)
    (codes, scales, bias), What = assert_quantize_exact(e0m4, oracle, W, G)
    ks = np.random.default_rng(61).integers(0, K, M)
    ks[0], ks[-1] = 0, K - 1
    X = np.zeros((M, K), dtype=np.float16)
    X[np.arange(M), ks] = 1.0
    Y = bits(e0m4.e0m4_matmul(to_dev(X), codes, scales, bias, N, K, G))
    assert np.array_equal(Y, What.view(np.uint16)[:, ks].T)


@pytest.mark.parametrize("M", [1, 64])
def test_all_ones_activations_give_row_sums(e0m4, oracle, M):
    N, K, G = 192, 1024, 64
    W = synth_inputs.weights(N, K, seed=62)
    (codes, scales, bias), What = assert_quantize_exact(e0m4, oracle, W, G)
    X = np.ones((M, K), dtype=np.float16)
    Y = e0m4.e0m4_matmul(to_dev(X), codes, scales, bias, N, K, G)
    sums = What.astype(np.float64).sum(axis=1)
    absdot = np.abs(What.astype(np.float64)).sum(axis=1)
    check_matmul(Y, np.tile(sums.astype(np.float16), (M, 1)), np.tile(absdot, (M, 1)))


@pytest.mark.parametrize("M", [1, 5, 200])
def test_matmul_is_deterministic(e0m4, M):
    N, K, G = 4096, 4096, 128
    W = synth_inputs.weights(N, K, seed=63)
    X = to_dev(synth_inputs.activations(M, K, seed=63))
    codes, scales, bias = e0m4.e0m4_quantize(to_dev(W), G)
    y1 = bits(e0m4.e0m4_matmul(X, codes, scales, bias, N, K, G))
    y2 = bits(e0m4.e0m4_matmul(X, codes, scales, bias, N, K, G))
    assert np.array_equal(y1, y2)


@pytest.mark.parametrize("M,G", [(8, 64), (5, 32), (8, 128)])
def test_few_rows_with_large_weights_take_the_gemm(e0m4, oracle, M, G):
    # M * N * K above 3.8e8 and no small-batch matrix-core kernel (other groups; at G = 128, that kernel switched
    # off): the 64 x 256 GEMM tile instead of the vector kernel
    if G == 128:
        e0m4.e0m4_set_knob("gemv_mfma", 1)
        try:
            run_matmul_case(e0m4, oracle, M, 1600, 32768, G, seed=611)
        finally:
            e0m4.e0m4_set_knob("gemv_mfma", 0)
    else:
        run_matmul_case(e0m4, oracle, M, 24000 if M == 5 else 12288, 4096, G, seed=610 + M, outliers=True)


@pytest.mark.parametrize("M", [1, 3, 20])
def test_longest_rows(e0m4, oracle, M):
    # K at its limit of 2^20: the decode kernel stages X in many segments, the GEMM runs 16384 K slices in 8 splits
    run_matmul_case(e0m4, oracle, M, 24, 1 << 20, 128, seed=600 + M)


def test_empty_problems(e0m4):
    X = torch.zeros((0, 128), dtype=torch.float16, device=DEV)
    codes, scales, bias = e0m4.alloc_packed(64, 128, 128, DEV)
    assert e0m4.e0m4_matmul(X, codes, scales, bias, 64, 128, 128).shape == (0, 64)
    # K = 0: the empty sum is zero
    X0 = torch.zeros((3, 0), dtype=torch.float16, device=DEV)
    c0, s0, b0 = e0m4.alloc_packed(70, 0, 128, DEV)
    Y = torch.full((3, 70), 7.0, dtype=torch.float16, device=DEV)
    e0m4.e0m4_matmul(X0, c0, s0, b0, 70, 0, 128, out=Y)
    assert not Y.cpu().numpy().any()
    # N = 0
    W0 = torch.zeros((0, 128), dtype=torch.float16, device=DEV)
    e0m4.e0m4_quantize(W0, 128)
    torch.cuda.synchronize()


# ------------------------------------------------------------------ small batches with dequantised weight operands
# (2 <= M <= 64, any group; by default it serves groups of 32 and 64 at 3 <= M <= 16; knob gemv_mfma = 4 forces the
# kernel wherever it can run)

DQ_SHAPES = [(203, 1664, 32), (203, 1664, 64), (203, 1664, 128), (1040, 4096, 64), (64, 128, 128), (17, 32, 32),
             (530, 13696, 64), (300, 8192, 128), (4608, 416, 32)]


@pytest.mark.parametrize("N,K,G", DQ_SHAPES)
@pytest.mark.parametrize("M", [2, 3, 8, 15, 16, 17, 24, 32, 33, 47, 64])
def test_small_batch_dequantised_operands_forced(e0m4, oracle, M, N, K, G):
    W = synth_inputs.weights(N, K, seed=900 + N + K + G)
    (codes, scales, bias), What = assert_quantize_exact(e0m4, oracle, W, G)
    X = synth_inputs.activations(M, K, seed=950 + M)
    ws = torch.empty(max(16, e0m4.e0m4_workspace_bytes(M, N, K, G)), dtype=torch.uint8, device=DEV)
    e0m4.e0m4_set_knob("gemv_mfma", 4)
    try:
        Y = e0m4.e0m4_matmul(to_dev(X), codes, scales, bias, N, K, G, workspace=ws)
        Y2 = e0m4.e0m4_matmul(to_dev(X), codes, scales, bias, N, K, G, workspace=ws)
    finally:
        e0m4.e0m4_set_knob("gemv_mfma", 0)
    Yref, absdot = oracle.matmul(X, What)
    check_matmul(Y, Yref, absdot, "dq M=%d N=%d K=%d G=%d" % (M, N, K, G))
    assert torch.equal(Y, Y2)


@pytest.mark.parametrize("G", [32, 64, 128])
@pytest.mark.parametrize("M", [3, 5, 16])
def test_small_batch_default_dispatch_and_one_hot(e0m4, oracle, M, G):
    N, K = 1040, 2048
    W = synth_inputs.weights(N, K, seed=970 + G)
    (codes, scales, bias), What = assert_quantize_exact(e0m4, oracle, W, G)
    assert e0m4.e0m4_workspace_bytes(M, N, K, G) == 0               # one of the small-batch kernels serves it
    X = synth_inputs.activations(M, K, seed=980 + M)
    Y = e0m4.e0m4_matmul(to_dev(X), codes, scales, bias, N, K, G)
    Yref, absdot = oracle.matmul(X, What)
    check_matmul(Y, Yref, absdot, "small batch M=%d G=%d" % (M, G))
    X1 = np.zeros((M, K), dtype=np.float16)
    ks = [(131 * m + 7) % K for m in range(M)]
    for m, k in enumerate(ks):
        X1[m, k] = 1.0
    Y1 = bits(e0m4.e0m4_matmul(to_dev(X1), codes, scales, bias, N, K, G))
    for m, k in enumerate(ks):
        assert np.array_equal(Y1[m] & 0x7FFF, What.view(np.uint16)[:, k] & 0x7FFF)


def test_small_batch_dequantised_operands_few_workgroups(e0m4, oracle):
    """Many row blocks per workgroup, K in several phases (the sums wait in LDS between phases)."""
    N, K, G, M = 2000, 6144, 64, 40
    W = synth_inputs.weights(N, K, seed=990)
    (codes, scales, bias), What = assert_quantize_exact(e0m4, oracle, W, G)
    X = synth_inputs.activations(M, K, seed=991)
    Yref, absdot = oracle.matmul(X, What)
    for target in (0, 7, 40):
        e0m4.e0m4_set_knob("gemv_mfma", 4)
        e0m4.e0m4_set_knob("gemv_workgroups", target)
        try:
            Y = e0m4.e0m4_matmul(to_dev(X), codes, scales, bias, N, K, G)
        finally:
            e0m4.e0m4_set_knob("gemv_mfma", 0)
            e0m4.e0m4_set_knob("gemv_workgroups", 0)
        check_matmul(Y, Yref, absdot, "dq target=%d" % target)
