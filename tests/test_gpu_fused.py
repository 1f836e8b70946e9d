"""Parity of e0m4_matmul_fused (rms-norm on X, SiLU-gated product of the output halves, residual add;
paper: section "Operator and lagging optimizations") with the CPU oracle, through the C ABI.

Tolerances.  Without the gated epilogue the output is linear in the sums a = sum_k x w and keeps the
matmul's bar, |y - ref| <= 1e-2 * max(1, sum_k |x w|).  With it, y = silu(g) * u, and an error e_g, e_u
of the two sums moves y by at most L |u| e_g + |silu(g)| e_u + L e_g e_u, L = 1.1 > max |silu'|; the
acceptance bar puts the matmul's bar in for e_g and e_u.  A second, much tighter quality bound uses what
the arithmetic allows: e = 2^-9 sum|x w| (fp32 accumulation, fp16 weights and activations), plus
2^-10 sum|x w| when the rows are normalised on the GPU (a normalised activation may round to the
neighbouring fp16 value), plus the final fp16 rounding of y."""
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
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def quantized(e0m4, oracle, N, K, G, seed, row_std=None, bits=4):
    W = synth_inputs.weights(N, K, seed=seed, row_std_range=row_std)
    if bits == 8:
        codes, _, _ = e0m4.e0m8_quantize(to_dev(W), G)
        oc, os_, ob = oracle.quantize_k(W, G, 8)
        return codes, oracle.dequant_k(oc, os_, ob, G, 8)
    codes, scales, bias = e0m4.e0m4_quantize(to_dev(W), G)
    oc, os_, ob = oracle.quantize(W, G)
    return codes, oracle.dequant(oc, os_, ob, G)


def check_fused(y_gpu, Yref, info, swiglu, normed, what):
    got = y_gpu.detach().cpu().numpy().astype(np.float64)
    ref = info["y"]
    assert got.shape == ref.shape, what
    err = np.abs(got - Yref.astype(np.float64))
    a, absdot = info["a"], info["absdot"]

    def bound(e):
        if not swiglu:
            return e
        h = a.shape[1] // 2
        g, u, eg, eu = a[:, :h], a[:, h:], e[:, :h], e[:, h:]
        sg = g / (1.0 + np.exp(-g))
        return 1.1 * np.abs(u) * eg + np.abs(sg) * eu + 1.1 * eg * eu

    accept = bound(1e-2 * np.maximum(1.0, absdot)) + 2.0 ** -10 * np.abs(ref) + 1e-6
    worst = np.unravel_index(np.argmax(err / accept), err.shape)
    assert (err <= accept).all(), "%s: worst at %s err %g tol %g" % (what, worst, err[worst], accept[worst])
    e = (2.0 ** -9 + (2.0 ** -10 if normed else 0.0)) * absdot + 1e-7
    tight = bound(e) + 2.0 ** -10 * np.abs(ref) + 1e-6
    assert (err <= tight).all(), "%s: quality bound: %g" % (what, (err / tight).max())


def run_fused(e0m4, oracle, M, N, K, G, seed, norm=False, swiglu=False, res=False, row_std=None, outliers=False,
              in_place=False, bits=4):
    codes, What = quantized(e0m4, oracle, N, K, G, seed, row_std, bits)
    X = synth_inputs.activations(M, K, seed=seed, outlier_frac=0.01 if outliers else 0.0)
    gamma = synth_inputs.norm_weight(K, seed) if norm else None
    n_out = N // 2 if swiglu else N
    R = synth_inputs.residual(M, n_out, seed) if res else None
    eps = 1e-5
    out = None
    r_dev = to_dev(R)
    if in_place:
        out = r_dev                                     # the residual stream is updated in place
    fn = e0m4.e0m8_matmul_fused if bits == 8 else e0m4.e0m4_matmul_fused
    Y = fn(to_dev(X), codes, N, K, G, rms_gamma=to_dev(gamma), rms_eps=eps,
           epilogue=e0m4.E0M4_EPILOGUE_SWIGLU if swiglu else e0m4.E0M4_EPILOGUE_NONE, residual=r_dev, out=out)
    Yref, info = oracle.matmul_fused(X, What, gamma=gamma, eps=eps, swiglu=swiglu, residual=R)
    torch.cuda.synchronize()
    what = "bits=%d M=%d N=%d K=%d G=%d norm=%d swiglu=%d res=%d" % (bits, M, N, K, G, norm, swiglu, res)
    check_fused(Y, Yref, info, swiglu, norm, what)
    return Y


COMBOS = [(True, False, False), (False, True, False), (False, False, True), (True, True, True), (True, False, True)]


@pytest.mark.parametrize("norm,swiglu,res", COMBOS)
@pytest.mark.parametrize("M", [1, 2, 5, 8])
def test_decode_kernel(e0m4, oracle, M, norm, swiglu, res):
    run_fused(e0m4, oracle, M, 320, 1152, 128, seed=300 + M, norm=norm, swiglu=swiglu, res=res)     # 9 k blocks, 10 pairs
    run_fused(e0m4, oracle, M, 1088, 4096, 128, seed=310 + M, norm=norm, swiglu=swiglu, res=res, outliers=True)


@pytest.mark.parametrize("norm,swiglu,res", COMBOS)
@pytest.mark.parametrize("M", [2, 5, 8])
def test_decode_vector_kernel_for_small_batches(e0m4, oracle, M, norm, swiglu, res):
    e0m4.e0m4_set_knob("gemv_mfma", 1)                  # group 128 would take the matrix-core kernel for M >= 2
    try:
        run_fused(e0m4, oracle, M, 320, 1152, 128, seed=305 + M, norm=norm, swiglu=swiglu, res=res)
    finally:
        e0m4.e0m4_set_knob("gemv_mfma", 0)


@pytest.mark.parametrize("norm,swiglu,res", COMBOS)
@pytest.mark.parametrize("M", [3, 4, 8, 9, 13, 16])
def test_small_batch_matrix_core_kernel(e0m4, oracle, M, norm, swiglu, res):
    run_fused(e0m4, oracle, M, 320, 1152, 128, seed=500 + M, norm=norm, swiglu=swiglu, res=res)     # 9 k blocks, 10 pairs
    run_fused(e0m4, oracle, M, 1088, 4096, 128, seed=510 + M, norm=norm, swiglu=swiglu, res=res, outliers=True)
    run_fused(e0m4, oracle, M, 333 if not swiglu else 448, 1664, 128, seed=520 + M, norm=norm, swiglu=swiglu, res=res)


@pytest.mark.parametrize("norm,swiglu,res", COMBOS)
@pytest.mark.parametrize("bits", [4, 8])
def test_small_batch_rows_longer_than_the_lds(e0m4, oracle, bits, norm, swiglu, res):
    # M rows of X do not fit the LDS: K in phases (the rms-norm sums run over all of K before the first phase)
    run_fused(e0m4, oracle, 16, 448, 5248 if bits == 4 else 5184, 128 if bits == 4 else 64, seed=540 + bits, norm=norm,
              swiglu=swiglu, res=res, bits=bits)
    run_fused(e0m4, oracle, 7, 1088, 16384, 128, seed=541 + bits, norm=norm, swiglu=swiglu, res=res, outliers=True,
              bits=bits)


@pytest.mark.parametrize("norm,swiglu,res", COMBOS)
@pytest.mark.parametrize("G,M", [(64, 2), (64, 5), (64, 8), (32, 3), (32, 4)])
def test_small_batch_groups_of_64_and_32_fused(e0m4, oracle, G, M, norm, swiglu, res):
    # groups of 64 and 32 on the matrix-core small-batch kernel (rows of X staged once per group of a block): the
    # default for the fused matmul at 3 <= M <= 8 (group 64) and 3 <= M <= 4 (group 32), forced at M = 2; whole rows,
    # and K in phases
    e0m4.e0m4_set_knob("gemv_mfma", 6)
    try:
        run_fused(e0m4, oracle, M, 320, 1152, G, seed=569 + M + G, norm=norm, swiglu=swiglu, res=res)
    finally:
        e0m4.e0m4_set_knob("gemv_mfma", 0)
    run_fused(e0m4, oracle, M, 448, 1664, G, seed=570 + M + G, norm=norm, swiglu=swiglu, res=res, outliers=True)
    run_fused(e0m4, oracle, M, 1088, 2048, G, seed=571 + M + G, norm=norm, swiglu=swiglu, res=res, row_std=(0.5, 2.0))
    run_fused(e0m4, oracle, M, 192, 8192, G, seed=572 + M + G, norm=norm, swiglu=swiglu, res=res)


@pytest.mark.parametrize("norm,swiglu,res", COMBOS)
@pytest.mark.parametrize("M", [17, 24, 32, 41, 64])
@pytest.mark.parametrize("bits", [4, 8])
def test_small_batch_chunks_of_rows(e0m4, oracle, bits, M, norm, swiglu, res):
    # 17 <= M <= 64 (8-bit: 32) on small weights: the small-batch kernel on equal chunks of at most 16 rows in one
    # launch; every chunk gets its rows of X, of the residual and of Y
    run_fused(e0m4, oracle, M, 448, 1664, 128, seed=545 + M, norm=norm, swiglu=swiglu, res=res, bits=bits)
    run_fused(e0m4, oracle, M, 1088 if swiglu else 1000, 4096 if bits == 4 else 2048, 128, seed=546 + M, norm=norm,
              swiglu=swiglu, res=res, outliers=True, bits=bits)


@pytest.mark.parametrize("M", [2, 6, 16])
def test_small_batch_matrix_core_kernel_reduction_per_row_block(e0m4, oracle, M):
    e0m4.e0m4_set_knob("gemv_mfma", 3)
    try:
        run_fused(e0m4, oracle, M, 1088, 2048, 128, seed=525 + M, norm=True, swiglu=True, res=True)
        run_fused(e0m4, oracle, M, 333, 1664, 128, seed=526 + M, norm=True, res=True)
    finally:
        e0m4.e0m4_set_knob("gemv_mfma", 0)


@pytest.mark.parametrize("waves", [4, 8, 16])
@pytest.mark.parametrize("target", [0, 3])
def test_small_batch_matrix_core_kernel_forced_shapes(e0m4, oracle, waves, target):
    e0m4.e0m4_set_knob("gemv_waves", waves)
    e0m4.e0m4_set_knob("gemv_workgroups", target)       # 3 workgroups: many pairs each, dealt unevenly
    try:
        run_fused(e0m4, oracle, 6, 2240, 2304, 128, seed=530 + waves, norm=True, swiglu=True, res=True)
        run_fused(e0m4, oracle, 16, 130, 4096, 128, seed=531 + waves, norm=True, res=True)
    finally:
        e0m4.e0m4_set_knob("gemv_waves", 0)
        e0m4.e0m4_set_knob("gemv_workgroups", 0)


@pytest.mark.parametrize("G", [32, 64])
def test_decode_kernel_other_groups(e0m4, oracle, G):
    run_fused(e0m4, oracle, 1, 448, 1760 if G == 32 else 1728, G, seed=320 + G, norm=True, swiglu=True, res=True)
    run_fused(e0m4, oracle, 3, 448, 1024, G, seed=321 + G, norm=True, swiglu=True, res=True)


@pytest.mark.parametrize("waves", [4, 8, 16])
@pytest.mark.parametrize("target", [0, 3, 100000])
def test_decode_kernel_forced_shapes(e0m4, oracle, waves, target):
    # 3 workgroups: many pairs of row blocks each, dealt unevenly; 100000: one pair (or row block) each
    e0m4.e0m4_set_knob("gemv_waves", waves)
    e0m4.e0m4_set_knob("gemv_workgroups", target)
    try:
        run_fused(e0m4, oracle, 1, 2240, 2304, 128, seed=330 + waves, norm=True, swiglu=True, res=True)
        run_fused(e0m4, oracle, 4, 704, 1152, 64, seed=331 + waves, swiglu=True)
        run_fused(e0m4, oracle, 2, 333, 1664, 128, seed=332 + waves, norm=True, res=True)      # N ends inside a row block
    finally:
        e0m4.e0m4_set_knob("gemv_waves", 0)
        e0m4.e0m4_set_knob("gemv_workgroups", 0)


@pytest.mark.parametrize("norm,swiglu,res", COMBOS)
def test_decode_kernel_one_wavefront_per_work_item(e0m4, oracle, norm, swiglu, res):
    run_fused(e0m4, oracle, 1, 12352, 5120, 128, seed=330, norm=norm, swiglu=swiglu, res=res)   # 10 wavefronts
    run_fused(e0m4, oracle, 1, 320, 6144, 64, seed=331, norm=norm, swiglu=swiglu, res=res)      # 12


def test_few_rows_with_large_weights_take_the_gemm(e0m4, oracle):
    run_fused(e0m4, oracle, 8, 12288, 4096, 64, seed=332, norm=True, swiglu=True, res=True)


def test_decode_kernel_long_rows(e0m4, oracle):
    # 8 rows of K = 16384 are staged in several segments: the norm's row sums come from memory, and the
    # gated epilogue (which needs whole rows in LDS) is served by the GEMM kernels instead
    # (group 64: the vector kernel; group 128: the small-batch kernel with K in phases)
    for G in (64, 128):
        run_fused(e0m4, oracle, 8, 130, 16384, G, seed=340, norm=True, res=True)
        run_fused(e0m4, oracle, 8, 128, 16384, G, seed=341, norm=True, swiglu=True, res=True)
    run_fused(e0m4, oracle, 1, 192, 32768, 128, seed=342, norm=True, swiglu=True)


def test_nothing_selected_equals_the_plain_matmul(e0m4, oracle):
    for M in (1, 6, 40):
        codes, What = quantized(e0m4, oracle, 200, 1152, 128, seed=350 + M)
        X = to_dev(synth_inputs.activations(M, 1152, seed=350 + M))
        y0 = e0m4.e0m4_matmul(X, codes, None, None, 200, 1152, 128)
        y1 = e0m4.e0m4_matmul_fused(X, codes, 200, 1152, 128)
        e0m4.e0m4_set_knob("gemv_mfma", 1)              # small batches on the vector kernel
        try:
            y0v = e0m4.e0m4_matmul(X, codes, None, None, 200, 1152, 128)
            y1v = e0m4.e0m4_matmul_fused(X, codes, 200, 1152, 128)
        finally:
            e0m4.e0m4_set_knob("gemv_mfma", 0)
        torch.cuda.synchronize()
        assert torch.equal(y1, y0) and torch.equal(y1v, y0v), M
        Yref, absdot = oracle.matmul(X.cpu().numpy(), What)
        assert np.all(np.abs(y0.cpu().numpy().astype(np.float64) - Yref.astype(np.float64)) <= 1e-2 * np.maximum(1, absdot))


# 1: small-tile kernel; pipelined kernel with tiles of 2: 256 x 256, 3: 128 x 128, 4: 64 x 256
@pytest.mark.parametrize("variant", [1, 2, 3, 4, 5])
@pytest.mark.parametrize("norm,swiglu,res", COMBOS)
def test_gemm_kernels(e0m4, oracle, variant, norm, swiglu, res):
    e0m4.e0m4_set_knob("gemm_variant", variant)
    try:
        run_fused(e0m4, oracle, 300, 640, 1024, 128, seed=360 + variant, norm=norm, swiglu=swiglu, res=res,
                  row_std=(0.5, 2.0), outliers=True)    # ragged in M; 320 outputs: 2.5 gated tiles of the large kernel
        run_fused(e0m4, oracle, 9, 192, 384, 64, seed=361 + variant, norm=norm, swiglu=swiglu, res=res)
        run_fused(e0m4, oracle, 130, 1088, 512, 32, seed=362 + variant, norm=norm, swiglu=swiglu, res=res)
    finally:
        e0m4.e0m4_set_knob("gemm_variant", 0)


@pytest.mark.parametrize("variant", [2, 3, 4, 5])
@pytest.mark.parametrize("splits", [2, 3, 8])
@pytest.mark.parametrize("norm,swiglu,res", COMBOS)
def test_gemm_split_along_k(e0m4, oracle, variant, splits, norm, swiglu, res):
    e0m4.e0m4_set_knob("gemm_variant", variant)
    e0m4.e0m4_set_knob("gemm_splits", splits)
    e0m4.e0m4_set_knob("gemm_split_order", 1 + splits % 2)      # work items by tile first, or by split first
    try:
        run_fused(e0m4, oracle, 257, 704, 1024, 128, seed=370 + splits, norm=norm, swiglu=swiglu, res=res)
    finally:
        e0m4.e0m4_set_knob("gemm_variant", 0)
        e0m4.e0m4_set_knob("gemm_splits", 0)
        e0m4.e0m4_set_knob("gemm_split_order", 0)


# the panelled tile numbering with the gated epilogue (a tile covers half as many output columns) and 11 row tiles of 64
@pytest.mark.parametrize("variant,panel", [(4, 0), (4, 3), (5, 1), (2, 2), (4, -1)])
def test_gemm_panelled_tile_numbering_with_epilogues(e0m4, oracle, variant, panel):
    e0m4.e0m4_set_knob("gemm_variant", variant)
    e0m4.e0m4_set_knob("gemm_panel", panel)
    try:
        run_fused(e0m4, oracle, 700, 640, 256, 128, seed=380 + variant, norm=True, swiglu=True, res=True)
        run_fused(e0m4, oracle, 700, 608, 256, 64, seed=381 + variant, norm=False, swiglu=False, res=True)
    finally:
        e0m4.e0m4_set_knob("gemm_variant", 0)
        e0m4.e0m4_set_knob("gemm_panel", 0)


def test_gemm_small_kernel_ragged_k(e0m4, oracle):
    run_fused(e0m4, oracle, 70, 256, 416, 32, seed=380, norm=True, swiglu=True, res=True)      # K = 6.5 slices of 64


# ---- the same operators on 8-bit codes (e0m8_matmul_fused)
@pytest.mark.parametrize("norm,swiglu,res", COMBOS)
@pytest.mark.parametrize("M", [1, 2, 5, 8])
def test_8bit_decode_kernel(e0m4, oracle, M, norm, swiglu, res):
    e0m4.e0m4_set_knob("gemv_mfma", 1)                  # M >= 2 would take the matrix-core kernel
    try:
        run_fused(e0m4, oracle, M, 320, 576, 64, seed=700 + M, norm=norm, swiglu=swiglu, res=res, bits=8)   # 9 blocks
        run_fused(e0m4, oracle, M, 1088, 2048, 128, seed=710 + M, norm=norm, swiglu=swiglu, res=res, outliers=True, bits=8)
        run_fused(e0m4, oracle, M, 192, 1088, 64, seed=720 + M, norm=norm, swiglu=swiglu, res=res, bits=8)  # 17 blocks
    finally:
        e0m4.e0m4_set_knob("gemv_mfma", 0)


@pytest.mark.parametrize("waves", [4, 8, 16])
@pytest.mark.parametrize("target", [0, 3, 100000])
def test_8bit_decode_kernel_forced_shapes(e0m4, oracle, waves, target):
    e0m4.e0m4_set_knob("gemv_waves", waves)
    e0m4.e0m4_set_knob("gemv_workgroups", target)
    try:
        for M in (1, 3):
            run_fused(e0m4, oracle, M, 448, 1600, 64, seed=730 + waves, norm=True, swiglu=True, res=True, bits=8)
    finally:
        e0m4.e0m4_set_knob("gemv_waves", 0)
        e0m4.e0m4_set_knob("gemv_workgroups", 0)


@pytest.mark.parametrize("norm,swiglu,res", COMBOS)
@pytest.mark.parametrize("M", [2, 3, 8, 9, 16])
def test_8bit_small_batch_matrix_core_kernel(e0m4, oracle, M, norm, swiglu, res):
    run_fused(e0m4, oracle, M, 320, 576, 64, seed=740 + M, norm=norm, swiglu=swiglu, res=res, bits=8)
    run_fused(e0m4, oracle, M, 1088, 2048, 128, seed=750 + M, norm=norm, swiglu=swiglu, res=res, outliers=True, bits=8)
    run_fused(e0m4, oracle, M, 333 if not swiglu else 448, 832, 64, seed=760 + M, norm=norm, swiglu=swiglu, res=res,
              bits=8)


@pytest.mark.parametrize("mode", [2, 3])
@pytest.mark.parametrize("waves", [4, 8, 16])
def test_8bit_small_batch_matrix_core_kernel_forced_shapes(e0m4, oracle, waves, mode):
    e0m4.e0m4_set_knob("gemv_waves", waves)
    e0m4.e0m4_set_knob("gemv_mfma", mode)               # 2: X from the LDS, 3: reduction per row block
    try:
        for M in (2, 11):
            run_fused(e0m4, oracle, M, 448, 1600, 64, seed=770 + waves, norm=True, swiglu=True, res=True, bits=8)
    finally:
        e0m4.e0m4_set_knob("gemv_waves", 0)
        e0m4.e0m4_set_knob("gemv_mfma", 0)


@pytest.mark.parametrize("variant,splits", [(2, 0), (3, 0), (4, 0), (5, 0), (2, 3), (3, 2), (4, 8), (5, 4)])
@pytest.mark.parametrize("norm,swiglu,res", COMBOS)
def test_8bit_gemm_kernels(e0m4, oracle, variant, splits, norm, swiglu, res):
    e0m4.e0m4_set_knob("gemm_variant", variant)
    e0m4.e0m4_set_knob("gemm_splits", splits)
    try:
        run_fused(e0m4, oracle, 300, 640, 1024, 128, seed=780 + variant, norm=norm, swiglu=swiglu, res=res,
                  row_std=(0.5, 2.0), outliers=True, bits=8)
        run_fused(e0m4, oracle, 17, 192, 384, 64, seed=781 + variant, norm=norm, swiglu=swiglu, res=res, bits=8)
    finally:
        e0m4.e0m4_set_knob("gemm_variant", 0)
        e0m4.e0m4_set_knob("gemm_splits", 0)


def test_8bit_larger_batches_need_whole_k_slices(e0m4):
    N, K, G = 128, 192, 64                              # K % 128 != 0: only the decode kernels take it
    codes, _, _ = e0m4.e0m8_quantize(to_dev(synth_inputs.weights(N, K, seed=1)), G)
    x = to_dev(synth_inputs.activations(40, K, seed=2))
    assert e0m4.e0m8_matmul_fused(x[:8].contiguous(), codes, N, K, G, epilogue=e0m4.E0M4_EPILOGUE_SWIGLU).shape == (8, 64)
    with pytest.raises(e0m4.E0M4Error, match="shape"):
        e0m4.e0m8_matmul_fused(x, codes, N, K, G, epilogue=e0m4.E0M4_EPILOGUE_SWIGLU)


def test_residual_in_place(e0m4, oracle):
    run_fused(e0m4, oracle, 1, 320, 1152, 128, seed=390, res=True, in_place=True)
    run_fused(e0m4, oracle, 5, 640, 1152, 128, seed=391, swiglu=True, res=True, in_place=True)
    run_fused(e0m4, oracle, 300, 640, 1024, 128, seed=392, norm=True, res=True, in_place=True)
    e0m4.e0m4_set_knob("gemm_variant", 2)
    e0m4.e0m4_set_knob("gemm_splits", 2)
    try:
        run_fused(e0m4, oracle, 257, 704, 1024, 128, seed=393, swiglu=True, res=True, in_place=True)
    finally:
        e0m4.e0m4_set_knob("gemm_variant", 0)
        e0m4.e0m4_set_knob("gemm_splits", 0)


def test_argument_errors(e0m4):
    x = torch.zeros((1, 128), dtype=torch.float16, device=DEV)
    codes = torch.zeros(e0m4.e0m4_codes_bytes(96, 128, 128), dtype=torch.uint8, device=DEV)
    with pytest.raises(e0m4.E0M4Error):                 # N / 2 is not a whole number of pairs of row blocks
        e0m4.e0m4_matmul_fused(x, codes, 96, 128, 128, epilogue=e0m4.E0M4_EPILOGUE_SWIGLU)
    with pytest.raises(e0m4.E0M4Error):                 # unknown epilogue
        e0m4.e0m4_matmul_fused(x, codes, 96, 128, 128, epilogue=7)
    big = torch.zeros((300, 128), dtype=torch.float16, device=DEV)
    gamma = torch.ones(128, dtype=torch.float16, device=DEV)
    with pytest.raises(e0m4.E0M4Error):                 # workspace too small for the normalised copy of X
        e0m4.e0m4_matmul_fused(big, codes, 96, 128, 128, rms_gamma=gamma,
                               workspace=torch.zeros(64, dtype=torch.uint8, device=DEV))


# ------------------------------------------------------------------ the benchmark's layer, full size

def sample_indices(count, total, tile, rng):
    fixed = {0, total - 1, tile - 1, tile, total // 2, max(total - tile, 0), max(total - tile - 1, 0)}
    fixed = {i for i in fixed if 0 <= i < total}
    extra = set(int(i) for i in rng.integers(0, total, max(count - len(fixed), 0)))
    return np.array(sorted(fixed | extra), dtype=np.int64)


FULL = [
    # name, N, K, norm, swiglu, res  (the four fused calls of a ChatGLM2-6B-shaped layer, as the benchmark issues them)
    ("qkv", 4608, 4096, True, False, False),
    ("attn_out", 4096, 4096, False, False, True),
    ("gate_up", 27392, 4096, True, True, False),
    ("down", 4096, 13696, False, False, True),
]


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("name,N,K,norm,swiglu,res", FULL, ids=[c[0] for c in FULL])
def test_full_size_layer(e0m4, oracle, name, N, K, norm, swiglu, res, bits):
    G, Mp = 128, 1024
    seed = 400 + N % 97 + K % 89 + (8 if bits == 8 else 0)
    # decode: the whole output
    run_fused(e0m4, oracle, 1, N, K, G, seed=seed, norm=norm, swiglu=swiglu, res=res, bits=bits)
    # prefill: sampled rows over all outputs, sampled output columns over all rows
    codes, What = quantized(e0m4, oracle, N, K, G, seed + 1, row_std=(0.5, 2.0), bits=bits)
    X = synth_inputs.activations(Mp, K, seed=seed + 1, outlier_frac=0.01)
    gamma = synth_inputs.norm_weight(K, seed + 1) if norm else None
    n_out = N // 2 if swiglu else N
    R = synth_inputs.residual(Mp, n_out, seed + 1) if res else None
    fn = e0m4.e0m8_matmul_fused if bits == 8 else e0m4.e0m4_matmul_fused
    Y = fn(to_dev(X), codes, N, K, G, rms_gamma=to_dev(gamma), rms_eps=1e-5,
           epilogue=e0m4.E0M4_EPILOGUE_SWIGLU if swiglu else e0m4.E0M4_EPILOGUE_NONE, residual=to_dev(R)).cpu().numpy()
    rng = np.random.default_rng(seed)
    ms = sample_indices(12, Mp, 128, rng)
    Yr, info = oracle.matmul_fused(X[ms], What, gamma=gamma, eps=1e-5, swiglu=swiglu,
                                   residual=None if R is None else R[ms])
    check_fused(torch.from_numpy(Y[ms]), Yr, info, swiglu, norm, name + " prefill rows")
    js = sample_indices(48, n_out, 128, rng)
    rows = np.concatenate([js, js + N // 2]) if swiglu else js
    Yc, info_c = oracle.matmul_fused(X, What[rows], gamma=gamma, eps=1e-5, swiglu=swiglu,
                                     residual=None if R is None else np.ascontiguousarray(R[:, js]))
    check_fused(torch.from_numpy(np.ascontiguousarray(Y[:, js])), Yc, info_c, swiglu, norm, name + " prefill cols")


def test_fused_layer_in_a_hip_graph_matches_eager(e0m4):
    """Graph replays of the fused decode calls reproduce the eager results bit for bit."""
    G, N, K = 128, 27392, 4096
    stream = torch.cuda.Stream()
    W = synth_inputs.weights_device(N, K, 7300, DEV)
    codes, _, _ = e0m4.e0m4_quantize(W, G)
    del W
    x = synth_inputs.activations_device(1, K, 7301, DEV)
    gamma = to_dev(synth_inputs.norm_weight(K, 7302))
    r = to_dev(synth_inputs.residual(1, N // 2, 7303))
    y = torch.empty((1, N // 2), dtype=torch.float16, device=DEV)

    def call(out, st=None):
        return e0m4.e0m4_matmul_fused(x, codes, N, K, G, rms_gamma=gamma, rms_eps=1e-5,
                                      epilogue=e0m4.E0M4_EPILOGUE_SWIGLU, residual=r, out=out, stream=st)

    want = call(None).clone()
    torch.cuda.synchronize()
    with torch.cuda.stream(stream):
        call(y, stream)
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            call(y, stream)
    for replay in range(3):
        y.fill_(float("nan"))
        torch.cuda.synchronize()
        with torch.cuda.stream(stream):
            graph.replay()
        stream.synchronize()
        assert torch.equal(y, want), "replay %d" % replay
