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
KNOBS = ("gemv_waves", "gemv_workgroups", "gemv_mfma", "gemm_variant", "gemm_splits")


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


def quantized(e0m4, oracle, N, K, G, seed, row_std=None):
    W = synth_inputs.weights(N, K, seed=seed, row_std_range=row_std)
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
              in_place=False):
    codes, What = quantized(e0m4, oracle, N, K, G, seed, row_std)
    X = synth_inputs.activations(M, K, seed=seed, outlier_frac=0.01 if outliers else 0.0)
    gamma = synth_inputs.norm_weight(K, seed) if norm else None
    n_out = N // 2 if swiglu else N
    R = synth_inputs.residual(M, n_out, seed) if res else None
    eps = 1e-5
    out = None
    r_dev = to_dev(R)
    if in_place:
        out = r_dev                                     # the residual stream is updated in place
    Y = e0m4.e0m4_matmul_fused(to_dev(X), codes, N, K, G, rms_gamma=to_dev(gamma), rms_eps=eps,
                               epilogue=e0m4.E0M4_EPILOGUE_SWIGLU if swiglu else e0m4.E0M4_EPILOGUE_NONE,
                               residual=r_dev, out=out)
    Yref, info = oracle.matmul_fused(X, What, gamma=gamma, eps=eps, swiglu=swiglu, residual=R)
    torch.cuda.synchronize()
    what = "M=%d N=%d K=%d G=%d norm=%d swiglu=%d res=%d" % (M, N, K, G, norm, swiglu, res)
    check_fused(Y, Yref, info, swiglu, norm, what)
    return Y


COMBOS = [(True, False, False), (False, True, False), (False, False, True), (True, True, True), (True, False, True)]


@pytest.mark.parametrize("norm,swiglu,res", COMBOS)
@pytest.mark.parametrize("M", [1, 2, 5, 8])
def test_decode_kernel(e0m4, oracle, M, norm, swiglu, res):
    run_fused(e0m4, oracle, M, 320, 1152, 128, seed=300 + M, norm=norm, swiglu=swiglu, res=res)     # 9 k blocks, 10 pairs
    run_fused(e0m4, oracle, M, 1088, 4096, 128, seed=310 + M, norm=norm, swiglu=swiglu, res=res, outliers=True)


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


def test_decode_kernel_long_rows(e0m4, oracle):
    # 8 rows of K = 16384 are staged in several segments: the norm's row sums come from memory, and the
    # gated epilogue (which needs whole rows in LDS) is served by the GEMM kernels instead
    run_fused(e0m4, oracle, 8, 130, 16384, 128, seed=340, norm=True, res=True)
    run_fused(e0m4, oracle, 8, 128, 16384, 128, seed=341, norm=True, swiglu=True, res=True)
    run_fused(e0m4, oracle, 1, 192, 32768, 128, seed=342, norm=True, swiglu=True)


def test_nothing_selected_equals_the_plain_matmul(e0m4, oracle):
    for M in (1, 6, 40):
        codes, What = quantized(e0m4, oracle, 200, 1152, 128, seed=350 + M)
        X = to_dev(synth_inputs.activations(M, 1152, seed=350 + M))
        y0 = e0m4.e0m4_matmul(X, codes, None, None, 200, 1152, 128)
        e0m4.e0m4_set_knob("gemv_mfma", 1)              # the fused entry point uses the vector kernel for M <= 8
        try:
            y0v = e0m4.e0m4_matmul(X, codes, None, None, 200, 1152, 128)
        finally:
            e0m4.e0m4_set_knob("gemv_mfma", 0)
        y1 = e0m4.e0m4_matmul_fused(X, codes, 200, 1152, 128)
        torch.cuda.synchronize()
        assert torch.equal(y1, y0v), M
        Yref, absdot = oracle.matmul(X.cpu().numpy(), What)
        assert np.all(np.abs(y0.cpu().numpy().astype(np.float64) - Yref.astype(np.float64)) <= 1e-2 * np.maximum(1, absdot))


@pytest.mark.parametrize("variant", [1, 2])           # 1: small-tile kernel, 2: pipelined 256 x 256 kernel
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


@pytest.mark.parametrize("splits", [2, 3, 8])
@pytest.mark.parametrize("norm,swiglu,res", COMBOS)
def test_gemm_split_along_k(e0m4, oracle, splits, norm, swiglu, res):
    e0m4.e0m4_set_knob("gemm_variant", 2)
    e0m4.e0m4_set_knob("gemm_splits", splits)
    try:
        run_fused(e0m4, oracle, 257, 704, 1024, 128, seed=370 + splits, norm=norm, swiglu=swiglu, res=res)
    finally:
        e0m4.e0m4_set_knob("gemm_variant", 0)
        e0m4.e0m4_set_knob("gemm_splits", 0)


def test_gemm_small_kernel_ragged_k(e0m4, oracle):
    run_fused(e0m4, oracle, 70, 256, 416, 32, seed=380, norm=True, swiglu=True, res=True)      # K = 6.5 slices of 64


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
