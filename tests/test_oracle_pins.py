"""Pins for the CPU oracle: every check here compares the oracle with something
other than itself -- values the paper's formula fixes, closed forms, exact
rational arithmetic, exhaustive enumeration, brute force on tiny groups, or an
independent library conversion.  No GPU needed.

Paper passages: section "E0M4 FP4 quantization" (quantization paragraph,
dequantization formula, Figure 2 caption) and Table 2.
"""
from fractions import Fraction
import os

import numpy as np
import pytest

import synth_inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")

F16_ONE = 0x3C00
F16_TWO = 0x4000


def f16_bits(x) -> int:
    return int(np.array(x, dtype=np.float16).view(np.uint16))


def bits_f16(b) -> float:
    return float(np.array(b, dtype=np.uint16).view(np.float16))


# ---------------------------------------------------------------- conversions

def test_half_to_double_exhaustive_vs_numpy(oracle):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    ref = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.half_bits_to_double(int(b)) for b in bits])
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], ref[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(ref[~nan]))


def test_double_to_half_rne_vs_numpy_and_midpoints(oracle):
    rng = np.random.default_rng(1)
    vals = list(np.ldexp(rng.uniform(-2, 2, 20000), rng.integers(-28, 18, 20000)))
    # every midpoint between consecutive positive halves and its two neighbours in fp64
    hb = np.arange(0, 0x7C00, 37, dtype=np.uint16)
    lo = hb.view(np.float16).astype(np.float64)
    hi = (hb + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    hi[np.isinf(hi)] = 65536.0
    mid = (lo + hi) / 2
    for v in (mid, np.nextafter(mid, 0), np.nextafter(mid, np.inf)):
        vals += list(v) + list(-v)
    vals += [0.0, -0.0, 65504.0, 65519.99, 65520.0, 65536.0, 1e9, 2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * 1.0001,
             2.0 ** -14, np.nextafter(2.0 ** -14, 0), 1.0 / 3.0]
    vals = np.array(vals, dtype=np.float64)
    with np.errstate(over="ignore"):
        ref = vals.astype(np.float16).view(np.uint16)
    got = np.array([oracle.double_to_half_bits(float(v)) for v in vals], dtype=np.uint16)
    assert np.array_equal(got, ref)


# ---------------------------------------------------------------- dequant

def test_code_table_matches_paper_formula(oracle):
    rows = [l.split() for l in open(os.path.join(GOLDEN, "e0m4_code_table.txt")) if l.strip() and l[0] != "#"]
    assert len(rows) == 16
    for c, hx, val in rows:
        c = int(c)
        assert oracle.w1_bits(c) == int(hx, 16)
        assert bits_f16(oracle.w1_bits(c)) == float(val) == 2 + c / 8
        # the two bitwise operations of the paper's formula
        assert oracle.w1_bits(c) == (0x4000 | (c << 6))


def test_decode_is_affine_exact_rational(oracle):
    """(w1 - bias) * scale with one rounding: compare against exact rational arithmetic."""
    rng = np.random.default_rng(2)
    scales = np.concatenate([rng.integers(0x0400, 0x7BFF, 300), [0x0400, 0x3C00, 0x7BFF, 0x2000, 0x0001, 0x03FF]])
    for sb in scales:
        s = Fraction(bits_f16(sb))
        for z in range(16):
            bb = 0x4000 | (z << 6)
            for c in range(16):
                exact = (Fraction(2) + Fraction(c, 8) - (Fraction(2) + Fraction(z, 8))) * s
                with np.errstate(over="ignore"):
                    want = f16_bits(np.float64(exact.numerator) / np.float64(exact.denominator))
                # numerator/denominator are small exact integers -> the fp64 quotient is exact
                assert oracle.decode_one(c, int(sb), bb) == want, (hex(sb), z, c)


def test_decode_monotone_in_code(oracle):
    rng = np.random.default_rng(3)
    for sb in rng.integers(0x0400, 0x7000, 200):
        for z in (0, 5, 15):
            bb = 0x4000 | (z << 6)
            v = [bits_f16(oracle.decode_one(c, int(sb), bb)) for c in range(16)]
            assert all(v[i] <= v[i + 1] for i in range(15))
            assert v[z] == 0.0


# ---------------------------------------------------------------- code extraction / rounding rule

def test_rounding_rule_exhaustive_over_binade(oracle):
    """All 1024 fp16 values of [2,4): code = round-half-up((v-2)*8) saturated at 15."""
    for b in range(0x4000, 0x4400):
        v = bits_f16(b)
        w0 = v - 2.0                                  # exactly representable in fp16
        assert bits_f16(f16_bits(w0)) == w0
        c = oracle.encode_one(f16_bits(w0), F16_ONE, F16_TWO)
        want = min(int(np.floor((v - 2.0) * 8 + 0.5)), 15)
        assert c == want, hex(b)
        # bit view of the same rule: four highest fraction bits plus the fifth
        assert c == min(((b >> 6) & 15) + ((b >> 5) & 1), 15)
        assert oracle.forward_bits(f16_bits(w0), F16_ONE, F16_TWO) == b


def test_forward_map_shares_sign_and_exponent(oracle):
    rng = np.random.default_rng(4)
    w = rng.integers(0, 65536, 20000).astype(np.uint16)
    w = w[np.isfinite(w.view(np.float16))]
    sb = rng.integers(0x0400, 0x7BFF, w.size)
    z = rng.integers(0, 16, w.size)
    for wi, si, zi in zip(w[:5000], sb, z):
        fb = oracle.forward_bits(int(wi), int(si), 0x4000 | (int(zi) << 6))
        assert fb >> 10 == 16, (hex(wi), hex(si), zi, hex(fb))   # sign 0, exponent field 16


# ---------------------------------------------------------------- fit

def _fit_exact_reference(w0: np.ndarray):
    """Independent statement of the fit in exact rationals (single roundings where the
    definition has them): returns (scale_bits, acceptable bias bit patterns)."""
    vals = [Fraction(float(v)) for v in w0]
    mn = min([Fraction(0)] + vals)
    mx = max([Fraction(0)] + vals)
    span = Fraction(0x43FF - 0x4000, 512)            # (4 - 2^-9) - 2
    s_exact = (mx - mn) / span
    return mn, mx, s_exact


def test_fit_scale_and_bias_against_exact_rationals(oracle):
    rng = np.random.default_rng(5)
    for trial in range(400):
        G = int(rng.choice([2, 4, 8, 64, 128]))
        std = float(rng.choice([1e-3, 0.02, 1.0, 50.0]))
        w0 = (rng.standard_normal(G) * std).astype(np.float16)
        if trial % 7 == 0:
            w0 = np.abs(w0)                          # one-signed group: range still contains 0
        if trial % 11 == 0:
            w0 = -np.abs(w0)
        sb, bb = oracle.fit_group(w0)
        mn, mx, s_exact = _fit_exact_reference(w0)
        s = Fraction(bits_f16(sb))
        # scale: fp32 divide then fp16 rounding -> within one fp16 ulp-half of the exact quotient
        if s_exact >= Fraction(1, 2 ** 14):
            assert abs(s - s_exact) <= s_exact * Fraction(1, 2 ** 11) * Fraction(1001, 1000)
        else:
            assert sb == 0x0400
        assert bb & 0x3F == 0 and (bb >> 10) == 16   # bias = 2 + z/8
        z = (bb >> 6) & 15
        # bias is the truncation (to eighths) of the image of zero, 2 - min/scale, clamped to the binade
        b_exact = min(max(Fraction(2) - mn / s, Fraction(2)), Fraction(2047, 512))
        z_floor = int((b_exact - 2) * 8)
        assert z in (z_floor, min(z_floor + 1, 15), max(z_floor - 1, 0))
        # and exactly floor unless b_exact is within rounding distance of a multiple of 1/8
        frac = (b_exact - 2) * 8 - z_floor
        if Fraction(1, 64) < frac < Fraction(63, 64):
            assert z == min(z_floor, 15)


def test_fit_closed_form_symmetric_group(oracle):
    # range [-1, 1]: scale = fp16(2 / 1.998046875), bias = trunc_8ths(2 + 1/scale)
    w0 = np.array([-1.0, 1.0, 0.25, -0.5], dtype=np.float16)
    sb, bb = oracle.fit_group(w0)
    s_exact = Fraction(2) / Fraction(1023, 512)
    assert sb == f16_bits(float(s_exact))
    s = Fraction(bits_f16(sb))
    assert s == Fraction(1025, 1024)
    # image of zero: 2 + 1024/1025 = 2.99902..., just above the midpoint 2.9990234375 between the
    # fp16 neighbours 2.998046875 and 3.0 -> the fp16 bias is 3.0, whose low fraction bits are already zero
    b16 = Fraction(bits_f16(f16_bits(float(2 + 1 / s))))
    assert b16 == 3
    assert bb == 0x4200


def test_bias_truncates_not_rounds(oracle):
    # range [-0.9, 1.1]: image of zero = 2 + 0.9/scale = 2.899..., i.e. 7.19 eighths -> z = 7;
    # range [-0.98, 1.02]: 2 + 0.979 -> 7.83 eighths: truncation keeps 7 where rounding would give 8
    for lo, hi, z_want in ((-0.9, 1.1, 7), (-0.98, 1.02, 7), (-0.3, 1.7, 2)):
        w0 = np.array([lo, hi, 0.0, 0.1], dtype=np.float16)
        sb, bb = oracle.fit_group(w0)
        s = Fraction(bits_f16(sb))
        img = (Fraction(2) - Fraction(float(w0[0])) / s - 2) * 8
        assert int(img) == z_want and bb == 0x4000 | (z_want << 6), (float(img), hex(bb))


# ---------------------------------------------------------------- round trip, nearest code, error bound

def test_fixed_parameter_round_trip_exhaustive(oracle):
    """encode(decode(c)) == c for every normal positive fp16 scale x 16 biases x 16 codes."""
    sb = np.arange(0x0400, 0x7C00, dtype=np.uint16)              # 30720 normal scales
    zz = np.arange(16, dtype=np.uint16)
    scales = np.repeat(sb, 16)[:, None]                           # [N,1], N = 30720*16
    bias = np.tile((0x4000 | (zz << 6)).astype(np.uint16), sb.size)[:, None]
    codes = np.tile(np.arange(16, dtype=np.uint8), (scales.shape[0], 1))
    with np.errstate(over="ignore"):
        What = oracle.dequant(codes, scales, bias, 16)
    finite = np.isfinite(What)
    assert finite.mean() > 0.9
    back = oracle.encode(What, scales, bias, 16)
    assert np.array_equal(back[finite], codes[finite])
    # hence dequant(quant(dequant(c))) == dequant(c) at fixed parameters
    again = oracle.dequant(back, scales, bias, 16)
    assert np.array_equal(again.view(np.uint16)[finite], What.view(np.uint16)[finite])


def _unclamped(w0, s, b):
    t = w0.astype(np.float64) / s + b
    return (t >= 2.0) & (t <= 4 - 2.0 ** -9)


@pytest.mark.parametrize("G", [2, 4, 8])
def test_brute_force_nearest_code_tiny_groups(oracle, G):
    rng = np.random.default_rng(100 + G)
    W = (rng.standard_normal((3000, G)) * 0.02).astype(np.float16)
    codes, scales, bias = oracle.quantize(W, G)
    s = scales.astype(np.float64)
    b = bias.astype(np.float64)
    levels = (2.0 + np.arange(16) / 8.0)[None, None, :]             # w1 of every code
    cand = (levels - b[:, :, None]) * s[:, :, None]                 # exact in fp64
    w = W.astype(np.float64)[:, :, None]
    best = np.abs(w - cand).min(axis=2)
    chosen = np.abs(w[:, :, 0] - np.take_along_axis(cand, codes[:, :, None].astype(np.int64), 2)[:, :, 0])
    step = s / 8.0
    ok = np.ones_like(W, dtype=bool)       # clamped elements take the end codes, which are nearest too
    assert 0.3 < _unclamped(W, s, b).mean() < 1.0
    # double rounding (fp32 -> fp16 -> 4 bit) may pick the other neighbour only within 1/32 step of a tie
    assert (chosen[ok] <= best[ok] + step.repeat(G, 1)[ok] / 32 + 1e-12).all()
    # and for the vast majority the chosen code is exactly the nearest one
    assert (chosen[ok] <= best[ok] + 1e-15).mean() > 0.97


def test_error_bound_closed_form(oracle):
    W = synth_inputs.weights(256, 1024, seed=7)
    for G in (64, 128):
        codes, scales, bias = oracle.quantize(W, G)
        What = oracle.dequant(codes, scales, bias, G).astype(np.float64)
        s = np.repeat(scales.astype(np.float64), G, axis=1)
        b = np.repeat(bias.astype(np.float64), G, axis=1)
        w = W.astype(np.float64)
        t = w / s + b
        err = np.abs(w - What)
        ulp_slop = np.abs(What) * 2.0 ** -11 + 2.0 ** -25
        inner = (t >= 2.0) & (t < 3.9375)
        top = (t >= 3.9375) & (t <= 4 - 2.0 ** -9)
        assert inner.mean() > 0.95
        assert (err[inner] <= (1 / 16 + 2.0 ** -10 + 1e-6) * s[inner] + ulp_slop[inner]).all()
        assert (err[top] <= (1 / 8) * s[top] + ulp_slop[top]).all()
        # clamped elements (below the binade after the bias was truncated) lose at most one step
        low = t < 2.0
        assert (err[low] <= (1 / 8 + 1e-6) * s[low] + ulp_slop[low]).all()
        assert (codes[low] == 0).all()


def test_codes_monotone_within_group(oracle):
    W = synth_inputs.weights(64, 512, seed=8)
    codes, _, _ = oracle.quantize(W, 128)
    Wg = W.reshape(64, 4, 128).astype(np.float64)
    cg = codes.reshape(64, 4, 128)
    order = np.argsort(Wg, axis=2, kind="stable")
    sorted_codes = np.take_along_axis(cg, order, 2).astype(np.int64)
    assert (np.diff(sorted_codes, axis=2) >= 0).all()


def test_quantize_groups_are_independent_and_match_scalar_path(oracle):
    rng = np.random.default_rng(9)
    N, K, G = 6, 512, 128
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float16)
    W[:, 128:256] *= np.float16(30.0)                               # one group far larger than its neighbours
    codes, scales, bias = oracle.quantize(W, G)
    for n in range(N):
        for g in range(K // G):
            grp = W[n, g * G:(g + 1) * G]
            sb, bb = oracle.fit_group(grp)
            assert scales.view(np.uint16)[n, g] == sb and bias.view(np.uint16)[n, g] == bb
            rng_g = float(max(grp.max(), 0)) - float(min(grp.min(), 0))
            assert abs(float(scales[n, g]) - rng_g / 1.998046875) <= rng_g * 1e-3
            for k in range(0, G, 17):
                assert codes[n, g * G + k] == oracle.encode_one(int(grp.view(np.uint16)[k]), sb, bb)
    assert scales[:, 1].astype(np.float64).min() > 5 * scales[:, 0].astype(np.float64).max()


# ---------------------------------------------------------------- Table 2 statistic

def _int4_asym_dequant(W: np.ndarray, G: int) -> np.ndarray:
    """Comparison format (not defined by the paper; stated assumption): asymmetric min/max
    INT4, 15 steps, rounded integer zero-point, round-to-nearest."""
    N, K = W.shape
    w = W.astype(np.float64).reshape(N, K // G, G)
    mn = np.minimum(w.min(axis=2, keepdims=True), 0)
    mx = np.maximum(w.max(axis=2, keepdims=True), 0)
    scale = (mx - mn) / 15.0
    scale[scale == 0] = 1.0
    zp = np.clip(np.round(-mn / scale), 0, 15)
    q = np.clip(np.round(w / scale) + zp, 0, 15)
    return ((q - zp) * scale).reshape(N, K)


def test_table2_mae_ratio_on_gaussian_weights(oracle):
    ratios = [float(l.split()[1]) for l in open(os.path.join(GOLDEN, "table2_mae_ratio.txt"))
              if l.strip() and l[0] != "#"]
    assert min(ratios) == 0.955 and max(ratios) == 0.957
    W = synth_inputs.weights(5000, 512, seed=10)                    # 20 000 groups of 128
    codes, scales, bias = oracle.quantize(W, 128)
    What = oracle.dequant(codes, scales, bias, 128).astype(np.float64)
    w = W.astype(np.float64)
    mae_e0m4 = np.abs(w - What).mean()
    mae_int4 = np.abs(w - _int4_asym_dequant(W, 128)).mean()
    ratio = mae_e0m4 / mae_int4
    assert min(ratios) - 0.003 <= ratio <= max(ratios) + 0.003, ratio


# ---------------------------------------------------------------- matmul

def test_matmul_tiny_exact_rational(oracle):
    rng = np.random.default_rng(11)
    for _ in range(40):
        M, N, K = int(rng.integers(1, 4)), int(rng.integers(1, 5)), int(rng.integers(1, 17))
        X = rng.standard_normal((M, K)).astype(np.float16)
        Wh = (rng.standard_normal((N, K)) * 0.05).astype(np.float16)
        Y, absdot = oracle.matmul(X, Wh)
        for m in range(M):
            for n in range(N):
                ex = sum(Fraction(float(X[m, k])) * Fraction(float(Wh[n, k])) for k in range(K))
                ea = sum(abs(Fraction(float(X[m, k])) * Fraction(float(Wh[n, k]))) for k in range(K))
                # fp64 accumulation of <=16 products of 11-bit numbers is exact here
                assert Y.view(np.uint16)[m, n] == f16_bits(float(ex))
                assert absdot[m, n] == float(ea)


def test_matmul_operand_orientation_and_special_inputs(oracle):
    rng = np.random.default_rng(12)
    M, N, K = 3, 7, 96
    X = rng.standard_normal((M, K)).astype(np.float16)
    Wh = (rng.standard_normal((N, K)) * 0.05).astype(np.float16)
    Y, absdot = oracle.matmul(X, Wh)
    assert Y.shape == (M, N) and absdot.shape == (M, N)
    ref = X.astype(np.float64) @ Wh.astype(np.float64).T
    assert np.array_equal(Y, ref.astype(np.float16))
    # one-hot activations pick out columns of What (rows of the weight matrix) bit-exactly
    E = np.zeros((2, K), dtype=np.float16)
    E[0, 5] = 1.0
    E[1, K - 1] = 1.0
    Y1, _ = oracle.matmul(E, Wh)
    assert np.array_equal(Y1[0].view(np.uint16), Wh[:, 5].view(np.uint16))
    assert np.array_equal(Y1[1].view(np.uint16), Wh[:, K - 1].view(np.uint16))
    # all-ones activations give the row sums
    ones = np.ones((1, K), dtype=np.float16)
    Y2, a2 = oracle.matmul(ones, Wh)
    assert np.array_equal(Y2[0], Wh.astype(np.float64).sum(axis=1).astype(np.float16))
    assert np.allclose(a2[0], np.abs(Wh.astype(np.float64)).sum(axis=1), rtol=1e-14)


def test_factored_form_is_within_tolerance_of_definition(oracle):
    """sum_g scale_g (sum x w1 - bias_g sum x) equals the definition up to the fp16 rounding of the
    dequantised weights: the identity the GPU kernels rely on."""
    G, K, N = 128, 1024, 32
    W = synth_inputs.weights(N, K, seed=13)
    X = synth_inputs.activations(2, K, seed=13)
    codes, scales, bias = oracle.quantize(W, G)
    What = oracle.dequant(codes, scales, bias, G)
    Y, absdot = oracle.matmul(X, What)
    w1 = 2.0 + codes.astype(np.float64) / 8.0
    x = X.astype(np.float64)
    acc = np.zeros((2, N))
    for g in range(K // G):
        sl = slice(g * G, (g + 1) * G)
        xs = x[:, sl].sum(axis=1)
        acc += scales[:, g].astype(np.float64)[None, :] * (x[:, sl] @ w1[:, sl].T
                                                             - bias[:, g].astype(np.float64)[None, :] * xs[:, None])
    exact_def = x @ What.astype(np.float64).T
    assert (np.abs(acc - exact_def) <= 2.0 ** -11 * absdot + 1e-12).all()


# ------------------------------------------------------------------ INT4 comparison format
# (paper: section "Evaluation of FP4 quantization".  The paper does not define its INT4 quantiser;
# the oracle's is the stated reading: asymmetric min/max, 15 steps, integer zero point, nearest.)

def test_int4_decode_is_the_e0m4_decoder_with_mapped_parameters(oracle):
    """(q - z) * s == ((2 + q/8) - (2 + z/8)) * (8 s): an INT4 group with integer zero point is an E0M4
    group with bias 2 + z/8 and scale 8 s, so the two decoders must agree bit for bit."""
    scale_bits = list(range(0x0400, 0x6C00, 37)) + [0x0400, 0x6BFF]          # 8 s stays finite
    for sb in scale_bits:
        s8 = oracle.double_to_half_bits(8.0 * oracle.half_bits_to_double(sb))
        assert oracle.half_bits_to_double(s8) == 8.0 * oracle.half_bits_to_double(sb)
        for z in range(16):
            zb = oracle.double_to_half_bits(float(z))
            bias_bits = 0x4000 | (z << 6)
            for q in range(16):
                assert oracle.int4_decode_one(q, sb, zb) == oracle.decode_one(q, s8, bias_bits), (sb, z, q)


def test_int4_code_is_the_nearest_level_by_brute_force(oracle):
    rng = np.random.default_rng(5)
    for G in (2, 4, 8, 32):
        W = (rng.standard_normal((400, G)) * rng.choice([1e-3, 0.02, 1.0, 300.0], (400, 1))).astype(np.float16)
        W[::7] = np.abs(W[::7])                                 # one-signed groups
        W[::11, 0] = 0.0
        codes, scales, zeros = oracle.int4_quantize(W, G)
        s = scales.astype(np.float64)
        z = zeros.astype(np.float64)
        assert ((z >= 0) & (z <= 15) & (z == np.round(z))).all()
        w = W.astype(np.float64)
        levels = (np.arange(16)[None, None, :] - z[:, :, None]) * s[:, :, None]       # [N, 1, 16]
        err = np.abs(w[:, :, None] - levels)                                             # [N, G, 16]
        chosen = np.take_along_axis(err, codes[:, :, None].astype(np.int64), axis=2)[:, :, 0]
        # nearest up to the fp32 rounding of w/s (a tie may go either way)
        assert (chosen <= err.min(axis=2) + 1e-6 * s).all()


def test_int4_invariants(oracle):
    W = synth_inputs.weights(64, 512, seed=12)
    W[3, 5] = 0.0
    W[9] = 0.0                                                  # all-zero row
    W[10] = np.float16(0.25)                                    # constant row
    for G in (32, 128):
        codes, scales, zeros = oracle.int4_quantize(W, G)
        What = oracle.int4_dequant(codes, scales, zeros, G)
        assert codes.max() <= 15
        g = 5 // G
        assert codes[3, 5] == int(zeros[3, g]) and What[3, 5] == 0          # an exact zero stays exactly zero
        assert not What[9].any()
        s = np.repeat(scales.astype(np.float64), G, axis=1)
        err = np.abs(W.astype(np.float64) - What.astype(np.float64))
        assert (err <= 1.0 * s + 1e-12).all()                    # ends of the range may clamp by up to a step
        assert np.median(err / s) < 0.3                          # typical error: a quarter of a step
        # monotone: larger weight, not smaller code (within a group)
        for n in (0, 17):
            w = W[n, :G].astype(np.float64)
            order = np.argsort(w, kind="stable")
            assert (np.diff(codes[n, :G][order].astype(int)) >= 0).all()


def test_int4_fit_scale_and_zero_point_against_exact_rationals(oracle):
    """The INT4 fit, group by group, against the stated definition in exact rationals: scale is the fp16
    rounding of (max - min)/15 over the range extended to 0; zero is round-half-to-even of -min/scale with the
    STORED fp16 scale, clamped to 0..15.  A fit that rounded half up, used the unrounded scale, forgot the
    extension to 0 or the clamp fails here."""
    def fit(w0):
        w0 = np.asarray(w0, dtype=np.float16)
        _, sc, ze = oracle.int4_quantize(w0.reshape(1, -1), w0.size)
        return Fraction(float(sc[0, 0])), int(ze[0, 0]), float(ze[0, 0])

    def rne(x: Fraction) -> int:
        f = x.numerator // x.denominator
        r = x - f
        if r > Fraction(1, 2) or (r == Fraction(1, 2) and f % 2 == 1):
            f += 1
        return f

    # hand-made groups whose scale is exactly 1: zero = rne(-min)
    for w0, z_want in (([-2.5, 12.5, 0.0, 1.0], 2),           # tie: half to even, not half up
                       ([-3.5, 11.5, 0.0, 1.0], 4),           # tie the other way
                       ([-15.0, -1.0, -2.0, -3.0], 15),       # all negative: range extended to 0, zero at the top
                       ([15.0, 1.0, 2.0, 3.0], 0),            # all positive: zero at the bottom
                       ([-7.25, 7.75, 0.0, 1.0], 7), ([-7.75, 7.25, 0.5, 1.0], 8)):
        s, z, zf = fit(w0)
        assert s == 1 and z == z_want and zf == z_want, (w0, s, zf)
    rng = np.random.default_rng(17)
    exact_checked = 0
    for trial in range(600):
        G = int(rng.choice([2, 4, 8, 64, 128]))
        std = float(rng.choice([1e-3, 0.02, 1.0, 50.0]))
        w0 = (rng.standard_normal(G) * std).astype(np.float16)
        if trial % 7 == 0:
            w0 = np.abs(w0)
        if trial % 11 == 0:
            w0 = -np.abs(w0)
        s, z, zf = fit(w0)
        vals = [Fraction(float(v)) for v in w0]
        mn, mx = min([Fraction(0)] + vals), max([Fraction(0)] + vals)
        s_exact = (mx - mn) / 15
        if s_exact >= Fraction(1, 2 ** 14):         # fp32 divide, then fp16 rounding: half an fp16 ulp (and a bit)
            assert abs(s - s_exact) <= s_exact * Fraction(1, 2 ** 11) * Fraction(1001, 1000)
        else:
            assert s == Fraction(1, 2 ** 14)
        assert zf == z and 0 <= z <= 15
        z_exact = -mn / s                           # with the stored scale
        want = min(max(rne(z_exact), 0), 15)
        frac = z_exact - (z_exact.numerator // z_exact.denominator)
        if abs(frac - Fraction(1, 2)) > Fraction(1, 2 ** 18):    # away from a tie the fp32 quotient cannot change the result
            assert z == want, (trial, float(z_exact), z)
            exact_checked += 1
        else:
            assert abs(z - z_exact) <= Fraction(1, 2) + Fraction(1, 2 ** 18)
    assert exact_checked > 550


def test_int4_agrees_with_the_plain_float64_definition_in_distribution(oracle):
    W = synth_inputs.weights(2000, 512, seed=13)
    codes, scales, zeros = oracle.int4_quantize(W, 128)
    What = oracle.int4_dequant(codes, scales, zeros, 128).astype(np.float64)
    w = W.astype(np.float64)
    mae_oracle = np.abs(w - What).mean()
    mae_plain = np.abs(w - _int4_asym_dequant(W, 128)).mean()   # float64, unrounded scale
    assert abs(mae_oracle / mae_plain - 1.0) < 0.005


def test_table2_mae_ratio_with_the_oracle_int4(oracle):
    W = synth_inputs.weights(5000, 512, seed=10)
    w = W.astype(np.float64)
    c, s, b = oracle.quantize(W, 128)
    mae_e0m4 = np.abs(w - oracle.dequant(c, s, b, 128).astype(np.float64)).mean()
    q, s4, z4 = oracle.int4_quantize(W, 128)
    mae_int4 = np.abs(w - oracle.int4_dequant(q, s4, z4, 128).astype(np.float64)).mean()
    assert abs(mae_e0m4 / mae_int4 - 0.955) <= 0.004


# ---------------------------------------------------------------------------------------------------
# Operators fused around the matmul (paper: section "Operator and lagging optimizations").  The oracle
# writes the textbook formulas in numpy; the pins tie them to closed forms and to torch's own CPU
# routines (an independent implementation), and the fused function to the composition of those.
# ---------------------------------------------------------------------------------------------------

def test_silu_closed_forms_and_library(oracle):
    import torch
    g = np.concatenate([np.linspace(-30, 30, 2001), [-800.0, 800.0, 0.0, -0.0]])
    s = oracle.silu(g)
    assert np.all(np.isfinite(s))
    assert s[-2] == 0.0 and s[-1] == 0.0
    np.testing.assert_allclose(s - oracle.silu(-g), g, rtol=0, atol=1e-12)         # silu(g) - silu(-g) = g
    assert s[-4] == 0.0 and s[-3] == 800.0                                          # tails: 0 and the identity
    # the one minimum of g*sigmoid(g): the derivative vanishes where g0 = -(1 + exp(g0)) = -1.2784645...,
    # and the value there is g0 + 1 = -exp(g0)
    fine = np.linspace(-1.3, -1.25, 200001)
    i = np.argmin(oracle.silu(fine))
    assert abs(fine[i] - (-1.2784645)) < 1e-5 and abs(oracle.silu(fine)[i] - (-0.2784645)) < 1e-7
    g0 = -1.0
    for _ in range(60):
        g0 = -(1.0 + np.exp(g0))
    assert abs(oracle.silu(np.array([g0]))[0] - (g0 + 1.0)) < 1e-15
    ref = torch.nn.functional.silu(torch.from_numpy(g)).numpy()
    np.testing.assert_allclose(s, ref, rtol=1e-14, atol=1e-300)


def test_rmsnorm_invariants_and_library(oracle):
    import torch
    rng = np.random.default_rng(5)
    X = rng.standard_normal((7, 96)).astype(np.float16)
    gamma = (1.0 + 0.2 * rng.standard_normal(96)).astype(np.float16)
    y = oracle.rmsnorm(X, gamma, 0.0)
    # with eps = 0 the normalised rows have mean square 1 before gamma, and scaling a row changes nothing
    np.testing.assert_allclose(np.mean((y / gamma.astype(np.float64)) ** 2, axis=1), 1.0, rtol=1e-13)
    np.testing.assert_allclose(oracle.rmsnorm((X * np.float16(4)).astype(np.float16), gamma, 0.0), y, rtol=1e-13)
    # eps sits inside the square root, next to the mean (not the sum) of squares
    x1 = np.full((1, 4), 2.0, np.float16)
    np.testing.assert_allclose(oracle.rmsnorm(x1, np.ones(4, np.float16), 5.0), np.full((1, 4), 2.0 / 3.0), rtol=1e-15)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(X.astype(np.float64)), (96,),
                                       torch.from_numpy(gamma.astype(np.float64)), 1e-5).numpy()
    np.testing.assert_allclose(oracle.rmsnorm(X, gamma, 1e-5), ref, rtol=1e-13)


def test_matmul_fused_reduces_to_the_plain_matmul(oracle):
    rng = np.random.default_rng(6)
    X = rng.standard_normal((3, 64)).astype(np.float16)
    W = rng.standard_normal((10, 64)).astype(np.float16)
    Y, info = oracle.matmul_fused(X, W)
    Yp, absdot = oracle.matmul(X, W)
    assert np.array_equal(Y.view(np.uint16), Yp.view(np.uint16))
    np.testing.assert_allclose(info["absdot"], absdot, rtol=1e-13)


def test_matmul_fused_is_the_composition_of_library_operators(oracle):
    import torch
    rng = np.random.default_rng(7)
    M, N, K = 5, 24, 128
    X = (3.0 * rng.standard_normal((M, K))).astype(np.float16)
    W = (0.1 * rng.standard_normal((N, K))).astype(np.float16)
    gamma = (1.0 + 0.3 * rng.standard_normal(K)).astype(np.float16)
    R = rng.standard_normal((M, N // 2)).astype(np.float16)
    Y, info = oracle.matmul_fused(X, W, gamma=gamma, eps=1e-5, swiglu=True, residual=R)
    t = lambda a: torch.from_numpy(np.asarray(a).astype(np.float64))
    xn = torch.nn.functional.rms_norm(t(X), (K,), t(gamma), 1e-5).to(torch.float16).to(torch.float64)
    a = torch.nn.functional.linear(xn, t(W))
    gate, up = torch.chunk(a, 2, dim=-1)                    # first half of the rows is the gate
    y = torch.nn.functional.silu(gate) * up + t(R)
    np.testing.assert_allclose(info["y"], y.numpy(), rtol=1e-12, atol=1e-13)
    assert np.array_equal(Y.view(np.uint16), y.to(torch.float16).numpy().view(np.uint16))
    # the two halves are not interchangeable, and the residual is added after the product
    W_swapped = np.concatenate([W[N // 2:], W[: N // 2]])
    Ys, _ = oracle.matmul_fused(X, W_swapped, gamma=gamma, eps=1e-5, swiglu=True, residual=R)
    assert not np.array_equal(Ys, Y)


def test_matmul_fused_special_cases(oracle):
    rng = np.random.default_rng(8)
    M, Nh, K = 2, 6, 32
    X = rng.standard_normal((M, K)).astype(np.float16)
    Wg = rng.standard_normal((Nh, K)).astype(np.float16)
    # up rows that make a[m, Nh + j] = sum of x: one-hot-free check that gate and up meet at the same j
    Wu = np.ones((Nh, K), np.float16)
    Y, info = oracle.matmul_fused(X, np.concatenate([Wg, Wu]), swiglu=True)
    sx = X.astype(np.float64).sum(axis=1, keepdims=True)
    g = X.astype(np.float64) @ Wg.astype(np.float64).T
    np.testing.assert_allclose(info["y"], oracle.silu(g) * sx, rtol=1e-13)
    # residual only: one rounding of the exact sum
    R = rng.standard_normal((M, 2 * Nh)).astype(np.float16)
    Yr, info_r = oracle.matmul_fused(X, np.concatenate([Wg, Wu]), residual=R)
    np.testing.assert_allclose(info_r["y"], info_r["a"] + R.astype(np.float64), rtol=0, atol=0)
    assert np.array_equal(Yr, (info_r["a"] + R.astype(np.float64)).astype(np.float16))
    # gamma = 1, eps = 0 on rows of equal magnitude: the norm divides by that magnitude
    Xc = np.where(rng.random((M, K)) < 0.5, -3.0, 3.0).astype(np.float16)
    Yn, info_n = oracle.matmul_fused(Xc, Wg, gamma=np.ones(K, np.float16), eps=0.0)
    np.testing.assert_allclose(info_n["a"], (Xc.astype(np.float64) / 3.0) @ Wg.astype(np.float64).T, rtol=1e-13)


# ---------------------------------------------------------------------------------------------------
# KV-cache append (paper: section "KV cache copy optimization"): writing the new rows at consecutive
# positions of the one big tensor must give what concatenating old cache and new rows gives.
# ---------------------------------------------------------------------------------------------------

def test_kv_append_equals_concatenation(oracle):
    rng = np.random.default_rng(11)
    max_seq, row, have, n_new = 40, 24, 17, 5
    old = rng.standard_normal((have, row)).astype(np.float16)
    new = rng.standard_normal((n_new, row)).astype(np.float16)
    cache = np.full((max_seq, row), np.float16(-7.0))
    cache[:have] = old
    out = oracle.kv_append(cache, new, np.arange(have, have + n_new))
    assert np.array_equal(out[: have + n_new], np.concatenate([old, new]))          # the operator it replaces
    assert np.array_equal(out[have + n_new:], cache[have + n_new:])                  # the rest is untouched
    assert np.array_equal(cache[have], np.full(row, np.float16(-7.0)))               # the input is not modified
    # arbitrary positions: row i lands at position_ids[i] and nowhere else; out-of-range rows are dropped
    pos = np.array([3, 39, 0, 40, -1])
    out2 = oracle.kv_append(cache, new, pos)
    for i, p in enumerate(pos):
        if 0 <= p < max_seq:
            assert np.array_equal(out2[p], new[i])
    untouched = [p for p in range(max_seq) if p not in (3, 39, 0)]
    assert np.array_equal(out2[untouched], cache[untouched])
    # decode: one row at a time, step after step, builds the same cache as one prefill-sized append
    step = cache
    for i in range(n_new):
        step = oracle.kv_append(step, new[i:i + 1], np.array([have + i]))
    assert np.array_equal(step, out)


# ---------------------------------------------------------------------------------------------------
# Other code widths, E0Mk (paper: closing remark of the section "E0M4 FP4 quantization").  The generic
# functions are written out separately in the oracle; at k = 4 they must be the E0M4 functions bit for
# bit, and for every k the rounding rule, the levels, nearest-level choice and the error bound are
# checked against their definitions.
# ---------------------------------------------------------------------------------------------------

def test_e0mk_at_four_bits_is_e0m4(oracle):
    W = synth_inputs.weights(64, 512, seed=21)
    W[0, :8] = [0.0, -0.0, 65504.0, -65504.0, 6e-8, -6e-8, 1.0, -1.0]
    for G in (32, 128):
        c4, s4, b4 = oracle.quantize(W, G)
        ck, sk, bk = oracle.quantize_k(W, G, 4)
        assert np.array_equal(c4, ck)
        assert np.array_equal(s4.view(np.uint16), sk.view(np.uint16))
        assert np.array_equal(b4.view(np.uint16), bk.view(np.uint16))
        assert np.array_equal(oracle.dequant(c4, s4, b4, G).view(np.uint16),
                              oracle.dequant_k(ck, sk, bk, G, 4).view(np.uint16))
    for c in range(16):
        assert oracle.w1_bits_k(c, 4) == oracle.w1_bits(c)


@pytest.mark.parametrize("bits", [1, 2, 3, 5, 8])
def test_e0mk_levels_and_rounding_rule_exhaustive(oracle, bits):
    top = (1 << bits) - 1
    # the 2^k levels are 2 + c / 2^(k-1): uniform over the binade, the paper's shift-and-or with 10 - k
    for c in range(top + 1):
        assert oracle.w1_bits_k(c, bits) == (0x4000 | (c << (10 - bits)))
        assert Fraction(bits_f16(oracle.w1_bits_k(c, bits))) == 2 + Fraction(c, 1 << (bits - 1))
    # all 1024 fp16 values of [2,4) under scale 1, bias 2: round half up in units of the step, saturated
    for b in range(0x4000, 0x4400):
        v = bits_f16(b)
        c = oracle.encode_one_k(f16_bits(v - 2.0), F16_ONE, F16_TWO, bits)
        assert c == min(int(np.floor((v - 2.0) * (1 << (bits - 1)) + 0.5)), top), hex(b)
        assert c == min(((b >> (10 - bits)) & top) + ((b >> (9 - bits)) & 1), top)


@pytest.mark.parametrize("bits", [2, 3, 8])
def test_e0mk_nearest_level_and_error_bound(oracle, bits):
    rng = np.random.default_rng(200 + bits)
    G = 8
    W = (rng.standard_normal((2000, G)) * 0.02).astype(np.float16)
    codes, scales, bias = oracle.quantize_k(W, G, bits)
    assert codes.max() <= (1 << bits) - 1
    s = scales.astype(np.float64)
    b = bias.astype(np.float64)
    # the bias keeps exactly its k highest fraction bits, so a zero weight decodes to exactly zero
    assert np.all((bias.view(np.uint16) & ((1 << (10 - bits)) - 1)) == 0)
    Wz = W.copy()
    Wz[:, 0] = 0
    cz, sz, bz = oracle.quantize_k(Wz, G, bits)
    assert np.all(oracle.dequant_k(cz, sz, bz, G, bits)[:, 0] == 0)
    levels = (2.0 + np.arange(1 << bits) / float(1 << (bits - 1)))[None, None, :]
    cand = (levels - b[:, :, None]) * s[:, :, None]
    w = W.astype(np.float64)[:, :, None]
    best = np.abs(w - cand).min(axis=2)
    chosen = np.abs(w[:, :, 0] - np.take_along_axis(cand, codes[:, :, None].astype(np.int64), 2)[:, :, 0])
    step = (s / float(1 << (bits - 1))).repeat(G, 1)
    # double rounding (fp32 -> fp16 -> k bits) can pick the other neighbour only near a tie: within one
    # fp16 ulp of the binade (2^-9) of it, i.e. 2^(k-10) of a step
    slack = step * 2.0 ** (bits - 10) + 1e-12
    assert (chosen <= best + slack).all()
    assert (chosen <= best + 1e-15).mean() > (0.97 if bits < 8 else 0.7)
    # decoded weights: fp16 values, within half a step (plus the rounding slop) unless clamped
    What = oracle.dequant_k(codes, scales, bias, G, bits).astype(np.float64)
    t = W.astype(np.float64) / s.repeat(G, 1) + b.repeat(G, 1)
    inner = (t >= 2.0) & (t < 4.0 - step / s.repeat(G, 1))
    err = np.abs(W.astype(np.float64) - What)
    assert (err[inner] <= 0.5 * step[inner] * (1 + 2.0 ** (bits - 9)) + np.abs(What[inner]) * 2.0 ** -11 + 2.0 ** -24).all()


def test_e0mk_monotone_and_round_trip(oracle):
    for bits in (2, 8):
        top = (1 << bits) - 1
        sb, bb = f16_bits(0.0123), oracle.w1_bits_k(top // 3, bits)
        vals = [bits_f16(oracle.decode_one_k(c, sb, bb, bits)) for c in range(top + 1)]
        assert all(a < b for a, b in zip(vals, vals[1:]))
        # dequant(quant(dequant(c))) == dequant(c) under fixed parameters
        for c in range(top + 1):
            w = oracle.decode_one_k(c, sb, bb, bits)
            c2 = oracle.encode_one_k(w, sb, bb, bits)
            assert oracle.decode_one_k(c2, sb, bb, bits) == w


def test_e0m8_mean_error_is_a_sixteenth_of_e0m4(oracle):
    W = synth_inputs.weights(128, 1024, seed=23)
    e = {}
    for bits in (4, 8):
        c, s, b = oracle.quantize_k(W, 128, bits)
        e[bits] = np.abs(W.astype(np.float64) - oracle.dequant_k(c, s, b, 128, bits).astype(np.float64)).mean()
    assert 12.0 < e[4] / e[8] < 17.0        # sixteen times finer steps; fp16 rounding of the result takes a little back
