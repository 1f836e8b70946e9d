"""Pins for the bfloat16 member of the format family in the CPU oracle.  The paper (closing remark of the
section "E0M4 FP4 quantization") only says that the approach carries over to other formats and widths; the
oracle's reading is the E0M4 definition with bfloat16's own numbers (7 fraction bits: shift 3, top of the
binade 4 - 2^-6, bias truncated to its four highest fraction bits).  Every check compares the oracle with
something other than itself: an independent library conversion (torch's CPU bfloat16), exact rational
arithmetic, exhaustive enumeration, brute force on tiny groups, closed forms.  No GPU needed."""
from fractions import Fraction

import numpy as np
import pytest

import synth_inputs

BF_ONE = 0x3F80
BF_TWO = 0x4000


def bf_val(b) -> float:
    """bfloat16 bit pattern -> value: the upper half of a binary32 (independent of the oracle)."""
    return float(np.array([int(b) << 16], dtype=np.uint32).view(np.float32)[0])


def bf_exact_bits(x: Fraction) -> int:
    """Exact rational -> bfloat16 bits, round to nearest even, normal range only; plain integer arithmetic."""
    assert x > 0
    e = 0
    while x >= 2:
        x /= 2
        e += 1
    while x < 1:
        x *= 2
        e -= 1
    m = x * 128                                      # in [128, 256)
    f = m.numerator // m.denominator
    r = m - f
    if r > Fraction(1, 2) or (r == Fraction(1, 2) and f % 2 == 1):
        f += 1
    if f == 256:
        f, e = 128, e + 1
    assert -126 <= e <= 127
    return ((e + 127) << 7) | (f - 128)


# ---------------------------------------------------------------- conversions

def test_bf16_to_double_exhaustive(oracle):
    bits = np.arange(65536, dtype=np.uint32)
    with np.errstate(invalid="ignore"):
        ref = (bits << 16).astype(np.uint32).view(np.float32).astype(np.float64)
    got = np.array([oracle.bf16_bits_to_double(int(b)) for b in bits])
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], ref[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(ref[~nan]))
    with np.errstate(invalid="ignore"):
        assert np.array_equal(oracle.bf16_to_float64(bits.astype(np.uint16))[~nan], ref[~nan])


def test_double_to_bf16_rne_vs_torch_and_midpoints(oracle):
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(1)
    vals = list(np.ldexp(rng.uniform(-2, 2, 20000), rng.integers(-140, 127, 20000)).astype(np.float32).astype(np.float64))
    hb = np.arange(0x0001, 0x7F7F, 29, dtype=np.uint32)
    lo = (hb << 16).astype(np.uint32).view(np.float32).astype(np.float64)
    hi = ((hb + 1) << 16).astype(np.uint32).view(np.float32).astype(np.float64)
    mid = (lo + hi) / 2                              # exact in fp64 and in fp32 (one more bit)
    for v in (mid, lo, hi):
        vals += list(v) + list(-v)
    vals += [0.0, -0.0, 2.0 ** -133, 2.0 ** -134, 2.0 ** -126, 3.984375, 3.9921875, float(np.float32(1.0 / 3.0))]
    vals = np.array(vals, dtype=np.float64)
    as_f32 = vals.astype(np.float32)
    assert np.array_equal(as_f32.astype(np.float64), vals)       # every test value is an exact binary32
    ref = torch.from_numpy(as_f32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([oracle.double_to_bf16_bits(float(v)) for v in vals], dtype=np.uint16)
    assert np.array_equal(got, ref)
    # the input generator's own rounding agrees with both
    assert np.array_equal(synth_inputs.to_bf16_bits(as_f32), ref)
    # values between binary32 neighbours, against exact rational rounding
    for _ in range(2000):
        x = Fraction(int(rng.integers(1, 1 << 40)), int(rng.integers(1, 1 << 40)))
        assert oracle.double_to_bf16_bits(x.numerator / x.denominator) in (bf_exact_bits(x),)


# ---------------------------------------------------------------- code table, decode

def test_bf16_code_table_is_the_formula_with_shift_three(oracle):
    for c in range(16):
        assert oracle.bf16_w1_bits(c) == (0x4000 | (c << 3)) == 0x4000 + 8 * c
        assert Fraction(bf_val(oracle.bf16_w1_bits(c))) == 2 + Fraction(c, 8)       # the same values as for fp16
    assert bf_val(0x407F) == 4 - 2.0 ** -6


def test_bf16_decode_is_affine_exact_rational(oracle):
    rng = np.random.default_rng(2)
    scales = np.concatenate([rng.integers(0x0080, 0x7F7F, 300), [0x0080, 0x3F80, 0x7F7F, 0x3C00, 0x4B00]])
    for sb in scales:
        s = Fraction(bf_val(sb))
        for z in range(16):
            bb = 0x4000 | (z << 3)
            for c in range(16):
                exact = Fraction(c - z, 8) * s
                got = oracle.bf16_decode_one(c, int(sb), bb)
                if exact == 0:
                    assert got in (0x0000, 0x8000)
                    continue
                mag = abs(exact)
                if mag >= Fraction(2) ** 128 * (1 - Fraction(1, 512)) or mag < Fraction(1, 2 ** 126):
                    continue                                    # overflow / subnormal results: not produced by real groups
                want = bf_exact_bits(mag) | (0x8000 if exact < 0 else 0)
                assert got == want, (hex(sb), z, c)
            v = [oracle.bf16_bits_to_double(oracle.bf16_decode_one(c, int(sb), bb)) for c in range(16)]
            assert all(v[i] <= v[i + 1] for i in range(15)) and v[z] == 0.0


# ---------------------------------------------------------------- rounding rule, fit, round trip

def test_bf16_rounding_rule_exhaustive_over_binade(oracle):
    """All 128 bfloat16 values of [2,4): code = round-half-up((v-2)*8) saturated at 15, i.e. fraction bits 6..3
    plus bit 2."""
    for b in range(0x4000, 0x4080):
        v = bf_val(b)
        w0 = v - 2.0
        w0b = int(synth_inputs.to_bf16_bits(np.array([w0], dtype=np.float32))[0])
        assert bf_val(w0b) == w0                                 # exactly representable
        c = oracle.bf16_encode_one(w0b, BF_ONE, BF_TWO)
        assert c == min(int(np.floor((v - 2.0) * 8 + 0.5)), 15), hex(b)
        assert c == min(((b >> 3) & 15) + ((b >> 2) & 1), 15)
        assert oracle.bf16_forward_bits(w0b, BF_ONE, BF_TWO) == b


def test_bf16_forward_map_shares_sign_and_exponent(oracle):
    rng = np.random.default_rng(4)
    for _ in range(5000):
        wb = int(rng.integers(0, 0x7F80)) | (int(rng.integers(0, 2)) << 15)
        sb = int(rng.integers(0x0080, 0x7F80))
        z = int(rng.integers(0, 16))
        fb = oracle.bf16_forward_bits(wb, sb, 0x4000 | (z << 3))
        assert fb >> 7 == 0x80, (hex(wb), hex(sb), z, hex(fb))   # sign 0, exponent field 128


def test_bf16_fit_against_exact_rationals(oracle):
    rng = np.random.default_rng(5)
    span = Fraction(0x407F - 0x4000, 64)                        # (4 - 2^-6) - 2
    exact_checked = 0
    for trial in range(400):
        G = int(rng.choice([2, 4, 8, 64, 128]))
        std = float(rng.choice([1e-3, 0.02, 1.0, 50.0]))
        w = rng.standard_normal(G).astype(np.float32) * np.float32(std)
        if trial % 7 == 0:
            w = np.abs(w)
        if trial % 11 == 0:
            w = -np.abs(w)
        wb = synth_inputs.to_bf16_bits(w)
        sb, bb = oracle.bf16_fit_group(wb)
        vals = [Fraction(bf_val(b)) for b in wb]
        mn, mx = min([Fraction(0)] + vals), max([Fraction(0)] + vals)
        s_exact = (mx - mn) / span
        s = Fraction(bf_val(sb))
        # fp32 divide, then one bfloat16 rounding: within half a bfloat16 ulp (and the fp32 rounding) of the quotient
        assert abs(s - s_exact) <= s_exact * Fraction(1, 2 ** 8) * Fraction(1001, 1000)
        assert bb & 0x7 == 0 and (bb >> 7) == 0x80              # bias = 2 + z/8
        z = (bb >> 3) & 15
        b_exact = min(max(Fraction(2) - mn / s, Fraction(2)), Fraction(255, 64))        # clamped to [2, 4 - 2^-6]
        z_floor = int((b_exact - 2) * 8)
        frac = (b_exact - 2) * 8 - z_floor
        # one bfloat16 ulp of the binade is 1/8 of a code step and rounding b moves it by half of that: away from a
        # multiple of 1/8 by more than that, the result is the truncation
        if Fraction(3, 32) < frac < Fraction(29, 32):
            assert z == min(z_floor, 15), (trial, float(b_exact), z)
            exact_checked += 1
        else:
            assert z in (z_floor, min(z_floor + 1, 15), max(z_floor - 1, 0))
    assert exact_checked > 200


def test_bf16_bias_truncates_and_exact_zero_stays_zero(oracle):
    # range [-0.98, 1.02] with scale about 1: image of zero near 2.98 -> 7.8 eighths: truncation keeps 7
    w = synth_inputs.to_bf16_bits(np.array([-0.98, 1.02, 0.0, 0.1], dtype=np.float32))
    sb, bb = oracle.bf16_fit_group(w)
    s = Fraction(bf_val(sb))
    img = (Fraction(2) - Fraction(bf_val(w[0])) / s - 2) * 8
    assert int(img) == 7 and bb == 0x4000 | (7 << 3), (float(img), hex(bb))
    codes, scales, bias = oracle.bf16_quantize(w.reshape(1, 4), 4)
    What = oracle.bf16_dequant(codes, scales, bias, 4)
    assert codes[0, 2] == 7 and What[0, 2] in (0x0000, 0x8000)
    # degenerate groups: all zero, constant
    z = np.zeros((1, 8), dtype=np.uint16)
    c, s_, b_ = oracle.bf16_quantize(z, 8)
    assert not c.any() and b_[0, 0] == 0x4000 and s_[0, 0] == 0x0080 and not oracle.bf16_dequant(c, s_, b_, 8).any()


def test_bf16_fixed_parameter_round_trip_exhaustive(oracle):
    """encode(decode(c)) == c for every normal positive bfloat16 scale x 16 biases x 16 codes whose decoded values
    are normal numbers."""
    sb = np.arange(0x0080, 0x7F80, dtype=np.uint16)             # 32512 normal scales
    zz = np.arange(16, dtype=np.uint16)
    scales = np.repeat(sb, 16)[:, None]
    bias = np.tile((0x4000 | (zz << 3)).astype(np.uint16), sb.size)[:, None]
    codes = np.tile(np.arange(16, dtype=np.uint8), (scales.shape[0], 1))
    What = oracle.bf16_dequant(codes, scales, bias, 16)
    mag = What & 0x7FFF
    usable = (mag < 0x7F80) & ((mag >= 0x0080) | (mag == 0))    # finite, and not subnormal
    assert usable.mean() > 0.9
    back = oracle.bf16_encode(What, scales, bias, 16)
    assert np.array_equal(back[usable], codes[usable])
    # hence dequant(quant(dequant(c))) == dequant(c) at fixed parameters
    again = oracle.bf16_dequant(back, scales, bias, 16)
    assert np.array_equal(again[usable], What[usable])


@pytest.mark.parametrize("G", [2, 4, 8])
def test_bf16_brute_force_nearest_code_tiny_groups(oracle, G):
    rng = np.random.default_rng(200 + G)
    W = synth_inputs.to_bf16_bits(rng.standard_normal((3000, G)).astype(np.float32) * np.float32(0.02))
    codes, scales, bias = oracle.bf16_quantize(W, G)
    s = oracle.bf16_to_float64(scales)
    b = oracle.bf16_to_float64(bias)
    levels = (2.0 + np.arange(16) / 8.0)[None, None, :]
    cand = (levels - b[:, :, None]) * s[:, :, None]
    w = oracle.bf16_to_float64(W)[:, :, None]
    best = np.abs(w - cand).min(axis=2)
    chosen = np.abs(w[:, :, 0] - np.take_along_axis(cand, codes[:, :, None].astype(np.int64), 2)[:, :, 0])
    step = (s / 8.0).repeat(G, 1)
    # double rounding (fp32 -> bfloat16 with 7 fraction bits -> 4 bits) can pick the other neighbour within
    # 1/8 of a step of a tie (one bfloat16 ulp of the binade is 1/8 of a code step)
    assert (chosen <= best + step / 8 + 1e-12).all()
    assert (chosen <= best + 1e-15).mean() > 0.85
    # the quantisation error itself: at most half a step plus that slack, one step for the clamped ends
    t = w[:, :, 0] / s.repeat(G, 1) + b.repeat(G, 1)
    inner = (t >= 2.0) & (t < 3.9375)
    assert inner.mean() > 0.3
    assert (chosen[inner] <= (1 / 16 + 1 / 64 + 1e-6) * 8 * step[inner]).all()


def test_bf16_codes_monotone_and_groups_independent(oracle):
    W = synth_inputs.weights_bf16(64, 512, seed=8)
    codes, scales, bias = oracle.bf16_quantize(W, 128)
    Wg = oracle.bf16_to_float64(W).reshape(64, 4, 128)
    order = np.argsort(Wg, axis=2, kind="stable")
    assert (np.diff(np.take_along_axis(codes.reshape(64, 4, 128), order, 2).astype(np.int64), axis=2) >= 0).all()
    # a group's result does not depend on its neighbours, and equals the scalar path
    c2, s2, b2 = oracle.bf16_quantize(W[:, 128:256], 128)
    assert np.array_equal(c2, codes[:, 128:256]) and np.array_equal(s2[:, 0], scales[:, 1]) and np.array_equal(b2[:, 0], bias[:, 1])
    sb, bb = oracle.bf16_fit_group(W[5, 256:384])
    assert (sb, bb) == (int(scales[5, 2]), int(bias[5, 2]))
    for k in range(256, 384, 17):
        assert codes[5, k] == oracle.bf16_encode_one(int(W[5, k]), sb, bb)


# ---------------------------------------------------------------- matmul

def test_bf16_matmul_tiny_exact_rational_and_special_inputs(oracle):
    rng = np.random.default_rng(9)
    M, N, K = 3, 5, 12
    X = synth_inputs.to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32))
    W = synth_inputs.to_bf16_bits(rng.standard_normal((N, K)).astype(np.float32) * np.float32(0.05))
    Y, absdot = oracle.bf16_matmul(X, W)
    for m in range(M):
        for n in range(N):
            exact = sum(Fraction(bf_val(X[m, k])) * Fraction(bf_val(W[n, k])) for k in range(K))
            want = (bf_exact_bits(abs(exact)) | (0x8000 if exact < 0 else 0)) if exact != 0 else 0
            assert int(Y[m, n]) == want
            assert abs(absdot[m, n] - float(sum(abs(Fraction(bf_val(X[m, k])) * Fraction(bf_val(W[n, k]))) for k in range(K)))) < 1e-12
    # operand orientation: a one-hot row of X picks column k of W^T, i.e. W[:, k]
    X1 = np.zeros((1, K), dtype=np.uint16)
    X1[0, 7] = BF_ONE
    Y1, _ = oracle.bf16_matmul(X1, W)
    assert np.array_equal(Y1[0], W[:, 7])
    ones = np.full((1, K), BF_ONE, dtype=np.uint16)
    Ys, _ = oracle.bf16_matmul(ones, W)
    ref = oracle.bf16_to_float64(W).sum(axis=1)
    assert np.array_equal(Ys[0], synth_inputs.to_bf16_bits(ref.astype(np.float32))) or \
        np.abs(oracle.bf16_to_float64(Ys[0]) - ref).max() <= np.abs(ref).max() * 2.0 ** -8
