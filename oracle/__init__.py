"""CPU oracle for the E0M4 quantised matmul -- TEST INFRASTRUCTURE ONLY.

Thin ctypes loader around ``e0m4_oracle.c`` (plain C, fp64 except where the
arithmetic decides an integer code).  Nothing here is part of the product:
only ``tests/``, the smoke check and the benchmark's CPU-baseline leg may
import this package, and this package imports nothing from the GPU library.

All arrays are numpy; fp16 data travels as ``uint16`` bit patterns or as
``float16`` arrays (viewed, never converted).  Layouts are the canonical ones:
``codes [N,K]`` one code (0..15) per byte, ``scales``/``bias`` ``[N, K/G]``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "e0m4_oracle.c")
_LIB = os.path.join(_HERE, "libe0m4_oracle.so")
_CFLAGS = ["-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC"]

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no GPU toolchain involved)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", *_CFLAGS, _SRC, "-o", tmp, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    L = ctypes.CDLL(_LIB)
    u16p = ctypes.POINTER(ctypes.c_uint16)
    u8p = ctypes.POINTER(ctypes.c_uint8)
    f64p = ctypes.POINTER(ctypes.c_double)
    i64 = ctypes.c_int64
    L.oracle_half_bits_to_double.restype = ctypes.c_double
    L.oracle_half_bits_to_double.argtypes = [ctypes.c_uint16]
    L.oracle_double_to_half_bits.restype = ctypes.c_uint16
    L.oracle_double_to_half_bits.argtypes = [ctypes.c_double]
    L.oracle_e0m4_w1_bits.restype = ctypes.c_uint16
    L.oracle_e0m4_w1_bits.argtypes = [ctypes.c_int]
    L.oracle_e0m4_decode_one.restype = ctypes.c_uint16
    L.oracle_e0m4_decode_one.argtypes = [ctypes.c_int, ctypes.c_uint16, ctypes.c_uint16]
    L.oracle_e0m4_encode_one.restype = ctypes.c_int
    L.oracle_e0m4_encode_one.argtypes = [ctypes.c_uint16, ctypes.c_uint16, ctypes.c_uint16]
    L.oracle_e0m4_forward_bits.restype = ctypes.c_uint16
    L.oracle_e0m4_forward_bits.argtypes = [ctypes.c_uint16, ctypes.c_uint16, ctypes.c_uint16]
    L.oracle_e0m4_fit_group.restype = None
    L.oracle_e0m4_fit_group.argtypes = [u16p, i64, u16p, u16p]
    L.oracle_e0m4_quantize.restype = None
    L.oracle_e0m4_quantize.argtypes = [u16p, i64, i64, i64, u8p, u16p, u16p]
    L.oracle_e0m4_encode.restype = None
    L.oracle_e0m4_encode.argtypes = [u16p, i64, i64, i64, u16p, u16p, u8p]
    L.oracle_e0m4_dequant.restype = None
    L.oracle_e0m4_dequant.argtypes = [u8p, u16p, u16p, i64, i64, i64, u16p]
    L.oracle_int4_decode_one.restype = ctypes.c_uint16
    L.oracle_int4_decode_one.argtypes = [ctypes.c_int, ctypes.c_uint16, ctypes.c_uint16]
    L.oracle_int4_encode_one.restype = ctypes.c_int
    L.oracle_int4_encode_one.argtypes = [ctypes.c_uint16, ctypes.c_uint16, ctypes.c_uint16]
    L.oracle_int4_quantize.restype = None
    L.oracle_int4_quantize.argtypes = [u16p, i64, i64, i64, u8p, u16p, u16p]
    L.oracle_int4_dequant.restype = None
    L.oracle_int4_dequant.argtypes = [u8p, u16p, u16p, i64, i64, i64, u16p]
    ci = ctypes.c_int
    L.oracle_e0mk_w1_bits.restype = ctypes.c_uint16
    L.oracle_e0mk_w1_bits.argtypes = [ci, ci]
    L.oracle_e0mk_decode_one.restype = ctypes.c_uint16
    L.oracle_e0mk_decode_one.argtypes = [ci, ctypes.c_uint16, ctypes.c_uint16, ci]
    L.oracle_e0mk_encode_one.restype = ci
    L.oracle_e0mk_encode_one.argtypes = [ctypes.c_uint16, ctypes.c_uint16, ctypes.c_uint16, ci]
    L.oracle_e0mk_fit_group.restype = None
    L.oracle_e0mk_fit_group.argtypes = [u16p, i64, ci, u16p, u16p]
    L.oracle_e0mk_quantize.restype = None
    L.oracle_e0mk_quantize.argtypes = [u16p, i64, i64, i64, ci, u8p, u16p, u16p]
    L.oracle_e0mk_dequant.restype = None
    L.oracle_e0mk_dequant.argtypes = [u8p, u16p, u16p, i64, i64, i64, ci, u16p]
    L.oracle_e0m4_matmul.restype = None
    L.oracle_e0m4_matmul.argtypes = [u16p, i64, u16p, i64, i64, u16p, f64p]
    L.oracle_bf16_bits_to_double.restype = ctypes.c_double
    L.oracle_bf16_bits_to_double.argtypes = [ctypes.c_uint16]
    L.oracle_double_to_bf16_bits.restype = ctypes.c_uint16
    L.oracle_double_to_bf16_bits.argtypes = [ctypes.c_double]
    L.oracle_bf16_w1_bits.restype = ctypes.c_uint16
    L.oracle_bf16_w1_bits.argtypes = [ctypes.c_int]
    for name in ("oracle_bf16_decode_one",):
        getattr(L, name).restype = ctypes.c_uint16
        getattr(L, name).argtypes = [ctypes.c_int, ctypes.c_uint16, ctypes.c_uint16]
    L.oracle_bf16_encode_one.restype = ctypes.c_int
    L.oracle_bf16_encode_one.argtypes = [ctypes.c_uint16, ctypes.c_uint16, ctypes.c_uint16]
    L.oracle_bf16_forward_bits.restype = ctypes.c_uint16
    L.oracle_bf16_forward_bits.argtypes = [ctypes.c_uint16, ctypes.c_uint16, ctypes.c_uint16]
    L.oracle_bf16_fit_group.restype = None
    L.oracle_bf16_fit_group.argtypes = [u16p, i64, u16p, u16p]
    L.oracle_bf16_quantize.restype = None
    L.oracle_bf16_quantize.argtypes = [u16p, i64, i64, i64, u8p, u16p, u16p]
    L.oracle_bf16_encode.restype = None
    L.oracle_bf16_encode.argtypes = [u16p, i64, i64, i64, u16p, u16p, u8p]
    L.oracle_bf16_dequant.restype = None
    L.oracle_bf16_dequant.argtypes = [u8p, u16p, u16p, i64, i64, i64, u16p]
    L.oracle_bf16_matmul.restype = None
    L.oracle_bf16_matmul.argtypes = [u16p, i64, u16p, i64, i64, u16p, f64p]
    L.oracle_num_threads.restype = ctypes.c_int
    L.oracle_set_num_threads.restype = ctypes.c_int
    L.oracle_set_num_threads.argtypes = [ctypes.c_int]
    _lib = L
    return L


def _u16(a: np.ndarray) -> np.ndarray:
    """View an fp16 / uint16 array as contiguous uint16 bit patterns."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    assert a.dtype == np.uint16, a.dtype
    return a


def _p(a: np.ndarray, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


# ---- scalar helpers (used by the pin tests) ---------------------------------

def half_bits_to_double(h: int) -> float:
    return _load().oracle_half_bits_to_double(int(h))


def double_to_half_bits(d: float) -> int:
    return _load().oracle_double_to_half_bits(float(d))


def w1_bits(c: int) -> int:
    """Bit pattern of the binade value of code c (paper: dequantization formula)."""
    return _load().oracle_e0m4_w1_bits(int(c))


def decode_one(c: int, scale_bits: int, bias_bits: int) -> int:
    return _load().oracle_e0m4_decode_one(int(c), int(scale_bits), int(bias_bits))


def encode_one(w0_bits: int, scale_bits: int, bias_bits: int) -> int:
    return _load().oracle_e0m4_encode_one(int(w0_bits), int(scale_bits), int(bias_bits))


def forward_bits(w0_bits: int, scale_bits: int, bias_bits: int) -> int:
    return _load().oracle_e0m4_forward_bits(int(w0_bits), int(scale_bits), int(bias_bits))


def fit_group(w0: np.ndarray):
    """(scale_bits, bias_bits) of one group (paper: quantization paragraph)."""
    w0 = _u16(w0).ravel()
    s = ctypes.c_uint16()
    b = ctypes.c_uint16()
    _load().oracle_e0m4_fit_group(_p(w0, ctypes.c_uint16), w0.size, ctypes.byref(s), ctypes.byref(b))
    return s.value, b.value


# ---- array entry points -----------------------------------------------------

def quantize(W: np.ndarray, group: int):
    """W [N,K] fp16 -> (codes u8 [N,K], scales f16 [N,K/G], bias f16 [N,K/G])."""
    Wb = _u16(W)
    N, K = Wb.shape
    assert K % group == 0
    codes = np.empty((N, K), np.uint8)
    scales = np.empty((N, K // group), np.uint16)
    bias = np.empty((N, K // group), np.uint16)
    _load().oracle_e0m4_quantize(_p(Wb, ctypes.c_uint16), N, K, group, _p(codes, ctypes.c_uint8),
                                 _p(scales, ctypes.c_uint16), _p(bias, ctypes.c_uint16))
    return codes, scales.view(np.float16), bias.view(np.float16)


def encode(W: np.ndarray, scales: np.ndarray, bias: np.ndarray, group: int) -> np.ndarray:
    """Codes of W under caller-supplied per-group parameters."""
    Wb, sb, bb = _u16(W), _u16(scales), _u16(bias)
    N, K = Wb.shape
    assert sb.shape == (N, K // group) and bb.shape == sb.shape
    codes = np.empty((N, K), np.uint8)
    _load().oracle_e0m4_encode(_p(Wb, ctypes.c_uint16), N, K, group, _p(sb, ctypes.c_uint16),
                               _p(bb, ctypes.c_uint16), _p(codes, ctypes.c_uint8))
    return codes


def dequant(codes: np.ndarray, scales: np.ndarray, bias: np.ndarray, group: int) -> np.ndarray:
    """codes u8 [N,K] + params [N,K/G] -> dequantised weights f16 [N,K]."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    sb, bb = _u16(scales), _u16(bias)
    N, K = codes.shape
    assert sb.shape == (N, K // group) and bb.shape == sb.shape
    out = np.empty((N, K), np.uint16)
    _load().oracle_e0m4_dequant(_p(codes, ctypes.c_uint8), _p(sb, ctypes.c_uint16), _p(bb, ctypes.c_uint16),
                                N, K, group, _p(out, ctypes.c_uint16))
    return out.view(np.float16)


# ---- INT4 comparison format (paper: section "Evaluation of FP4 quantization") ----

def int4_decode_one(q: int, scale_bits: int, zero_bits: int) -> int:
    return _load().oracle_int4_decode_one(q, scale_bits, zero_bits)


def int4_encode_one(w0_bits: int, scale_bits: int, zero_bits: int) -> int:
    return _load().oracle_int4_encode_one(w0_bits, scale_bits, zero_bits)


def int4_quantize(W: np.ndarray, group: int):
    """W [N,K] fp16 -> (codes u8 [N,K], scales f16 [N,K/G], zeros f16 [N,K/G], integer-valued 0..15)."""
    Wb = _u16(W)
    N, K = Wb.shape
    assert K % group == 0
    codes = np.empty((N, K), np.uint8)
    scales = np.empty((N, K // group), np.uint16)
    zeros = np.empty((N, K // group), np.uint16)
    _load().oracle_int4_quantize(_p(Wb, ctypes.c_uint16), N, K, group, _p(codes, ctypes.c_uint8),
                                 _p(scales, ctypes.c_uint16), _p(zeros, ctypes.c_uint16))
    return codes, scales.view(np.float16), zeros.view(np.float16)


def int4_dequant(codes: np.ndarray, scales: np.ndarray, zeros: np.ndarray, group: int) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    sb, zb = _u16(scales), _u16(zeros)
    N, K = codes.shape
    assert sb.shape == (N, K // group) and zb.shape == sb.shape
    out = np.empty((N, K), np.uint16)
    _load().oracle_int4_dequant(_p(codes, ctypes.c_uint8), _p(sb, ctypes.c_uint16), _p(zb, ctypes.c_uint16),
                                N, K, group, _p(out, ctypes.c_uint16))
    return out.view(np.float16)


def matmul(X: np.ndarray, What: np.ndarray, want_absdot: bool = True):
    """Y[m,n] = fp16(sum_k X[m,k] What[n,k]) in fp64; also sum_k |x w| per output."""
    Xb, Wb = _u16(X), _u16(What)
    M, K = Xb.shape
    N, K2 = Wb.shape
    assert K == K2
    Y = np.empty((M, N), np.uint16)
    absdot = np.empty((M, N), np.float64) if want_absdot else None
    _load().oracle_e0m4_matmul(_p(Xb, ctypes.c_uint16), M, _p(Wb, ctypes.c_uint16), N, K,
                               _p(Y, ctypes.c_uint16),
                               _p(absdot, ctypes.c_double) if want_absdot else None)
    return (Y.view(np.float16), absdot) if want_absdot else Y.view(np.float16)


def num_threads() -> int:
    return _load().oracle_num_threads()


def set_num_threads(n: int) -> bool:
    """Threads used by the parallel loops from now on (for timing on one thread); False without OpenMP."""
    return bool(_load().oracle_set_num_threads(int(n)))


# --------------------------------------------------------------------------------------------------
# Operators fused around the matmul (paper: section "Operator and lagging optimizations": the small
# operators of rms-norm are fused into one, element-wise operators are fused into their neighbours).
# The paper names the operators and gives no formulas; they are the textbook ones, written out in
# fp64 with numpy:
#   rms-norm   x'[k] = x[k] * gamma[k] / sqrt(mean_k(x^2) + eps)
#   SiLU       silu(g) = g / (1 + exp(-g))
#   gated unit y[j] = silu(a[j]) * a[N/2 + j]     (first half of the rows: gate, second half: up)
#   residual   y = a + r
# --------------------------------------------------------------------------------------------------

def silu(g: np.ndarray) -> np.ndarray:
    """g * sigmoid(g) in fp64, written so that exp never overflows."""
    g = np.asarray(g, np.float64)
    e = np.exp(-np.abs(g))                      # in (0, 1]
    sig = np.where(g >= 0, 1.0 / (1.0 + e), e / (1.0 + e))
    return g * sig


def rmsnorm(X: np.ndarray, gamma: np.ndarray, eps: float) -> np.ndarray:
    """Row-wise rms-norm of X [M,K] with weight gamma [K]; fp64 result (not rounded)."""
    x = np.asarray(X).astype(np.float64)
    g = np.asarray(gamma).astype(np.float64)
    ms = np.mean(x * x, axis=1, keepdims=True)
    return x * g[None, :] / np.sqrt(ms + float(eps))


def matmul_fused(X: np.ndarray, What: np.ndarray, gamma=None, eps: float = 0.0, swiglu: bool = False,
                 residual=None):
    """The matmul with its neighbours folded in, each step the plain definition in fp64:

    1. if gamma is given, X is replaced by fp16(rmsnorm(X, gamma, eps)) (the normalised activation is an
       fp16 tensor, as it is when the operator runs on its own);
    2. a[m,n] = sum_k X[m,k] * What[n,k];
    3. if swiglu, y[m,j] = silu(a[m,j]) * a[m, N/2 + j] for j < N/2, else y = a;
    4. if residual is given, y += residual;
    5. one rounding to fp16.

    Returns (Y fp16, info) where info holds what the acceptance tolerance is stated in: 'a' (fp64 sums of
    step 2), 'absdot' (sum_k |x w| per entry of a) and 'y' (the fp64 result before step 5).
    """
    Xh = np.asarray(X)
    assert Xh.dtype == np.float16 and np.asarray(What).dtype == np.float16
    if gamma is not None:
        Xh = rmsnorm(Xh, gamma, eps).astype(np.float16)
    xd = Xh.astype(np.float64)
    wd = np.asarray(What).astype(np.float64)
    a = xd @ wd.T
    absdot = np.abs(xd) @ np.abs(wd).T
    if swiglu:
        N = wd.shape[0]
        assert N % 2 == 0
        y = silu(a[:, : N // 2]) * a[:, N // 2:]
    else:
        y = a
    if residual is not None:
        r = np.asarray(residual)
        assert r.dtype == np.float16 and r.shape == y.shape
        y = y + r.astype(np.float64)
    with np.errstate(over="ignore"):
        Y = y.astype(np.float16)
    return Y, {"a": a, "absdot": absdot, "y": y}


# --------------------------------------------------------------------------------------------------
# KV-cache append (paper: section "KV cache copy optimization"): one tensor of the maximum sequence
# length holds the cache, sequence position first; the rows produced for the new tokens are written in
# place at the positions given by position_ids, which replaces concatenating old cache and new rows.
# --------------------------------------------------------------------------------------------------

def kv_append(cache: np.ndarray, new_rows: np.ndarray, position_ids: np.ndarray) -> np.ndarray:
    """Returns the cache [max_seq, row] after writing new_rows[i] to row position_ids[i], one row at a
    time in order (a position outside [0, max_seq) leaves the cache untouched for that row)."""
    out = np.array(cache, copy=True)
    for i in range(new_rows.shape[0]):
        p = int(position_ids[i])
        if 0 <= p < out.shape[0]:
            for e in range(new_rows.shape[1]):
                out[p, e] = new_rows[i, e]
    return out


# --------------------------------------------------------------------------------------------------
# Other code widths, E0Mk with 1 <= k <= 8 (paper: the closing remark of the section "E0M4 FP4
# quantization").  Same definition with the k highest fraction bits in place of four.
# --------------------------------------------------------------------------------------------------

def w1_bits_k(c: int, bits: int) -> int:
    return int(_load().oracle_e0mk_w1_bits(int(c), int(bits)))


def decode_one_k(c: int, scale_bits: int, bias_bits: int, bits: int) -> int:
    return int(_load().oracle_e0mk_decode_one(int(c), int(scale_bits), int(bias_bits), int(bits)))


def encode_one_k(w0_bits: int, scale_bits: int, bias_bits: int, bits: int) -> int:
    return int(_load().oracle_e0mk_encode_one(int(w0_bits), int(scale_bits), int(bias_bits), int(bits)))


def fit_group_k(w0: np.ndarray, bits: int):
    w0 = _u16(w0)
    sb, bb = ctypes.c_uint16(0), ctypes.c_uint16(0)
    _load().oracle_e0mk_fit_group(_p(w0, ctypes.c_uint16), w0.size, int(bits), ctypes.byref(sb), ctypes.byref(bb))
    return int(sb.value), int(bb.value)


def quantize_k(W: np.ndarray, group: int, bits: int):
    """W [N,K] fp16 -> (codes [N,K] uint8 in 0..2^bits-1, scales, bias [N,K/group] fp16)."""
    Wb = _u16(W)
    N, K = Wb.shape
    assert K % group == 0 and 1 <= bits <= 8
    codes = np.empty((N, K), np.uint8)
    scales = np.empty((N, K // group), np.uint16)
    bias = np.empty((N, K // group), np.uint16)
    _load().oracle_e0mk_quantize(_p(Wb, ctypes.c_uint16), N, K, group, int(bits), _p(codes, ctypes.c_uint8),
                                 _p(scales, ctypes.c_uint16), _p(bias, ctypes.c_uint16))
    return codes, scales.view(np.float16), bias.view(np.float16)


def dequant_k(codes: np.ndarray, scales: np.ndarray, bias: np.ndarray, group: int, bits: int) -> np.ndarray:
    codes = np.ascontiguousarray(codes, np.uint8)
    N, K = codes.shape
    sb, bb = _u16(scales), _u16(bias)
    assert sb.shape == (N, K // group) and bb.shape == sb.shape
    out = np.empty((N, K), np.uint16)
    _load().oracle_e0mk_dequant(_p(codes, ctypes.c_uint8), _p(sb, ctypes.c_uint16), _p(bb, ctypes.c_uint16),
                                N, K, group, int(bits), _p(out, ctypes.c_uint16))
    return out.view(np.float16)


# --------------------------------------------------------------------------------------------------
# The same construction on bfloat16 (see the C source for the reading).  numpy has no bfloat16 type:
# every bfloat16 array here is a uint16 array of bit patterns.
# --------------------------------------------------------------------------------------------------

def bf16_bits_to_double(h: int) -> float:
    return _load().oracle_bf16_bits_to_double(h)


def double_to_bf16_bits(d: float) -> int:
    return _load().oracle_double_to_bf16_bits(d)


def bf16_w1_bits(c: int) -> int:
    return _load().oracle_bf16_w1_bits(c)


def bf16_decode_one(c: int, scale_bits: int, bias_bits: int) -> int:
    return _load().oracle_bf16_decode_one(c, scale_bits, bias_bits)


def bf16_encode_one(w0_bits: int, scale_bits: int, bias_bits: int) -> int:
    return _load().oracle_bf16_encode_one(w0_bits, scale_bits, bias_bits)


def bf16_forward_bits(w0_bits: int, scale_bits: int, bias_bits: int) -> int:
    return _load().oracle_bf16_forward_bits(w0_bits, scale_bits, bias_bits)


def bf16_fit_group(w0_bits: np.ndarray):
    w = np.ascontiguousarray(w0_bits, dtype=np.uint16)
    sb, bb = ctypes.c_uint16(0), ctypes.c_uint16(0)
    _load().oracle_bf16_fit_group(_p(w, ctypes.c_uint16), w.size, ctypes.byref(sb), ctypes.byref(bb))
    return sb.value, bb.value


def bf16_quantize(W_bits: np.ndarray, group: int):
    """W_bits [N,K] bfloat16 bit patterns -> (codes u8 [N,K], scale bits u16 [N,K/G], bias bits u16 [N,K/G])."""
    Wb = np.ascontiguousarray(W_bits, dtype=np.uint16)
    N, K = Wb.shape
    assert K % group == 0
    codes = np.empty((N, K), np.uint8)
    scales = np.empty((N, K // group), np.uint16)
    bias = np.empty((N, K // group), np.uint16)
    _load().oracle_bf16_quantize(_p(Wb, ctypes.c_uint16), N, K, group, _p(codes, ctypes.c_uint8),
                                 _p(scales, ctypes.c_uint16), _p(bias, ctypes.c_uint16))
    return codes, scales, bias


def bf16_encode(W_bits: np.ndarray, scales: np.ndarray, bias: np.ndarray, group: int) -> np.ndarray:
    """Codes of W under given per-group parameters (bit patterns), no fitting."""
    Wb = np.ascontiguousarray(W_bits, dtype=np.uint16)
    sb = np.ascontiguousarray(scales, dtype=np.uint16)
    bb = np.ascontiguousarray(bias, dtype=np.uint16)
    N, K = Wb.shape
    codes = np.empty((N, K), np.uint8)
    _load().oracle_bf16_encode(_p(Wb, ctypes.c_uint16), N, K, group, _p(sb, ctypes.c_uint16), _p(bb, ctypes.c_uint16),
                               _p(codes, ctypes.c_uint8))
    return codes


def bf16_dequant(codes: np.ndarray, scales: np.ndarray, bias: np.ndarray, group: int) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    sb = np.ascontiguousarray(scales, dtype=np.uint16)
    bb = np.ascontiguousarray(bias, dtype=np.uint16)
    N, K = codes.shape
    out = np.empty((N, K), np.uint16)
    _load().oracle_bf16_dequant(_p(codes, ctypes.c_uint8), _p(sb, ctypes.c_uint16), _p(bb, ctypes.c_uint16), N, K, group,
                                _p(out, ctypes.c_uint16))
    return out


def bf16_matmul(X_bits: np.ndarray, What_bits: np.ndarray):
    """Y bits [M,N] = bf16(sum_k X[m,k] What[n,k]) in fp64, and sum_k |x w| per output."""
    Xb = np.ascontiguousarray(X_bits, dtype=np.uint16)
    Wb = np.ascontiguousarray(What_bits, dtype=np.uint16)
    M, K = Xb.shape
    N, K2 = Wb.shape
    assert K == K2
    Y = np.empty((M, N), np.uint16)
    absdot = np.empty((M, N), np.float64)
    _load().oracle_bf16_matmul(_p(Xb, ctypes.c_uint16), M, _p(Wb, ctypes.c_uint16), N, K, _p(Y, ctypes.c_uint16),
                               _p(absdot, ctypes.c_double))
    return Y, absdot


def bf16_to_float64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of an array of bfloat16 bit patterns (a bfloat16 is the upper half of a binary32)."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)
