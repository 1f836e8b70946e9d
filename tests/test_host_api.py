"""Host-side checks of libe0m4 that need no GPU: the library loads, exports every
symbol the public header declares, sizes are what the header says, and every
argument error is caught before anything could be launched."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "e0m4.h")


@pytest.fixture(scope="module")
def L():
    from paper_2403_20041_amd import binding, build

    if not os.path.exists(binding.LIB_PATH):
        build.build_library(verbose=False)
    return binding.lib()


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(e0m[348]_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported(L):
    names = declared_symbols()
    assert {"e0m4_quantize", "e0m4_dequant", "e0m4_matmul", "e0m4_unpack_codes", "e0m4_encode",
            "e0m4_codes_bytes", "e0m4_params_elems", "e0m4_workspace_bytes", "e0m4_abi_version",
            "e0m4_strerror", "e0m4_last_hip_error", "e0m4_set_knob"} <= set(names)
    for n in names:
        assert hasattr(L, n), n
    assert L.e0m4_abi_version() == 4


def test_size_functions(L):
    blk = 1024 + 64                                         # 16 rows x 128 k of codes + 16 (scale, bias) pairs at G=128
    assert L.e0m4_codes_bytes(4096, 4096, 128) == 256 * 32 * blk
    assert L.e0m4_codes_bytes(1, 32, 32) == 1024 + 256      # rows padded to 16, k padded to 128, 4 sub-groups
    assert L.e0m4_codes_bytes(17, 192, 64) == 2 * 2 * (1024 + 128)
    assert L.e0m4_codes_bytes(0, 4096, 128) == 0
    assert L.e0m4_codes_bytes(64, 48, 32) == 0              # K not a multiple of 32
    assert L.e0m4_codes_bytes(64, 128, 100) == 0
    assert L.e0m4_params_elems(4096, 4096, 128) == 32 * 4096
    assert L.e0m4_params_elems(100, 256, 64) == 400
    assert L.e0m4_params_elems(100, 256, 48) == 0
    assert L.e0m4_workspace_bytes(1, 4096, 4096, 128) == 0  # small M: partial sums never leave the chip
    assert L.e0m4_workspace_bytes(8, 151936, 4096, 128) == 0
    # few tiles and a long K: a K split (the number by the library's estimate of the launch), one fp32 [M, N] slab each
    for M, N, K in ((1024, 4096, 13696), (512, 4096, 4096), (128, 4608, 4096), (256, 4096, 13696)):
        need = L.e0m4_workspace_bytes(M, N, K, 128)
        assert need % (M * N * 4) == 0 and 2 <= need // (M * N * 4) <= 8, (M, N, K, need)
    # short K and many columns: enough whole tiles for every compute unit, unsplit
    assert L.e0m4_workspace_bytes(1024, 16384, 2048, 128) == 0
    assert L.e0m4_workspace_bytes(2048, 32768, 5120, 128) == 0          # 1024 tiles, four whole rounds of 256: no split
    # 132 large tiles with a long K, shared out by K ranges over the 256 compute units: their counters, then one
    # 256 x 256 fp32 slab for each compute unit and one more for each shared tile
    assert L.e0m4_workspace_bytes(1024, 8448, 13696, 128) == 1024 + (256 + 132) * 256 * 256 * 4
    assert L.e0m4_workspace_bytes(1024, 4096, 4160, 64) == 0            # K not a multiple of 128: other kernel


def test_size_queries_of_empty_and_invalid_problems(L):
    """Every size query answers 0 for an empty or invalid problem and never faults (a query with N = 0 once
    divided by a tile count of zero)."""
    L.e0m4_fused_workspace_bytes.restype = ctypes.c_size_t
    L.e0m4_fused_workspace_bytes.argtypes = [ctypes.c_int64] * 3 + [ctypes.c_int] * 3
    L.e0m8_fused_workspace_bytes.restype = ctypes.c_size_t
    L.e0m8_fused_workspace_bytes.argtypes = [ctypes.c_int64] * 3 + [ctypes.c_int] * 3
    L.e0m8_workspace_bytes.restype = ctypes.c_size_t
    L.e0m8_workspace_bytes.argtypes = [ctypes.c_int64] * 3 + [ctypes.c_int]
    for M in (0, 1, 8, 16, 24, 64, 1000, 1024, 4096, -3):
        for N, K in ((0, 4096), (4096, 0), (0, 0), (-1, 128), (128, -128), (128, 100)):
            assert L.e0m4_workspace_bytes(M, N, K, 128) == 0, (M, N, K)
            assert L.e0m8_workspace_bytes(M, N, K, 128) == 0, (M, N, K)
            for norm in (0, 1):
                for epi in (0, 1):
                    assert L.e0m4_fused_workspace_bytes(M, N, K, 128, norm, epi) == 0, (M, N, K)
                    assert L.e0m8_fused_workspace_bytes(M, N, K, 128, norm, epi) == 0, (M, N, K)
    for M in (0, -1):
        assert L.e0m4_workspace_bytes(M, 4096, 4096, 128) == 0
        assert L.e0m8_workspace_bytes(M, 4096, 4096, 128) == 0
        assert L.e0m4_fused_workspace_bytes(M, 4096, 4096, 128, 1, 1) == 0
    assert L.e0m4_workspace_bytes(1024, 4096, 4096, 48) == 0            # bad group
    assert L.e0m4_codes_bytes(0, 0, 128) == 0 and L.e0m4_params_elems(0, 128, 128) == 0
    assert L.e0m8_codes_bytes(0, 128, 128) == 0


def test_knobs_belong_to_the_calling_thread(L):
    """A diagnostic knob set by one thread changes neither the size queries nor the dispatch of another."""
    import threading

    shape = (1024, 4096, 13696, 128)
    base = L.e0m4_workspace_bytes(*shape)
    assert base > 0 and base % (1024 * 4096 * 4) == 0
    seen = {}

    def other():
        assert L.e0m4_set_knob(b"gemm_splits", 3) == 0
        seen["other"] = L.e0m4_workspace_bytes(*shape)
        # left set on purpose: it must die with the thread

    th = threading.Thread(target=other)
    th.start()
    th.join()
    assert seen["other"] == 3 * 1024 * 4096 * 4 != base
    assert L.e0m4_workspace_bytes(*shape) == base


def test_error_codes_before_any_launch(L):
    p = ctypes.c_void_p(0x1000)         # aligned, never dereferenced: every call below fails validation first
    odd = ctypes.c_void_p(0x1008)
    null = ctypes.c_void_p(0)
    ERR_NULL, ERR_SHAPE, ERR_GROUP, ERR_ALIGN, ERR_WS = -1, -2, -3, -4, -5
    assert L.e0m4_quantize(p, 64, 100, 128, p, p, p, null) == ERR_SHAPE      # K % 32
    assert L.e0m4_quantize(p, 64, 192, 128, p, p, p, null) == ERR_SHAPE      # K % group
    assert L.e0m4_quantize(p, -1, 128, 128, p, p, p, null) == ERR_SHAPE
    assert L.e0m4_quantize(p, 64, 128, 16, p, p, p, null) == ERR_GROUP
    assert L.e0m4_quantize(p, 64, 128, 256, p, p, p, null) == ERR_GROUP
    assert L.e0m4_quantize(null, 64, 128, 128, p, p, p, null) == ERR_NULL
    assert L.e0m4_quantize(p, 64, 128, 128, p, null, p, null) == ERR_NULL
    assert L.e0m4_quantize(odd, 64, 128, 128, p, p, p, null) == ERR_ALIGN
    assert L.e0m4_encode(p, 64, 128, 128, null, p, p, null) == ERR_NULL
    assert L.e0m4_dequant(p, p, p, 64, 128, 128, null, null) == ERR_NULL
    assert L.e0m4_dequant(p, p, p, 64, 128, 128, odd, null) == ERR_ALIGN
    assert L.e0m4_unpack_codes(p, 64, 130, 32, p, null) == ERR_SHAPE
    assert L.e0m4_matmul(p, 1, p, p, p, 64, 100, 128, p, null, 0, null) == ERR_SHAPE
    assert L.e0m4_matmul(p, -1, p, p, p, 64, 128, 128, p, null, 0, null) == ERR_SHAPE
    assert L.e0m4_matmul(p, 1, p, p, p, 64, (1 << 20) + 128, 128, p, null, 0, null) == ERR_SHAPE     # K above its limit
    assert L.e0m4_quantize(p, (1 << 31) + 1, 128, 128, p, p, p, null) == ERR_SHAPE
    assert L.e0m4_matmul(null, 1, p, p, p, 64, 128, 128, p, null, 0, null) == ERR_NULL
    assert L.e0m4_matmul(p, 1, p, p, p, 64, 128, 128, odd, null, 0, null) == ERR_ALIGN
    assert L.e0m4_matmul(p, 1, null, p, p, 64, 128, 128, p, null, 0, null) == ERR_NULL
    assert ERR_WS == -5
    # empty problems succeed without touching anything
    assert L.e0m4_quantize(null, 0, 128, 128, null, null, null, null) == 0
    assert L.e0m4_matmul(null, 0, null, null, null, 64, 128, 128, null, null, 0, null) == 0
    assert L.e0m4_matmul(null, 4, null, null, null, 0, 128, 128, null, null, 0, null) == 0
    for code in (0, -1, -2, -3, -4, -5, -6, -99):
        assert L.e0m4_strerror(code)
    assert L.e0m4_set_knob(b"no_such_knob", 1) == ERR_SHAPE
    assert L.e0m4_set_knob(b"gemv_waves", 0) == 0


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    from paper_2403_20041_amd import binding

    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "libe0m4.so"))
    with pytest.raises(RuntimeError, match="not built"):
        binding.lib()


def test_product_does_not_import_oracle():
    pkg = os.path.join(ROOT, "paper_2403_20041_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".hpp", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), os.path.join(dirpath, f)
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c", ".h")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2403_20041_amd" not in text and "libe0m4.so" not in text


def test_fused_matmul_validation_and_workspace(L):
    L.e0m4_matmul_fused.restype = ctypes.c_int
    L.e0m4_matmul_fused.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_float, ctypes.c_void_p,
                                    ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
                                    ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    L.e0m4_fused_workspace_bytes.restype = ctypes.c_size_t
    L.e0m4_fused_workspace_bytes.argtypes = [ctypes.c_int64] * 3 + [ctypes.c_int] * 3
    p, odd, null = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1008), ctypes.c_void_p(0)
    ERR_NULL, ERR_SHAPE, ERR_GROUP, ERR_ALIGN, ERR_WS = -1, -2, -3, -4, -5
    NONE, SWIGLU = 0, 1
    f = L.e0m4_matmul_fused
    assert f(p, 1, null, 0.0, p, 128, 100, 128, NONE, null, p, null, 0, null) == ERR_SHAPE       # K % 32
    assert f(p, 1, null, 0.0, p, 128, 128, 48, NONE, null, p, null, 0, null) == ERR_GROUP
    assert f(p, 1, null, 0.0, p, 128, 128, 128, 2, null, p, null, 0, null) == ERR_SHAPE          # unknown epilogue
    assert f(p, 1, null, 0.0, p, 96, 128, 128, SWIGLU, null, p, null, 0, null) == ERR_SHAPE      # N not a multiple of 64
    assert f(p, 1, null, 0.0, p, 128, 0, 128, NONE, null, p, null, 0, null) == ERR_SHAPE         # nothing to contract
    assert f(null, 1, null, 0.0, p, 128, 128, 128, NONE, null, p, null, 0, null) == ERR_NULL
    assert f(p, 1, null, 0.0, p, 128, 128, 128, NONE, null, null, null, 0, null) == ERR_NULL
    assert f(p, 1, odd, 0.0, p, 128, 128, 128, NONE, null, p, null, 0, null) == ERR_ALIGN        # gamma
    assert f(p, 1, null, 0.0, p, 128, 128, 128, NONE, odd, p, null, 0, null) == ERR_ALIGN        # residual
    assert f(p, 300, p, 0.0, p, 128, 128, 128, NONE, null, p, null, 0, null) == ERR_NULL         # GEMM path needs a workspace
    assert f(p, 300, p, 0.0, p, 128, 128, 128, NONE, null, p, p, 64, null) == ERR_WS
    assert f(null, 0, null, 0.0, null, 128, 128, 128, SWIGLU, null, null, null, 0, null) == 0    # empty problem
    w = L.e0m4_fused_workspace_bytes
    assert w(1, 27392, 4096, 128, 1, SWIGLU) == 0               # decode: everything stays in the one kernel
    assert w(8, 4096, 4096, 128, 1, NONE) == 0
    assert w(16, 4096, 16384, 128, 1, SWIGLU) == 0              # X longer than the LDS: still one kernel (K in phases)
    assert w(17, 4096, 16384, 128, 1, SWIGLU) > 0               # GEMM path: normalised copy of X
    assert w(24, 4096, 4096, 128, 1, NONE) == 0                 # two chunks of rows on the small-batch kernel
    assert w(48, 4096, 4096, 128, 1, NONE) == 0                 # three chunks: three rounds of its 256 workgroups, small weights
    assert w(64, 4096, 4096, 128, 1, NONE) > 0                  # four rounds: the GEMM, with its normalised copy of X
    assert w(64, 4608, 4096, 128, 1, NONE) == 0                 # 144 workgroups: four chunks make three rounds
    assert L.e0m4_workspace_bytes(24, 4096, 4096, 128) == 0
    assert L.e0m4_workspace_bytes(24, 27392, 4096, 128) > 0     # large weights: the GEMM, split along K
    assert w(1024, 27392, 4096, 128, 1, SWIGLU) == 1024 * 4096 * 2         # normalised X; enough tiles, no K split
    assert w(1024, 27392, 4096, 128, 0, SWIGLU) == 0
    assert w(1024, 4096, 13696, 128, 0, NONE) == L.e0m4_workspace_bytes(1024, 4096, 13696, 128) > 0
    assert w(1024, 4096, 13696, 128, 1, NONE) == 1024 * 13696 * 2 + L.e0m4_workspace_bytes(1024, 4096, 13696, 128)
    assert w(1024, 4096, 4096, 128, 1, 5) == 0


def test_kv_append_validation(L):
    L.e0m4_kv_append.restype = ctypes.c_int
    L.e0m4_kv_append.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64,
                                 ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p]
    p, odd, null = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1004), ctypes.c_void_p(0)
    ERR_NULL, ERR_SHAPE, ERR_ALIGN = -1, -2, -4
    f = L.e0m4_kv_append
    assert f(p, 16, 12, p, 1, 16, p, null) == ERR_SHAPE         # row not a multiple of 8
    assert f(p, 16, 16, p, 1, 20, p, null) == ERR_SHAPE         # source stride not a multiple of 8
    assert f(p, 16, 16, p, 1, 8, p, null) == ERR_SHAPE          # source stride shorter than a row
    assert f(p, -1, 16, p, 1, 16, p, null) == ERR_SHAPE
    assert f(null, 16, 16, p, 1, 16, p, null) == ERR_NULL
    assert f(p, 16, 16, p, 1, 16, null, null) == ERR_NULL
    assert f(p, 16, 16, ctypes.c_void_p(0x1008), 1, 16, p, null) == ERR_ALIGN
    assert f(p, 16, 16, p, 1, 16, odd, null) == ERR_ALIGN       # position_ids are 8-byte integers
    assert f(null, 16, 16, null, 0, 16, null, null) == 0        # nothing to append


def test_e0m8_validation_and_sizes(L):
    for name, res, args in (("e0m8_codes_bytes", ctypes.c_size_t, [ctypes.c_int64, ctypes.c_int64, ctypes.c_int]),
                            ("e0m8_quantize", ctypes.c_int, [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int]
                             + [ctypes.c_void_p] * 4),
                            ("e0m8_dequant", ctypes.c_int, [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int,
                                                            ctypes.c_void_p, ctypes.c_void_p]),
                            ("e0m8_matmul", ctypes.c_int, [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64,
                                                           ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
                                                           ctypes.c_size_t, ctypes.c_void_p]),
                            ("e0m8_workspace_bytes", ctypes.c_size_t, [ctypes.c_int64] * 3 + [ctypes.c_int])):
        getattr(L, name).restype = res
        getattr(L, name).argtypes = args
    p, odd, null = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1008), ctypes.c_void_p(0)
    ERR_NULL, ERR_SHAPE, ERR_GROUP, ERR_ALIGN = -1, -2, -3, -4
    blk = 1024 + 64                                         # 16 rows x 64 weights + 16 (scale, bias) words
    assert L.e0m8_codes_bytes(4096, 4096, 128) == 256 * 64 * blk      # twice the 4-bit size
    assert L.e0m8_codes_bytes(17, 192, 64) == 2 * 3 * blk
    assert L.e0m8_codes_bytes(64, 200, 64) == 0
    assert L.e0m8_codes_bytes(64, 128, 32) == 0
    assert L.e0m8_quantize(p, 64, 128, 32, p, p, p, null) == ERR_GROUP
    assert L.e0m8_quantize(p, 64, 200, 64, p, p, p, null) == ERR_SHAPE
    assert L.e0m8_quantize(p, 64, (1 << 19) + 128, 128, p, p, p, null) == ERR_SHAPE     # K above its limit
    assert L.e0m8_quantize(null, 64, 128, 64, p, p, p, null) == ERR_NULL
    assert L.e0m8_quantize(odd, 64, 128, 64, p, p, p, null) == ERR_ALIGN
    assert L.e0m8_dequant(p, 64, 128, 64, null, null) == ERR_NULL
    assert L.e0m8_matmul(p, 1, p, 64, 128, 64, odd, null, 0, null) == ERR_ALIGN
    assert L.e0m8_matmul(p, 40, p, 68, 192, 64, p, null, 0, null) == ERR_SHAPE          # row chunks of Y need N % 8 == 0
    assert L.e0m8_matmul(null, 0, null, 64, 128, 64, null, null, 0, null) == 0
    assert L.e0m8_matmul(p, 1024, p, 4096, 13696, 128, p, null, 0, null) == -5          # split K: workspace needed
    assert L.e0m8_workspace_bytes(8, 4096, 4096, 128) == 0
    assert L.e0m8_workspace_bytes(1024, 4096, 13696, 128) == L.e0m4_workspace_bytes(1024, 4096, 13696, 128) > 0
    assert L.e0m8_workspace_bytes(1024, 4096, 192, 64) == 0                             # K % 128 != 0: decode kernel, row chunks
    # the fused matmul on 8-bit codes
    L.e0m8_fused_workspace_bytes.restype = ctypes.c_size_t
    L.e0m8_fused_workspace_bytes.argtypes = [ctypes.c_int64] * 3 + [ctypes.c_int] * 3
    L.e0m8_matmul_fused.restype = ctypes.c_int
    L.e0m8_matmul_fused.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_float, ctypes.c_void_p,
                                    ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
                                    ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    assert L.e0m8_matmul_fused(p, 1, null, 0.0, p, 96, 128, 64, 1, null, p, null, 0, null) == ERR_SHAPE   # gated: N % 64
    assert L.e0m8_matmul_fused(p, 1, null, 0.0, p, 128, 128, 64, 7, null, p, null, 0, null) == ERR_SHAPE  # epilogue
    assert L.e0m8_matmul_fused(p, 1, null, 0.0, p, 128, 128, 32, 0, null, p, null, 0, null) == ERR_GROUP
    assert L.e0m8_matmul_fused(p, 1, odd, 0.0, p, 128, 128, 64, 0, null, p, null, 0, null) == ERR_ALIGN
    assert L.e0m8_matmul_fused(p, 1, null, 0.0, p, 128, 128, 64, 0, odd, p, null, 0, null) == ERR_ALIGN
    assert L.e0m8_matmul_fused(null, 1, null, 0.0, p, 128, 128, 64, 0, null, p, null, 0, null) == ERR_NULL
    assert L.e0m8_matmul_fused(null, 0, null, 0.0, null, 128, 128, 64, 0, null, null, null, 0, null) == 0
    assert L.e0m8_matmul_fused(p, 40, null, 0.0, p, 128, 192, 64, 0, null, p, null, 0, null) == ERR_SHAPE  # M > 16: K % 128
    assert L.e0m8_matmul_fused(p, 1024, p, 1e-5, p, 4096, 4096, 128, 0, null, p, null, 0, null) == ERR_NULL  # workspace
    assert L.e0m8_fused_workspace_bytes(8, 27392, 4096, 128, 1, 1) == 0
    assert (L.e0m8_fused_workspace_bytes(1024, 4096, 4096, 128, 1, 0) - L.e0m8_fused_workspace_bytes(1024, 4096, 4096, 128, 0, 0)
            == 1024 * 4096 * 2)                                                         # the normalised copy of X
    assert L.e0m8_fused_workspace_bytes(1024, 4096, 13696, 128, 0, 0) == L.e0m4_fused_workspace_bytes(1024, 4096, 13696, 128, 0, 0) > 0
