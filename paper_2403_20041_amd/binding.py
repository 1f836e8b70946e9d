"""ctypes binding of libe0m4: argument marshalling only.

Every function has the name of the C entry point it calls (see
``include/e0m4.h``) and does nothing but turn torch tensors into device
pointers and sizes; all arithmetic happens in the HIP kernels.  torch is used
for device memory and streams.  There is no CPU fallback: if the shared
library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libe0m4.so")

_lib = None


class E0M4Error(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = lib().e0m4_strerror(code).decode()
        if code == -6:
            msg += ": " + lib().e0m4_last_hip_error().decode()
        super().__init__("%s failed (%d): %s" % (where, code, msg))


def lib() -> ctypes.CDLL:
    """Load libe0m4.so (built in-tree by ``paper_2403_20041_amd.build``); fails loudly if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            "libe0m4.so is not built: run `python -m paper_2403_20041_amd.build` (needs hipcc); "
            "there is no fallback path")
    L = ctypes.CDLL(LIB_PATH)
    vp, i64, ci, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t
    L.e0m4_abi_version.restype = ci
    L.e0m4_abi_version.argtypes = []
    L.e0m4_strerror.restype = ctypes.c_char_p
    L.e0m4_strerror.argtypes = [ci]
    L.e0m4_last_hip_error.restype = ctypes.c_char_p
    L.e0m4_last_hip_error.argtypes = []
    L.e0m4_codes_bytes.restype = sz
    L.e0m4_codes_bytes.argtypes = [i64, i64, ci]
    L.e0m4_params_elems.restype = sz
    L.e0m4_params_elems.argtypes = [i64, i64, ci]
    L.e0m4_workspace_bytes.restype = sz
    L.e0m4_workspace_bytes.argtypes = [i64, i64, i64, ci]
    L.e0m4_quantize.restype = ci
    L.e0m4_quantize.argtypes = [vp, i64, i64, ci, vp, vp, vp, vp]
    L.e0m4_encode.restype = ci
    L.e0m4_encode.argtypes = [vp, i64, i64, ci, vp, vp, vp, vp]
    L.e0m4_dequant.restype = ci
    L.e0m4_dequant.argtypes = [vp, vp, vp, i64, i64, ci, vp, vp]
    L.e0m4_unpack_codes.restype = ci
    L.e0m4_unpack_codes.argtypes = [vp, i64, i64, ci, vp, vp]
    L.e0m4_matmul.restype = ci
    L.e0m4_matmul.argtypes = [vp, i64, vp, vp, vp, i64, i64, ci, vp, vp, sz, vp]
    L.e0m4_matmul_static.restype = ci
    L.e0m4_matmul_static.argtypes = [vp, i64, vp, i64, i64, ci, vp, vp]
    L.e0m4_fused_workspace_bytes.restype = sz
    L.e0m4_fused_workspace_bytes.argtypes = [i64, i64, i64, ci, ci, ci]
    L.e0m4_matmul_fused.restype = ci
    L.e0m4_matmul_fused.argtypes = [vp, i64, vp, ctypes.c_float, vp, i64, i64, ci, ci, vp, vp, vp, sz, vp]
    L.e0m8_codes_bytes.restype = sz
    L.e0m8_codes_bytes.argtypes = [i64, i64, ci]
    L.e0m8_quantize.restype = ci
    L.e0m8_quantize.argtypes = [vp, i64, i64, ci, vp, vp, vp, vp]
    L.e0m8_dequant.restype = ci
    L.e0m8_dequant.argtypes = [vp, i64, i64, ci, vp, vp]
    L.e0m8_unpack_codes.restype = ci
    L.e0m8_unpack_codes.argtypes = [vp, i64, i64, ci, vp, vp]
    L.e0m8_matmul.restype = ci
    L.e0m8_matmul.argtypes = [vp, i64, vp, i64, i64, ci, vp, vp, sz, vp]
    L.e0m8_fused_workspace_bytes.restype = sz
    L.e0m8_fused_workspace_bytes.argtypes = [i64, i64, i64, ci, ci, ci]
    L.e0m8_matmul_fused.restype = ci
    L.e0m8_matmul_fused.argtypes = [vp, i64, vp, ctypes.c_float, vp, i64, i64, ci, ci, vp, vp, vp, sz, vp]
    L.e0m8_workspace_bytes.restype = sz
    L.e0m8_workspace_bytes.argtypes = [i64, i64, i64, ci]
    L.e0m4_kv_append.restype = ci
    L.e0m4_kv_append.argtypes = [vp, i64, i64, vp, i64, i64, vp, vp]
    L.e0m4_int4_quantize.restype = ci
    L.e0m4_int4_quantize.argtypes = [vp, i64, i64, ci, vp, vp, vp, vp]
    L.e0m4_int4_dequant.restype = ci
    L.e0m4_int4_dequant.argtypes = [vp, i64, i64, ci, vp, vp]
    L.e0m4_int4_gemv.restype = ci
    L.e0m4_int4_gemv.argtypes = [vp, vp, i64, i64, ci, vp, vp]
    for name in ("e0m3_quantize", "e0m4_bf16_quantize", "e0m4_bf16_encode"):
        getattr(L, name).restype = ci
        getattr(L, name).argtypes = [vp, i64, i64, ci, vp, vp, vp, vp]
    L.e0m3_unpack_codes.restype = ci
    L.e0m3_unpack_codes.argtypes = [vp, i64, i64, ci, vp, vp]
    L.e0m4_bf16_dequant.restype = ci
    L.e0m4_bf16_dequant.argtypes = [vp, i64, i64, ci, vp, vp]
    L.e0m4_bf16_matmul.restype = ci
    L.e0m4_bf16_matmul.argtypes = [vp, i64, vp, i64, i64, ci, vp, vp]
    L.e0m4_set_knob.restype = ci
    L.e0m4_set_knob.argtypes = [ctypes.c_char_p, ci]
    if L.e0m4_abi_version() != 4:
        raise RuntimeError("libe0m4 ABI version mismatch")
    _lib = L
    return L


def _stream(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _empty(shape, dtype, device, stream, what: str):
    """torch.empty for a buffer that the kernels enqueued on `stream` will use.  The caching allocator ties a
    block to the stream that was current when it was allocated, so the buffer is allocated with `stream`
    current; a raw stream handle that is not the current stream cannot be made current here, and the caller
    must then own the buffer."""
    if stream is None:
        return torch.empty(shape, dtype=dtype, device=device)
    if hasattr(stream, "cuda_stream"):
        with torch.cuda.stream(stream):
            return torch.empty(shape, dtype=dtype, device=device)
    if int(stream) == torch.cuda.current_stream(device).cuda_stream:
        return torch.empty(shape, dtype=dtype, device=device)
    raise ValueError("%s: pass a caller-owned tensor when `stream` is a raw handle other than torch's current stream"
                     % what)


def _ptr(t) -> int:
    return 0 if t is None else t.data_ptr()


def _check(rc: int, where: str):
    if rc != 0:
        raise E0M4Error(rc, where)


def _need(t: torch.Tensor, dtype, shape, name: str):
    if t.dtype != dtype or tuple(t.shape) != tuple(shape) or not t.is_contiguous() or not t.is_cuda:
        raise ValueError("%s must be a contiguous cuda %s tensor of shape %s, got %s %s on %s"
                         % (name, dtype, tuple(shape), t.dtype, tuple(t.shape), t.device))


def e0m4_codes_bytes(N: int, K: int, group: int) -> int:
    return lib().e0m4_codes_bytes(N, K, group)


def e0m4_params_elems(N: int, K: int, group: int) -> int:
    return lib().e0m4_params_elems(N, K, group)


def e0m4_workspace_bytes(M: int, N: int, K: int, group: int) -> int:
    return lib().e0m4_workspace_bytes(M, N, K, group)


def e0m4_set_knob(name: str, value: int) -> None:
    _check(lib().e0m4_set_knob(name.encode(), int(value)), "e0m4_set_knob")


def alloc_packed(N: int, K: int, group: int, device):
    """Uninitialised output buffers for e0m4_quantize: (codes u8, scales f16 [N,K/G], bias f16 [N,K/G])."""
    codes = torch.empty(max(e0m4_codes_bytes(N, K, group), 16), dtype=torch.uint8, device=device)
    scales = torch.empty((N, K // group), dtype=torch.float16, device=device)
    bias = torch.empty((N, K // group), dtype=torch.float16, device=device)
    return codes, scales, bias


def e0m4_quantize(W: torch.Tensor, group: int, out=None, stream=None):
    """W [N,K] fp16 -> (codes, scales, bias); see include/e0m4.h."""
    N, K = W.shape
    _need(W, torch.float16, (N, K), "W")
    codes, scales, bias = out if out is not None else alloc_packed(N, K, group, W.device)
    _check(lib().e0m4_quantize(_ptr(W), N, K, group, _ptr(codes), _ptr(scales), _ptr(bias), _stream(stream)),
           "e0m4_quantize")
    return codes, scales, bias


def e0m4_encode(W: torch.Tensor, scales: torch.Tensor, bias: torch.Tensor, group: int, codes=None, stream=None):
    N, K = W.shape
    _need(W, torch.float16, (N, K), "W")
    _need(scales, torch.float16, (N, K // group), "scales")
    _need(bias, torch.float16, (N, K // group), "bias")
    if codes is None:
        codes = torch.empty(max(e0m4_codes_bytes(N, K, group), 16), dtype=torch.uint8, device=W.device)
    _check(lib().e0m4_encode(_ptr(W), N, K, group, _ptr(scales), _ptr(bias), _ptr(codes), _stream(stream)),
           "e0m4_encode")
    return codes


def e0m4_dequant(codes, scales, bias, N: int, K: int, group: int, out=None, stream=None) -> torch.Tensor:
    if out is None:
        out = torch.empty((N, K), dtype=torch.float16, device=codes.device)
    _need(out, torch.float16, (N, K), "out")
    _check(lib().e0m4_dequant(_ptr(codes), _ptr(scales), _ptr(bias), N, K, group, _ptr(out), _stream(stream)),
           "e0m4_dequant")
    return out


def e0m4_unpack_codes(codes, N: int, K: int, group: int, out=None, stream=None) -> torch.Tensor:
    if out is None:
        out = torch.empty((N, K), dtype=torch.uint8, device=codes.device)
    _need(out, torch.uint8, (N, K), "out")
    _check(lib().e0m4_unpack_codes(_ptr(codes), N, K, group, _ptr(out), _stream(stream)), "e0m4_unpack_codes")
    return out


def e0m4_matmul(X, codes, scales, bias, N: int, K: int, group: int, out=None, workspace=None, stream=None):
    """Y [M,N] fp16 = X [M,K] fp16 times the dequantised weights, transposed."""
    M = X.shape[0]
    _need(X, torch.float16, (M, K), "X")
    if out is None:
        out = _empty((M, N), torch.float16, X.device, stream, "out")
    _need(out, torch.float16, (M, N), "out")
    need = e0m4_workspace_bytes(M, N, K, group)
    if workspace is None and need > 0:
        workspace = _empty(need, torch.uint8, X.device, stream, "workspace")
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().e0m4_matmul(_ptr(X), M, _ptr(codes), _ptr(scales), _ptr(bias), N, K, group, _ptr(out),
                             _ptr(workspace), ws_bytes, _stream(stream)), "e0m4_matmul")
    return out


E0M4_STATIC_SCRATCH_BYTES = 128 << 20


def e0m4_matmul_static(X, codes, N: int, K: int, group: int, out, stream=None):
    """e0m4_matmul without a workspace argument: the library's own fixed scratch array serves the split along
    K.  `out` is required, so that the call itself allocates nothing."""
    M = X.shape[0]
    _need(X, torch.float16, (M, K), "X")
    _need(out, torch.float16, (M, N), "out")
    _check(lib().e0m4_matmul_static(_ptr(X), M, _ptr(codes), N, K, group, _ptr(out), _stream(stream)),
           "e0m4_matmul_static")
    return out


E0M4_EPILOGUE_NONE = 0
E0M4_EPILOGUE_SWIGLU = 1


def e0m4_fused_workspace_bytes(M: int, N: int, K: int, group: int, with_rmsnorm: bool, epilogue: int) -> int:
    return lib().e0m4_fused_workspace_bytes(M, N, K, group, 1 if with_rmsnorm else 0, epilogue)


def e0m4_matmul_fused(X, codes, N: int, K: int, group: int, rms_gamma=None, rms_eps: float = 0.0,
                      epilogue: int = E0M4_EPILOGUE_NONE, residual=None, out=None, workspace=None, stream=None):
    """The matmul with rms-norm on X, the SiLU-gated product of the two output halves and a residual add
    folded in (each optional; see include/e0m4.h).  Y is [M, N/2] with the gated epilogue, else [M, N]."""
    M = X.shape[0]
    _need(X, torch.float16, (M, K), "X")
    n_out = N // 2 if epilogue == E0M4_EPILOGUE_SWIGLU else N
    if rms_gamma is not None:
        _need(rms_gamma, torch.float16, (K,), "rms_gamma")
    if residual is not None:
        _need(residual, torch.float16, (M, n_out), "residual")
    if out is None:
        out = _empty((M, n_out), torch.float16, X.device, stream, "out")
    _need(out, torch.float16, (M, n_out), "out")
    need = e0m4_fused_workspace_bytes(M, N, K, group, rms_gamma is not None, epilogue)
    if workspace is None and need > 0:
        workspace = _empty(need, torch.uint8, X.device, stream, "workspace")
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().e0m4_matmul_fused(_ptr(X), M, _ptr(rms_gamma), float(rms_eps), _ptr(codes), N, K, group, epilogue,
                                   _ptr(residual), _ptr(out), _ptr(workspace), ws_bytes, _stream(stream)),
           "e0m4_matmul_fused")
    return out


def e0m4_kv_append(cache, new_rows, position_ids, stream=None):
    """cache [max_seq, row] fp16 is updated in place: cache[position_ids[i]] = new_rows[i].  new_rows may be a
    column slice of a wider matrix (last dimension contiguous); position_ids is an int64 device tensor."""
    max_seq, row = cache.shape
    n_new = new_rows.shape[0]
    if cache.dtype != torch.float16 or new_rows.dtype != torch.float16 or position_ids.dtype != torch.int64:
        raise TypeError("e0m4_kv_append: cache and new_rows must be float16, position_ids int64")
    if not cache.is_contiguous() or new_rows.shape[1] != row or new_rows.stride(1) != 1 or \
            not position_ids.is_contiguous() or position_ids.numel() != n_new:
        raise ValueError("e0m4_kv_append: bad shapes or strides")
    _check(lib().e0m4_kv_append(_ptr(cache), max_seq, row, _ptr(new_rows), n_new, new_rows.stride(0),
                                _ptr(position_ids), _stream(stream)), "e0m4_kv_append")
    return cache


# ---- E0M8, the 8-bit member of the family (see include/e0m4.h) ---------------------------------------

def e0m8_codes_bytes(N: int, K: int, group: int) -> int:
    return lib().e0m8_codes_bytes(N, K, group)


def e0m8_quantize(W: torch.Tensor, group: int, stream=None):
    """W [N,K] fp16 -> (codes packed uint8, scales [N,K/group] fp16, bias [N,K/group] fp16)."""
    N, K = W.shape
    _need(W, torch.float16, (N, K), "W")
    nbytes = e0m8_codes_bytes(N, K, group)
    if nbytes == 0 and N * K > 0:
        raise ValueError("e0m8_quantize: unsupported shape or group")
    codes = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=W.device)
    scales = torch.empty((N, max(K // group, 1)), dtype=torch.float16, device=W.device)
    bias = torch.empty_like(scales)
    _check(lib().e0m8_quantize(_ptr(W), N, K, group, _ptr(codes), _ptr(scales), _ptr(bias), _stream(stream)),
           "e0m8_quantize")
    return codes, scales, bias


def e0m8_dequant(codes, N: int, K: int, group: int, out=None, stream=None) -> torch.Tensor:
    if out is None:
        out = torch.empty((N, K), dtype=torch.float16, device=codes.device)
    _need(out, torch.float16, (N, K), "out")
    _check(lib().e0m8_dequant(_ptr(codes), N, K, group, _ptr(out), _stream(stream)), "e0m8_dequant")
    return out


def e0m8_unpack_codes(codes, N: int, K: int, group: int, stream=None) -> torch.Tensor:
    out = torch.empty((N, K), dtype=torch.uint8, device=codes.device)
    _check(lib().e0m8_unpack_codes(_ptr(codes), N, K, group, _ptr(out), _stream(stream)), "e0m8_unpack_codes")
    return out


def e0m8_workspace_bytes(M: int, N: int, K: int, group: int) -> int:
    return lib().e0m8_workspace_bytes(M, N, K, group)


def e0m8_matmul(X, codes, N: int, K: int, group: int, out=None, workspace=None, stream=None) -> torch.Tensor:
    """Y [M,N] fp16 = X [M,K] fp16 times the dequantised 8-bit weights, transposed."""
    M = X.shape[0]
    _need(X, torch.float16, (M, K), "X")
    if out is None:
        out = _empty((M, N), torch.float16, X.device, stream, "out")
    _need(out, torch.float16, (M, N), "out")
    need = e0m8_workspace_bytes(M, N, K, group)
    if workspace is None and need > 0:
        workspace = _empty(need, torch.uint8, X.device, stream, "workspace")
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().e0m8_matmul(_ptr(X), M, _ptr(codes), N, K, group, _ptr(out), _ptr(workspace), ws_bytes,
                             _stream(stream)), "e0m8_matmul")
    return out


def e0m8_matmul_fused(X, codes, N: int, K: int, group: int, rms_gamma=None, rms_eps: float = 0.0,
                      epilogue: int = E0M4_EPILOGUE_NONE, residual=None, out=None, workspace=None, stream=None):
    """e0m4_matmul_fused on 8-bit codes."""
    M = X.shape[0]
    _need(X, torch.float16, (M, K), "X")
    n_out = N // 2 if epilogue == E0M4_EPILOGUE_SWIGLU else N
    if rms_gamma is not None:
        _need(rms_gamma, torch.float16, (K,), "rms_gamma")
    if residual is not None:
        _need(residual, torch.float16, (M, n_out), "residual")
    if out is None:
        out = _empty((M, n_out), torch.float16, X.device, stream, "out")
    _need(out, torch.float16, (M, n_out), "out")
    need = lib().e0m8_fused_workspace_bytes(M, N, K, group, 1 if rms_gamma is not None else 0, epilogue)
    if workspace is None and need > 0:
        workspace = _empty(need, torch.uint8, X.device, stream, "workspace")
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().e0m8_matmul_fused(_ptr(X), M, _ptr(rms_gamma), float(rms_eps), _ptr(codes), N, K, group, epilogue,
                                   _ptr(residual), _ptr(out), _ptr(workspace), ws_bytes, _stream(stream)),
           "e0m8_matmul_fused")
    return out


# ---- INT4 twin (see include/e0m4.h) ------------------------------------------------------------

def e0m4_int4_quantize(W: torch.Tensor, group: int, out=None, stream=None):
    """W [N,K] fp16 -> (codes, scales, zeros) in the INT4 comparison format."""
    N, K = W.shape
    _need(W, torch.float16, (N, K), "W")
    codes, scales, zeros = out if out is not None else alloc_packed(N, K, group, W.device)
    _check(lib().e0m4_int4_quantize(_ptr(W), N, K, group, _ptr(codes), _ptr(scales), _ptr(zeros), _stream(stream)),
           "e0m4_int4_quantize")
    return codes, scales, zeros


def e0m4_int4_dequant(codes, N: int, K: int, group: int, out=None, stream=None) -> torch.Tensor:
    if out is None:
        out = torch.empty((N, K), dtype=torch.float16, device=codes.device)
    _need(out, torch.float16, (N, K), "out")
    _check(lib().e0m4_int4_dequant(_ptr(codes), N, K, group, _ptr(out), _stream(stream)), "e0m4_int4_dequant")
    return out


def e0m4_int4_gemv(X, codes, N: int, K: int, group: int, out=None, stream=None) -> torch.Tensor:
    """Y [1,N] fp16 = X [1,K] fp16 times the dequantised INT4 weights, transposed."""
    _need(X, torch.float16, (1, K), "X")
    if out is None:
        out = torch.empty((1, N), dtype=torch.float16, device=X.device)
    _need(out, torch.float16, (1, N), "out")
    _check(lib().e0m4_int4_gemv(_ptr(X), _ptr(codes), N, K, group, _ptr(out), _stream(stream)), "e0m4_int4_gemv")
    return out


# ---- E0M3 (3-bit codes in 4-bit slots) and E0M4 on bfloat16 (see include/e0m4.h) -----------------

def e0m3_quantize(W: torch.Tensor, group: int, stream=None):
    """W [N,K] fp16 -> (codes, scales, bias); the buffer is read by e0m4_dequant / e0m4_matmul unchanged."""
    N, K = W.shape
    _need(W, torch.float16, (N, K), "W")
    codes, scales, bias = alloc_packed(N, K, group, W.device)
    _check(lib().e0m3_quantize(_ptr(W), N, K, group, _ptr(codes), _ptr(scales), _ptr(bias), _stream(stream)),
           "e0m3_quantize")
    return codes, scales, bias


def e0m3_unpack_codes(codes, N: int, K: int, group: int, stream=None) -> torch.Tensor:
    out = torch.empty((N, K), dtype=torch.uint8, device=codes.device)
    _check(lib().e0m3_unpack_codes(_ptr(codes), N, K, group, _ptr(out), _stream(stream)), "e0m3_unpack_codes")
    return out


def e0m4_bf16_quantize(W: torch.Tensor, group: int, stream=None):
    """W [N,K] bfloat16 -> (codes, scales bf16 [N,K/G], bias bf16 [N,K/G])."""
    N, K = W.shape
    _need(W, torch.bfloat16, (N, K), "W")
    codes = torch.empty(max(e0m4_codes_bytes(N, K, group), 16), dtype=torch.uint8, device=W.device)
    scales = torch.empty((N, K // group), dtype=torch.bfloat16, device=W.device)
    bias = torch.empty((N, K // group), dtype=torch.bfloat16, device=W.device)
    _check(lib().e0m4_bf16_quantize(_ptr(W), N, K, group, _ptr(codes), _ptr(scales), _ptr(bias), _stream(stream)),
           "e0m4_bf16_quantize")
    return codes, scales, bias


def e0m4_bf16_encode(W: torch.Tensor, scales: torch.Tensor, bias: torch.Tensor, group: int, stream=None):
    N, K = W.shape
    _need(W, torch.bfloat16, (N, K), "W")
    _need(scales, torch.bfloat16, (N, K // group), "scales")
    _need(bias, torch.bfloat16, (N, K // group), "bias")
    codes = torch.empty(max(e0m4_codes_bytes(N, K, group), 16), dtype=torch.uint8, device=W.device)
    _check(lib().e0m4_bf16_encode(_ptr(W), N, K, group, _ptr(scales), _ptr(bias), _ptr(codes), _stream(stream)),
           "e0m4_bf16_encode")
    return codes


def e0m4_bf16_dequant(codes, N: int, K: int, group: int, out=None, stream=None) -> torch.Tensor:
    if out is None:
        out = torch.empty((N, K), dtype=torch.bfloat16, device=codes.device)
    _need(out, torch.bfloat16, (N, K), "out")
    _check(lib().e0m4_bf16_dequant(_ptr(codes), N, K, group, _ptr(out), _stream(stream)), "e0m4_bf16_dequant")
    return out


def e0m4_bf16_matmul(X, codes, N: int, K: int, group: int, out=None, stream=None) -> torch.Tensor:
    """Y [M,N] bfloat16 = X [M,K] bfloat16 times the dequantised weights, transposed."""
    M = X.shape[0]
    _need(X, torch.bfloat16, (M, K), "X")
    if out is None:
        out = _empty((M, N), torch.bfloat16, X.device, stream, "out")
    _need(out, torch.bfloat16, (M, N), "out")
    _check(lib().e0m4_bf16_matmul(_ptr(X), M, _ptr(codes), N, K, group, _ptr(out), _stream(stream)), "e0m4_bf16_matmul")
    return out
