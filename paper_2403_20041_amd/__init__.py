"""E0M4 FP4 weight-only quantised matmul for MI355X: Python face of libe0m4.

The package holds the HIP sources (``csrc/``), the in-tree build
(``build.py``) and a ctypes binding with the same names as the C entry points.
"""
from .binding import (  # noqa: F401
    E0M4_EPILOGUE_NONE,
    E0M4_EPILOGUE_SWIGLU,
    E0M4_STATIC_SCRATCH_BYTES,
    E0M4Error,
    alloc_packed,
    e0m4_codes_bytes,
    e0m4_dequant,
    e0m4_encode,
    e0m4_fused_workspace_bytes,
    e0m4_int4_dequant,
    e0m4_int4_gemv,
    e0m4_int4_quantize,
    e0m4_kv_append,
    e0m4_matmul,
    e0m4_matmul_static,
    e0m4_matmul_fused,
    e0m4_params_elems,
    e0m4_quantize,
    e0m4_set_knob,
    e0m4_unpack_codes,
    e0m4_workspace_bytes,
    e0m8_codes_bytes,
    e0m8_dequant,
    e0m8_matmul,
    e0m8_matmul_fused,
    e0m8_quantize,
    e0m8_unpack_codes,
    e0m8_workspace_bytes,
    lib,
)
