"""e0m4_matmul_static, the entry point for callers that cannot allocate: through the C ABI it must reproduce
e0m4_matmul bit for bit (same kernels, fixed reduction order) on calls in a row that share the library's one
scratch array, the later ones with smaller inputs; it must reject what does not fit the array; and it must not
allocate device memory."""
import ctypes

import numpy as np
import pytest

import synth_inputs
from test_gpu_parity import DEV, bits, check_matmul, e0m4, to_dev, torch  # noqa: F401

pytestmark = pytest.mark.gpu

G = 128
# (M, N, K): split-K GEMM with the large tile, the same with a smaller input, the flat tile, a decode call
# (no scratch at all), a GEMM with enough tiles to need none, and one whose 132 tiles are shared out evenly over the
# compute units (counters and one fp32 slab per compute unit and per tile: 97 MiB of the array)
CALLS = [(1024, 1280, 4096), (640, 1040, 2048), (300, 520, 2048), (1, 1040, 2048), (512, 8192, 256), (1024, 8448, 13696)]


def test_static_scratch_matmul_matches_the_workspace_form(e0m4, oracle):
    L = e0m4.lib()
    stream = torch.cuda.current_stream().cuda_stream
    prepared = []
    for i, (M, N, K) in enumerate(CALLS):
        W = synth_inputs.weights_device(N, K, 4100 + i, DEV)
        codes, _, _ = e0m4.e0m4_quantize(W, G)
        X = synth_inputs.activations_device(M, K, 4200 + i, DEV)
        need = e0m4.e0m4_workspace_bytes(M, N, K, G)
        ws = torch.empty(max(need, 16), dtype=torch.uint8, device=DEV)
        want = e0m4.e0m4_matmul(X, codes, None, None, N, K, G, workspace=ws)
        got = torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV)
        prepared.append((M, N, K, X, codes, want, got, need))
    assert prepared[0][7] > prepared[1][7] > prepared[2][7] > 0 and prepared[3][7] == 0
    assert prepared[5][7] == 1024 + (256 + 132) * 256 * 256 * 4 <= e0m4.E0M4_STATIC_SCRATCH_BYTES
    # the first call on a device is the set-up call: it looks up the address of the library's scratch array
    # (the runtime binds the array's 128 MiB to the device then); nothing after it may allocate
    M, N, K, X, codes, want, got, need = prepared[0]
    assert L.e0m4_matmul_static(X.data_ptr(), M, codes.data_ptr(), N, K, G, got.data_ptr(), stream) == 0
    torch.cuda.synchronize()
    mem_before = torch.cuda.memory_allocated(), torch.cuda.memory_reserved()
    free_before = torch.cuda.mem_get_info()[0]
    for rnd in range(2):                                # twice over: the array keeps the last call's contents
        for M, N, K, X, codes, want, got, need in prepared:
            rc = L.e0m4_matmul_static(X.data_ptr(), M, codes.data_ptr(), N, K, G, got.data_ptr(), stream)
            assert rc == 0, (rc, M, N, K)
    torch.cuda.synchronize()
    assert (torch.cuda.memory_allocated(), torch.cuda.memory_reserved()) == mem_before
    assert torch.cuda.mem_get_info()[0] >= free_before - (1 << 20)      # nothing was allocated behind torch's back either
    for M, N, K, X, codes, want, got, need in prepared:
        assert np.array_equal(bits(got), bits(want)), (M, N, K)
    # and against the oracle, on the smaller split-K case
    M, N, K, X, codes, want, got, need = prepared[2]
    Wd = e0m4.e0m4_dequant(codes, None, None, N, K, G).cpu().numpy()
    Yref, absdot = oracle.matmul(X.cpu().numpy(), Wd)
    check_matmul(got, Yref, absdot, "static scratch")


def test_static_scratch_matmul_rejects_what_does_not_fit(e0m4):
    L = e0m4.lib()
    p = ctypes.c_void_p(0x1000)
    M, N, K = 2048, 8192, 4096                          # 256 large tiles: no split by default ...
    assert e0m4.e0m4_workspace_bytes(M, N, K, G) == 0
    e0m4.e0m4_set_knob("gemm_splits", 4)                # ... four slabs of 64 MiB when forced: twice the array
    try:
        assert e0m4.e0m4_workspace_bytes(M, N, K, G) > e0m4.E0M4_STATIC_SCRATCH_BYTES
        assert L.e0m4_matmul_static(p, M, p, N, K, G, p, None) == -5        # nothing was enqueued
    finally:
        e0m4.e0m4_set_knob("gemm_splits", 0)
    assert L.e0m4_matmul_static(p, 1, p, 64, 100, G, p, None) == -2         # same shape rules as e0m4_matmul
    assert L.e0m4_matmul_static(None, 1024, p, 1280, 4096, G, p, None) == -1
    assert L.e0m4_matmul_static(None, 0, None, 64, 128, G, None, None) == 0
