"""Two host threads, each on its own stream, issue e0m4_matmul at the same time: the library keeps no
state between calls (the diagnostic knobs belong to the calling thread), so both must match the oracle, with
one thread forcing kernel variants through its knobs while the other runs the defaults."""
import threading

import numpy as np
import pytest

import synth_inputs
from test_gpu_parity import DEV, check_matmul, e0m4, to_dev, torch  # noqa: F401

pytestmark = pytest.mark.gpu


def test_matmul_from_two_threads_on_two_streams(e0m4, oracle):
    G = 128
    cases = [(1, 1040, 2048, 31), (300, 520, 2048, 32)]            # decode kernel; GEMM, split along K
    prepared = []
    for M, N, K, seed in cases:
        W = synth_inputs.weights(N, K, seed=seed)
        X = synth_inputs.activations(M, K, seed=seed + 1)
        oc, os_, ob = oracle.quantize(W, G)
        What = oracle.dequant(oc, os_, ob, G)
        Yref, absdot = oracle.matmul(X, What)
        codes, _, _ = e0m4.e0m4_quantize(to_dev(W), G)
        prepared.append((M, N, K, to_dev(X), codes, Yref, absdot))
    torch.cuda.synchronize()
    default_ws = e0m4.e0m4_workspace_bytes(300, 520, 2048, G)
    results, errors = {}, []
    start = threading.Barrier(2)

    def worker(idx, knobs):
        try:
            M, N, K, X, codes, _, _ = prepared[idx]
            torch.cuda.set_device(0)
            stream = torch.cuda.Stream()
            for name, value in knobs:
                e0m4.e0m4_set_knob(name, value)
            need = e0m4.e0m4_workspace_bytes(M, N, K, G)        # this thread's own view
            with torch.cuda.stream(stream):
                ws = torch.empty(max(need, 16), dtype=torch.uint8, device=DEV)
                outs = []
                start.wait()
                for _ in range(8):
                    outs.append(e0m4.e0m4_matmul(X, codes, None, None, N, K, G, workspace=ws, stream=stream))
            stream.synchronize()
            results[idx] = (outs, need)
        except Exception as exc:               # noqa: BLE001
            errors.append((idx, repr(exc)))
            try:
                start.abort()
            except Exception:                   # noqa: BLE001
                pass

    threads = [threading.Thread(target=worker, args=(0, [("gemv_waves", 4)])),
               threading.Thread(target=worker, args=(1, []))]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    assert results[1][1] == default_ws                  # the other thread's knobs did not leak into this one
    for idx, (M, N, K, X, codes, Yref, absdot) in enumerate(prepared):
        outs, _ = results[idx]
        for y in outs:
            check_matmul(y, Yref, absdot, "thread %d" % idx)
        for y in outs[1:]:
            assert torch.equal(y, outs[0])              # deterministic under concurrency
    assert e0m4.e0m4_workspace_bytes(300, 520, 2048, G) == default_ws       # and not into the main thread
