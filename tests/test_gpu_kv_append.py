"""Parity of e0m4_kv_append (paper: section "KV cache copy optimization") with the CPU oracle, bit for bit,
through the C ABI: the whole cache is compared, so rows that must stay untouched are covered too."""
import numpy as np
import pytest

import synth_inputs

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

DEV = "cuda:0"


@pytest.fixture(scope="module")
def e0m4():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (run with -m 'not gpu' elsewhere)")
    import paper_2403_20041_amd as pkg

    pkg.lib()                                   # raises if the HIP library is not built
    return pkg


def run_case(e0m4, oracle, max_seq, row, n_new, ld, col, pos, seed):
    cache = synth_inputs.activations(max_seq, row, seed=seed)
    wide = synth_inputs.activations(n_new, ld, seed=seed + 1)              # e.g. the QKV projection's output
    new = wide[:, col:col + row]
    want = oracle.kv_append(cache, new, pos)
    c_dev = torch.from_numpy(cache).to(DEV)
    w_dev = torch.from_numpy(wide).to(DEV)
    p_dev = torch.from_numpy(np.asarray(pos, dtype=np.int64)).to(DEV)
    e0m4.e0m4_kv_append(c_dev, w_dev[:, col:col + row], p_dev)
    torch.cuda.synchronize()
    got = c_dev.cpu().numpy()
    assert np.array_equal(got.view(np.uint16), want.view(np.uint16))


def test_decode_step_chatglm2_shape(e0m4, oracle):
    # one new token; K and V of a position side by side (2 x 2 heads x 128), taken from the QKV output columns
    run_case(e0m4, oracle, 300, 512, 1, 4608, 4096, [123], seed=600)
    run_case(e0m4, oracle, 300, 512, 1, 4608, 4096, [0], seed=601)
    run_case(e0m4, oracle, 300, 512, 1, 4608, 4096, [299], seed=602)


def test_prefill_consecutive_positions(e0m4, oracle):
    run_case(e0m4, oracle, 400, 512, 257, 4608, 4096, np.arange(10, 267), seed=610)
    run_case(e0m4, oracle, 2048, 256, 1024, 256, 0, np.arange(1024), seed=611)        # contiguous source


def test_scattered_and_out_of_range_positions(e0m4, oracle):
    rng = np.random.default_rng(5)
    pos = rng.permutation(200)[:37].astype(np.int64)
    pos[5], pos[11], pos[20] = -1, 200, 1 << 40                                        # skipped rows
    run_case(e0m4, oracle, 200, 72, 37, 136, 64, pos, seed=620)                       # 9 pieces per row, ragged last workgroup


def test_small_and_empty(e0m4, oracle):
    run_case(e0m4, oracle, 3, 8, 2, 8, 0, [2, 0], seed=630)
    cache = torch.ones((4, 8), dtype=torch.float16, device=DEV)
    e0m4.e0m4_kv_append(cache, torch.empty((0, 8), dtype=torch.float16, device=DEV),
                        torch.empty(0, dtype=torch.int64, device=DEV))
    torch.cuda.synchronize()
    assert bool((cache == 1).all())


def test_decode_steps_build_the_prefill_cache(e0m4, oracle):
    max_seq, row, n = 64, 256, 20
    rows = torch.from_numpy(synth_inputs.activations(n, row, seed=640)).to(DEV)
    a = torch.zeros((max_seq, row), dtype=torch.float16, device=DEV)
    b = torch.zeros_like(a)
    e0m4.e0m4_kv_append(a, rows, torch.arange(n, dtype=torch.int64, device=DEV))
    for i in range(n):
        e0m4.e0m4_kv_append(b, rows[i:i + 1], torch.tensor([i], dtype=torch.int64, device=DEV))
    torch.cuda.synchronize()
    assert torch.equal(a, b) and torch.equal(a[:n], rows) and bool((a[n:] == 0).all())


def test_argument_errors(e0m4):
    cache = torch.zeros((8, 16), dtype=torch.float16, device=DEV)
    rows = torch.zeros((2, 24), dtype=torch.float16, device=DEV)
    pos = torch.zeros(2, dtype=torch.int64, device=DEV)
    with pytest.raises(e0m4.E0M4Error):                 # source columns start at an odd 16-byte boundary
        e0m4.e0m4_kv_append(cache, rows[:, 4:20], pos)
    with pytest.raises(e0m4.E0M4Error):                 # row length not a multiple of 8
        e0m4.e0m4_kv_append(torch.zeros((8, 12), dtype=torch.float16, device=DEV),
                            torch.zeros((2, 12), dtype=torch.float16, device=DEV), pos)
