"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module holds no arithmetic of the E0M4 method: it only draws random
fp16 matrices with the shapes and value distributions of the workloads
(linear layers of ChatGLM2-6B-, Gemma-2B- and 14B-class decoders) and hands the
same bits to the CPU oracle and to the GPU library.

numpy side: counter-based Philox streams keyed by the seed, so a (seed, shape)
pair always yields the same bits on any machine.  torch side (benchmark only,
where billions of weights are needed): the device generator seeded the same
way; those tensors never meet the oracle except through an explicit copy.
"""
from __future__ import annotations

import numpy as np

# (name, N, K) per projection; N = out features, K = in features.
CHATGLM2_6B = [("qkv", 4608, 4096), ("attn_out", 4096, 4096), ("ffn_gate_up", 27392, 4096), ("ffn_down", 4096, 13696)]
GEMMA_2B = [("qkv", 2560, 2048), ("attn_out", 2048, 2048), ("ffn_gate_up", 32768, 2048), ("ffn_down", 2048, 16384)]
GEMMA_2B_LM_HEAD = ("lm_head", 256000, 2048)
DENSE_14B = [("qkv", 15360, 5120), ("attn_out", 5120, 5120), ("ffn_gate_up", 27392, 5120), ("ffn_down", 5120, 13696)]
# weight shapes [K, N] of the latency comparison between E0M4 and INT4 (paper: Table 1), M = 1
TABLE1_SHAPES = [(4096, 4096), (4096, 11008), (11008, 4096)]
CHATGLM2_LAYERS = 28
DENSE_14B_LAYERS = 40
GEMMA_2B_LAYERS = 18

W_STD = 0.02


def _rng(seed: int, stream: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[int(seed), int(stream)]))


def weights(N: int, K: int, seed: int, std: float = W_STD, row_std_range=None) -> np.ndarray:
    """W [N,K] fp16 ~ N(0, std); optionally each row's std is multiplied by a
    factor drawn uniformly from row_std_range (prefill workload)."""
    g = _rng(seed, 1)
    W = g.standard_normal((N, K), dtype=np.float32) * np.float32(std)
    if row_std_range is not None:
        lo, hi = row_std_range
        r = _rng(seed, 2).uniform(lo, hi, size=(N, 1)).astype(np.float32)
        W *= r
    return W.astype(np.float16)


def activations(M: int, K: int, seed: int, outlier_frac: float = 0.0, outlier_scale: float = 20.0) -> np.ndarray:
    """X [M,K] fp16 ~ N(0,1); optionally a fraction of the K channels (chosen
    once per seed) is multiplied by outlier_scale (activation outliers)."""
    g = _rng(seed, 3)
    X = g.standard_normal((M, K), dtype=np.float32)
    if outlier_frac > 0.0:
        n_out = max(1, int(round(outlier_frac * K)))
        ch = _rng(seed, 4).choice(K, size=n_out, replace=False)
        X[:, ch] *= np.float32(outlier_scale)
    return X.astype(np.float16)


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 array -> bfloat16 bit patterns (uint16), round to nearest even; a change of storage type only."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)


def weights_bf16(N: int, K: int, seed: int, std: float = W_STD) -> np.ndarray:
    """W [N,K] ~ N(0, std) as bfloat16 bit patterns (uint16)."""
    return to_bf16_bits(_rng(seed, 1).standard_normal((N, K), dtype=np.float32) * np.float32(std))


def activations_bf16(M: int, K: int, seed: int) -> np.ndarray:
    """X [M,K] ~ N(0,1) as bfloat16 bit patterns (uint16)."""
    return to_bf16_bits(_rng(seed, 3).standard_normal((M, K), dtype=np.float32))


def norm_weight(K: int, seed: int) -> np.ndarray:
    """rms-norm weight gamma [K] fp16 ~ 1 + 0.1 N(0,1) (trained norm weights sit around one)."""
    return (1.0 + 0.1 * _rng(seed, 5).standard_normal(K, dtype=np.float32)).astype(np.float16)


def residual(M: int, N: int, seed: int) -> np.ndarray:
    """Residual-stream values [M,N] fp16 ~ N(0,1)."""
    return _rng(seed, 6).standard_normal((M, N), dtype=np.float32).astype(np.float16)


def layer_seed(layer: int, proj: int) -> int:
    return layer * 4 + proj


# ---- device-side generation for the benchmark (torch is plumbing here) -------

def weights_device(N: int, K: int, seed: int, device, std: float = W_STD, row_std_range=None):
    import torch

    g = torch.Generator(device=device)
    g.manual_seed(int(seed) * 2 + 1)
    W = torch.randn((N, K), generator=g, device=device, dtype=torch.float32) * std
    if row_std_range is not None:
        lo, hi = row_std_range
        r = torch.rand((N, 1), generator=g, device=device, dtype=torch.float32) * (hi - lo) + lo
        W = W * r
    return W.to(torch.float16)


def activations_device(M: int, K: int, seed: int, device, outlier_frac: float = 0.0, outlier_scale: float = 20.0):
    import torch

    g = torch.Generator(device=device)
    g.manual_seed(int(seed) * 2)
    X = torch.randn((M, K), generator=g, device=device, dtype=torch.float32)
    if outlier_frac > 0.0:
        n_out = max(1, int(round(outlier_frac * K)))
        ch = torch.randperm(K, generator=g, device=device)[:n_out]
        X[:, ch] *= outlier_scale
    return X.to(torch.float16)
