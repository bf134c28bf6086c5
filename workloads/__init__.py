"""Seeded synthetic inputs for the DGQ A8W4 linear layer.

This module serves both the CPU oracle and the HIP path.  It only draws random
numbers and names layer shapes; none of the method's arithmetic (quantizers,
packing, matmul, epilogue) lives here.

The tensors stand in for the LLaMA linear layers and their activations that the
paper evaluates end to end (Section 4.3, Fig. 4): same shapes, Gaussian values,
and a small fraction of activation channels carrying large outliers, which is
the activation structure the paper's smoothing (Section 3.4) is aimed at.
"""
from __future__ import annotations

import numpy as np

# (K, N) of the four linears of one decoder layer: fused qkv, attention output,
# fused gate+up, down.  K is the paper's h (input channels), N its o.
LLAMA_SHAPES = {
    "7b": {"qkv": (4096, 12288), "o": (4096, 4096), "gate_up": (4096, 22016), "down": (11008, 4096)},
    "13b": {"qkv": (5120, 15360), "o": (5120, 5120), "gate_up": (5120, 27648), "down": (13824, 5120)},
    "65b": {"qkv": (8192, 24576), "o": (8192, 8192), "gate_up": (8192, 44032), "down": (22016, 8192)},
}

# Activation outlier recipe per model size: (fraction of channels, multiplier).
OUTLIERS = {"7b": (0.01, 20.0), "13b": (0.01, 20.0), "65b": (0.005, 50.0)}


def activations(M: int, K: int, seed: int, outlier_frac: float = 0.01,
                outlier_mult: float = 20.0) -> np.ndarray:
    """fp16 [M, K]: N(0,1), with round(outlier_frac*K) channels multiplied by outlier_mult."""
    rng = np.random.default_rng([seed, 0xA])
    x = rng.standard_normal((M, K), dtype=np.float32)
    n_out = int(round(outlier_frac * K))
    if n_out > 0:
        ch = rng.choice(K, size=n_out, replace=False)
        x[:, ch] *= np.float32(outlier_mult)
    return x.astype(np.float16)


def weights(K: int, N: int, seed: int, std: float = 0.02) -> np.ndarray:
    """fp16 [K, N] (paper orientation h x o, N contiguous): N(0, std)."""
    rng = np.random.default_rng([seed, 0xB])
    w = rng.standard_normal((K, N), dtype=np.float32)
    w *= np.float32(std)
    return w.astype(np.float16)


def integer_weights(K: int, N: int, group: int, seed: int):
    """Already-quantized operands drawn uniformly over their whole legal range.

    Returns (w4 int8 [K,N] in [-8,7], s2 uint8 [K/group,N] in [1,15],
    s1 float32 [N] in [1e-3, 3e-3)).  Used to exercise every nibble/scale value,
    which Gaussian weights (group scales concentrate near 12..15) do not.
    """
    rng = np.random.default_rng([seed, 0xC])
    w4 = rng.integers(-8, 8, size=(K, N), dtype=np.int8)
    s2 = rng.integers(1, 16, size=(K // group, N), dtype=np.uint8)
    s1 = (1e-3 * (1.0 + 2.0 * rng.random(N, dtype=np.float32))).astype(np.float32)
    return w4, s2, s1


def integer_activations(M: int, K: int, seed: int):
    """int8 [M,K] uniform in [-127,127] and positive fp32 per-token scales [M]."""
    rng = np.random.default_rng([seed, 0xD])
    xq = rng.integers(-127, 128, size=(M, K), dtype=np.int8)
    sx = (0.01 * (1.0 + rng.random(M, dtype=np.float32))).astype(np.float32)
    return xq, sx
