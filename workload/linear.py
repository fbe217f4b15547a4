"""Seeded inputs for the TP-shard-selecting linear layer: bfloat16 activations
and a full weight matrix, as uint16 bit patterns.  Input generation only."""
from __future__ import annotations

import numpy as np

from .splitmix import SplitMix64

# (n_out, n_in, split) of the four linear layers of a decoder block; split "out" =
# column-parallel, "in" = row-parallel.  8B: hidden 4096, 32 query + 8 KV heads of
# 128, MLP 14336 (the paper's Llama-3.1-8B); 14B: hidden 5120, 40 + 8 heads, MLP 13824.
LAYERS = {
    "8b_qkv": (6144, 4096, "out"),
    "8b_o": (4096, 4096, "in"),
    "8b_gate_up": (28672, 4096, "out"),
    "8b_down": (4096, 14336, "in"),
    "14b_qkv": (7168, 5120, "out"),
    "14b_o": (5120, 5120, "in"),
    "14b_gate_up": (27648, 5120, "out"),
    "14b_down": (5120, 13824, "in"),
}


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bfloat16 bit patterns (finite inputs)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (r >> np.uint32(16)).astype(np.uint16)


def f32_to_f16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> IEEE float16 bit patterns."""
    return np.ascontiguousarray(a, dtype=np.float32).astype(np.float16).view(np.uint16)


def linear_inputs(seed: int, M: int, n_out: int, n_in: int, x_cols: int | None = None, dtype: str = "bf16"):
    """X [M][x_cols] uniform in [-2, 2), W [n_out][n_in] uniform in [-0.04, 0.04),
    both rounded to bfloat16 (or float16); returned as uint16 arrays."""
    rng = SplitMix64(seed)
    x_cols = x_cols or n_in
    f32_to_bf16_bits_ = f32_to_bf16_bits if dtype == "bf16" else f32_to_f16_bits
    X = f32_to_bf16_bits_((rng.uniform(M * x_cols) * 4.0 - 2.0).astype(np.float32)).reshape(M, x_cols)
    W = np.empty(n_out * n_in, dtype=np.uint16)
    step = 1 << 22
    for s in range(0, W.size, step):
        n = min(step, W.size - s)
        W[s:s + n] = f32_to_bf16_bits_((rng.uniform(n) * 0.08 - 0.04).astype(np.float32))
    return X, W.reshape(n_out, n_in)


def linear_inputs_int(seed: int, M: int, n_out: int, n_in: int, x_cols: int | None = None, dtype: str = "bf16",
                      amax: int = 8):
    """Integer-valued inputs: X and W uniform over the integers -amax .. amax, stored
    as bfloat16 (or float16), which holds them exactly.  Every product is then an
    integer of at most amax^2 and every partial sum of up to 2^24 / amax^2 of
    them is exact in fp32 in any order, so a layer that accumulates in fp32 and
    rounds once has exactly one correct 16-bit result."""
    if not 1 <= amax <= 16:
        raise ValueError("amax must be in 1..16")
    rng = SplitMix64(seed)
    x_cols = x_cols or n_in
    to_bits = f32_to_bf16_bits if dtype == "bf16" else f32_to_f16_bits
    X = to_bits((rng.integers(-amax, amax, M * x_cols)).astype(np.float32)).reshape(M, x_cols)
    W = np.empty(n_out * n_in, dtype=np.uint16)
    step = 1 << 22
    for s in range(0, W.size, step):
        n = min(step, W.size - s)
        W[s:s + n] = to_bits(rng.integers(-amax, amax, n).astype(np.float32))
    return X, W.reshape(n_out, n_in)
