"""CPU oracle for the TP-shard-selecting linear layer: TEST INFRASTRUCTURE ONLY.

Sec. 3.2.1 of the paper ("Zero-Overhead TP Weight Switching"): every GPU keeps
ONE full copy of each weight matrix and, at TP level N, rank r computes with
the r-th 1/N of it, picked at execution time (rank 0 uses the first half under
TP2, the first quarter under TP4).  The paper does not say along which axis a
given layer is cut; the reading used here is the usual tensor-parallel pair:

  split = "out" (column-parallel: QKV, gate, up projections)
      Y[M, n_out/N] = X[M, n_in] . W[r*n_out/N : (r+1)*n_out/N, :]^T
  split = "in"  (row-parallel: attention-output and down projections)
      Y[M, n_out]   = X[M, n_in/N] . W[:, r*n_in/N : (r+1)*n_in/N]^T
      (a partial sum; the all-reduce over ranks is outside this operation)

with W stored [n_out][n_in] (row-major, as a linear layer's weight) in a
16-bit float format.  Everything is computed in float64 from the exact values
of the 16-bit inputs: slice, then numpy matmul.  `abs_bound` is the same
product on absolute values, which the tolerance of the GPU comparison scales
with.  Pins: tests/test_oracle_shard_linear.py.
"""
from __future__ import annotations

import numpy as np


def bf16_to_f64(u16: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> float64, exactly: a bfloat16 is the
    upper half of an IEEE binary32."""
    u = np.ascontiguousarray(u16, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def f16_to_f64(u16: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(u16, dtype=np.uint16).view(np.float16).astype(np.float64)


def shard_bounds(n: int, tp: int, rank: int):
    """[lo, hi) of the rank-th 1/tp of an axis of length n."""
    if tp <= 0 or n % tp != 0 or not 0 <= rank < tp:
        raise ValueError("axis length must be a multiple of tp and 0 <= rank < tp")
    per = n // tp
    return rank * per, (rank + 1) * per


def shard_linear(X: np.ndarray, W: np.ndarray, tp: int, rank: int, split: str):
    """X, W: float64 arrays holding the exact input values.  Returns (Y, abs_bound)."""
    n_out, n_in = W.shape
    if split == "out":
        lo, hi = shard_bounds(n_out, tp, rank)
        Ws = W[lo:hi, :]
        if X.shape[1] != n_in:
            raise ValueError("X must have n_in columns")
    elif split == "in":
        lo, hi = shard_bounds(n_in, tp, rank)
        Ws = W[:, lo:hi]
        if X.shape[1] != hi - lo:
            raise ValueError("X must have n_in/tp columns")
    else:
        raise ValueError(split)
    return X @ Ws.T, np.abs(X) @ np.abs(Ws).T


def tolerance(Y: np.ndarray, abs_bound: np.ndarray, k: int, out_bits: int = 8) -> np.ndarray:
    """Allowed |error| per output for fp32 accumulation of k products in any order
    followed by one rounding to a float with `out_bits` explicit mantissa bits
    (8 for bfloat16, 11 for float16 counts the hidden bit already: pass 11).

    fp32 summation in any order: |err| <= (k * 2^-24) * sum|x*w| to first order;
    the final rounding adds at most 2^-(out_bits+1) * |y|.  Both are doubled."""
    acc = (k * 2.0 ** -23) * abs_bound
    return 2.0 ** -out_bits * (np.abs(Y) + acc) + acc
