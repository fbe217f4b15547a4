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
product on absolute values, which the worst-case tolerance of the GPU
comparison scales with; `product_norm` is the Euclidean norm of the products
of one output, which the tight (typical-error) tolerance scales with.
`round_to_bits` rounds an exact float64 result once, to nearest even, to the
16-bit output format: for inputs whose products and partial sums are all exact
in fp32 (small integers) it is the bit pattern the layer must return.
Pins: tests/test_oracle_shard_linear.py.
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


def _shard(X: np.ndarray, W: np.ndarray, tp: int, rank: int, split: str) -> np.ndarray:
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
    return Ws


def shard_linear(X: np.ndarray, W: np.ndarray, tp: int, rank: int, split: str):
    """X, W: float64 arrays holding the exact input values.  Returns (Y, abs_bound)."""
    Ws = _shard(X, W, tp, rank, split)
    return X @ Ws.T, np.abs(X) @ np.abs(Ws).T


def product_norm(X: np.ndarray, W: np.ndarray, tp: int, rank: int, split: str) -> np.ndarray:
    """sqrt(sum_k (x_k w_k)^2) per output: the size a partial sum of the products
    typically reaches (the products of one output largely cancel)."""
    Ws = _shard(X, W, tp, rank, split)
    return np.sqrt((X * X) @ (Ws * Ws).T)


def _fmt(fmt: str):
    """(explicit mantissa bits, minimum normal exponent, first exponent that overflows)."""
    if fmt == "bf16":
        return 7, -126, 128
    if fmt == "f16":
        return 10, -14, 16
    raise ValueError(fmt)


def ulp(y: np.ndarray, fmt: str) -> np.ndarray:
    """Spacing of the format's values around |y| (subnormal spacing below the smallest normal)."""
    m, emin, _ = _fmt(fmt)
    a = np.abs(np.asarray(y, dtype=np.float64))
    _, e = np.frexp(a)                                             # |y| = f * 2^e, f in [0.5, 1)
    e = np.where(a == 0, emin, np.maximum(e - 1, emin))            # exponent of the leading bit
    return np.ldexp(1.0, e - m)


def round_to_bits(y: np.ndarray, fmt: str) -> np.ndarray:
    """One round-to-nearest-even of exact float64 values to bfloat16 / float16,
    returned as uint16 bit patterns (overflow gives infinity)."""
    m, emin, emax = _fmt(fmt)
    y = np.asarray(y, dtype=np.float64)
    q = ulp(y, fmt)
    r = np.rint(y / q) * q                       # rint rounds halves to even; y / q is exact (q a power of two)
    r = np.where(np.abs(r) >= np.ldexp(1.0, emax), np.copysign(np.inf, y), r)
    r = np.where(r == 0, np.copysign(0.0, y), r)
    if fmt == "bf16":
        with np.errstate(over="ignore"):
            return (r.astype(np.float32).view(np.uint32) >> np.uint32(16)).astype(np.uint16)   # r is representable: exact
    with np.errstate(over="ignore"):
        return r.astype(np.float16).view(np.uint16)


def tolerance(Y: np.ndarray, abs_bound: np.ndarray, k: int, out_bits: int = 8) -> np.ndarray:
    """Allowed |error| per output for fp32 accumulation of k products in any order
    followed by one rounding to a float with `out_bits` explicit mantissa bits
    (8 for bfloat16, 11 for float16 counts the hidden bit already: pass 11).

    fp32 summation in any order: |err| <= (k * 2^-24) * sum|x*w| to first order;
    the final rounding adds at most 2^-(out_bits+1) * |y|.  Both are doubled."""
    acc = (k * 2.0 ** -23) * abs_bound
    return 2.0 ** -out_bits * (np.abs(Y) + acc) + acc


def tight_tolerance(Y: np.ndarray, prod_norm: np.ndarray, k: int, fmt: str) -> np.ndarray:
    """Allowed |error| per output for a layer that really accumulates in fp32 and
    rounds once to nearest: half a unit in the last place of the output format
    (the one rounding), plus what fp32 accumulation typically adds.  Each of the
    k additions errs by at most 2^-24 of a partial sum; partial sums are of the
    size of `prod_norm` (products cancel), and k such errors add like a random
    walk: about sqrt(k) * 2^-24 * prod_norm.  Eight times that is allowed, plus
    2^-5 of the half ulp for the rare result whose fp32 sum falls on the other
    side of a rounding boundary than the exact one.  Unlike `tolerance` this is
    not a worst-case bound, but one dropped or doubled product of typical size
    already exceeds it at every reduction length the layer is used with."""
    return (0.5 + 2.0 ** -5) * ulp(Y, fmt) + 8.0 * np.sqrt(float(k)) * 2.0 ** -24 * prod_norm
