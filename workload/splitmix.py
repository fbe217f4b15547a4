"""SplitMix64 as a counter-based generator (Steele, Lea, Flood 2014).

The k-th output of a stream seeded with ``s`` is ``mix64(s + (k+1)*GAMMA)``:
it depends on (s, k) only, so any slice of a stream can be produced without
its prefix.  That is what lets a 92 GiB pool be filled on the GPU and any
small part of it be recomputed on the host.

Pool fill pattern ("stateless fill"): a pool is viewed as little-endian
64-bit words; word ``k`` of the pool holds stream output ``k`` of the stream
seeded with ``mix64(seed)``.  A 16-bit element ``i`` is therefore bits
``16*(i%4) .. 16*(i%4)+15`` of word ``i//4``.
"""
from __future__ import annotations

import numpy as np

GAMMA = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB
_MASK = (1 << 64) - 1


def mix64(z: int) -> int:
    """SplitMix64 output function on a Python int (mod 2**64)."""
    z &= _MASK
    z = ((z ^ (z >> 30)) * _M1) & _MASK
    z = ((z ^ (z >> 27)) * _M2) & _MASK
    return z ^ (z >> 31)


def _mix64_np(z: np.ndarray) -> np.ndarray:
    z = z.copy()
    z ^= z >> np.uint64(30)
    z *= np.uint64(_M1)
    z ^= z >> np.uint64(27)
    z *= np.uint64(_M2)
    z ^= z >> np.uint64(31)
    return z


def stream_words(state0: int, start: int, count: int) -> np.ndarray:
    """Outputs ``start .. start+count-1`` of the stream with initial state ``state0``."""
    with np.errstate(over="ignore"):
        k = np.arange(start + 1, start + 1 + count, dtype=np.uint64)
        z = k * np.uint64(GAMMA) + np.uint64(state0 & _MASK)
        return _mix64_np(z)


def fill_key(seed: int) -> int:
    """Initial state of the fill stream of ``seed``."""
    return mix64(seed)


def fill_words(seed: int, start_word: int, count: int) -> np.ndarray:
    """Words ``start_word ..`` of the stateless fill pattern of ``seed`` (uint64)."""
    return stream_words(fill_key(seed), start_word, count)


def fill_pool_u16(seed: int, n_elems: int, chunk_words: int = 1 << 22) -> np.ndarray:
    """A whole pool of ``n_elems`` 16-bit elements (``n_elems`` multiple of 4)."""
    if n_elems % 4:
        raise ValueError("pool size must be a multiple of 4 elements (8 bytes)")
    n_words = n_elems // 4
    out = np.empty(n_words, dtype="<u8")
    for s in range(0, n_words, chunk_words):
        c = min(chunk_words, n_words - s)
        out[s:s + c] = fill_words(seed, s, c)
    return out.view("<u2")


class SplitMix64:
    """Sequential view of one stream (for lengths, permutations, samples)."""

    def __init__(self, seed: int):
        self.state0 = mix64(seed ^ 0xA5A5A5A5A5A5A5A5)
        self.pos = 0

    def words(self, count: int) -> np.ndarray:
        w = stream_words(self.state0, self.pos, count)
        self.pos += count
        return w

    def uniform(self, count: int) -> np.ndarray:
        """Doubles in [0, 1) from the top 53 bits."""
        return (self.words(count) >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))

    def integers(self, lo: int, hi: int, count: int) -> np.ndarray:
        """Integers in [lo, hi] (inclusive); modulo bias is irrelevant here."""
        span = np.uint64(hi - lo + 1)
        return (self.words(count) % span).astype(np.int64) + lo

    def permutation(self, n: int) -> np.ndarray:
        """A permutation of 0..n-1: stable argsort of n stream words."""
        return np.argsort(self.words(n), kind="stable").astype(np.int64)
