"""C twin of the stateless pool fill for the host (ctypes + gcc).

Input generation only.  ``build()`` compiles workload/fill_host.c into
workload/libnts_fill_host.so; ``fill_words_fast`` returns the same words as
``splitmix.fill_words`` about twenty times faster, which is what lets every
slab of a 92 GiB pool be regenerated on the host.  The call releases the GIL,
so several slabs can be produced by a thread pool.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

from .splitmix import fill_key

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "fill_host.c")
LIB = os.path.join(HERE, "libnts_fill_host.so")
_lib = None


def build(force: bool = False) -> str:
    if force or not os.path.exists(LIB) or os.path.getmtime(LIB) < os.path.getmtime(SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-shared", "-fPIC", SRC, "-o", LIB])
    return LIB


def _clib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        u64 = ctypes.c_uint64
        _lib.wl_fill_words_host.argtypes = [ctypes.c_void_p, u64, u64, u64]
        _lib.wl_fill_words_host.restype = None
    return _lib


def fill_words_fast(seed: int, start_word: int, count: int, out: np.ndarray | None = None) -> np.ndarray:
    """Words ``start_word .. start_word+count-1`` of the fill pattern of ``seed`` (uint64)."""
    if out is None:
        out = np.empty(count, dtype="<u8")
    if out.dtype != np.dtype("<u8") or out.size != count or not out.flags.c_contiguous:
        raise ValueError("out must be a contiguous uint64 array of `count` words")
    _clib().wl_fill_words_host(out.ctypes.data, start_word, count, fill_key(seed))
    return out
