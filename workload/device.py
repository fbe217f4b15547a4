"""Device-side twin of the stateless pool fill (torch tensors + a small HIP library).

Input generation only.  ``build()`` compiles workload/fill_gpu.hip with hipcc
for gfx950 into workload/libnts_fill.so; the functions below need a GPU.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

from .splitmix import fill_key

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "fill_gpu.hip")
LIB = os.path.join(HERE, "libnts_fill.so")
_lib = None


def build(force: bool = True) -> str:
    if force or not os.path.exists(LIB):
        subprocess.check_call(["hipcc", "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared",
                               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                               SRC, "-o", LIB], stderr=subprocess.DEVNULL)
    return LIB


def _clib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB):
            build()
        import torch  # noqa: F401  (first, so that this library binds to the HIP runtime torch ships)
        _lib = ctypes.CDLL(LIB)
        u64, vp = ctypes.c_uint64, ctypes.c_void_p
        _lib.wl_fill_words.argtypes = [vp, u64, u64, u64, vp]
        _lib.wl_fill_words.restype = ctypes.c_int
        _lib.wl_count_mismatch.argtypes = [vp, u64, u64, u64, vp, vp]
        _lib.wl_count_mismatch.restype = ctypes.c_int
    return _lib


def fill_tensor(t, seed: int, start_word: int = 0) -> None:
    """Fill a contiguous device tensor (byte size a multiple of 8) with the
    stateless pattern of ``seed``, as if it began at word ``start_word``."""
    import torch
    nbytes = t.numel() * t.element_size()
    if not t.is_contiguous() or nbytes % 8:
        raise ValueError("tensor must be contiguous with a byte size multiple of 8")
    rc = _clib().wl_fill_words(t.data_ptr(), start_word, nbytes // 8, fill_key(seed),
                               torch.cuda.current_stream().cuda_stream)
    if rc:
        raise RuntimeError(f"wl_fill_words failed with HIP error {rc}")


def count_mismatch(t, seed: int, start_word: int = 0) -> int:
    """Number of 8-byte words of ``t`` that differ from the pattern of ``seed``."""
    import torch
    nbytes = t.numel() * t.element_size()
    if not t.is_contiguous() or nbytes % 8:
        raise ValueError("tensor must be contiguous with a byte size multiple of 8")
    cnt = torch.zeros(1, dtype=torch.int64, device=t.device)
    rc = _clib().wl_count_mismatch(t.data_ptr(), start_word, nbytes // 8, fill_key(seed),
                                   cnt.data_ptr(), torch.cuda.current_stream().cuda_stream)
    if rc:
        raise RuntimeError(f"wl_count_mismatch failed with HIP error {rc}")
    return int(cnt.item())
