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
        _lib.wl_mfma_probe.argtypes = [vp, ctypes.c_uint32, ctypes.c_uint32, u64, vp]
        _lib.wl_mfma_probe.restype = ctypes.c_int
        _lib.wl_read_probe.argtypes = [vp, u64, vp, vp]
        _lib.wl_read_probe.restype = ctypes.c_int
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


def mfma_ceiling_tflops(seconds: float = 0.25) -> float:
    """bf16 TFLOP/s the matrix cores sustain on pseudo-random operands with nothing else going on
    (registers only; 1024 workgroups of four wavefronts, each a 128 x 128 accumulator tile), timed
    over about ``seconds`` of back-to-back launches so that the clock settles where the power limit
    puts it."""
    import torch
    wgs, iters = 1024, 4096
    out = torch.empty(wgs * 256, dtype=torch.float32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    flops = wgs * 4 * iters * 16 * 32768.0

    def launch():
        rc = _clib().wl_mfma_probe(out.data_ptr(), wgs, iters, fill_key(99), st)
        if rc:
            raise RuntimeError(f"wl_mfma_probe failed with HIP error {rc}")

    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    launch()
    torch.cuda.synchronize()
    e0.record(); launch(); e1.record(); torch.cuda.synchronize()
    n = max(2, int(seconds / (e0.elapsed_time(e1) * 1e-3)))
    for _ in range(n):                      # settle
        launch()
    e0.record()
    for _ in range(n):
        launch()
    e1.record()
    torch.cuda.synchronize()
    return flops * n / (e0.elapsed_time(e1) * 1e-3) / 1e12


def read_ceiling_gbs(n_bytes: int = 1 << 30) -> float:
    """GB/s of a read-only stream over ``n_bytes`` of HBM (eight 16-byte non-temporal loads per lane)."""
    import torch
    buf = torch.empty(2 * n_bytes, dtype=torch.uint8, device="cuda").fill_(5)     # two halves: no reuse from a cache
    sink = torch.zeros(1024, dtype=torch.int32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream

    def launch(i):
        rc = _clib().wl_read_probe(buf.data_ptr() + (i & 1) * n_bytes, n_bytes, sink.data_ptr(), st)
        if rc:
            raise RuntimeError(f"wl_read_probe failed with HIP error {rc}")

    for i in range(4):
        launch(i)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    n = 20
    e0.record()
    for i in range(n):
        launch(i)
    e1.record()
    torch.cuda.synchronize()
    return n_bytes * n / (e0.elapsed_time(e1) * 1e-3) / 1e9
