"""Helpers shared by the GPU parity tests: pools on the device and on the host
from the same stateless fill, and the oracle's expected result per layer."""
from __future__ import annotations

import ctypes

import numpy as np

from oracle import kvmig as orc
from workload import fill_words
from workload.configs import PairCase


def np_dtype(e: int):
    return {1: np.uint8, 2: np.uint16, 4: np.uint32}[e]


def host_layers(case: PairCase, side: str, layers, L=None, D=None) -> np.ndarray:
    """Layers ``layers`` of a pool, [len(layers)][2][S][H_local][D], from the fill."""
    sh = case.shape
    D = D or sh.D
    S, Hl, seed = ((case.S_src, case.Hs, case.seed_src) if side == "src"
                   else (case.S_dst, case.Hd, case.seed_dst))
    layer_bytes = 2 * S * Hl * D * sh.e
    assert layer_bytes % 8 == 0
    out = np.empty((len(layers), layer_bytes // 8), dtype="<u8")
    for i, l in enumerate(layers):
        out[i] = fill_words(seed, l * (layer_bytes // 8), layer_bytes // 8)
    return out.view(np_dtype(sh.e)).reshape(len(layers), 2, S, Hl, D)


def device_pool(case: PairCase, side: str, L=None, D=None):
    """The whole pool as a flat uint8 device tensor filled with the same pattern."""
    import torch
    from workload import device as wdev
    sh = case.shape
    L, D = L or sh.L, D or sh.D
    S, Hl, seed = ((case.S_src, case.Hs, case.seed_src) if side == "src"
                   else (case.S_dst, case.Hd, case.seed_dst))
    t = torch.empty(L * 2 * S * Hl * D * sh.e, dtype=torch.uint8, device="cuda")
    wdev.fill_tensor(t, seed)
    return t


def slab_bytes(case: PairCase, side: str, D=None) -> int:
    sh = case.shape
    D = D or sh.D
    S, Hl = (case.S_src, case.Hs) if side == "src" else (case.S_dst, case.Hd)
    return S * Hl * D * sh.e


def make_plan(b, ctx, case: PairCase, L=None, D=None, staging_bytes=0, flags=None):
    sh = case.shape
    so, do, w = b.nts_route(sh.H, case.Ns, case.rs, case.Nd, case.rd)
    return b.nts_plan_create(
        ctx, L=L or sh.L, D=D or sh.D, elem_bytes=sh.e, page_size=case.p, Hs=case.Hs, Hd=case.Hd,
        src_head_off=so, dst_head_off=do, w=w, S_src=case.S_src, S_dst=case.S_dst,
        ctx_len=case.ctx_len, src_pages=case.src_pages, dst_pages=case.dst_pages,
        staging_bytes=staging_bytes,
        flags=b.NTS_VALIDATE_UNIQUE_DST if flags is None else flags)


def oracle_slots(case: PairCase):
    return (orc.flatten(case.ctx_len, case.src_pages, case.p),
            orc.flatten(case.ctx_len, case.dst_pages, case.p))


def to_host(t) -> np.ndarray:
    return t.cpu().numpy()
