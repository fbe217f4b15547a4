"""CPU oracle for the KV-migration hot path: TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the bench's cpu_baseline leg may import this
module.  It shares no code with the HIP path and never imports it.

What is computed follows Sec. 3.2.2 of the paper ("Aggregated and Pipelined KV
Migration"):

* ``head_interval`` / ``route``: under TP level N the KV heads are split evenly
  over the N GPUs of a group; a switch moves, from source rank to destination
  rank, the heads both intervals have in common.
* ``flatten``: the metadata exchanged before the transfer (request, context
  length, pages) turned into one slot per migrated token.
* ``runs``: the migrated tokens cut into maximal runs that sit in neighbouring
  slots on both sides (with small pages a request's KV is scattered over many
  regions, with a contiguous per-request layout over few: the two layouts of
  the paper's microbenchmark).
* ``pack`` / ``unpack`` / ``migrate_direct``: plain loops in C
  (``kvmig_oracle.c``) that gather the moved head slice of every token into a
  contiguous stream, scatter such a stream into the destination pool, or do
  both at once.
* ``Cluster``: several virtual GPUs in host memory, for the worked
  TP1 -> TP2 -> TP4 example of Fig. "KV Conversion" and its reversal.

All of it is pinned in tests/test_oracle_pins.py and
tests/test_oracle_cluster.py; nothing is "parity unpinned".
"""
from __future__ import annotations

import ctypes
from dataclasses import dataclass, field
from typing import Callable, Dict, List, Sequence, Tuple

import numpy as np

from . import build as _build

_lib = None


def _clib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(_build.build())
        i64, vp = ctypes.c_int64, ctypes.c_void_p
        _lib.orc_pack.argtypes = [vp, i64, i64, i64, i64, i64, vp, i64, i64, i64, vp]
        _lib.orc_pack.restype = None
        _lib.orc_unpack.argtypes = [vp, i64, i64, i64, i64, i64, vp, i64, i64, i64, vp]
        _lib.orc_unpack.restype = None
        _lib.orc_migrate_direct.argtypes = [vp, i64, i64, i64, vp, i64, i64, i64,
                                            i64, i64, i64, i64, vp, vp, i64]
        _lib.orc_migrate_direct.restype = None
    return _lib


# ----------------------------------------------------------------------------
# routing (integer, host)
# ----------------------------------------------------------------------------

def head_interval(H: int, N: int, r: int) -> Tuple[int, int]:
    """Global heads [a, b) held by rank ``r`` of a group at TP level ``N``
    (even split on the head dimension, Sec. 3.2.2)."""
    if N <= 0 or H % N != 0 or not 0 <= r < N:
        raise ValueError("H must be a multiple of N and 0 <= r < N")
    per = H // N
    return r * per, (r + 1) * per


def route(H: int, Ns: int, rs: int, Nd: int, rd: int) -> Tuple[int, int, int]:
    """Heads to move from source rank ``rs`` (TP ``Ns``) to destination rank ``rd``
    (TP ``Nd``): returns (src_head_off, dst_head_off, w) with offsets local to
    each GPU's own head range; w == 0 means nothing moves between the two."""
    sa, sb = head_interval(H, Ns, rs)
    da, db = head_interval(H, Nd, rd)
    a, b = max(sa, da), min(sb, db)
    if b <= a:
        return 0, 0, 0
    return a - sa, a - da, b - a


# ----------------------------------------------------------------------------
# flattening (integer, host)
# ----------------------------------------------------------------------------

def flatten(ctx_len: Sequence[int], pages: Sequence[int], p: int) -> np.ndarray:
    """Slot of every migrated token, requests in caller order, tokens in
    position order.  ``pages`` is CSR by request with ceil(ctx_len/p) page ids
    each; token t of a request sits in slot pages[t // p] * p + t % p.  A last,
    partly filled page contributes only its valid tokens."""
    out: List[int] = []
    at = 0
    if any(int(n) < 0 for n in ctx_len):
        raise ValueError("negative context length")
    if sum((int(n) + p - 1) // p for n in ctx_len) != len(pages):
        raise ValueError("page table length does not match the context lengths")
    for n in ctx_len:
        n = int(n)
        n_pg = (n + p - 1) // p
        for t in range(n):
            out.append(int(pages[at + t // p]) * p + t % p)
        at += n_pg
    return np.asarray(out, dtype=np.int32)


def runs(sslot: Sequence[int], dslot: Sequence[int]) -> np.ndarray:
    """Start index of every run, then T: ``[s_0 = 0, s_1, ..., s_{n-1}, T]`` (just
    ``[0]`` for no tokens).  Token j continues the run of token j-1 exactly when
    it sits in the next slot on the source side AND in the next slot on the
    destination side; otherwise it starts a run.  When a fragment is a whole
    token row on both sides, a run is one contiguous region per (layer, K|V):
    the regions a per-region copy has to issue (Sec. 3.2.2, the fragmented
    against the contiguous layout)."""
    if len(sslot) != len(dslot):
        raise ValueError("slot lists differ in length")
    out: List[int] = []
    for j in range(len(sslot)):
        if j == 0 or int(sslot[j]) != int(sslot[j - 1]) + 1 or int(dslot[j]) != int(dslot[j - 1]) + 1:
            out.append(j)
    out.append(len(sslot))
    return np.asarray(out if len(sslot) else [0], dtype=np.int32)


# ----------------------------------------------------------------------------
# byte movers (plain C loops)
# ----------------------------------------------------------------------------

def _chk_pool(pool: np.ndarray):
    if pool.ndim != 5 or pool.shape[1] != 2 or not pool.flags.c_contiguous:
        raise ValueError("pool must be a C-contiguous [L][2][S][H_local][D] array")
    return pool.shape[0], pool.shape[2], pool.shape[3], pool.shape[4], pool.dtype.itemsize


def _chk_slots(slots: np.ndarray, S: int) -> np.ndarray:
    slots = np.ascontiguousarray(slots, dtype=np.int32)
    if slots.size and (slots.min() < 0 or slots.max() >= S):
        raise ValueError("slot outside the pool")
    return slots


def pack(src: np.ndarray, sslot: np.ndarray, src_head_off: int, w: int) -> np.ndarray:
    """stream[l][c][j][h][x] = src[l][c][sslot[j]][src_head_off + h][x]."""
    L, S, Hs, D, e = _chk_pool(src)
    sslot = _chk_slots(sslot, S)
    if w <= 0 or src_head_off < 0 or src_head_off + w > Hs:
        raise ValueError("head slice outside the source's heads")
    T = sslot.size
    stream = np.empty((L, 2, T, w, D), dtype=src.dtype)
    _clib().orc_pack(src.ctypes.data, L, S, Hs, D, e, sslot.ctypes.data, T,
                     src_head_off, w, stream.ctypes.data)
    return stream


def unpack(stream: np.ndarray, dst: np.ndarray, dslot: np.ndarray, dst_head_off: int) -> None:
    """dst[l][c][dslot[j]][dst_head_off + h][x] = stream[l][c][j][h][x], in place."""
    L, S, Hd, D, e = _chk_pool(dst)
    dslot = _chk_slots(dslot, S)
    T, w = dslot.size, stream.shape[3]
    if stream.shape != (L, 2, T, w, D) or stream.dtype != dst.dtype or not stream.flags.c_contiguous:
        raise ValueError("stream does not match the destination geometry")
    if dst_head_off < 0 or dst_head_off + w > Hd:
        raise ValueError("head slice outside the destination's heads")
    if np.unique(dslot).size != T:
        raise ValueError("destination slots must be distinct")
    _clib().orc_unpack(stream.ctypes.data, L, S, Hd, D, e, dslot.ctypes.data, T,
                       dst_head_off, w, dst.ctypes.data)


def migrate(src, dst, sslot, dslot, src_head_off, dst_head_off, w) -> None:
    """unpack(pack(src)) into ``dst``."""
    unpack(pack(src, sslot, src_head_off, w), dst, dslot, dst_head_off)


def migrate_direct(src, dst, sslot, dslot, src_head_off, dst_head_off, w) -> None:
    """The same migration as one loop nest from pool to pool (no stream)."""
    L, Ss, Hs, D, e = _chk_pool(src)
    L2, Sd, Hd, D2, e2 = _chk_pool(dst)
    if (L, D, e) != (L2, D2, e2):
        raise ValueError("pools disagree on layers, head dim or element size")
    sslot, dslot = _chk_slots(sslot, Ss), _chk_slots(dslot, Sd)
    if sslot.size != dslot.size:
        raise ValueError("slot lists differ in length")
    if w <= 0 or src_head_off < 0 or src_head_off + w > Hs or dst_head_off < 0 or dst_head_off + w > Hd:
        raise ValueError("head slice outside a pool's heads")
    if np.unique(dslot).size != dslot.size:
        raise ValueError("destination slots must be distinct")
    _clib().orc_migrate_direct(src.ctypes.data, Ss, Hs, src_head_off, dst.ctypes.data, Sd, Hd,
                               dst_head_off, L, D, e, w, sslot.ctypes.data, dslot.ctypes.data,
                               sslot.size)


def migrated_element_source(j_of_dslot: Dict[int, int], sslot: np.ndarray, dst_slot: int,
                            dst_head: int, src_head_off: int, dst_head_off: int, w: int):
    """For one destination (slot, local head): the source (slot, local head) whose
    bytes it must hold after the migration, or None if the migration leaves it
    untouched.  Used to check single outputs of pools too large to copy back."""
    h = dst_head - dst_head_off
    if not 0 <= h < w:
        return None
    j = j_of_dslot.get(int(dst_slot))
    if j is None:
        return None
    return int(sslot[j]), src_head_off + h


# ----------------------------------------------------------------------------
# several virtual GPUs (worked example of Fig. "KV Conversion")
# ----------------------------------------------------------------------------

@dataclass
class VGpu:
    pool: np.ndarray                                  # [L][2][S][H_local][D]
    slots: Dict[int, np.ndarray] = field(default_factory=dict)   # request -> slot per token


@dataclass
class Cluster:
    """G virtual GPUs.  ``groups[k]`` lists the GPUs of TP group k in rank
    order; ``home[req]`` is the group a request runs on.  Every GPU of a
    group holds, for each of the group's requests, its own H/N heads."""
    L: int
    H: int
    D: int
    S: int
    dtype: np.dtype
    groups: List[List[int]]
    home: Dict[int, int]
    ctx: Dict[int, int]
    gpus: Dict[int, VGpu]

    def tp_of(self, group: int) -> int:
        return len(self.groups[group])

    def gather_request(self, req: int) -> np.ndarray:
        """Full KV of a request, [L][2][ctx][H][D], reassembled from its group."""
        g = self.home[req]
        N = self.tp_of(g)
        out = np.zeros((self.L, 2, self.ctx[req], self.H, self.D), dtype=self.dtype)
        for r, gpu in enumerate(self.groups[g]):
            a, b = head_interval(self.H, N, r)
            v = self.gpus[gpu]
            out[:, :, :, a:b, :] = v.pool[:, :, v.slots[req], :, :]
        return out


def transition_pairs(H: int, old_groups, new_groups, home_old: Dict[int, int],
                     home_new: Dict[int, int]):
    """All (src gpu, dst gpu, requests, src_head_off, dst_head_off, w) of a switch:
    every GPU of a request's old group against every GPU of its new group,
    kept when the two head intervals overlap."""
    table: Dict[Tuple[int, int], List[int]] = {}
    for req, go in home_old.items():
        gn = home_new[req]
        for s in old_groups[go]:
            for d in new_groups[gn]:
                table.setdefault((s, d, go, gn), []).append(req)
    out = []
    for (s, d, go, gn), reqs in sorted(table.items()):
        Ns, Nd = len(old_groups[go]), len(new_groups[gn])
        so, do, w = route(H, Ns, old_groups[go].index(s), Nd, new_groups[gn].index(d))
        if w > 0:
            out.append((s, d, sorted(reqs), so, do, w))
    return out


def transition(cl: Cluster, new_groups: List[List[int]], home_new: Dict[int, int],
               alloc: Callable[[int, int], np.ndarray], sentinel: Callable[[int, tuple], np.ndarray],
               mover=None) -> Cluster:
    """Switch ``cl`` to ``new_groups``.  Every destination writes into a fresh
    pool (pre-filled by ``sentinel(gpu, shape)``); ``alloc(gpu, n)`` hands out
    ``n`` distinct free slots of that GPU's new pool.  ``mover`` defaults to
    the oracle's own unpack-after-pack."""
    mover = mover or migrate
    new_gpus: Dict[int, VGpu] = {}
    for g, members in enumerate(new_groups):
        Hl = cl.H // len(members)
        for gpu in members:
            new_gpus[gpu] = VGpu(pool=sentinel(gpu, (cl.L, 2, cl.S, Hl, cl.D)))
    for req, gn in home_new.items():               # one slot list per (request, new GPU)
        for gpu in new_groups[gn]:
            new_gpus[gpu].slots[req] = np.asarray(alloc(gpu, cl.ctx[req]), dtype=np.int32)
    for s, d, reqs, so, do, w in transition_pairs(cl.H, cl.groups, new_groups, cl.home, home_new):
        sslot = np.concatenate([cl.gpus[s].slots[r] for r in reqs]) if reqs else np.zeros(0, np.int32)
        dslot = np.concatenate([new_gpus[d].slots[r] for r in reqs]) if reqs else np.zeros(0, np.int32)
        if sslot.size:
            mover(cl.gpus[s].pool, new_gpus[d].pool, sslot, dslot, so, do, w)
    return Cluster(L=cl.L, H=cl.H, D=cl.D, S=cl.S, dtype=cl.dtype, groups=[list(m) for m in new_groups],
                   home=dict(home_new), ctx=dict(cl.ctx), gpus=new_gpus)
