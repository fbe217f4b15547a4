"""Helpers shared by the GPU parity tests: pools on the device and on the host
from the same stateless fill, and the oracle's expected result per layer."""
from __future__ import annotations

import ctypes

import numpy as np

import threading
from concurrent.futures import ThreadPoolExecutor

from oracle import kvmig as orc
from workload import SplitMix64, fill_words, fill_words_fast
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


def compare_every_layer(case: PairCase, dst_d, sslot, dslot, workers: int = 10, label: str = "",
                        direct: bool = False) -> float:
    """Every byte of the destination pool against the oracle, layer by layer.

    The oracle's loops are independent per layer, so each layer is one job of a
    thread pool: regenerate that layer of the source pool and of the
    destination's sentinel fill on the host (stateless fill), run the oracle's
    migration on the pair, copy the GPU's layer back and compare all bytes,
    untouched ones included.  Host memory stays at three layers per worker
    whatever the pool size.  ``direct`` picks the oracle's pool-to-pool loop
    instead of unpack-after-pack (they are pinned to each other; the former
    needs no stream-sized temporary).  Returns the seconds the oracle's
    migration calls took, summed over layers."""
    import torch
    sh = case.shape
    so, do, w = orc.route(sh.H, case.Ns, case.rs, case.Nd, case.rd)
    dt = np_dtype(sh.e)
    src_words = 2 * case.S_src * case.Hs * sh.D * sh.e // 8
    dst_words = 2 * case.S_dst * case.Hd * sh.D * sh.e // 8
    assert (2 * case.S_src * case.Hs * sh.D * sh.e) % 8 == 0 and (2 * case.S_dst * case.Hd * sh.D * sh.e) % 8 == 0
    local = threading.local()
    oracle_seconds = [0.0]
    lock = threading.Lock()
    dst_bytes = dst_d.view(torch.uint8).reshape(-1)

    def one_layer(l):
        import time
        if not hasattr(local, "src"):
            local.src = np.empty(src_words, dtype="<u8")
            local.want = np.empty(dst_words, dtype="<u8")
            local.got = np.empty(dst_words, dtype="<u8")
        fill_words_fast(case.seed_src, l * src_words, src_words, local.src)
        fill_words_fast(case.seed_dst, l * dst_words, dst_words, local.want)
        src = local.src.view(dt).reshape(1, 2, case.S_src, case.Hs, sh.D)
        want = local.want.view(dt).reshape(1, 2, case.S_dst, case.Hd, sh.D)
        t0 = time.perf_counter()
        (orc.migrate_direct if direct else orc.migrate)(src, want, sslot, dslot, so, do, w)
        dt_oracle = time.perf_counter() - t0
        torch.from_numpy(local.got.view(np.uint8)).copy_(dst_bytes[l * dst_words * 8:(l + 1) * dst_words * 8])
        same = np.array_equal(local.got, local.want)
        with lock:
            oracle_seconds[0] += dt_oracle
        return l, same

    bad = []
    with ThreadPoolExecutor(max_workers=min(workers, sh.L)) as ex:
        for l, same in ex.map(one_layer, range(sh.L)):
            if l % 8 == 7 or not same:
                print(f"    {label or case.name}: layers ..{l} compared with the oracle", flush=True)
            if not same:
                bad.append(l)
    assert not bad, (label or case.name, "layers differ from the oracle", bad)
    return oracle_seconds[0]


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


def draw_case(seed):
    rng = SplitMix64(9000 + seed)
    u = lambda lo, hi: int(rng.integers(lo, hi, 1)[0])
    e = (1, 2, 2, 2, 4)[u(0, 4)]
    D = (8, 16, 32, 64, 128, 24, 40)[u(0, 6)]
    while (D * e) % 4:
        D += 1
    L = u(1, 5)
    tps = (1, 2, 4, 8)
    Ns, Nd = tps[u(0, 3)], tps[u(0, 3)]
    H = max(Ns, Nd) * (1, 1, 2, 3)[u(0, 3)]
    rs = u(0, Ns - 1)
    # pick a destination rank whose interval overlaps the source's
    cands = [rd for rd in range(Nd) if orc.route(H, Ns, rs, Nd, rd)[2] > 0]
    rd = cands[u(0, len(cands) - 1)]
    p = (1, 1, 2, 4, 16)[u(0, 4)]
    n_req = u(1, 6)
    ctx_len = rng.integers(0, 70, n_req).astype(np.int32)
    if ctx_len.sum() == 0:
        ctx_len[0] = 5
    n_pg = int(((ctx_len.astype(np.int64) + p - 1) // p).sum())
    pool_pages_s = n_pg + u(1, 40)
    pool_pages_d = n_pg + u(0, 40)
    src_pages = rng.permutation(pool_pages_s)[:n_pg].astype(np.int32)
    if u(0, 3) == 0 and n_pg > 2:                      # shared source pages are legal
        src_pages[1] = src_pages[0]
    dst_pages = rng.permutation(pool_pages_d)[:n_pg].astype(np.int32)
    pad_s, pad_d = (0, 0, 16, 48)[u(0, 3)], (0, 0, 16, 32)[u(0, 3)]
    staging = (0, 1, 4096, 20000, 1 << 20)[u(0, 4)]
    return dict(e=e, D=D, L=L, H=H, Ns=Ns, rs=rs, Nd=Nd, rd=rd, p=p, ctx_len=ctx_len, src_pages=src_pages,
                dst_pages=dst_pages, S_src=pool_pages_s * p, S_dst=pool_pages_d * p, pad_s=pad_s, pad_d=pad_d,
                staging=staging, seed=seed)


def draw_mid_case(seed):
    """Like draw_case at a few thousand tokens and fragments of 256 B to 2 KiB: sizes at which a
    launch has thousands of workgroups, wavefronts cover several small fragments, token counts are
    odd (a wavefront may straddle two slabs) and chunks can exceed the kernels' workgroup groups."""
    rng = SplitMix64(77000 + seed)
    u = lambda lo, hi: int(rng.integers(lo, hi, 1)[0])
    e = (1, 2, 2)[u(0, 2)]
    D = (64, 128)[u(0, 1)]
    L = u(2, 4)
    tps = (1, 2, 4, 8)
    Ns, Nd = tps[u(0, 3)], tps[u(0, 3)]
    H = max(Ns, Nd) * (1, 2, 4, 8)[u(0, 3)]
    rs = u(0, Ns - 1)
    cands = [rd for rd in range(Nd) if orc.route(H, Ns, rs, Nd, rd)[2] > 0]
    rd = cands[u(0, len(cands) - 1)]
    p = (1, 1, 4, 16)[u(0, 3)]
    n_req = u(3, 9)
    ctx_len = rng.integers(300, 1500, n_req).astype(np.int32)
    ctx_len[0] |= 1
    ctx_len[-1] += 1 - int(ctx_len.sum()) % 2          # an odd total
    n_pg = int(((ctx_len.astype(np.int64) + p - 1) // p).sum())
    pool_pages_s = n_pg + u(1, 400)
    pool_pages_d = n_pg + u(0, 400)
    src_pages = rng.permutation(pool_pages_s)[:n_pg].astype(np.int32)
    dst_pages = rng.permutation(pool_pages_d)[:n_pg].astype(np.int32)
    pad_s, pad_d = (0, 16)[u(0, 1)], (0, 32)[u(0, 1)]
    staging = (0, (9 << 20) + 4 * u(1, 5000), (3 << 20) + 4 * u(1, 5000), 1 << 20)[u(0, 3)]
    return dict(e=e, D=D, L=L, H=H, Ns=Ns, rs=rs, Nd=Nd, rd=rd, p=p, ctx_len=ctx_len, src_pages=src_pages,
                dst_pages=dst_pages, S_src=pool_pages_s * p, S_dst=pool_pages_d * p, pad_s=pad_s, pad_d=pad_d,
                staging=staging, seed=seed)


def random_case_host(c, routed):
    """Host side of a drawn case: 2L separately allocated, row-padded arrays per
    pool, the oracle's slot lists, stream and expected destination.  ``routed``
    is the (src_head_off, dst_head_off, w) the library computed; it must equal
    the oracle's."""
    e, D, L, H = c["e"], c["D"], c["L"], c["H"]
    Hs, Hd = H // c["Ns"], H // c["Nd"]
    so, do, w = routed
    assert (so, do, w) == orc.route(H, c["Ns"], c["rs"], c["Nd"], c["rd"]) and w > 0
    dt = np_dtype(e)
    rng = SplitMix64(c["seed"])
    row_s, row_d = Hs * D * e, Hd * D * e
    st_s, st_d = row_s + c["pad_s"], row_d + c["pad_d"]
    S_s, S_d = c["S_src"], c["S_dst"]
    src_arr = [rng.words((S_s * st_s + 7) // 8).view(np.uint8)[:S_s * st_s].copy() for _ in range(2 * L)]
    dst_arr = [rng.words((S_d * st_d + 7) // 8).view(np.uint8)[:S_d * st_d].copy() for _ in range(2 * L)]
    src_h = np.stack([a.reshape(S_s, st_s)[:, :row_s].copy().view(dt).reshape(S_s, Hs, D) for a in src_arr]
                     ).reshape(L, 2, S_s, Hs, D)
    dst_h = np.stack([a.reshape(S_d, st_d)[:, :row_d].copy().view(dt).reshape(S_d, Hd, D) for a in dst_arr]
                     ).reshape(L, 2, S_d, Hd, D)
    sslot = orc.flatten(c["ctx_len"], c["src_pages"], c["p"])
    dslot = orc.flatten(c["ctx_len"], c["dst_pages"], c["p"])
    stream = orc.pack(np.ascontiguousarray(src_h), sslot, so, w)
    want = dst_h.copy()
    orc.unpack(stream, want, dslot, do)
    return dict(e=e, D=D, L=L, Hs=Hs, Hd=Hd, so=so, do=do, w=w, st_s=st_s, st_d=st_d, row_s=row_s, row_d=row_d,
                S_s=S_s, S_d=S_d, src_arr=src_arr, dst_arr=dst_arr, sslot=sslot, dslot=dslot, stream=stream,
                want=want)


def random_case_plan_args(b, c, h):
    return dict(L=h["L"], D=h["D"], elem_bytes=h["e"], page_size=c["p"], Hs=h["Hs"], Hd=h["Hd"],
                src_head_off=h["so"], dst_head_off=h["do"], w=h["w"], S_src=h["S_s"], S_dst=h["S_d"],
                ctx_len=c["ctx_len"], src_pages=c["src_pages"], dst_pages=c["dst_pages"],
                src_token_stride=h["st_s"], dst_token_stride=h["st_d"], staging_bytes=c["staging"],
                flags=b.NTS_VALIDATE_UNIQUE_DST)
