"""Concrete synthetic instances of the five benchmark configurations.

Every instance ("pair case") describes ONE source-GPU -> destination-GPU
migration: the model's KV geometry, the tensor-parallel coordinates of both
ends, the per-request context lengths and the two page tables.  Which heads
move (the routing step) and which slot each token lives in (the flattening
step) are part of the method and are NOT computed here: a case only carries
(H, Ns, rs, Nd, rd), lengths and page ids.

Shapes follow the paper's KV-migration microbenchmark (Sec. 3.2.2): 16-bit KV
of an 8B Llama-class model (32 layers, 8 KV heads, head dim 128, so 128 KiB
per token), 4096 to 40960 tokens, token-granular pages that are fully
fragmented or contiguous per request.  Request lengths are drawn at the scale
of the prompt lengths the paper quotes for its traces (Sec. 4, Workloads).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List

import numpy as np

from .splitmix import SplitMix64


@dataclass(frozen=True)
class ModelShape:
    L: int          # layers
    H: int          # KV heads of the whole model
    D: int          # head dimension (elements)
    e: int          # bytes per element

    @property
    def token_bytes(self) -> int:
        return 2 * self.L * self.H * self.D * self.e


M8B = ModelShape(L=32, H=8, D=128, e=2)


@dataclass
class PairCase:
    name: str
    shape: ModelShape
    p: int                      # page size in tokens
    Ns: int                     # TP level of the source group
    rs: int                     # rank of the source GPU in its group
    Nd: int                     # TP level of the destination group
    rd: int                     # rank of the destination GPU in its group
    S_src: int                  # source pool capacity in token slots
    S_dst: int                  # destination pool capacity in token slots
    ctx_len: np.ndarray         # int32 [n_req]
    src_pages: np.ndarray       # int32, CSR by request, ceil(ctx_len/p) each
    dst_pages: np.ndarray       # int32, same shape
    seed_src: int               # stateless-fill seed of the source pool
    seed_dst: int               # stateless-fill seed of the destination pool (sentinel)
    layout: str = "fragmented"
    notes: str = ""

    @property
    def T(self) -> int:
        return int(self.ctx_len.sum())

    @property
    def Hs(self) -> int:
        return self.shape.H // self.Ns

    @property
    def Hd(self) -> int:
        return self.shape.H // self.Nd

    def pool_elems(self, side: str) -> int:
        S, Hl = (self.S_src, self.Hs) if side == "src" else (self.S_dst, self.Hd)
        return self.shape.L * 2 * S * Hl * self.shape.D

    def pool_bytes(self, side: str) -> int:
        return self.pool_elems(side) * self.shape.e


# ----------------------------------------------------------------------------
# request lengths
# ----------------------------------------------------------------------------

def _rescale_to_sum(x: np.ndarray, total: int) -> np.ndarray:
    x = x.astype(np.float64)
    y = np.floor(x * (total / x.sum())).astype(np.int64)
    y = np.maximum(y, 1)
    diff = total - int(y.sum())
    i = 0
    n = len(y)
    while diff != 0:
        k = i % n
        if diff > 0:
            y[k] += 1
            diff -= 1
        elif y[k] > 1:
            y[k] -= 1
            diff += 1
        i += 1
    return y.astype(np.int32)


def lengths_uniform(rng: SplitMix64, n_req: int, lo: int, hi: int, total: int) -> np.ndarray:
    """n_req lengths uniform in [lo, hi], rescaled so they sum to ``total``."""
    return _rescale_to_sum(rng.integers(lo, hi, n_req), total)


def lengths_zipf(rng: SplitMix64, n_req: int, s: float, total: int) -> np.ndarray:
    """Lengths proportional to rank**-s over ranks 1..n_req, in shuffled order."""
    w = 1.0 / np.arange(1, n_req + 1, dtype=np.float64) ** s
    y = _rescale_to_sum(w * 1e6, total)
    return y[rng.permutation(n_req)].astype(np.int32)


# ----------------------------------------------------------------------------
# page tables (page ids; for p == 1 a page id is a token slot)
# ----------------------------------------------------------------------------

def _n_pages(ctx_len: np.ndarray, p: int) -> np.ndarray:
    return (ctx_len.astype(np.int64) + p - 1) // p


def _request_starts(counts: np.ndarray) -> np.ndarray:
    out = np.zeros(len(counts) + 1, dtype=np.int64)
    np.cumsum(counts, out=out[1:])
    return out


def slots_fragmented(rng: SplitMix64, ctx_len: np.ndarray, p: int, n_pool_pages: int) -> np.ndarray:
    """Distinct random pages; no two consecutive pages of a request are neighbours.

    This is the "fully fragmented" layout: every page of a request is an
    isolated region of the pool.
    """
    cnt = _n_pages(ctx_len, p)
    n = int(cnt.sum())
    if n > n_pool_pages:
        raise ValueError("pool too small")
    pages = rng.permutation(n_pool_pages)[:n].copy()
    if n < 4:
        return pages.astype(np.int32)
    starts = _request_starts(cnt)
    same_req = np.ones(n - 1, dtype=bool)
    same_req[starts[1:-1][(starts[1:-1] > 0) & (starts[1:-1] < n)] - 1] = False
    for _ in range(64):
        bad = np.nonzero(same_req & (np.abs(pages[1:] - pages[:-1]) == 1))[0]
        if len(bad) == 0:
            return pages.astype(np.int32)
        for j in bad:                      # swap the second of the pair far away
            k = int((j + 1 + n // 2 + int(rng.integers(0, 7, 1)[0])) % n)
            pages[j + 1], pages[k] = pages[k], pages[j + 1]
    raise RuntimeError("could not remove adjacent pages")


def slots_contiguous(rng: SplitMix64, ctx_len: np.ndarray, p: int, n_pool_pages: int) -> np.ndarray:
    """Each request's pages are consecutive; requests sit at shuffled positions
    with the pool's free pages spread between them."""
    cnt = _n_pages(ctx_len, p)
    n_req = len(cnt)
    n = int(cnt.sum())
    free = n_pool_pages - n
    if free < 0:
        raise ValueError("pool too small")
    order = rng.permutation(n_req)
    gaps = np.zeros(n_req + 1, dtype=np.int64)
    if free:
        cuts = np.sort(rng.integers(0, free, n_req))
        gaps[:n_req] = np.diff(np.concatenate([[0], cuts]))
    pos = 0
    start_of = np.zeros(n_req, dtype=np.int64)
    for slot, r in enumerate(order):
        pos += int(gaps[slot])
        start_of[r] = pos
        pos += int(cnt[r])
    out = np.empty(n, dtype=np.int32)
    starts = _request_starts(cnt)
    for r in range(n_req):
        out[starts[r]:starts[r + 1]] = np.arange(start_of[r], start_of[r] + cnt[r])
    return out


def slots_zipf_runs(rng: SplitMix64, ctx_len: np.ndarray, p: int, n_pool_pages: int,
                    s: float = 1.1, cap: int = 256) -> np.ndarray:
    """Pages laid out as runs whose lengths follow a Zipf(s) law capped at ``cap``.

    Runs never span two requests.  The runs and the pool's free pages are
    shuffled together, so long contiguous stretches and isolated pages mix.
    """
    cnt = _n_pages(ctx_len, p)
    n = int(cnt.sum())
    free = n_pool_pages - n
    if free < 0:
        raise ValueError("pool too small")
    pmf = 1.0 / np.arange(1, cap + 1, dtype=np.float64) ** s
    cdf = np.cumsum(pmf / pmf.sum())
    runs: List[int] = []
    for c in cnt:
        left = int(c)
        while left > 0:
            draw = rng.uniform(max(8, left // 4 + 1))
            lens = np.searchsorted(cdf, draw) + 1
            for ln in lens:
                ln = int(min(ln, left))
                runs.append(ln)
                left -= ln
                if left == 0:
                    break
    runs_a = np.asarray(runs, dtype=np.int64)
    n_items = len(runs_a) + free
    item_len = np.ones(n_items, dtype=np.int64)
    item_len[:len(runs_a)] = runs_a
    order = rng.permutation(n_items)                   # order[k] = item at position k
    pos_len = item_len[order]
    pos_start = np.concatenate([[0], np.cumsum(pos_len)[:-1]])
    start_of_item = np.empty(n_items, dtype=np.int64)
    start_of_item[order] = pos_start
    out = np.empty(n, dtype=np.int32)
    at = 0
    for k, ln in enumerate(runs_a):
        out[at:at + ln] = np.arange(start_of_item[k], start_of_item[k] + ln)
        at += int(ln)
    return out


def pages_from_slots(slots: np.ndarray) -> np.ndarray:
    """For p == 1 a slot list is already a page table."""
    return np.ascontiguousarray(slots, dtype=np.int32)


def random_pages(rng: SplitMix64, ctx_len: np.ndarray, p: int, n_pool_pages: int, layout: str) -> np.ndarray:
    if layout == "fragmented":
        return slots_fragmented(rng, ctx_len, p, n_pool_pages)
    if layout == "contiguous":
        return slots_contiguous(rng, ctx_len, p, n_pool_pages)
    if layout == "zipf_runs":
        return slots_zipf_runs(rng, ctx_len, p, n_pool_pages)
    raise ValueError(layout)


# ----------------------------------------------------------------------------
# the configurations
# ----------------------------------------------------------------------------

CONFIG_NAMES = ("c1", "c2", "c3", "c3b", "c3c", "c3d", "c4", "c5")

# (Ns, rs, Nd, rd) of the TP-switch shapes used as companions: the moved slice
# is 8, 4, 2, 1, 2, 4, 8 heads wide respectively.
_TRANSITIONS = {
    "1to1": (1, 0, 1, 0),
    "1to2": (1, 0, 2, 1),
    "2to4": (2, 1, 4, 2),
    "4to8": (4, 3, 8, 7),
    "8to4": (8, 2, 4, 1),
    "4to2": (4, 1, 2, 0),
    "2to1": (2, 1, 1, 0),
}


def _round_up(x: int, m: int) -> int:
    return -(-x // m) * m


def _pair(name, shape, p, tr, S_src, S_dst, ctx_len, layout, rng, seed, notes="") -> PairCase:
    Ns, rs, Nd, rd = _TRANSITIONS[tr]
    src_pages = random_pages(rng, ctx_len, p, S_src // p, layout)
    dst_layout = "fragmented" if layout != "contiguous" else "contiguous"
    dst_pages = random_pages(rng, ctx_len, p, S_dst // p, dst_layout)
    return PairCase(name=name, shape=shape, p=p, Ns=Ns, rs=rs, Nd=Nd, rd=rd,
                    S_src=S_src, S_dst=S_dst, ctx_len=ctx_len.astype(np.int32),
                    src_pages=src_pages, dst_pages=dst_pages,
                    seed_src=seed * 1000 + 17, seed_dst=seed * 1000 + 91,
                    layout=layout, notes=notes)


def make_case(name: str, shape: ModelShape = M8B, p: int = 1, tokens: int | None = None) -> List[PairCase]:
    """Pair cases of configuration ``name``.

    c1  seed 0: 160 tokens, 8 requests, 256-slot pools, every TP-switch shape.
    c2  seed 1: 16384 tokens, 16 requests, 20480-slot pools, full and half slice.
    c3  seed 2: headline, 40960 tokens, 40 requests, 49152-slot pools, all 8 heads.
    c3b seed 2: 4096 tokens (the microbenchmark's smallest payload).
    c3c seed 2: headline size, contiguous-per-request layout.
    c3d seed 2: headline size, slices of 4, 2 and 1 heads (TP 1->2, 2->4, 4->8).
    c4  seed 3: headline size, Zipf(1.1) request lengths over 512 requests,
                Zipf(1.1) page-run lengths, four destinations of Zipf(1.1) shares.
    c5  seed 4: 720896 tokens, 704 requests, 753664-slot pools (2 x 92 GiB).
    ``tokens`` overrides the token count (pools scale with it) for reduced runs.
    """
    if name == "c1":
        rng = SplitMix64(0)
        T = tokens or 160
        ctx = lengths_uniform(rng, 8, 1, 40, T)
        S = _round_up(max(256, (T * 8) // 5), p)
        return [_pair(f"c1_{tr}", shape, p, tr, S, S, ctx, "fragmented", rng, 0)
                for tr in ("1to2", "1to1", "2to4", "4to8", "8to4", "4to2", "2to1")]
    if name == "c2":
        rng = SplitMix64(1)
        T = tokens or 16384
        ctx = lengths_uniform(rng, 16, 512, 1536, T)
        S = _round_up((T * 5) // 4, p)
        return [_pair(f"c2_{tr}", shape, p, tr, S, S, ctx, "fragmented", rng, 1)
                for tr in ("1to1", "1to2")]
    if name in ("c3", "c3b", "c3c", "c3d"):
        rng = SplitMix64(2)
        T = tokens or (4096 if name == "c3b" else 40960)
        n_req = max(1, T // 1024)
        ctx = lengths_uniform(rng, n_req, 512, 1536, T)
        S = _round_up((T * 6) // 5, p)
        if name == "c3c":
            return [_pair("c3c_1to1", shape, p, "1to1", S, S, ctx, "contiguous", rng, 2)]
        if name == "c3d":
            return [_pair(f"c3d_{tr}", shape, p, tr, S, S, ctx, "fragmented", rng, 2)
                    for tr in ("1to2", "2to4", "4to8")]
        return [_pair(f"{name}_1to1", shape, p, "1to1", S, S, ctx, "fragmented", rng, 2)]
    if name == "c4":
        rng = SplitMix64(3)
        T = tokens or 40960
        n_req = 512 if T >= 4096 else max(4, T // 8)
        ctx = lengths_zipf(rng, n_req, 1.1, T)
        S = _round_up((T * 6) // 5, p)
        src_pages_all = slots_zipf_runs(rng, ctx, p, S // p)
        # destinations: requests dealt out so that token shares follow Zipf(1.1) over 4 ranks
        share = 1.0 / np.arange(1, 5, dtype=np.float64) ** 1.1
        share /= share.sum()
        target = share * T
        got = np.zeros(4)
        dest = np.zeros(n_req, dtype=np.int64)
        for r in np.argsort(-ctx, kind="stable"):
            d = int(np.argmax(target - got))
            dest[r] = d
            got[d] += ctx[r]
        cnt = _n_pages(ctx, p)
        starts = _request_starts(cnt)
        cases = []
        for d in range(4):
            reqs = np.nonzero(dest == d)[0]
            ctx_d = ctx[reqs]
            sp = (np.concatenate([src_pages_all[starts[r]:starts[r + 1]] for r in reqs])
                  if len(reqs) else np.zeros(0, np.int32))
            dp = slots_fragmented(rng, ctx_d, p, S // p)
            cases.append(PairCase(name=f"c4_dst{d}", shape=shape, p=p, Ns=1, rs=0, Nd=1, rd=0,
                                  S_src=S, S_dst=S, ctx_len=ctx_d.astype(np.int32),
                                  src_pages=sp.astype(np.int32), dst_pages=dp,
                                  seed_src=3017, seed_dst=3091 + d, layout="zipf_runs",
                                  notes=f"destination {d} of 4"))
        return cases
    if name == "c5":
        rng = SplitMix64(4)
        T = tokens or 720896
        n_req = max(1, T // 1024)
        ctx = lengths_uniform(rng, n_req, 512, 1536, T)
        S = _round_up((T * 23) // 22, p)
        return [_pair("c5_1to1", shape, p, "1to1", S, S, ctx, "fragmented", rng, 4)]
    raise ValueError(f"unknown configuration {name!r}")
