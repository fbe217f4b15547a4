"""Seeded random geometries: every case draws a model shape, page size, TP pair,
request mix, pool sizes, row padding and staging size, runs pack, the pipelined
migration and the pool-to-pool kernel through the C ABI and compares whole
outputs with the oracle, bit for bit."""
import numpy as np
import pytest

from oracle import kvmig as orc
from workload import SplitMix64

pytestmark = pytest.mark.gpu
N_CASES = 64


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


@pytest.fixture(scope="module")
def env():
    import torch
    from paper_2605_05467_amd import binding as b
    ctx = b.nts_init(0)
    yield torch, b, ctx
    b.nts_free(ctx)


@pytest.mark.parametrize("seed", range(N_CASES))
def test_random_geometry(env, seed):
    torch, b, ctx = env
    c = draw_case(seed)
    e, D, L, H = c["e"], c["D"], c["L"], c["H"]
    Hs, Hd = H // c["Ns"], H // c["Nd"]
    so, do, w = b.nts_route(H, c["Ns"], c["rs"], c["Nd"], c["rd"])
    assert (so, do, w) == orc.route(H, c["Ns"], c["rs"], c["Nd"], c["rd"]) and w > 0
    dt = {1: np.uint8, 2: np.uint16, 4: np.uint32}[e]
    rng = SplitMix64(seed)
    row_s, row_d = Hs * D * e, Hd * D * e
    st_s, st_d = row_s + c["pad_s"], row_d + c["pad_d"]
    S_s, S_d = c["S_src"], c["S_dst"]
    # 2L separate arrays per pool, rows padded to the token stride
    src_arr = [rng.words((S_s * st_s + 7) // 8).view(np.uint8)[:S_s * st_s].copy() for _ in range(2 * L)]
    dst_arr = [rng.words((S_d * st_d + 7) // 8).view(np.uint8)[:S_d * st_d].copy() for _ in range(2 * L)]
    src_h = np.stack([a.reshape(S_s, st_s)[:, :row_s].copy().view(dt).reshape(S_s, Hs, D) for a in src_arr]
                     ).reshape(L, 2, S_s, Hs, D)
    dst_h = np.stack([a.reshape(S_d, st_d)[:, :row_d].copy().view(dt).reshape(S_d, Hd, D) for a in dst_arr]
                     ).reshape(L, 2, S_d, Hd, D)
    sslot = orc.flatten(c["ctx_len"], c["src_pages"], c["p"])
    dslot = orc.flatten(c["ctx_len"], c["dst_pages"], c["p"])
    stream_h = orc.pack(np.ascontiguousarray(src_h), sslot, so, w)
    want = dst_h.copy()
    orc.unpack(stream_h, want, dslot, do)

    src_d = [torch.from_numpy(a).cuda() for a in src_arr]
    kw = dict(L=L, D=D, elem_bytes=e, page_size=c["p"], Hs=Hs, Hd=Hd, src_head_off=so, dst_head_off=do, w=w,
              S_src=S_s, S_dst=S_d, ctx_len=c["ctx_len"], src_pages=c["src_pages"], dst_pages=c["dst_pages"],
              src_token_stride=st_s, dst_token_stride=st_d, staging_bytes=c["staging"],
              flags=b.NTS_VALIDATE_UNIQUE_DST)
    plan = b.nts_plan_create(ctx, **kw)
    try:
        info = b.nts_plan_info(plan)
        s, d = b.nts_plan_slots(plan)
        assert np.array_equal(s, sslot) and np.array_equal(d, dslot)
        assert info.X == stream_h.nbytes
        st = torch.cuda.current_stream().cuda_stream
        sp = [t.data_ptr() for t in src_d]
        out = torch.full((max(info.X, 16),), 0xA5, dtype=torch.uint8, device="cuda")
        b.nts_run_pack(plan, sp, out.data_ptr(), st)
        torch.cuda.synchronize()
        assert out.cpu().numpy()[:info.X].tobytes() == stream_h.tobytes()
        for which in ("migrate", "direct", "unpack"):
            dst_d = [torch.from_numpy(a).cuda() for a in dst_arr]
            dp = [t.data_ptr() for t in dst_d]
            if which == "migrate":
                staging = torch.empty(max(2 * info.chunk_bytes, 16), dtype=torch.uint8, device="cuda")
                b.nts_run_migrate(plan, sp, dp, staging.data_ptr(), st)
            elif which == "direct":
                b.nts_run_migrate_direct(plan, sp, dp, st)
            else:
                b.nts_run_unpack(plan, out.data_ptr(), dp, st)
            torch.cuda.synchronize()
            for i in range(2 * L):
                got = dst_d[i].cpu().numpy().reshape(S_d, st_d)
                assert got[:, :row_d].tobytes() == want.reshape(2 * L, S_d, -1)[i].tobytes(), (which, i, c)
                assert np.array_equal(got[:, row_d:], dst_arr[i].reshape(S_d, st_d)[:, row_d:])   # padding untouched
    finally:
        b.nts_plan_free(plan)
