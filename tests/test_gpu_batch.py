"""nts_run_migrate_batch: several (source, destination) pairs as one pipeline
(Sec. 3.2.2: a TP switch is a list of pairs).  The result must equal the
oracle's migration of every pair, whatever mix of geometries, vector widths,
chunk counts and empty plans shares the two staging buffers."""
import numpy as np
import pytest

from gpu_util import draw_case, random_case_host, random_case_plan_args
from oracle import kvmig as orc
from workload import SplitMix64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    from paper_2605_05467_amd import binding as b
    ctx = b.nts_init(0)
    yield torch, b, ctx
    b.nts_free(ctx)


def _check_pair(h, dst_d, tag):
    L, S_d, st_d, row_d = h["L"], h["S_d"], h["st_d"], h["row_d"]
    for i in range(2 * L):
        got = dst_d[i].cpu().numpy().reshape(S_d, st_d)
        assert got[:, :row_d].tobytes() == h["want"].reshape(2 * L, S_d, -1)[i].tobytes(), (tag, i)
        assert np.array_equal(got[:, row_d:], h["dst_arr"][i].reshape(S_d, st_d)[:, row_d:]), (tag, i)


@pytest.mark.parametrize("first", [0, 7, 14, 21, 28, 35])
def test_batch_of_unrelated_pairs_equals_the_oracle_pair_by_pair(env, first):
    """The staging area has exactly the size nts_batch_staging_bytes names (the
    documented contract, mixed vector widths included) and is followed by guard
    bytes that must stay as they were."""
    torch, b, ctx = env
    st = torch.cuda.current_stream().cuda_stream
    plans, stabs, dtabs, hosts, dsts, keep = [], [], [], [], [], []
    try:
        for seed in range(first, first + 7):
            c = draw_case(seed)
            if seed % 7 == 3:
                c["ctx_len"] = np.zeros_like(c["ctx_len"])          # a pair with nothing to move
                c["src_pages"] = c["src_pages"][:0]
                c["dst_pages"] = c["dst_pages"][:0]
            h = random_case_host(c, b.nts_route(c["H"], c["Ns"], c["rs"], c["Nd"], c["rd"]))
            src_d = [torch.from_numpy(a).cuda() for a in h["src_arr"]]
            dst_d = [torch.from_numpy(a).cuda() for a in h["dst_arr"]]
            args = random_case_plan_args(b, c, h)
            if seed % 2:                                   # every other pair moves its tokens in destination order
                args["flags"] |= b.NTS_ORDER_BY_DST
            plans.append(b.nts_plan_create(ctx, **args))
            stabs.append([t.data_ptr() for t in src_d])
            dtabs.append([t.data_ptr() for t in dst_d])
            hosts.append(h)
            dsts.append(dst_d)
            keep.append(src_d)
        infos = [b.nts_plan_info(p) for p in plans]
        need = b.nts_batch_staging_bytes(plans)
        assert need == 2 * max((i.chunk_bytes + 15) // 16 * 16 for i in infos if i.F)
        guard = 4096
        staging = torch.full((need + guard,), 0xA5, dtype=torch.uint8, device="cuda")
        b.nts_run_migrate_batch(plans, stabs, dtabs, staging.data_ptr(), st)
        torch.cuda.synchronize()
        assert bool((staging[need:] == 0xA5).all()), "wrote past the documented staging size"
        for k, (h, dst_d) in enumerate(zip(hosts, dsts)):
            _check_pair(h, dst_d, (first, k))
        for h, src_d in zip(hosts, keep):                              # sources untouched
            for a, t in zip(h["src_arr"], src_d):
                assert t.cpu().numpy().tobytes() == a.tobytes()
    finally:
        for p in plans:
            b.nts_plan_free(p)


def test_batch_staging_contract_with_a_12_byte_fragment(env):
    """A 12-byte fragment forces 4-byte vectors and a chunk size that is no
    multiple of 16; next to a plan with 16-byte vectors the second buffer must
    still start aligned and end inside nts_batch_staging_bytes."""
    torch, b, ctx = env
    st = torch.cuda.current_stream().cuda_stream
    L, S, T = 2, 64, 40
    rng = SplitMix64(515)
    plans, stabs, dtabs, want, dsts = [], [], [], [], []
    try:
        for D, e, H, B in ((3, 4, 1, 60), (8, 2, 2, 64)):          # 12-byte and 32-byte fragments
            dt = {2: np.uint16, 4: np.uint32}[e]
            src = (rng.words(L * 2 * S * H * D) & np.uint64(np.iinfo(dt).max)).astype(dt).reshape(L, 2, S, H, D)
            dst = (rng.words(L * 2 * S * H * D) & np.uint64(np.iinfo(dt).max)).astype(dt).reshape(L, 2, S, H, D)
            ss, ds = rng.permutation(S)[:T].astype(np.int32), rng.permutation(S)[:T].astype(np.int32)
            exp = dst.copy()
            orc.migrate(src, exp, ss, ds, 0, 0, H)
            sd = torch.from_numpy(src.view(np.uint8).reshape(-1)).cuda()
            dd = torch.from_numpy(dst.view(np.uint8).reshape(-1)).cuda()
            plans.append(b.nts_plan_create(ctx, L=L, D=D, elem_bytes=e, page_size=1, Hs=H, Hd=H, src_head_off=0,
                                           dst_head_off=0, w=H, S_src=S, S_dst=S, ctx_len=[T], src_pages=ss,
                                           dst_pages=ds, staging_bytes=B, flags=b.NTS_VALIDATE_UNIQUE_DST))
            stabs.append(b.layer_ptrs(sd.data_ptr(), L, S * H * D * e))
            dtabs.append(b.layer_ptrs(dd.data_ptr(), L, S * H * D * e))
            want.append((dst, exp))
            dsts.append((sd, dd))
        infos = [b.nts_plan_info(p) for p in plans]
        assert infos[0].vec_bytes == 4 and infos[0].chunk_bytes == 60 and infos[1].vec_bytes == 16
        need = b.nts_batch_staging_bytes(plans)
        assert need == 2 * 64
        staging = torch.full((need + 256,), 0xA5, dtype=torch.uint8, device="cuda")
        b.nts_run_migrate_batch(plans, stabs, dtabs, staging.data_ptr(), st)
        torch.cuda.synchronize()
        assert bool((staging[need:] == 0xA5).all())
        for (sd, dd), (dst, exp) in zip(dsts, want):
            assert dd.cpu().numpy().tobytes() == exp.tobytes()
    finally:
        for p in plans:
            b.nts_plan_free(p)


def _build_cluster(G, H, L, D, S, ctx_of_req, rng):
    gpus = {g: orc.VGpu(pool=np.full((L, 2, S, H, D), 0xDEAD, np.uint16)) for g in range(G)}
    free = {g: list(rng.permutation(S)) for g in range(G)}
    home = {}
    for r, n in ctx_of_req.items():
        g = r % G
        kv = (rng.words(L * 2 * n * H * D) & np.uint64(0xFFFF)).astype(np.uint16).reshape(L, 2, n, H, D)
        slots = np.array([free[g].pop() for _ in range(n)], np.int32)
        gpus[g].slots[r] = slots
        gpus[g].pool[:, :, slots] = kv
        home[r] = g
    return orc.Cluster(L=L, H=H, D=D, S=S, dtype=np.uint16, groups=[[g] for g in range(G)], home=home,
                       ctx=dict(ctx_of_req), gpus=gpus)


def test_whole_tp_switch_as_one_batch_matches_the_oracle_cluster(env):
    """Four virtual GPUs, TP1 -> 2 -> 4 -> 2 -> 1: every step's pairs (several
    sources writing different head ranges of one destination pool included) go
    through ONE batch call; pools compared with the oracle's cluster."""
    torch, b, ctx = env
    st = torch.cuda.current_stream().cuda_stream
    G, H, L, D, S = 4, 8, 3, 16, 128
    ctx_of_req = {r: int(n) for r, n in enumerate(SplitMix64(77).integers(1, 12, 2 * G))}
    cl = _build_cluster(G, H, L, D, S, ctx_of_req, SplitMix64(177))
    first_home = dict(cl.home)
    dev = {g: torch.from_numpy(cl.gpus[g].pool.view(np.int16)).cuda() for g in range(G)}
    for step, size in enumerate((2, 4, 2, 1)):
        new_groups = [list(range(i, i + size)) for i in range(0, G, size)]
        home_new = {r: first_home[r] // size for r in ctx_of_req}
        rng, free = SplitMix64(2000 + step), {}

        def alloc(gpu, n):
            if gpu not in free:
                free[gpu] = list(rng.permutation(S))
            return [free[gpu].pop() for _ in range(n)]

        new = orc.transition(cl, new_groups, home_new, alloc, lambda gpu, shape: np.full(shape, 0xBEEF, np.uint16))
        Hn = H // size
        new_dev = {g: torch.full((L, 2, S, Hn, D), 0xBEEF - 0x10000, dtype=torch.int16, device="cuda")
                   for g in range(G)}
        plans, stabs, dtabs = [], [], []
        try:
            for s, d, reqs, so_o, do_o, w_o in orc.transition_pairs(H, cl.groups, new_groups, cl.home, home_new):
                go, gn = cl.home[reqs[0]], home_new[reqs[0]]
                Ns, Nd = len(cl.groups[go]), len(new_groups[gn])
                so, do, w = b.nts_route(H, Ns, cl.groups[go].index(s), Nd, new_groups[gn].index(d))
                assert (so, do, w) == (so_o, do_o, w_o)
                Hs = H // Ns
                sslot = np.concatenate([cl.gpus[s].slots[r] for r in reqs])
                dslot = np.concatenate([new.gpus[d].slots[r] for r in reqs])
                plans.append(b.nts_plan_create(ctx, L=L, D=D, elem_bytes=2, page_size=1, Hs=Hs, Hd=Hn,
                                               src_head_off=so, dst_head_off=do, w=w, S_src=S, S_dst=S,
                                               ctx_len=[len(sslot)], src_pages=sslot, dst_pages=dslot,
                                               staging_bytes=2048,
                                               flags=b.NTS_VALIDATE_UNIQUE_DST | (b.NTS_ORDER_BY_DST if (s + d + step) % 2 else 0)))
                stabs.append(b.layer_ptrs(dev[s].data_ptr(), L, S * Hs * D * 2))
                dtabs.append(b.layer_ptrs(new_dev[d].data_ptr(), L, S * Hn * D * 2))
            assert len(plans) >= G
            staging = torch.empty(b.nts_batch_staging_bytes(plans), dtype=torch.uint8, device="cuda")
            b.nts_run_migrate_batch(plans, stabs, dtabs, staging.data_ptr(), st)
            torch.cuda.synchronize()
        finally:
            for p in plans:
                b.nts_plan_free(p)
        for g in range(G):
            got = new_dev[g].cpu().numpy().view(np.uint16)
            assert got.tobytes() == new.gpus[g].pool.tobytes(), (step, g)
        cl, dev = new, new_dev


def test_batch_argument_errors(env):
    torch, b, ctx = env
    st = torch.cuda.current_stream().cuda_stream
    L, D, S = 2, 16, 32
    pool = lambda: torch.zeros(L * 2 * S * 4 * D * 2, dtype=torch.uint8, device="cuda")
    A, B, C = pool(), pool(), pool()
    tab = lambda t: b.layer_ptrs(t.data_ptr(), L, S * 4 * D * 2)
    mk = lambda c: b.nts_plan_create(c, L=L, D=D, elem_bytes=2, page_size=1, Hs=4, Hd=4, src_head_off=0,
                                     dst_head_off=0, w=4, S_src=S, S_dst=S, ctx_len=[3], src_pages=[1, 5, 9],
                                     dst_pages=[2, 4, 6], staging_bytes=1024, flags=b.NTS_VALIDATE_UNIQUE_DST)
    p1, p2 = mk(ctx), mk(ctx)
    other = b.nts_init(0)
    p3 = mk(other)
    staging = torch.empty(4096, dtype=torch.uint8, device="cuda")
    try:
        b.nts_run_migrate_batch([], [], [], 0, st)                       # an empty batch is legal
        # A -> B and B -> C in one batch: the second pair would read what the first writes
        with pytest.raises(b.NtsError) as ei:
            b.nts_run_migrate_batch([p1, p2], [tab(A), tab(B)], [tab(B), tab(C)], staging.data_ptr(), st)
        assert ei.value.status == b.NTS_EALIAS
        with pytest.raises(b.NtsError) as ei:                             # staging inside a pool
            b.nts_run_migrate_batch([p1], [tab(A)], [tab(B)], A.data_ptr(), st)
        assert ei.value.status == b.NTS_EALIAS
        with pytest.raises(b.NtsError) as ei:
            b.nts_run_migrate_batch([p1, p3], [tab(A), tab(A)], [tab(B), tab(C)], staging.data_ptr(), st)
        assert ei.value.status == b.NTS_EINVAL
        with pytest.raises(b.NtsError) as ei:
            b.nts_run_migrate_batch([p1], [tab(A)], [tab(B)], 0, st)
        assert ei.value.status == b.NTS_EINVAL
        # two sources into one destination pool is fine (plan order decides overlapping bytes)
        b.nts_run_migrate_batch([p1, p2], [tab(A), tab(C)], [tab(B), tab(B)], staging.data_ptr(), st)
        torch.cuda.synchronize()
    finally:
        for p in (p1, p2, p3):
            b.nts_plan_free(p)
        b.nts_free(other)
