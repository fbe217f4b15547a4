"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle
on the same seeded inputs.  Byte movers: the bar is bit-exact."""
import numpy as np
import pytest

from oracle import kvmig as orc
from workload import M8B, ModelShape, fill_pool_u16, make_case, SplitMix64
from workload.configs import PairCase, random_pages, lengths_uniform

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def b():
    from paper_2605_05467_amd import binding
    return binding


@pytest.fixture(scope="module")
def ctx(b):
    c = b.nts_init(0)
    yield c
    b.nts_free(c)


@pytest.fixture(scope="module")
def torch():
    import torch
    return torch


def _expected_full(case, L, D):
    """Oracle result on whole pools (small cases only)."""
    from gpu_util import host_layers, oracle_slots
    so, do, w = orc.route(case.shape.H, case.Ns, case.rs, case.Nd, case.rd)
    src = host_layers(case, "src", range(L), D=D)
    dst = host_layers(case, "dst", range(L), D=D).copy()
    sslot, dslot = oracle_slots(case)
    stream = orc.pack(src, sslot, so, w)
    orc.unpack(stream, dst, dslot, do)
    return src, stream, dst


def test_device_fill_matches_host_fill(torch):
    from workload import device as wdev
    from workload import fill_words
    t = torch.empty(8 * 100003, dtype=torch.uint8, device="cuda")
    wdev.fill_tensor(t, 1234, start_word=77)
    got = t.cpu().numpy().view("<u8")
    assert np.array_equal(got, fill_words(1234, 77, 100003))
    assert wdev.count_mismatch(t, 1234, start_word=77) == 0
    t[8 * 5] ^= 1
    assert wdev.count_mismatch(t, 1234, start_word=77) == 1


def test_measurement_probes_run_and_report_plausible_ceilings(torch):
    """The two probes bench.py --linear reports as measured ceilings (matrix cores alone on
    random operands; a read-only HBM stream) launch, finish and land between a loose floor
    and the chip's nominal peaks."""
    from workload import device as wdev
    t = wdev.mfma_ceiling_tflops(0.05)
    g = wdev.read_ceiling_gbs(256 << 20)
    assert 500.0 < t <= 2500.0 * 1.02, t
    assert 2000.0 < g <= 8000.0 * 1.02, g


@pytest.mark.parametrize("p", [1, 4, 16])
def test_plan_flattening_matches_oracle(b, ctx, p):
    from gpu_util import make_plan, oracle_slots
    rng = SplitMix64(40 + p)
    ctx_len = np.array([0, 5, 17, 0, 1, 64, 33, 0], np.int32)
    S = 256
    case = PairCase(name="t", shape=M8B, p=p, Ns=1, rs=0, Nd=2, rd=1, S_src=S, S_dst=S, ctx_len=ctx_len,
                    src_pages=random_pages(rng, ctx_len, p, S // p, "fragmented"),
                    dst_pages=random_pages(rng, ctx_len, p, S // p, "fragmented"),
                    seed_src=1, seed_dst=2)
    plan = make_plan(b, ctx, case, L=2)
    try:
        s, d = b.nts_plan_slots(plan)
        es, ed = oracle_slots(case)
        assert np.array_equal(s, es) and np.array_equal(d, ed)
        info = b.nts_plan_info(plan)
        assert info.T == int(ctx_len.sum()) and info.F == info.T * 4
        assert info.frag_bytes == 4 * 128 * 2 and info.X == info.F * info.frag_bytes
    finally:
        b.nts_plan_free(plan)


@pytest.mark.parametrize("idx", range(7))
def test_c1_pack_unpack_migrate(b, ctx, torch, idx):
    """Configuration 1 (~1e4 fragments), every TP-switch shape, whole outputs."""
    from gpu_util import device_pool, make_plan, slab_bytes, to_host
    case = make_case("c1")[idx]
    sh = case.shape
    src_h, stream_h, dst_h = _expected_full(case, sh.L, sh.D)
    src_d, dst_d = device_pool(case, "src"), device_pool(case, "dst")
    assert np.array_equal(to_host(src_d).view(np.uint16), src_h.reshape(-1))
    sp = b.layer_ptrs(src_d.data_ptr(), sh.L, slab_bytes(case, "src"))
    dp = b.layer_ptrs(dst_d.data_ptr(), sh.L, slab_bytes(case, "dst"))
    plan = make_plan(b, ctx, case)
    try:
        info = b.nts_plan_info(plan)
        assert info.X == stream_h.nbytes
        out = torch.zeros(info.X, dtype=torch.uint8, device="cuda")
        st = torch.cuda.current_stream().cuda_stream
        b.nts_run_pack(plan, sp, out.data_ptr(), st)
        torch.cuda.synchronize()
        assert to_host(out).tobytes() == stream_h.tobytes()
        b.nts_run_unpack(plan, out.data_ptr(), dp, st)
        torch.cuda.synchronize()
        assert to_host(dst_d).tobytes() == dst_h.tobytes()
        assert np.array_equal(to_host(src_d).view(np.uint16), src_h.reshape(-1))   # source untouched
    finally:
        b.nts_plan_free(plan)
    # the pipelined migration gives the same pool for any staging size
    for B in (0, info.frag_bytes, 7 * info.frag_bytes, 65536 + 512, 1 << 20):
        dst2 = device_pool(case, "dst")
        dp2 = b.layer_ptrs(dst2.data_ptr(), sh.L, slab_bytes(case, "dst"))
        if B == info.frag_bytes and info.F > 4096:
            B = info.frag_bytes * 3
        plan = make_plan(b, ctx, case, staging_bytes=B)
        try:
            i2 = b.nts_plan_info(plan)
            staging = torch.empty(2 * i2.chunk_bytes, dtype=torch.uint8, device="cuda")
            b.nts_run_migrate(plan, sp, dp2, staging.data_ptr(), torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
            assert to_host(dst2).tobytes() == dst_h.tobytes(), B
        finally:
            b.nts_plan_free(plan)


def test_chunks_concatenate_to_the_stream(b, ctx, torch):
    from gpu_util import device_pool, make_plan, slab_bytes, to_host
    case = make_case("c1")[0]
    sh = case.shape
    _, stream_h, _ = _expected_full(case, sh.L, sh.D)
    src_d = device_pool(case, "src")
    sp = b.layer_ptrs(src_d.data_ptr(), sh.L, slab_bytes(case, "src"))
    plan = make_plan(b, ctx, case, staging_bytes=300 * 1024 + 4)     # 293 fragments per chunk
    try:
        info = b.nts_plan_info(plan)
        assert info.chunk_frags == (300 * 1024 + 4) // info.frag_bytes
        parts = []
        for k in range(info.n_chunks):
            buf = torch.full((info.chunk_bytes,), 0xA5, dtype=torch.uint8, device="cuda")
            b.nts_run_pack_chunk(plan, sp, k, buf.data_ptr(), torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
            n = min(info.chunk_frags, info.F - k * info.chunk_frags) * info.frag_bytes
            h = to_host(buf)
            assert (h[n:] == 0xA5).all()                              # nothing past the chunk
            parts.append(h[:n])
        assert np.concatenate(parts).tobytes() == stream_h.tobytes()
    finally:
        b.nts_plan_free(plan)


def test_chunk_by_chunk_pack_then_unpack_equals_the_migration(b, ctx, torch):
    """What a sender and a receiver do around their transport: chunk k packed into one of two
    buffers, unpacked from it on the other side; ragged chunk size, last chunk short."""
    from gpu_util import device_pool, make_plan, slab_bytes, to_host
    for case in make_case("c1")[:3]:
        sh = case.shape
        _, _, dst_h = _expected_full(case, sh.L, sh.D)
        src_d, dst_d = device_pool(case, "src"), device_pool(case, "dst")
        sp = b.layer_ptrs(src_d.data_ptr(), sh.L, slab_bytes(case, "src"))
        dp = b.layer_ptrs(dst_d.data_ptr(), sh.L, slab_bytes(case, "dst"))
        plan = make_plan(b, ctx, case, staging_bytes=200 * 1024 + 12)
        try:
            info = b.nts_plan_info(plan)
            assert info.n_chunks > 3 and info.F % info.chunk_frags != 0
            bufs = torch.full((2, info.chunk_bytes + 64), 0xA5, dtype=torch.uint8, device="cuda")
            st = torch.cuda.current_stream().cuda_stream
            for k in range(info.n_chunks):
                p_ = bufs[k & 1].data_ptr()
                b.nts_run_pack_chunk(plan, sp, k, p_, st)
                b.nts_run_unpack_chunk(plan, p_, k, dp, st)
            torch.cuda.synchronize()
            assert to_host(dst_d).tobytes() == dst_h.tobytes()
            assert (to_host(bufs)[:, info.chunk_bytes:] == 0xA5).all()      # nothing past a chunk
        finally:
            b.nts_plan_free(plan)


@pytest.mark.parametrize("shape,tr,p,T", [
    (ModelShape(L=3, H=8, D=64, e=1), (1, 0, 2, 1), 1, 300),      # fp8 KV, 256 B fragments
    (ModelShape(L=2, H=6, D=40, e=2), (1, 0, 2, 0), 2, 157),      # 240 B fragments: 48 B-aligned -> 16 B vectors
    (ModelShape(L=2, H=6, D=20, e=2), (2, 1, 1, 0), 4, 97),       # 120 B fragments -> 8 B vectors
    (ModelShape(L=2, H=3, D=1, e=4), (1, 0, 1, 0), 1, 513),       # 12 B fragments -> 4 B vectors
    (ModelShape(L=5, H=32, D=128, e=2), (1, 0, 1, 0), 16, 200),   # 8 KiB fragments: several column steps
    (ModelShape(L=2, H=12, D=128, e=2), (1, 0, 4, 3), 1, 333),    # 3 heads: 768 B, 48 of 64 lanes
    (ModelShape(L=1, H=8, D=128, e=4), (4, 1, 8, 2), 1, 1),       # a single token
    (ModelShape(L=96, H=2, D=32, e=2), (1, 0, 2, 1), 1, 61),      # NTS_MAX_LAYERS: the whole by-value pointer table in use
])
def test_other_geometries(b, ctx, torch, shape, tr, p, T):
    from gpu_util import device_pool, make_plan, slab_bytes, to_host
    rng = SplitMix64(T)
    n_req = min(5, T)
    ctx_len = lengths_uniform(rng, n_req, 1, 50, T)
    S = ((T + n_req * p) * 2 // p + 1) * p
    Ns, rs, Nd, rd = tr
    case = PairCase(name="g", shape=shape, p=p, Ns=Ns, rs=rs, Nd=Nd, rd=rd, S_src=S, S_dst=S,
                    ctx_len=ctx_len, src_pages=random_pages(rng, ctx_len, p, S // p, "fragmented"),
                    dst_pages=random_pages(rng, ctx_len, p, S // p, "fragmented"), seed_src=5, seed_dst=6)
    if (2 * S * case.Hs * shape.D * shape.e) % 8 or (2 * S * case.Hd * shape.D * shape.e) % 8:
        pytest.skip("layer size not a multiple of the fill word")
    _, stream_h, dst_h = _expected_full(case, shape.L, shape.D)
    src_d, dst_d = device_pool(case, "src"), device_pool(case, "dst")
    sp = b.layer_ptrs(src_d.data_ptr(), shape.L, slab_bytes(case, "src"))
    dp = b.layer_ptrs(dst_d.data_ptr(), shape.L, slab_bytes(case, "dst"))
    plan = make_plan(b, ctx, case, staging_bytes=40000)
    try:
        info = b.nts_plan_info(plan)
        out = torch.zeros(info.X, dtype=torch.uint8, device="cuda")
        b.nts_run_pack(plan, sp, out.data_ptr(), torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        assert to_host(out).tobytes() == stream_h.tobytes()
        staging = torch.empty(2 * info.chunk_bytes, dtype=torch.uint8, device="cuda")
        b.nts_run_migrate(plan, sp, dp, staging.data_ptr(), torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        assert to_host(dst_d).tobytes() == dst_h.tobytes()
    finally:
        b.nts_plan_free(plan)


def test_separate_layer_allocations_and_padded_rows(b, ctx, torch):
    """2L independent allocations with a token stride wider than a row."""
    from gpu_util import to_host
    L, H, D, e, S, T = 3, 4, 32, 2, 64, 50
    row = H * D * e
    stride = row + 64
    rng = SplitMix64(9)
    ctx_len = np.array([20, 30], np.int32)
    sp_h = rng.permutation(S)[:T].astype(np.int32)
    dp_h = rng.permutation(S)[:T].astype(np.int32)
    src_h = [(rng.words(S * stride // 8)).view(np.uint8).copy() for _ in range(2 * L)]
    dst_h = [(rng.words(S * stride // 8)).view(np.uint8).copy() for _ in range(2 * L)]
    src_d = [torch.from_numpy(a).cuda() for a in src_h]
    dst_d = [torch.from_numpy(a).cuda() for a in dst_h]
    so, do, w = b.nts_route(H, 1, 0, 1, 0)
    plan = b.nts_plan_create(ctx, L=L, D=D, elem_bytes=e, page_size=1, Hs=H, Hd=H, src_head_off=so,
                             dst_head_off=do, w=w, S_src=S, S_dst=S, ctx_len=ctx_len, src_pages=sp_h,
                             dst_pages=dp_h, src_token_stride=stride, dst_token_stride=stride,
                             staging_bytes=4096, flags=b.NTS_VALIDATE_UNIQUE_DST)
    try:
        info = b.nts_plan_info(plan)
        staging = torch.empty(2 * info.chunk_bytes, dtype=torch.uint8, device="cuda")
        b.nts_run_migrate(plan, [t.data_ptr() for t in src_d], [t.data_ptr() for t in dst_d],
                          staging.data_ptr(), torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
    finally:
        b.nts_plan_free(plan)
    # oracle on the row part of each array (the padding is not KV and must not change)
    for i in range(2 * L):
        s2 = src_h[i].reshape(S, stride)[:, :row].copy().view(np.uint16).reshape(1, 1, S, H, D)
        d2 = dst_h[i].reshape(S, stride)[:, :row].copy().view(np.uint16).reshape(1, 1, S, H, D)
        s2 = np.concatenate([s2, s2], axis=1)
        d2 = np.concatenate([d2, d2], axis=1).copy()
        orc.migrate_direct(np.ascontiguousarray(s2), d2, orc.flatten(ctx_len, sp_h, 1),
                           orc.flatten(ctx_len, dp_h, 1), so, do, w)
        got = to_host(dst_d[i]).reshape(S, stride)
        assert got[:, :row].tobytes() == d2[0, 0].tobytes()
        assert np.array_equal(got[:, row:], dst_h[i].reshape(S, stride)[:, row:])


def test_error_paths_and_empty_plans(b, ctx, torch):
    kw = dict(L=2, D=128, elem_bytes=2, page_size=1, Hs=8, Hd=4, src_head_off=4, dst_head_off=0, w=4,
              S_src=32, S_dst=32, flags=b.NTS_VALIDATE_UNIQUE_DST)
    ok = dict(ctx_len=[3, 2], src_pages=[1, 2, 3, 4, 5], dst_pages=[9, 8, 7, 6, 5])

    def status(**over):
        args = {**kw, **ok, **over}
        try:
            plan = b.nts_plan_create(ctx, **args)
        except b.NtsError as e:
            return e.status
        b.nts_plan_free(plan)
        return 0

    assert status() == 0
    assert status(src_pages=[1, 2, 3, 4, 32]) == b.NTS_ERANGE
    assert status(dst_pages=[9, 8, -1, 6, 5]) == b.NTS_ERANGE
    assert status(dst_pages=[9, 8, 7, 9, 5]) == b.NTS_EDUP
    assert status(dst_pages=[9, 8, 7, 9, 5], flags=0) == 0           # not checked unless asked
    assert status(src_pages=[1, 1, 1, 1, 1]) == 0                     # shared source pages are fine
    assert status(w=0) == b.NTS_EINVAL
    assert status(src_head_off=5) == b.NTS_EINVAL
    assert status(dst_head_off=1) == b.NTS_EINVAL
    assert status(elem_bytes=3) == b.NTS_EINVAL
    assert status(L=b.NTS_MAX_LAYERS + 1) == b.NTS_EINVAL
    assert status(ctx_len=[3, -2]) == b.NTS_EINVAL
    assert status(page_size=3) == b.NTS_EINVAL                        # pool not a multiple of p
    assert status(D=1, elem_bytes=1, w=1, src_head_off=0) == b.NTS_EINVAL   # 1-byte fragments
    assert status(src_token_stride=(1 << 30) + 16) == b.NTS_EINVAL    # sizes that could leave 64 bits
    assert status(dst_token_stride=1 << 31) == b.NTS_EINVAL
    assert status(D=(1 << 20) + 4) == b.NTS_EINVAL
    assert status(Hs=(1 << 16) + 8) == b.NTS_EINVAL
    assert status(src_token_stride=8 * 128 * 2 + 64) == 0             # padded rows are fine
    # zero tokens: legal, run calls are no-ops
    plan = b.nts_plan_create(ctx, **{**kw, "ctx_len": [0, 0], "src_pages": [], "dst_pages": []})
    info = b.nts_plan_info(plan)
    assert (info.T, info.F, info.X, info.n_chunks) == (0, 0, 0, 0)
    z = torch.zeros(16, dtype=torch.uint8, device="cuda")
    tab = [z.data_ptr()] * 4
    b.nts_run_pack(plan, tab, 0)
    b.nts_run_unpack(plan, 0, tab)
    b.nts_run_migrate(plan, tab, tab, 0)
    b.nts_plan_free(plan)
    plan = b.nts_plan_create(ctx, **{**kw, "ctx_len": [], "src_pages": [], "dst_pages": []})
    assert b.nts_plan_info(plan).T == 0
    b.nts_plan_free(plan)
    # aliasing pools are rejected
    plan = b.nts_plan_create(ctx, **{**kw, **ok, "Hd": 8, "dst_head_off": 0})
    pool = torch.zeros(2 * 2 * 32 * 8 * 128 * 2, dtype=torch.uint8, device="cuda")
    tab = b.layer_ptrs(pool.data_ptr(), 2, 32 * 8 * 128 * 2)
    staging = torch.zeros(2 * b.nts_plan_info(plan).chunk_bytes, dtype=torch.uint8, device="cuda")
    with pytest.raises(b.NtsError) as ei:
        b.nts_run_migrate(plan, tab, tab, staging.data_ptr())
    assert ei.value.status == b.NTS_EALIAS
    with pytest.raises(b.NtsError) as ei:
        b.nts_run_pack(plan, tab, 0)
    assert ei.value.status == b.NTS_EINVAL
    with pytest.raises(b.NtsError) as ei:
        b.nts_run_pack_chunk(plan, tab, 99, staging.data_ptr())
    assert ei.value.status == b.NTS_EINVAL
    b.nts_plan_free(plan)
    torch.cuda.synchronize()


@pytest.mark.parametrize("seed", range(24))
def test_direct_in_destination_order_matches_oracle_on_drawn_cases(b, ctx, torch, seed):
    """NTS_ORDER_BY_DST: the pool-to-pool kernel walks the tokens in ascending
    destination-slot order.  The result must not change: drawn geometries (1-, 2- and
    4-byte elements, pages of 1 to 16 tokens, padded rows, 2L separate allocations,
    shared source pages, pools whose slot count is no multiple of 32 or of 256 x 32),
    every pool byte compared, and every other run call of such a plan unaffected."""
    from gpu_util import draw_case, random_case_host, random_case_plan_args
    c = draw_case(500 + seed)
    h = random_case_host(c, b.nts_route(c["H"], c["Ns"], c["rs"], c["Nd"], c["rd"]))
    args = random_case_plan_args(b, c, h)
    with pytest.raises(b.NtsError) as ei:                    # the ranking needs validated, distinct slots
        b.nts_plan_create(ctx, **{**args, "flags": b.NTS_ORDER_BY_DST})
    assert ei.value.status == b.NTS_EINVAL
    args["flags"] = b.NTS_VALIDATE_UNIQUE_DST | b.NTS_ORDER_BY_DST | (b.NTS_DETECT_RUNS if seed % 2 else 0)
    plan = b.nts_plan_create(ctx, **args)
    st = torch.cuda.current_stream().cuda_stream
    try:
        s, d = b.nts_plan_slots(plan)
        assert np.array_equal(s, h["sslot"]) and np.array_equal(d, h["dslot"])      # the lists themselves keep token order
        src_d = [torch.from_numpy(a).cuda() for a in h["src_arr"]]
        for call in ("direct", "staged"):
            dst_d = [torch.from_numpy(a).cuda() for a in h["dst_arr"]]
            stab, dtab = [t.data_ptr() for t in src_d], [t.data_ptr() for t in dst_d]
            if call == "direct":
                b.nts_run_migrate_direct(plan, stab, dtab, st)
            else:
                info = b.nts_plan_info(plan)
                staging = torch.empty(2 * info.chunk_bytes, dtype=torch.uint8, device="cuda")
                b.nts_run_migrate(plan, stab, dtab, staging.data_ptr(), st)
            torch.cuda.synchronize()
            L, S_d, st_d, row_d = h["L"], h["S_d"], h["st_d"], h["row_d"]
            for i in range(2 * L):
                got = dst_d[i].cpu().numpy().reshape(S_d, st_d)
                assert got[:, :row_d].tobytes() == h["want"].reshape(2 * L, S_d, -1)[i].tobytes(), (call, seed, i)
                assert np.array_equal(got[:, row_d:], h["dst_arr"][i].reshape(S_d, st_d)[:, row_d:]), (call, seed, i)
    finally:
        b.nts_plan_free(plan)


@pytest.mark.parametrize("idx", [0, 1, 3, 4])
def test_direct_and_memcpy_baseline_match_oracle(b, ctx, torch, idx):
    """The pool-to-pool kernel and the per-fragment memcpy baseline produce the
    oracle's direct migration (config 1 shapes, whole pools)."""
    from gpu_util import device_pool, host_layers, make_plan, oracle_slots, slab_bytes, to_host
    case = make_case("c1")[idx]
    sh = case.shape
    so, do, w = orc.route(sh.H, case.Ns, case.rs, case.Nd, case.rd)
    src_h = host_layers(case, "src", range(sh.L))
    want = host_layers(case, "dst", range(sh.L)).copy()
    sslot, dslot = oracle_slots(case)
    orc.migrate_direct(src_h, want, sslot, dslot, so, do, w)
    src_d = device_pool(case, "src")
    sp = b.layer_ptrs(src_d.data_ptr(), sh.L, slab_bytes(case, "src"))
    plan = make_plan(b, ctx, case)
    try:
        st = torch.cuda.current_stream().cuda_stream
        dst_d = device_pool(case, "dst")
        b.nts_run_migrate_direct(plan, sp, b.layer_ptrs(dst_d.data_ptr(), sh.L, slab_bytes(case, "dst")), st)
        torch.cuda.synchronize()
        assert to_host(dst_d).tobytes() == want.tobytes()
        for merge in (False, True):
            dst_d = device_pool(case, "dst")
            n = b.nts_run_memcpy_baseline(plan, sp, b.layer_ptrs(dst_d.data_ptr(), sh.L, slab_bytes(case, "dst")),
                                          merge, st)
            torch.cuda.synchronize()
            assert to_host(dst_d).tobytes() == want.tobytes()
            assert n == case.T * sh.L * 2          # fully fragmented: nothing to merge
        with pytest.raises(b.NtsError) as ei:
            b.nts_run_migrate_direct(plan, sp, sp, st)
        assert ei.value.status in (b.NTS_EALIAS, b.NTS_EINVAL)
    finally:
        b.nts_plan_free(plan)


def test_memcpy_baseline_merges_contiguous_runs(b, ctx, torch):
    from gpu_util import device_pool, host_layers, make_plan, oracle_slots, slab_bytes, to_host
    rng = SplitMix64(31)
    ctx_len = np.array([40, 1, 25], np.int32)
    S = 128
    case = PairCase(name="runs", shape=ModelShape(L=2, H=8, D=128, e=2), p=1, Ns=1, rs=0, Nd=1, rd=0,
                    S_src=S, S_dst=S, ctx_len=ctx_len,
                    src_pages=random_pages(rng, ctx_len, 1, S, "contiguous"),
                    dst_pages=random_pages(rng, ctx_len, 1, S, "contiguous"), seed_src=7, seed_dst=8)
    sh = case.shape
    src_h = host_layers(case, "src", range(sh.L))
    want = host_layers(case, "dst", range(sh.L)).copy()
    sslot, dslot = oracle_slots(case)
    orc.migrate_direct(src_h, want, sslot, dslot, 0, 0, 8)
    src_d, dst_d = device_pool(case, "src"), device_pool(case, "dst")
    plan = make_plan(b, ctx, case)
    try:
        n = b.nts_run_memcpy_baseline(plan, b.layer_ptrs(src_d.data_ptr(), sh.L, slab_bytes(case, "src")),
                                      b.layer_ptrs(dst_d.data_ptr(), sh.L, slab_bytes(case, "dst")), True,
                                      torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
    finally:
        b.nts_plan_free(plan)
    assert to_host(dst_d).tobytes() == want.tobytes()
    # runs break where either side's slots stop being consecutive: count them on the host
    runs = 1 + int(np.sum((np.diff(sslot) != 1) | (np.diff(dslot) != 1)))
    assert n == runs * sh.L * 2 and runs <= 5


@pytest.mark.parametrize("layout,p,n_req,mean_len", [("contiguous", 1, 40, 3000), ("fragmented", 1, 40, 3000),
                                                     ("fragmented", 16, 300, 400), ("zipf_runs", 1, 64, 1500),
                                                     ("contiguous", 4, 3, 50)])
def test_run_detection_equals_oracle(b, ctx, torch, layout, p, n_req, mean_len):
    """NTS_DETECT_RUNS: the device-built run list is the oracle's, entry for entry, on layouts
    with few long runs, with one run per token, with one run per page and with a skewed mix;
    sizes span several hundred 256-token blocks (more than one pass of the block scan) down
    to a single partial block."""
    rng = SplitMix64(1234 + p + n_req)
    ctx_len = lengths_uniform(rng, n_req, max(1, mean_len // 2), mean_len * 3 // 2, n_req * mean_len)
    n_pages = int(((ctx_len.astype(np.int64) + p - 1) // p).sum())
    S = (n_pages + 64) * p * 2
    src_pages = random_pages(rng, ctx_len, p, S // p, layout)
    dst_pages = random_pages(rng, ctx_len, p, S // p, "fragmented" if layout == "fragmented" else "contiguous")
    kw = dict(L=1, D=32, elem_bytes=2, page_size=p, Hs=2, Hd=2, src_head_off=0, dst_head_off=0, w=2, S_src=S,
              S_dst=S, ctx_len=ctx_len, src_pages=src_pages, dst_pages=dst_pages)
    plan = b.nts_plan_create(ctx, flags=b.NTS_VALIDATE_UNIQUE_DST | b.NTS_DETECT_RUNS, **kw)
    plain = b.nts_plan_create(ctx, flags=b.NTS_VALIDATE_UNIQUE_DST, **kw)
    try:
        sslot, dslot = orc.flatten(ctx_len, src_pages, p), orc.flatten(ctx_len, dst_pages, p)
        want = orc.runs(sslot, dslot)
        info = b.nts_plan_info(plan)
        assert info.T == len(sslot) and info.n_runs == len(want) - 1
        assert np.array_equal(b.nts_plan_runs(plan), want)
        assert b.nts_plan_info(plain).n_runs == 0
        with pytest.raises(b.NtsError) as ei:
            b.nts_plan_runs(plain)
        assert ei.value.status == b.NTS_EINVAL
    finally:
        b.nts_plan_free(plan)
        b.nts_plan_free(plain)


def test_run_flag_changes_no_result_and_feeds_the_memcpy_baseline(b, ctx, torch):
    """Same migration with and without NTS_DETECT_RUNS: identical bytes from the pipelined path,
    the pool-to-pool kernel and the merged per-region baseline, and the baseline issues one copy
    per run and (layer, K|V) either way.  A zero-token plan has zero runs."""
    from gpu_util import device_pool, host_layers, make_plan, oracle_slots, slab_bytes, to_host
    rng = SplitMix64(77)
    ctx_len = np.array([300, 0, 17, 1, 260], np.int32)
    S = 1024
    case = PairCase(name="runs", shape=ModelShape(L=3, H=4, D=64, e=2), p=1, Ns=1, rs=0, Nd=1, rd=0,
                    S_src=S, S_dst=S, ctx_len=ctx_len,
                    src_pages=random_pages(rng, ctx_len, 1, S, "zipf_runs"),
                    dst_pages=random_pages(rng, ctx_len, 1, S, "contiguous"), seed_src=17, seed_dst=18)
    sh = case.shape
    src_h = host_layers(case, "src", range(sh.L))
    want = host_layers(case, "dst", range(sh.L)).copy()
    sslot, dslot = oracle_slots(case)
    orc.migrate_direct(src_h, want, sslot, dslot, 0, 0, 4)
    n_runs = len(orc.runs(sslot, dslot)) - 1
    src_d = device_pool(case, "src")
    sp = b.layer_ptrs(src_d.data_ptr(), sh.L, slab_bytes(case, "src"))
    st = torch.cuda.current_stream().cuda_stream
    for flags in (b.NTS_VALIDATE_UNIQUE_DST, b.NTS_VALIDATE_UNIQUE_DST | b.NTS_DETECT_RUNS):
        plan = make_plan(b, ctx, case, staging_bytes=1 << 16, flags=flags)
        try:
            info = b.nts_plan_info(plan)
            assert info.n_runs == (n_runs if flags & b.NTS_DETECT_RUNS else 0)
            staging = torch.empty(2 * info.chunk_bytes, dtype=torch.uint8, device="cuda")
            for which in ("migrate", "direct", "memcpy"):
                dst_d = device_pool(case, "dst")
                dp = b.layer_ptrs(dst_d.data_ptr(), sh.L, slab_bytes(case, "dst"))
                if which == "migrate":
                    b.nts_run_migrate(plan, sp, dp, staging.data_ptr(), st)
                elif which == "direct":
                    b.nts_run_migrate_direct(plan, sp, dp, st)
                else:
                    assert b.nts_run_memcpy_baseline(plan, sp, dp, True, st) == n_runs * sh.L * 2
                torch.cuda.synchronize()
                assert to_host(dst_d).tobytes() == want.tobytes(), (flags, which)
        finally:
            b.nts_plan_free(plan)
    empty = b.nts_plan_create(ctx, L=1, D=32, elem_bytes=2, page_size=1, Hs=2, Hd=2, src_head_off=0, dst_head_off=0,
                              w=2, S_src=8, S_dst=8, ctx_len=np.zeros(2, np.int32), src_pages=np.zeros(0, np.int32),
                              dst_pages=np.zeros(0, np.int32), flags=b.NTS_DETECT_RUNS)
    try:
        assert b.nts_plan_info(empty).n_runs == 0 and b.nts_plan_runs(empty).tolist() == [0]
    finally:
        b.nts_plan_free(empty)


def test_migrate_can_be_captured_in_a_hip_graph(b, ctx, torch):
    """run calls allocate nothing and never synchronise, so a caller may record
    them into a HIP graph: several replays, with eager work in between, all
    give the eager result."""
    from gpu_util import device_pool, make_plan, slab_bytes, to_host
    from workload import device as wdev
    case = make_case("c1")[0]
    sh = case.shape
    _, _, dst_h = _expected_full(case, sh.L, sh.D)
    src_d, dst_d = device_pool(case, "src"), device_pool(case, "dst")
    sp = b.layer_ptrs(src_d.data_ptr(), sh.L, slab_bytes(case, "src"))
    dp = b.layer_ptrs(dst_d.data_ptr(), sh.L, slab_bytes(case, "dst"))
    plan = make_plan(b, ctx, case, staging_bytes=1 << 20)
    try:
        info = b.nts_plan_info(plan)
        staging = torch.empty(2 * info.chunk_bytes, dtype=torch.uint8, device="cuda")

        def run():
            b.nts_run_migrate(plan, sp, dp, staging.data_ptr(), torch.cuda.current_stream().cuda_stream)

        run()
        torch.cuda.synchronize()
        assert to_host(dst_d).tobytes() == dst_h.tobytes()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            run()
        for _ in range(3):
            wdev.fill_tensor(dst_d, case.seed_dst)          # eager work between replays
            staging.fill_(0x5A)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert to_host(dst_d).tobytes() == dst_h.tobytes()
        del graph
    finally:
        b.nts_plan_free(plan)


def test_one_plan_on_many_streams_then_freed(b, ctx, torch):
    """A plan remembers the streams it has work on so that freeing it is ordered behind that
    work; with more streams than its fixed record holds the free waits for the device.  Ten
    streams in turn, the last run left unsynchronised before the free, a new plan right after."""
    from gpu_util import device_pool, make_plan, slab_bytes, to_host
    from workload import device as wdev
    case = make_case("c1")[0]
    sh = case.shape
    _, _, dst_h = _expected_full(case, sh.L, sh.D)
    src_d, dst_d = device_pool(case, "src"), device_pool(case, "dst")
    sp = b.layer_ptrs(src_d.data_ptr(), sh.L, slab_bytes(case, "src"))
    dp = b.layer_ptrs(dst_d.data_ptr(), sh.L, slab_bytes(case, "dst"))
    streams = [torch.cuda.Stream() for _ in range(10)]
    plan = make_plan(b, ctx, case, staging_bytes=1 << 20)
    info = b.nts_plan_info(plan)
    staging = torch.empty(2 * info.chunk_bytes, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    try:
        for i, s in enumerate(streams):
            b.nts_run_migrate(plan, sp, dp, staging.data_ptr(), s.cuda_stream)
            if i + 1 < len(streams):
                s.synchronize()
                assert to_host(dst_d).tobytes() == dst_h.tobytes()
                wdev.fill_tensor(dst_d, case.seed_dst)
                torch.cuda.synchronize()
    finally:
        b.nts_plan_free(plan)
    other = make_plan(b, ctx, case, staging_bytes=1 << 20)   # may take over the freed plan's block
    try:
        torch.cuda.synchronize()
        assert to_host(dst_d).tobytes() == dst_h.tobytes()
    finally:
        b.nts_plan_free(other)
