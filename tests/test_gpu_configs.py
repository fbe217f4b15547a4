"""GPU parity at the benchmark configurations, in the launch configuration
bench.py times (route + plan + double-buffered migrate, 64 MiB staging).

Every configuration is compared whole: all bytes of the destination pool,
untouched ones included, against the oracle.  Configuration 2 holds both pools
on the host at once; the larger ones (3, its companions, 4, and the two 92 GiB
pools of 5) go layer by layer through a thread pool (layers are independent in
the oracle's loops; each job regenerates its layer of both pools from the
stateless fill, runs the oracle and compares that layer of the GPU's pool), so
host memory stays at a few layers.  Before that, as fast pre-checks: randomly
sampled single elements the oracle locates one by one, with the value taken
from the stateless fill's closed form, and two properties that hold at any
size (the source pool is unchanged; exactly payload-many words of the
destination differ from its sentinel fill).
"""
import numpy as np
import pytest

from oracle import kvmig as orc
from workload import SplitMix64, fill_words, make_case

pytestmark = pytest.mark.gpu
STAGING = 64 << 20


@pytest.fixture(scope="module")
def env():
    import torch
    from paper_2605_05467_amd import binding as b
    from workload import device as wdev
    ctx = b.nts_init(0)
    staging = torch.empty(2 * STAGING, dtype=torch.uint8, device="cuda")
    yield torch, b, wdev, ctx, staging
    del staging
    torch.cuda.empty_cache()
    b.nts_free(ctx)


def migrate_on_gpu(env, case, src_d=None):
    from gpu_util import device_pool, make_plan, slab_bytes
    torch, b, wdev, ctx, staging = env
    sh = case.shape
    if src_d is None:
        src_d = device_pool(case, "src")
    dst_d = device_pool(case, "dst")
    sp = b.layer_ptrs(src_d.data_ptr(), sh.L, slab_bytes(case, "src"))
    dp = b.layer_ptrs(dst_d.data_ptr(), sh.L, slab_bytes(case, "dst"))
    # bench.py's plan flags: validated destination slots, tokens moved in destination order
    plan = make_plan(b, ctx, case, staging_bytes=STAGING, flags=b.NTS_VALIDATE_UNIQUE_DST | b.NTS_ORDER_BY_DST)
    try:
        info = b.nts_plan_info(plan)
        s, d = b.nts_plan_slots(plan)
        b.nts_run_migrate(plan, sp, dp, staging.data_ptr(), torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
    finally:
        b.nts_plan_free(plan)
    return src_d, dst_d, info, s, d


def check_properties(env, case, src_d, dst_d, info):
    torch, b, wdev, ctx, _ = env
    assert wdev.count_mismatch(src_d, case.seed_src) == 0, "source pool changed"
    changed = wdev.count_mismatch(dst_d, case.seed_dst)
    assert changed == info.X // 8, (changed, info.X // 8)


def _fill_elem(seed, lin):
    word = int(fill_words(seed, lin // 4, 1)[0])
    return (word >> (16 * (lin % 4))) & 0xFFFF


def check_samples(env, case, dst_d, sslot, dslot, n=400, seed=99):
    torch = env[0]
    sh = case.shape
    assert sh.e == 2
    so, do, w = orc.route(sh.H, case.Ns, case.rs, case.Nd, case.rd)
    rng = SplitMix64(seed)
    j_of = {int(s): j for j, s in enumerate(dslot)}
    used = np.zeros(case.S_dst, bool)
    used[dslot] = True
    free = np.nonzero(~used)[0]
    coords = []
    for k in range(n):
        l = int(rng.integers(0, sh.L - 1, 1)[0])
        c = int(rng.integers(0, 1, 1)[0])
        if k % 3 != 2 or len(free) == 0:
            slot = int(dslot[int(rng.integers(0, len(dslot) - 1, 1)[0])])
        else:
            slot = int(free[int(rng.integers(0, len(free) - 1, 1)[0])])
        h = int(rng.integers(0, case.Hd - 1, 1)[0])
        x = int(rng.integers(0, sh.D - 1, 1)[0])
        coords.append((l, c, slot, h, x))
    lin_dst = np.array([((((l * 2 + c) * case.S_dst + s) * case.Hd + h) * sh.D + x) for l, c, s, h, x in coords], np.int64)
    got = dst_d.view(torch.int16)[torch.from_numpy(lin_dst).cuda()].cpu().numpy().view(np.uint16)
    for k, (l, c, slot, h, x) in enumerate(coords):
        srcpos = orc.migrated_element_source(j_of, sslot, slot, h, so, do, w)
        if srcpos is None:
            want = _fill_elem(case.seed_dst, int(lin_dst[k]))
        else:
            s_slot, s_head = srcpos
            want = _fill_elem(case.seed_src, (((l * 2 + c) * case.S_src + s_slot) * case.Hs + s_head) * sh.D + x)
        assert int(got[k]) == want, (case.name, coords[k])


def test_config2_whole_outputs(env):
    from gpu_util import compare_every_layer, oracle_slots
    for case in make_case("c2"):
        print(f"  {case.name}", flush=True)
        sh = case.shape
        src_d, dst_d, info, s, d = migrate_on_gpu(env, case)
        es, ed = oracle_slots(case)
        assert np.array_equal(s, es) and np.array_equal(d, ed)
        assert info.F == case.T * sh.L * 2
        check_properties(env, case, src_d, dst_d, info)
        compare_every_layer(case, dst_d, es, ed)
        del src_d, dst_d


@pytest.mark.parametrize("staging_bytes", [(20 << 20) + 3 * 2048, (9 << 20) + 1024])
def test_config2_chunks_that_end_inside_a_workgroup_group(env, staging_bytes):
    """The stage kernel hands its workgroups out in aligned groups of 8192 (8 MiB of stream) and
    leaves the ragged end of a job in plain order: chunks of 20 MiB + 3 fragments (two groups and a
    tail) and of 9 MiB + 1 KiB (one group and a tail), with and without the destination ranking."""
    from gpu_util import compare_every_layer, device_pool, make_plan, oracle_slots, slab_bytes
    torch, b, wdev, ctx, staging = env
    for case in make_case("c2"):
        sh = case.shape
        es, ed = oracle_slots(case)
        src_d = device_pool(case, "src")
        sp = b.layer_ptrs(src_d.data_ptr(), sh.L, slab_bytes(case, "src"))
        for flags in (b.NTS_VALIDATE_UNIQUE_DST, b.NTS_VALIDATE_UNIQUE_DST | b.NTS_ORDER_BY_DST):
            print(f"  {case.name} staging {staging_bytes} flags {flags}", flush=True)
            dst_d = device_pool(case, "dst")
            dp = b.layer_ptrs(dst_d.data_ptr(), sh.L, slab_bytes(case, "dst"))
            plan = make_plan(b, ctx, case, staging_bytes=staging_bytes, flags=flags)
            try:
                info = b.nts_plan_info(plan)
                assert info.chunk_bytes // 1024 > 8192 and (info.chunk_bytes // 1024) % 8192 != 0
                assert 2 * info.chunk_bytes <= staging.numel()
                b.nts_run_migrate(plan, sp, dp, staging.data_ptr(), torch.cuda.current_stream().cuda_stream)
                torch.cuda.synchronize()
            finally:
                b.nts_plan_free(plan)
            check_properties(env, case, src_d, dst_d, info)
            compare_every_layer(case, dst_d, es, ed)
            del dst_d
        del src_d


def test_config2_chunk_calls_at_size(env):
    """Chunk-by-chunk pack -> unpack through two buffers (the calls a sender and a receiver would
    use) at 1e6 fragments, with chunks that end inside a group of the kernels' workgroup mapping;
    every byte of the destination pool against the oracle."""
    from gpu_util import compare_every_layer, device_pool, make_plan, oracle_slots, slab_bytes
    torch, b, wdev, ctx, staging = env
    st = torch.cuda.current_stream().cuda_stream
    for case in make_case("c2"):
        sh = case.shape
        es, ed = oracle_slots(case)
        src_d, dst_d = device_pool(case, "src"), device_pool(case, "dst")
        sp = b.layer_ptrs(src_d.data_ptr(), sh.L, slab_bytes(case, "src"))
        dp = b.layer_ptrs(dst_d.data_ptr(), sh.L, slab_bytes(case, "dst"))
        plan = make_plan(b, ctx, case, staging_bytes=(18 << 20) + 5 * 1024)
        try:
            info = b.nts_plan_info(plan)
            assert (info.chunk_bytes // 1024) % 8192 != 0 and 2 * info.chunk_bytes <= staging.numel()
            print(f"  {case.name}: {info.n_chunks} chunks of {info.chunk_bytes} bytes", flush=True)
            for k in range(info.n_chunks):
                p_ = staging.data_ptr() + (k & 1) * info.chunk_bytes
                b.nts_run_pack_chunk(plan, sp, k, p_, st)
                b.nts_run_unpack_chunk(plan, p_, k, dp, st)
            torch.cuda.synchronize()
        finally:
            b.nts_plan_free(plan)
        check_properties(env, case, src_d, dst_d, info)
        compare_every_layer(case, dst_d, es, ed)
        del src_d, dst_d


@pytest.mark.parametrize("name", ["c3", "c3b", "c3c", "c3d"])
def test_config3_headline_and_companions(env, name):
    from gpu_util import compare_every_layer, oracle_slots
    for case in make_case(name):
        src_d, dst_d, info, s, d = migrate_on_gpu(env, case)
        es, ed = oracle_slots(case)
        assert np.array_equal(s, es) and np.array_equal(d, ed)
        if name == "c3":
            assert info.X == 5 * 2 ** 30 and info.F == 2621440 and info.n_chunks == 80
        if name == "c3b":
            assert info.X == 2 ** 29
        check_properties(env, case, src_d, dst_d, info)
        check_samples(env, case, dst_d, es, ed)
        compare_every_layer(case, dst_d, es, ed)
        # the pool-to-pool kernel on the same pools, in token order and in destination order
        from gpu_util import make_plan, slab_bytes
        torch, b, wdev, ctx, _ = env
        sh = case.shape
        sp = b.layer_ptrs(src_d.data_ptr(), sh.L, slab_bytes(case, "src"))
        dp = b.layer_ptrs(dst_d.data_ptr(), sh.L, slab_bytes(case, "dst"))
        for flags in (b.NTS_VALIDATE_UNIQUE_DST, b.NTS_VALIDATE_UNIQUE_DST | b.NTS_ORDER_BY_DST):
            wdev.fill_tensor(dst_d, case.seed_dst)
            plan = make_plan(b, ctx, case, staging_bytes=STAGING, flags=flags)
            try:
                b.nts_run_migrate_direct(plan, sp, dp, torch.cuda.current_stream().cuda_stream)
                torch.cuda.synchronize()
            finally:
                b.nts_plan_free(plan)
            compare_every_layer(case, dst_d, es, ed, label=f"{case.name} pool-to-pool flags={flags}", direct=True)
        del src_d, dst_d


def test_config4_skewed_four_destinations(env):
    from gpu_util import compare_every_layer, oracle_slots
    cases = make_case("c4")
    src_d = None
    total_F = 0
    for case in cases:
        src_d, dst_d, info, s, d = migrate_on_gpu(env, case, src_d)
        es, ed = oracle_slots(case)
        assert np.array_equal(s, es) and np.array_equal(d, ed)
        total_F += info.F
        check_properties(env, case, src_d, dst_d, info)
        check_samples(env, case, dst_d, es, ed, n=200)
        compare_every_layer(case, dst_d, es, ed)
        del dst_d
    assert total_F == 2621440


def test_config4_as_one_batch_call(env):
    """Configuration 4 the way bench.py runs a workload of several pairs: all four plans made first, then one
    nts_run_migrate_batch through the two staging buffers; every byte of the four destination pools against
    the oracle."""
    from gpu_util import compare_every_layer, device_pool, make_plan, oracle_slots, slab_bytes
    torch, b, wdev, ctx, staging = env
    cases = make_case("c4")
    sh = cases[0].shape
    src_d = device_pool(cases[0], "src")
    sp = b.layer_ptrs(src_d.data_ptr(), sh.L, slab_bytes(cases[0], "src"))
    dsts = [device_pool(c, "dst") for c in cases]
    dps = [b.layer_ptrs(d.data_ptr(), sh.L, slab_bytes(c, "dst")) for c, d in zip(cases, dsts)]
    plans = [make_plan(b, ctx, c, staging_bytes=STAGING, flags=b.NTS_VALIDATE_UNIQUE_DST | b.NTS_ORDER_BY_DST)
             for c in cases]
    try:
        b.nts_run_migrate_batch(plans, [sp] * len(cases), dps, staging.data_ptr(),
                                torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
    finally:
        for p in plans:
            b.nts_plan_free(p)
    assert wdev.count_mismatch(src_d, cases[0].seed_src) == 0, "source pool changed"
    for c, d in zip(cases, dsts):
        es, ed = oracle_slots(c)
        compare_every_layer(c, d, es, ed, label=f"c4 batch, destination rank {c.rd}")
    del src_d, dsts


@pytest.mark.parametrize("ranked", [False, True])
def test_whole_stream_pack_and_unpack_beyond_one_launch(env, ranked):
    """nts_run_pack and nts_run_unpack on a 33 GiB stream (config 5's recipe at 270,336 tokens): more
    than 2^31 lanes, so each call takes two launches; the stream keeps the caller's token order
    whether or not the plan is ranked.  Every byte of the destination pool against the oracle."""
    from gpu_util import compare_every_layer, device_pool, make_plan, oracle_slots, slab_bytes
    torch, b, wdev, ctx, _ = env
    case = make_case("c5", tokens=270336)[0]
    sh = case.shape
    free, total = torch.cuda.mem_get_info()
    need = case.pool_bytes("src") + case.pool_bytes("dst") + case.T * sh.L * 2 * sh.H * sh.D * sh.e + (1 << 30)
    if free < need:
        pytest.skip(f"needs {need >> 30} GiB of free HBM, {free >> 30} GiB available")
    es, ed = oracle_slots(case)
    src_d, dst_d = device_pool(case, "src"), device_pool(case, "dst")
    sp = b.layer_ptrs(src_d.data_ptr(), sh.L, slab_bytes(case, "src"))
    dp = b.layer_ptrs(dst_d.data_ptr(), sh.L, slab_bytes(case, "dst"))
    flags = b.NTS_VALIDATE_UNIQUE_DST | (b.NTS_ORDER_BY_DST if ranked else 0)
    plan = make_plan(b, ctx, case, staging_bytes=STAGING, flags=flags)
    try:
        info = b.nts_plan_info(plan)
        assert info.X > 32 << 30                       # 16-byte lanes: more than 2^31 of them
        stream = torch.empty(info.X, dtype=torch.uint8, device="cuda")
        st = torch.cuda.current_stream().cuda_stream
        b.nts_run_pack(plan, sp, stream.data_ptr(), st)
        b.nts_run_unpack(plan, stream.data_ptr(), dp, st)
        torch.cuda.synchronize()
    finally:
        b.nts_plan_free(plan)
    del stream
    check_properties(env, case, src_d, dst_d, info)
    compare_every_layer(case, dst_d, es, ed, label=f"33 GiB stream, ranked={ranked}")
    del src_d, dst_d
    torch.cuda.empty_cache()


def test_config5_roofline_size(env):
    """Two 92 GiB pools, 88 GiB payload: every byte of the destination pool
    against the oracle, layer by layer, for the double-buffered pipeline and for
    the pool-to-pool kernel; sampled elements and the any-size properties first."""
    from gpu_util import compare_every_layer, oracle_slots
    torch = env[0]
    free, total = torch.cuda.mem_get_info()
    case = make_case("c5")[0]
    need = case.pool_bytes("src") + case.pool_bytes("dst") + (1 << 30)
    if free < need:
        pytest.skip(f"needs {need >> 30} GiB of free HBM, {free >> 30} GiB available")
    src_d, dst_d, info, s, d = migrate_on_gpu(env, case)
    es, ed = oracle_slots(case)
    assert np.array_equal(s, es) and np.array_equal(d, ed)
    assert info.F == 46137344 and info.X == 88 * 2 ** 30
    check_properties(env, case, src_d, dst_d, info)
    check_samples(env, case, dst_d, es, ed, n=600)
    compare_every_layer(case, dst_d, es, ed, label="c5 pipeline", direct=True)
    # the pool-to-pool kernel at this size needs three launches (fewer than 2^31 lanes each)
    from gpu_util import slab_bytes
    from workload import device as wdev
    b, ctx = env[1], env[3]
    wdev.fill_tensor(dst_d, case.seed_dst)
    sh = case.shape
    sp = b.layer_ptrs(src_d.data_ptr(), sh.L, slab_bytes(case, "src"))
    dp = b.layer_ptrs(dst_d.data_ptr(), sh.L, slab_bytes(case, "dst"))
    from gpu_util import make_plan
    # ... walking the tokens in ascending destination-slot order (the flag changes no result)
    plan = make_plan(b, ctx, case, staging_bytes=STAGING, flags=b.NTS_VALIDATE_UNIQUE_DST | b.NTS_ORDER_BY_DST)
    try:
        b.nts_run_migrate_direct(plan, sp, dp, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        check_properties(env, case, src_d, dst_d, info)
        check_samples(env, case, dst_d, es, ed, n=600, seed=7)
        compare_every_layer(case, dst_d, es, ed, label="c5 pool-to-pool", direct=True)
        # one chunk of the stream, far into it, against the oracle's pack of that layer
        k = info.n_chunks - 3
        buf = torch.empty(info.chunk_bytes, dtype=torch.uint8, device="cuda")
        b.nts_run_pack_chunk(plan, sp, k, buf.data_ptr(), torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        q0 = k * info.chunk_frags
        lc, j0 = divmod(q0, info.T)
        assert j0 + info.chunk_frags <= info.T            # the chunk lies inside one (layer, K|V) slab
        from gpu_util import host_layers
        so, do, w = orc.route(sh.H, case.Ns, case.rs, case.Nd, case.rd)
        src_l = host_layers(case, "src", [lc // 2])
        want = orc.pack(src_l, es[j0:j0 + info.chunk_frags], so, w)[0, lc % 2]
        assert buf.cpu().numpy().tobytes() == want.tobytes()
    finally:
        b.nts_plan_free(plan)
    del src_d, dst_d
    torch.cuda.empty_cache()


@pytest.mark.parametrize("variant", ["p16", "fp8", "70b"])
def test_other_kv_geometries_at_size(env, variant):
    """16-token pages, 1-byte elements and an 80-layer model at 8192 tokens."""
    from gpu_util import compare_every_layer, oracle_slots
    from workload import M8B, ModelShape
    if variant == "p16":
        case = make_case("c3", shape=M8B, p=16, tokens=8192)[0]
    elif variant == "fp8":
        case = make_case("c3", shape=ModelShape(L=32, H=8, D=128, e=1), tokens=8192)[0]
    else:
        case = make_case("c3", shape=ModelShape(L=80, H=8, D=128, e=2), tokens=8192)[0]
    src_d, dst_d, info, s, d = migrate_on_gpu(env, case)
    es, ed = oracle_slots(case)
    assert np.array_equal(s, es) and np.array_equal(d, ed)
    check_properties(env, case, src_d, dst_d, info)
    compare_every_layer(case, dst_d, es, ed)
    if case.shape.e == 2:
        check_samples(env, case, dst_d, es, ed, n=200)


def test_back_to_back_pairs_without_synchronising(env):
    """Plans of different sizes created, run and freed back to back with no
    synchronisation in between (what bench.py does for configuration 4): a freed
    plan's device block is recycled by the next plan only after the kernels
    that still read it have finished."""
    from gpu_util import compare_every_layer, device_pool, make_plan, oracle_slots, slab_bytes
    torch, b, wdev, ctx, staging = env
    cases = make_case("c4", tokens=8192)
    assert len({c.T for c in cases}) > 1
    sh = cases[0].shape
    src_d = device_pool(cases[0], "src")
    sp = b.layer_ptrs(src_d.data_ptr(), sh.L, slab_bytes(cases[0], "src"))
    dsts = [device_pool(c, "dst") for c in cases]
    stream = torch.cuda.current_stream().cuda_stream
    infos = []
    for _ in range(3):
        infos = []
        for case, dst_d in zip(cases, dsts):
            plan = make_plan(b, ctx, case, staging_bytes=STAGING)
            infos.append(b.nts_plan_info(plan))
            b.nts_run_migrate(plan, sp, b.layer_ptrs(dst_d.data_ptr(), sh.L, slab_bytes(case, "dst")),
                              staging.data_ptr(), stream)
            b.nts_plan_free(plan)
    torch.cuda.synchronize()
    for case, dst_d, info in zip(cases, dsts, infos):
        es, ed = oracle_slots(case)
        check_properties(env, case, src_d, dst_d, info)
        compare_every_layer(case, dst_d, es, ed)
        check_samples(env, case, dst_d, es, ed, n=100)
