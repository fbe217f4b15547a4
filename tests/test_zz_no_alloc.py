"""nts_run_migrate_static: the allocation-free variant of nts_run_migrate whose
two staging buffers live in a static device array.  Its destination pool must
equal, bit for bit, what nts_run_migrate writes with a caller-provided staging
area (and what the oracle computes), on two calls in a row, the second with a
smaller input."""
import numpy as np
import pytest

from oracle import kvmig as orc
from workload import make_case

pytestmark = pytest.mark.gpu


def _pools(b, case):
    from gpu_util import device_pool, slab_bytes
    sh = case.shape
    src_d, dst_a, dst_b = device_pool(case, "src"), device_pool(case, "dst"), device_pool(case, "dst")
    tab = lambda t, side: b.layer_ptrs(t.data_ptr(), sh.L, slab_bytes(case, side))
    return src_d, dst_a, dst_b, tab(src_d, "src"), tab(dst_a, "dst"), tab(dst_b, "dst")


def test_static_staging_matches_caller_staging_twice_second_smaller():
    import torch
    from gpu_util import host_layers, make_plan, oracle_slots
    from paper_2605_05467_amd import binding as b
    ctx = b.nts_init(0)
    st = torch.cuda.current_stream().cuda_stream
    try:
        # first 4096 tokens through 2 x 16 MiB (the largest the static area takes), then 700 tokens through 2 x 1 MiB
        for tokens, staging_bytes in ((4096, b.NTS_STATIC_STAGING_BYTES // 2), (700, 1 << 20)):
            case = make_case("c3", tokens=tokens)[0]
            sh = case.shape
            src_d, dst_a, dst_b, sp, dpa, dpb = _pools(b, case)
            plan = make_plan(b, ctx, case, staging_bytes=staging_bytes)
            try:
                info = b.nts_plan_info(plan)
                assert 2 * info.chunk_bytes <= b.NTS_STATIC_STAGING_BYTES and info.n_chunks >= 4
                staging = torch.empty(2 * info.chunk_bytes, dtype=torch.uint8, device="cuda")
                b.nts_run_migrate_static(plan, sp, dpa, st)
                b.nts_run_migrate(plan, sp, dpb, staging.data_ptr(), st)
                torch.cuda.synchronize()
                assert torch.equal(dst_a, dst_b), tokens
                # and both equal the oracle on a few whole layers
                es, ed = oracle_slots(case)
                so, do, w = orc.route(sh.H, case.Ns, case.rs, case.Nd, case.rd)
                layer_bytes = 2 * case.S_dst * case.Hd * sh.D * sh.e
                for l in (0, sh.L - 1):
                    want = host_layers(case, "dst", [l]).copy()
                    orc.migrate(host_layers(case, "src", [l]), want, es, ed, so, do, w)
                    assert dst_a[l * layer_bytes:(l + 1) * layer_bytes].cpu().numpy().tobytes() == want.tobytes()
            finally:
                b.nts_plan_free(plan)
            del src_d, dst_a, dst_b, staging
    finally:
        b.nts_free(ctx)


def test_static_staging_rejects_plans_that_do_not_fit():
    import torch
    from gpu_util import make_plan
    from paper_2605_05467_amd import binding as b
    ctx = b.nts_init(0)
    try:
        case = make_case("c3", tokens=2048)[0]
        src_d, dst_a, dst_b, sp, dpa, dpb = _pools(b, case)
        plan = make_plan(b, ctx, case, staging_bytes=b.NTS_STATIC_STAGING_BYTES // 2 + 4096)
        try:
            before = dst_a.clone()
            with pytest.raises(b.NtsError) as ei:
                b.nts_run_migrate_static(plan, sp, dpa, torch.cuda.current_stream().cuda_stream)
            assert ei.value.status == b.NTS_EINVAL
            assert "NTS_STATIC_STAGING_BYTES" in b.nts_last_error(ctx)
            torch.cuda.synchronize()
            assert torch.equal(dst_a, before)
        finally:
            b.nts_plan_free(plan)
        with pytest.raises(b.NtsError):
            b.nts_run_migrate_static(0, sp, dpa, 0)
        # a plan with nothing to move is a no-op whatever its (default, 64 MiB) chunk geometry
        empty = b.nts_plan_create(ctx, L=1, D=32, elem_bytes=2, page_size=1, Hs=2, Hd=2, src_head_off=0, dst_head_off=0,
                                  w=2, S_src=8, S_dst=8, ctx_len=np.zeros(2, np.int32), src_pages=np.zeros(0, np.int32),
                                  dst_pages=np.zeros(0, np.int32))
        try:
            b.nts_run_migrate_static(empty, sp, dpa, 0)
        finally:
            b.nts_plan_free(empty)
    finally:
        b.nts_free(ctx)
