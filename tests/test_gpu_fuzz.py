"""Seeded random geometries: every case draws a model shape, page size, TP pair,
request mix, pool sizes, row padding and staging size (every other case also asks
for run detection, every third for the destination ranking: pack and unpack must
keep the caller's token order all the same), runs pack, the pipelined
migration and the pool-to-pool kernel through the C ABI and compares whole
outputs with the oracle, bit for bit."""
import numpy as np
import pytest

from gpu_util import draw_case, random_case_host, random_case_plan_args
from oracle import kvmig as orc

pytestmark = pytest.mark.gpu
N_CASES = 64


@pytest.fixture(scope="module")
def env():
    import torch
    from paper_2605_05467_amd import binding as b
    ctx = b.nts_init(0)
    yield torch, b, ctx
    b.nts_free(ctx)


@pytest.mark.parametrize("seed", range(N_CASES))
def test_random_geometry(env, seed):
    run_drawn_case(env, draw_case(seed), seed)


@pytest.mark.parametrize("seed", range(10))
def test_random_geometry_at_a_few_thousand_tokens(env, seed):
    """Drawn geometries at sizes where a launch has thousands of workgroups: fragments of 256 B to
    2 KiB (several per wavefront), odd token counts, chunks of 1 to 64 MiB."""
    from gpu_util import draw_mid_case
    run_drawn_case(env, draw_mid_case(seed), seed)


def run_drawn_case(env, c, seed):
    torch, b, ctx = env
    h = random_case_host(c, b.nts_route(c["H"], c["Ns"], c["rs"], c["Nd"], c["rd"]))
    L, st_d, row_d, S_d = h["L"], h["st_d"], h["row_d"], h["S_d"]
    src_arr, dst_arr, sslot, dslot, stream_h, want = (h[k] for k in ("src_arr", "dst_arr", "sslot", "dslot",
                                                                      "stream", "want"))
    src_d = [torch.from_numpy(a).cuda() for a in src_arr]
    kw = random_case_plan_args(b, c, h)
    if seed % 2:
        kw["flags"] |= b.NTS_DETECT_RUNS
    if seed % 3 == 0:                     # every third case moves its tokens in destination order where it may
        kw["flags"] |= b.NTS_ORDER_BY_DST
    plan = b.nts_plan_create(ctx, **kw)
    try:
        info = b.nts_plan_info(plan)
        s, d = b.nts_plan_slots(plan)
        assert np.array_equal(s, sslot) and np.array_equal(d, dslot)
        if seed % 2:
            assert np.array_equal(b.nts_plan_runs(plan), orc.runs(sslot, dslot))
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
