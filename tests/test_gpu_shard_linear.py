"""GPU parity of the TP-shard-selecting linear layer against its fp64 oracle.

Random inputs: two tolerances, both from oracle.shard_linear.  `tolerance` is
the worst-case bound (fp32 accumulation of K products in any order plus one
rounding); it grows with K and no longer notices a dropped product from
K = 4096 on.  `tight_tolerance` is half an output ulp plus the error fp32
accumulation typically makes (random-walk model, eight-fold margin); a dropped
or doubled product exceeds it at every K.  Every element must be inside both.

Integer inputs (|x|, |w| <= 8, exact in bf16 / fp16): every product and every
fp32 partial sum is exact whatever the order, so the result must equal the
oracle's fp64 result rounded once to nearest even, bit for bit."""
import numpy as np
import pytest

from linear_cases import CASES
from oracle import shard_linear as osl
from workload.linear import LAYERS, linear_inputs, linear_inputs_int

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    from paper_2605_05467_amd import binding as b
    ctx = b.nts_init(0)
    yield torch, b, ctx
    b.nts_free(ctx)


def run_case(env, M, n_out, n_in, tp, rank, split, seed=1, pad=0, dtype="bf16", pad_y=None, exact=False):
    """exact=False: random real inputs, result inside both tolerances.
    exact=True: integer inputs, result bit-identical to the once-rounded oracle."""
    torch, b, ctx = env
    k = n_in if split == "out" else n_in // tp
    nn = n_out // tp if split == "out" else n_out
    Xh, Wh = (linear_inputs_int if exact else linear_inputs)(seed, M, n_out, n_in, x_cols=k, dtype=dtype)
    decode = osl.bf16_to_f64 if dtype == "bf16" else osl.f16_to_f64
    ldx, ldw, ldy = k + pad, n_in + pad, nn + (pad if pad_y is None else pad_y)
    Xp = np.zeros((M, ldx), np.uint16); Xp[:, :k] = Xh
    Wp = np.zeros((n_out, ldw), np.uint16); Wp[:, :n_in] = Wh
    Xd = torch.from_numpy(Xp.view(np.int16)).cuda()
    Wd = torch.from_numpy(Wp.view(np.int16)).cuda()
    Yd = torch.full((M, ldy), 12345, dtype=torch.int16, device="cuda")
    sp = b.NTS_SPLIT_OUT if split == "out" else b.NTS_SPLIT_IN
    kw = dict(M=M, n_out=n_out, n_in=n_in, tp=tp, rank=rank, split=sp, ldx=ldx, ldw=ldw, ldy=ldy,
              dtype=b.NTS_BF16 if dtype == "bf16" else b.NTS_F16)
    ws_bytes = b.nts_shard_linear_workspace(**kw)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")
    b.nts_shard_linear(ctx, Xd.data_ptr(), Wd.data_ptr(), Yd.data_ptr(), workspace=ws.data_ptr(),
                       workspace_bytes=ws_bytes, hip_stream=torch.cuda.current_stream().cuda_stream, **kw)
    torch.cuda.synchronize()
    Yg = Yd.cpu().numpy().view(np.uint16)
    X64, W64 = decode(Xh), decode(Wh)
    want, bound = osl.shard_linear(X64, W64, tp, rank, split)
    if ldy > nn:
        assert np.all(Yg[:, nn:] == 12345)                     # nothing written past the output width
    if exact:
        assert k * 64 < 2 ** 24                                 # every partial sum is an exact fp32 integer
        want_bits = osl.round_to_bits(want, dtype)
        same = Yg[:, :nn] == want_bits
        assert same.all(), (int((~same).sum()), np.argwhere(~same)[:4].tolist())
        return 0.0
    got = decode(Yg[:, :nn])
    tol = osl.tolerance(want, bound, k, out_bits=8 if dtype == "bf16" else 11)
    tight = osl.tight_tolerance(want, osl.product_norm(X64, W64, tp, rank, split), k, dtype)
    err = np.abs(got - want)
    assert np.all(err <= tol), (float((err / tol).max()), np.unravel_index(np.argmax(err / tol), err.shape))
    assert np.all(err <= tight), (float((err / tight).max()), np.unravel_index(np.argmax(err / tight), err.shape))
    return float((err / tight).max())


@pytest.mark.parametrize("M", [1, 7, 16, 33, 64])
@pytest.mark.parametrize("split", ["out", "in"])
def test_small_batches_ragged_shapes(env, M, split):
    run_case(env, M, 96, 512, 2, 1, split, seed=M)
    run_case(env, M, 208, 1024 + 64, 1, 0, split, seed=M + 100, pad=8)
    run_case(env, M, 96, 4096, 4, 3, split, seed=M + 200)


@pytest.mark.parametrize("layer", sorted(LAYERS))
def test_decoder_layer_shapes_decode_batch(env, layer):
    n_out, n_in, split = LAYERS[layer]
    run_case(env, 8, n_out, n_in, 4, 2, split, seed=5)


def test_argument_errors(env):
    torch, b, ctx = env
    z = torch.zeros(64 * 64, dtype=torch.int16, device="cuda")
    ok = dict(M=4, n_out=64, n_in=64, tp=1, rank=0, split=b.NTS_SPLIT_OUT)

    def status(**over):
        try:
            b.nts_shard_linear(ctx, z.data_ptr(), z.data_ptr(), z.data_ptr(), **{**ok, **over})
        except b.NtsError as e:
            return e.status
        return 0

    assert status() == 0
    assert status(tp=3) == b.NTS_EINVAL
    assert status(rank=1) == b.NTS_EINVAL
    assert status(n_in=72) == b.NTS_EINVAL            # reduction length not a multiple of 64
    assert status(split=7) == b.NTS_EINVAL
    assert status(ldw=60) == b.NTS_EINVAL
    assert status(ldw=1 << 23) == b.NTS_EINVAL          # row strides stay below 2^23 elements
    assert status(M=0) == b.NTS_EINVAL
    torch.cuda.synchronize()


@pytest.mark.parametrize("M", [65, 96, 130, 192, 200, 256, 300, 777])
@pytest.mark.parametrize("split", ["out", "in"])
def test_large_batches_tile_edges(env, M, split):
    """Wide batches on small shards: several batch tiles per weight block, K
    splits, ragged edges in both output dimensions."""
    run_case(env, M, 96, 512, 2, 1, split, seed=M)
    run_case(env, M, 528, 1024 + 64, 1, 0, split, seed=M + 100, pad=8)
    run_case(env, M, 1024, 2048, 4, 3, split, seed=M + 200)


@pytest.mark.parametrize("case", CASES, ids=lambda c: "M%d_N%d_K%d_%s%dx%d%s_kw%d" % (c[:3] + ("tiled" if c[7] else "tile",) + c[3:5] + ("_split" if c[5] else "", c[6])))
@pytest.mark.parametrize("split", ["out", "in"])
def test_every_kernel_variant(env, case, split):
    """One shard shape per instantiated kernel variant (tile height x workgroup
    width, with and without a K split, one and several batch tiles; the decode
    kernel's row blocks x wavefronts per K range), selected at
    TP level 2 from a full matrix twice the shard, as rank 1; the variant each
    shape reaches is pinned by the CPU suite."""
    torch, b, ctx = env
    M, Nn, K, rows, cols, is_split, k_waves, tiled = case
    n_out, n_in = (2 * Nn, K) if split == "out" else (Nn, 2 * K)
    sp = b.NTS_SPLIT_OUT if split == "out" else b.NTS_SPLIT_IN
    pad = 8 if M % 2 else 0
    l = b.nts_shard_linear_launch(M=M, n_out=n_out, n_in=n_in, tp=2, rank=1, split=sp, ldx=K + pad,
                                  ldw=n_in + pad, ldy=Nn + pad)
    assert (l.tile_rows, l.tile_cols, l.k_splits > 1, l.k_waves, bool(l.tiled)) == (rows, cols, is_split, k_waves, tiled)
    run_case(env, M, n_out, n_in, 2, 1, split, seed=M + Nn, pad=pad,
             dtype="f16" if (M + Nn // 8) % 3 == 0 else "bf16")
    # and bit-exact on integer inputs, in both element formats
    run_case(env, M, n_out, n_in, 2, 1, split, seed=M + Nn + 1, pad=pad, dtype="bf16", exact=True)
    run_case(env, M, n_out, n_in, 2, 1, split, seed=M + Nn + 2, pad=pad, dtype="f16", exact=True)


@pytest.mark.parametrize("M", [520, 777])
@pytest.mark.parametrize("split", ["out", "in"])
def test_tiled_kernel_ragged_edges(env, M, split):
    """Outputs of this size go to the tiled matrix-core kernel (in whichever tile
    shape the library picks for them): ragged edges in both output dimensions,
    both element formats."""
    tp = 2
    n_out, n_in = (2 * 19000, 256) if split == "out" else (19000, 2 * 256)
    run_case(env, M, n_out, n_in, tp, 1, split, seed=M + 7)
    run_case(env, M, n_out, n_in, tp, 0, split, seed=M + 8, dtype="f16")


@pytest.mark.parametrize("M,n_out,n_in", [(1, 8, 64), (300, 8, 64), (20000, 264, 128), (20000, 520, 128),
                                          (3, 40, 16384), (257, 24, 64)])
@pytest.mark.parametrize("split", ["out", "in"])
def test_extreme_aspect_ratios(env, M, n_out, n_in, split):
    """Outputs narrower than one weight tile, batches of tens of thousands of rows on
    a few columns (streaming kernel with many batch tiles, and the tiled kernel
    with a single ragged tile column), one slab of reduction and hundreds."""
    run_case(env, M, n_out * 2 if split == "out" else n_out, n_in if split == "out" else n_in * 2, 2, 1, split,
             seed=M + n_out)


@pytest.mark.parametrize("M", [1, 9, 16, 40, 300])
def test_output_width_not_a_multiple_of_four(env, M):
    """Output widths of 4k+1, +2, +3 columns in a padded Y (the row stride must be a multiple
    of eight, the width need not): the scalar edge of the 8-byte and 16-byte stores of the
    decode, streaming and split-K paths."""
    for nn, k in ((1001, 1600), (1002, 256), (1743, 12352), (37, 64)):
        run_case(env, M, nn, k, 1, 0, "out", seed=M + nn, pad_y=8 - nn % 8)


@pytest.mark.parametrize("layer", ["8b_qkv", "8b_down", "14b_o"])
def test_decoder_layer_shapes_prefill_batch(env, layer):
    n_out, n_in, split = LAYERS[layer]
    run_case(env, 1024, n_out, n_in, 2, 1, split, seed=9)


@pytest.mark.parametrize("M", [1, 16, 40, 64, 300])
@pytest.mark.parametrize("split", ["out", "in"])
def test_float16_elements(env, M, split):
    run_case(env, M, 208, 1024 + 128, 2, 1, split, seed=M + 300, pad=8, dtype="f16")
    run_case(env, M, 1024, 2048, 4, 3, split, seed=M + 400, dtype="f16")


@pytest.mark.parametrize("layer", ["8b_qkv", "8b_o", "8b_gate_up", "8b_down"])
def test_bench_shapes_sampled_rows(env, layer):
    """The shapes bench.py --linear times (full 8B layer, rank tp-1 at TP 1 and 8,
    decode, short-prefill and prefill batches), each checked on eight whole output
    rows that the oracle computes from the full weight matrix."""
    torch, b, ctx = env
    n_out, n_in, split = LAYERS[layer]
    Xh, Wh = linear_inputs(77, 4096, n_out, n_in)
    Wf = osl.bf16_to_f64(Wh)
    Wd = torch.from_numpy(Wh.view(np.int16)).cuda()
    sp = b.NTS_SPLIT_OUT if split == "out" else b.NTS_SPLIT_IN
    rng = np.random.default_rng(5)
    for tp in (1, 8):
        k = n_in if split == "out" else n_in // tp
        nn = n_out // tp if split == "out" else n_out
        for M in (16, 256, 4096):
            Xm = np.ascontiguousarray(Xh[:M, :k])
            Xd = torch.from_numpy(Xm.view(np.int16)).cuda()
            Yd = torch.empty((M, nn), dtype=torch.int16, device="cuda")
            kw = dict(M=M, n_out=n_out, n_in=n_in, tp=tp, rank=tp - 1, split=sp)
            ws_bytes = b.nts_shard_linear_workspace(**kw)
            ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")
            b.nts_shard_linear(ctx, Xd.data_ptr(), Wd.data_ptr(), Yd.data_ptr(), workspace=ws.data_ptr(),
                               workspace_bytes=ws_bytes, hip_stream=torch.cuda.current_stream().cuda_stream, **kw)
            torch.cuda.synchronize()
            rows = np.unique(np.concatenate([[0, 1, M // 2, M - 1], rng.integers(0, M, 4)]))
            Xr = osl.bf16_to_f64(Xm[rows])
            want, bound = osl.shard_linear(Xr, Wf, tp, tp - 1, split)
            got = osl.bf16_to_f64(Yd[torch.from_numpy(rows).cuda()].cpu().numpy().view(np.uint16))
            tol = osl.tolerance(want, bound, k, out_bits=8)
            tight = osl.tight_tolerance(want, osl.product_norm(Xr, Wf, tp, tp - 1, split), k, "bf16")
            err = np.abs(got - want)
            assert got.shape == want.shape == (len(rows), nn)
            assert np.all(err <= tol), (layer, tp, M, float((err / tol).max()))
            assert np.all(err <= tight), (layer, tp, M, float((err / tight).max()))


@pytest.mark.parametrize("layer", ["8b_qkv", "8b_o", "8b_gate_up", "8b_down", "14b_qkv", "14b_down"])
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_bench_shapes_bit_exact_on_integer_inputs(env, layer, dtype):
    """Full 8B / 14B layers (reductions of 4096 ... 14336 terms at TP1), every batch
    size bench.py --linear times, TP 1 and 4: integer inputs, so the sampled whole
    output rows must equal the once-rounded oracle bit for bit.  The batches must
    between them reach the decode, streaming and tiled kernels, with and without a
    split reduction."""
    torch, b, ctx = env
    n_out, n_in, split = LAYERS[layer]
    Xh, Wh = linear_inputs_int(91, 4096, n_out, n_in, dtype=dtype)
    decode = osl.bf16_to_f64 if dtype == "bf16" else osl.f16_to_f64
    Wf = decode(Wh)
    Wd = torch.from_numpy(Wh.view(np.int16)).cuda()
    sp = b.NTS_SPLIT_OUT if split == "out" else b.NTS_SPLIT_IN
    rng = np.random.default_rng(6)
    seen = set()
    for tp in (1, 4):
        k = n_in if split == "out" else n_in // tp
        nn = n_out // tp if split == "out" else n_out
        for M in (1, 16, 64, 256, 1024, 4096):
            Xm = np.ascontiguousarray(Xh[:M, :k])
            Xd = torch.from_numpy(Xm.view(np.int16)).cuda()
            Yd = torch.full((M, nn), 12345, dtype=torch.int16, device="cuda")
            kw = dict(M=M, n_out=n_out, n_in=n_in, tp=tp, rank=tp - 1, split=sp,
                      dtype=b.NTS_BF16 if dtype == "bf16" else b.NTS_F16)
            how = b.nts_shard_linear_launch(**kw)
            seen.add(("tiled" if how.tiled else "decode" if how.tile_rows == 16 else "stream", how.k_splits > 1))
            ws_bytes = b.nts_shard_linear_workspace(**kw)
            ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")
            b.nts_shard_linear(ctx, Xd.data_ptr(), Wd.data_ptr(), Yd.data_ptr(), workspace=ws.data_ptr(),
                               workspace_bytes=ws_bytes, hip_stream=torch.cuda.current_stream().cuda_stream, **kw)
            torch.cuda.synchronize()
            rows = np.unique(np.concatenate([[0, M // 2, M - 1], rng.integers(0, M, 5)]))
            want, _ = osl.shard_linear(decode(Xm[rows]), Wf, tp, tp - 1, split)
            got = Yd[torch.from_numpy(rows).cuda()].cpu().numpy().view(np.uint16)
            same = got == osl.round_to_bits(want, dtype)
            assert same.all(), (layer, tp, M, int((~same).sum()), np.argwhere(~same)[:4].tolist())
    assert {kind for kind, _ in seen} >= {"stream", "tiled"}
    if layer == "8b_down":
        assert ("stream", True) in seen and ("decode", False) in seen


@pytest.mark.parametrize("block", range(6))
def test_random_shapes(env, block):
    """Seeded random batch sizes, output widths (multiples of 8), reduction lengths,
    TP levels, ranks, split axes and element formats: whichever kernel and
    configuration each shape gets must stay within the tolerance."""
    from workload import SplitMix64
    rng = SplitMix64(9100 + block)
    u = lambda lo, hi: int(rng.integers(lo, hi, 1)[0])
    for i in range(12):
        big = block >= 4                                  # the last blocks aim at the tiled kernel
        M = ((257, 300, 512, 777, 1024, 1500) if big else
             (1, 2, 3, 5, 8, 13, 16, 17, 31, 32, 33, 64, 100, 129, 200, 256))[u(0, 5 if big else 15)]
        tp = (1, 2, 4)[u(0, 2)]
        split = ("out", "in")[u(0, 1)]
        nn = 8 * (u(800, 3000) if big else u(1, 700))
        k = 64 * (u(1, 6) if big else u(1, 40 if M > 64 else 120))
        n_out, n_in = (nn * tp, k) if split == "out" else (nn, k * tp)
        run_case(env, M, n_out, n_in, tp, u(0, tp - 1), split, seed=block * 100 + i,
                 dtype=("bf16", "f16")[u(0, 1)])


@pytest.mark.parametrize("M,n_out,n_in,tp,split", [(16, 6144, 4096, 1, "out"), (16, 4096, 14336, 2, "in"), (1, 4096, 14336, 1, "in"),
                                                   (64, 4096, 4096, 4, "in"), (300, 2048, 2048, 1, "out"),
                                                   (1024, 6144, 4096, 1, "out")])
def test_tuned_configuration_keeps_parity(env, M, n_out, n_in, tp, split):
    """nts_shard_linear_tune times the candidate configurations and remembers the
    fastest; whichever it picks, the layer's result must stay inside both tolerances
    on random inputs and bit-exact on integer inputs, the tuning call itself must
    leave the right result in Y, and later calls must use what was remembered
    (and fall back to the default when their workspace is too small for it)."""
    torch, b, _ = env
    ctx = b.nts_init(0)                                   # a context of its own: tuning is remembered per context
    try:
        sp = b.NTS_SPLIT_OUT if split == "out" else b.NTS_SPLIT_IN
        k = n_in if split == "out" else n_in // tp
        nn = n_out // tp if split == "out" else n_out
        kw = dict(M=M, n_out=n_out, n_in=n_in, tp=tp, rank=tp - 1, split=sp)
        assert b.nts_shard_linear_tuned(ctx, **kw) is None
        ws = torch.empty(8 * M * nn * 4 + 16, dtype=torch.uint8, device="cuda")      # room for up to eight K splits
        st = torch.cuda.current_stream().cuda_stream
        for exact in (False, True):
            Xh, Wh = (linear_inputs_int if exact else linear_inputs)(60 + M, M, n_out, n_in, x_cols=k)
            Xd = torch.from_numpy(Xh.view(np.int16)).cuda()
            Wd = torch.from_numpy(Wh.view(np.int16)).cuda()
            X64, W64 = osl.bf16_to_f64(Xh), osl.bf16_to_f64(Wh)
            want, bound = osl.shard_linear(X64, W64, tp, tp - 1, split)
            tight = osl.tight_tolerance(want, osl.product_norm(X64, W64, tp, tp - 1, split), k, "bf16")

            def check(Yd, tag):
                got_bits = Yd.cpu().numpy().view(np.uint16)
                if exact:
                    assert np.array_equal(got_bits, osl.round_to_bits(want, "bf16")), tag
                else:
                    assert np.all(np.abs(osl.bf16_to_f64(got_bits) - want) <= tight), tag

            Yd = torch.full((M, nn), 12345, dtype=torch.int16, device="cuda")
            if not exact:
                more = [Wd.clone() for _ in range(M % 3)]               # one, two or three weight matrices
                picked = b.nts_shard_linear_tune(ctx, Xd.data_ptr(), [Wd.data_ptr()] + [w.data_ptr() for w in more],
                                                 Yd.data_ptr(), workspace=ws.data_ptr(),
                                                 workspace_bytes=ws.numel() - 16, hip_stream=st, **kw)
                torch.cuda.synchronize()
                check(Yd, "result left by the tuning call")
                kept = b.nts_shard_linear_tuned(ctx, **kw)
                assert kept is not None
                assert [getattr(kept, f) for f in ("tiled", "tile_rows", "tile_cols", "k_splits", "k_waves")] == \
                       [getattr(picked, f) for f in ("tiled", "tile_rows", "tile_cols", "k_splits", "k_waves")]
                assert picked.k_splits <= 8
                Yd.fill_(12345)
            b.nts_shard_linear(ctx, Xd.data_ptr(), Wd.data_ptr(), Yd.data_ptr(), workspace=ws.data_ptr(),
                               workspace_bytes=ws.numel() - 16, hip_stream=st, **kw)
            torch.cuda.synchronize()
            check(Yd, "tuned configuration")
            # with only the default's workspace the call still works (tuned if it fits, default otherwise)
            need = b.nts_shard_linear_workspace(**kw)
            Yd.fill_(12345)
            b.nts_shard_linear(ctx, Xd.data_ptr(), Wd.data_ptr(), Yd.data_ptr(), workspace=ws.data_ptr() if need else 0,
                               workspace_bytes=need, hip_stream=st, **kw)
            torch.cuda.synchronize()
            check(Yd, "default-sized workspace")
    finally:
        b.nts_free(ctx)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_all_five_tile_shapes_give_the_same_bits(env, dtype):
    """The tiled kernel's five tile shapes, each named explicitly through
    nts_shard_linear_with, on one problem that is ragged for all of them (700 rows,
    1000 columns of a TP-2 shard, row padding): integer inputs, so every shape must
    produce the oracle's once-rounded result bit for bit, and nothing past the row."""
    torch, b, ctx = env
    M, n_out, n_in, tp = 700, 2000, 320, 2
    nn, pad = n_out // tp, 8
    kw = dict(M=M, n_out=n_out, n_in=n_in, tp=tp, rank=1, split=b.NTS_SPLIT_OUT, ldy=nn + pad,
              dtype=b.NTS_BF16 if dtype == "bf16" else b.NTS_F16)
    Xh, Wh = linear_inputs_int(4242, M, n_out, n_in, x_cols=n_in, dtype=dtype)
    decode = osl.bf16_to_f64 if dtype == "bf16" else osl.f16_to_f64
    want, _ = osl.shard_linear(decode(Xh), decode(Wh), tp, 1, "out")
    bits = osl.round_to_bits(want, dtype)
    Xd = torch.from_numpy(Xh.view(np.int16)).cuda()
    Wd = torch.from_numpy(Wh.view(np.int16)).cuda()
    st = torch.cuda.current_stream().cuda_stream
    proto = b.nts_shard_linear_launch(**kw)
    for rows, cols in [(256, 256), (256, 192), (256, 128), (128, 192), (128, 128)]:
        how = type(proto)(tiled=1, tile_rows=rows, tile_cols=cols, k_splits=1, slabs_ahead=proto.slabs_ahead, k_waves=1)
        Yd = torch.full((M, nn + pad), 12345, dtype=torch.int16, device="cuda")
        b.nts_shard_linear_with(ctx, how, Xd.data_ptr(), Wd.data_ptr(), Yd.data_ptr(), hip_stream=st, **kw)
        torch.cuda.synchronize()
        got = Yd.cpu().numpy().view(np.uint16)
        assert np.array_equal(got[:, :nn], bits), (rows, cols)
        assert np.all(got[:, nn:] == 12345), (rows, cols)
    # a tile taller than the batch is refused, as in the default choice
    small = dict(kw, M=200)
    how = type(proto)(tiled=1, tile_rows=256, tile_cols=192, k_splits=1, slabs_ahead=proto.slabs_ahead, k_waves=1)
    with pytest.raises(b.NtsError):
        b.nts_shard_linear_with(ctx, how, Xd.data_ptr(), Wd.data_ptr(), Yd.data_ptr(), hip_stream=st, **small)


@pytest.mark.parametrize("M,n_out,n_in,tp,split,dtype", [
    (1, 4096, 14336, 1, "in", "bf16"), (16, 6144, 4096, 1, "out", "bf16"), (9, 1000, 12352, 1, "out", "f16"),
    (64, 4096, 4096, 4, "in", "bf16"), (130, 4104, 6144, 1, "out", "f16"), (300, 2048, 2048, 1, "out", "bf16"),
    (1024, 6144, 4096, 1, "out", "bf16"), (520, 2056, 512, 2, "in", "bf16")])
def test_every_candidate_configuration_computes_the_layer(env, M, n_out, n_in, tp, split, dtype):
    """nts_shard_linear_candidates lists what the tuner may pick for a shape; each of
    them, run through nts_shard_linear_with, must give the layer's result: inside the
    tight tolerance on random inputs and bit-exact on integer inputs.  The first
    candidate is the default; a description the library has no kernel for is refused;
    remembering one makes nts_shard_linear use it."""
    torch, b, _ = env
    ctx = b.nts_init(0)
    try:
        sp = b.NTS_SPLIT_OUT if split == "out" else b.NTS_SPLIT_IN
        k = n_in if split == "out" else n_in // tp
        nn = n_out // tp if split == "out" else n_out
        pad = 8 if nn % 8 == 0 else 8 - nn % 8
        kw = dict(M=M, n_out=n_out, n_in=n_in, tp=tp, rank=tp - 1, split=sp, ldy=nn + pad,
                  dtype=b.NTS_BF16 if dtype == "bf16" else b.NTS_F16)
        cands = b.nts_shard_linear_candidates(**kw)
        fields = ("tiled", "tile_rows", "tile_cols", "k_splits", "slabs_ahead", "k_waves")
        key = lambda c: tuple(getattr(c, f) for f in fields)
        assert 1 <= len(cands) <= 16 and len({key(c) for c in cands}) == len(cands)
        assert key(cands[0]) == key(b.nts_shard_linear_launch(**kw))
        decode = osl.bf16_to_f64 if dtype == "bf16" else osl.f16_to_f64
        st = torch.cuda.current_stream().cuda_stream
        ws = torch.empty(32 * M * nn * 4 + 16, dtype=torch.uint8, device="cuda")
        for exact in (False, True):
            Xh, Wh = (linear_inputs_int if exact else linear_inputs)(70 + M, M, n_out, n_in, x_cols=k, dtype=dtype)
            Xd = torch.from_numpy(Xh.view(np.int16)).cuda()
            Wd = torch.from_numpy(Wh.view(np.int16)).cuda()
            X64, W64 = decode(Xh), decode(Wh)
            want, _ = osl.shard_linear(X64, W64, tp, tp - 1, split)
            tight = osl.tight_tolerance(want, osl.product_norm(X64, W64, tp, tp - 1, split), k, dtype)
            for c in cands:
                Yd = torch.full((M, nn + pad), 12345, dtype=torch.int16, device="cuda")
                b.nts_shard_linear_with(ctx, c, Xd.data_ptr(), Wd.data_ptr(), Yd.data_ptr(), workspace=ws.data_ptr(),
                                        workspace_bytes=ws.numel() - 16, hip_stream=st, **kw)
                torch.cuda.synchronize()
                got = Yd.cpu().numpy().view(np.uint16)
                assert np.all(got[:, nn:] == 12345), key(c)
                if exact:
                    assert np.array_equal(got[:, :nn], osl.round_to_bits(want, dtype)), key(c)
                else:
                    assert np.all(np.abs(decode(got[:, :nn]) - want) <= tight), key(c)
        # a split that needs workspace is refused without it; a description with no kernel behind it is refused
        split_c = [c for c in cands if c.k_splits > 1]
        if split_c:
            with pytest.raises(b.NtsError):
                b.nts_shard_linear_with(ctx, split_c[0], Xd.data_ptr(), Wd.data_ptr(), Yd.data_ptr(), hip_stream=st, **kw)
        bogus = type(cands[0])(tiled=0, tile_rows=160, tile_cols=128, k_splits=1, slabs_ahead=3, k_waves=1)
        with pytest.raises(b.NtsError) as ei:
            b.nts_shard_linear_with(ctx, bogus, Xd.data_ptr(), Wd.data_ptr(), Yd.data_ptr(), hip_stream=st, **kw)
        assert ei.value.status == b.NTS_EINVAL
        # remember / forget
        last = cands[-1]
        b.nts_shard_linear_remember(ctx, last, **kw)
        assert key(b.nts_shard_linear_tuned(ctx, **kw)) == key(last)
        b.nts_shard_linear_remember(ctx, None, **kw)
        assert b.nts_shard_linear_tuned(ctx, **kw) is None
    finally:
        b.nts_free(ctx)


@pytest.mark.parametrize("split", ["out", "in"])
def test_shard_view_feeds_a_gemm_library(env, split):
    """The view nts_shard_linear_view names is the shard itself: a library GEMM on that view of the
    full, row-padded weight matrix gives the layer's result (integer inputs, so both are exact and
    must agree bit for bit with the once-rounded oracle)."""
    torch, b, ctx = env
    M, n_out, n_in, tp, rank, pad = 48, 512, 768, 4, 2, 8
    k = n_in if split == "out" else n_in // tp
    nn = n_out // tp if split == "out" else n_out
    Xh, Wh = linear_inputs_int(5, M, n_out, n_in, x_cols=k, dtype="bf16")
    ldw = n_in + pad
    Wp = np.zeros((n_out, ldw), np.uint16); Wp[:, :n_in] = Wh
    Xd = torch.from_numpy(Xh.view(np.int16)).cuda().view(torch.bfloat16)
    Wd = torch.from_numpy(Wp.view(np.int16)).cuda().view(torch.bfloat16)
    sp = b.NTS_SPLIT_OUT if split == "out" else b.NTS_SPLIT_IN
    off, rows, cols, rs = b.nts_shard_linear_view(M=M, n_out=n_out, n_in=n_in, tp=tp, rank=rank, split=sp, ldw=ldw)
    assert (rows, cols, rs) == (nn, k, ldw)
    view = torch.as_strided(Wd.reshape(-1), (rows, cols), (rs, 1), off)
    Y = torch.matmul(Xd, view.t())
    torch.cuda.synchronize()
    want, _ = osl.shard_linear(osl.bf16_to_f64(Xh), osl.bf16_to_f64(Wh), tp, rank, split)
    got = Y.view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(got, osl.round_to_bits(want, "bf16"))
