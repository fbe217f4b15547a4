"""Pins of the CPU oracle against what the paper and plain mathematics fix.

None of these tests calls the oracle to produce its own expected value: the
expected side is the paper's worked example (tests/golden), a NumPy library
routine (take / fancy assignment), a literal dictionary model, or a closed
form of the stateless fill.
"""
import itertools
import os

import numpy as np
import pytest

from oracle import kvmig as orc
from workload import SplitMix64, fill_pool_u16, fill_words, make_case, M8B

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rand_pool(rng, L, S, Hl, D, dtype=np.uint16):
    n = L * 2 * S * Hl * D
    bits = rng.words(n)
    return (bits & np.uint64(np.iinfo(dtype).max)).astype(dtype).reshape(L, 2, S, Hl, D)


# ------------------------------------------------------------------- runs ---

def test_runs_of_a_hand_written_example():
    """Written out by hand: source slots break after index 2 and 5, destination
    slots after index 4 (and 2): boundaries at 0, 3, 5, 6."""
    s = [10, 11, 12, 40, 41, 42, 7, 8]
    d = [20, 21, 22, 30, 31, 50, 51, 52]
    #    run 0       | run 1 | r2 | run 3
    assert orc.runs(s, d).tolist() == [0, 3, 5, 6, 8]
    assert orc.runs([], []).tolist() == [0]
    assert orc.runs([5], [9]).tolist() == [0, 1]
    with pytest.raises(ValueError):
        orc.runs([1, 2], [1])


def test_runs_closed_forms_of_the_two_layouts():
    """Contiguous per-request layout with a gap between requests on either
    side: one run per non-empty request.  Token-granular pages placed so that
    no two neighbours are adjacent: one run per token.  Pages of p tokens in
    such a placement: one run per page (a last partial page included)."""
    ctx_len = [40, 0, 1, 25]
    src_pages, dst_pages, at_s, at_d = [], [], 3, 500
    for n in ctx_len:
        src_pages += list(range(at_s, at_s + n))
        dst_pages += list(range(at_d, at_d + n))
        at_s += n + 2                                   # a gap on the source side only
        at_d += n
    s, d = orc.flatten(ctx_len, src_pages, 1), orc.flatten(ctx_len, dst_pages, 1)
    assert orc.runs(s, d).tolist() == [0, 40, 41, 66]
    T = 50
    odd = [2 * j for j in range(T)]                     # every other slot: never adjacent
    assert orc.runs(odd, list(range(T))).tolist() == list(range(T + 1))
    assert orc.runs(list(range(T)), odd).tolist() == list(range(T + 1))
    p, n_tok = 4, 22                                    # 5 full pages and a page of 2
    pages = [3 * i for i in range(6)]
    s = orc.flatten([n_tok], pages, p)
    assert orc.runs(s, s).tolist() == [0, 4, 8, 12, 16, 20, 22]


@pytest.mark.parametrize("seed", range(6))
def test_runs_partition_is_valid_and_maximal(seed):
    """Brute force on random slot lists with planted runs: inside a run both
    sides advance by one; across every boundary at least one side does not;
    the runs tile [0, T)."""
    rng = SplitMix64(700 + seed)
    s, d = [], []
    while len(s) < 300:
        n = int(rng.integers(1, 9, 1)[0])
        a, b = int(rng.integers(0, 5000, 1)[0]), int(rng.integers(0, 5000, 1)[0])
        s += list(range(a, a + n))
        d += list(range(b, b + n)) if rng.integers(0, 4, 1)[0] else list(range(b + n, b, -1))
    r = orc.runs(s, d).tolist()
    T = len(s)
    assert r[0] == 0 and r[-1] == T and all(x < y for x, y in zip(r, r[1:]))
    for a, b in zip(r, r[1:]):
        assert all(s[j] == s[j - 1] + 1 and d[j] == d[j - 1] + 1 for j in range(a + 1, b))
        if b < T:
            assert s[b] != s[b - 1] + 1 or d[b] != d[b - 1] + 1


# ---------------------------------------------------------------- routing ---

def test_route_reproduces_paper_worked_example():
    """Sec. 3.2.2: the seven moves the text spells out for 4 GPUs / 8 heads."""
    rows = []
    with open(os.path.join(GOLDEN, "tp_switch_example.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                step, s, d, a, b = line.split()
                rows.append((step, int(s), int(d), int(a), int(b)))
    assert len(rows) == 7
    H = 8
    steps = {
        "TP1->TP2": ([[1], [2], [3], [4]], [[1, 2], [3, 4]], {1: 0, 2: 0, 3: 1, 4: 1}),
        "TP2->TP4": ([[1, 2], [3, 4]], [[1, 2, 3, 4]], {1: 0, 2: 0, 3: 0, 4: 0}),
    }
    for step, s, d, a, b in rows:
        old, new, newgroup_of_gpu = steps[step]
        go = next(i for i, g in enumerate(old) if s in g)
        gn = newgroup_of_gpu[d]
        assert d in new[gn]
        so, do, w = orc.route(H, len(old[go]), old[go].index(s), len(new[gn]), new[gn].index(d))
        sa, _ = orc.head_interval(H, len(old[go]), old[go].index(s))
        da, _ = orc.head_interval(H, len(new[gn]), new[gn].index(d))
        assert w == b - a + 1, (step, s, d)
        assert sa + so == a and da + do == a, (step, s, d)


def test_route_full_pair_table_of_the_example():
    """The example's complete table (stated moves plus the ones "and so on"
    implies): cross-GPU moves only, as (src, dst, first, last)."""
    H = 8
    # one request per original GPU
    old, new = [[1], [2], [3], [4]], [[1, 2], [3, 4]]
    pairs = orc.transition_pairs(H, old, new, {10: 0, 20: 1, 30: 2, 40: 3}, {10: 0, 20: 0, 30: 1, 40: 1})
    got = sorted((s, d, orc.head_interval(H, 1, 0)[0] + so, w) for s, d, _, so, _, w in pairs if s != d)
    assert got == [(1, 2, 4, 4), (2, 1, 0, 4), (3, 4, 4, 4), (4, 3, 0, 4)]
    stay = sorted((s, so, w) for s, d, _, so, _, w in pairs if s == d)
    assert stay == [(1, 0, 4), (2, 4, 4), (3, 0, 4), (4, 4, 4)]
    old, new = [[1, 2], [3, 4]], [[1, 2, 3, 4]]
    pairs = orc.transition_pairs(H, old, new, {10: 0, 30: 1}, {10: 0, 30: 0})
    got = set()
    for s, d, reqs, so, do, w in pairs:
        first = orc.head_interval(H, 2, old[0].index(s) if s in old[0] else old[1].index(s))[0] + so
        got.add((s, d, first, first + w - 1))
    want = {(1, 1, 0, 1), (3, 1, 0, 1), (1, 2, 2, 3), (3, 2, 2, 3),
            (2, 3, 4, 5), (4, 3, 4, 5), (2, 4, 6, 7), (4, 4, 6, 7)}
    assert got == want


@pytest.mark.parametrize("H", [8, 16, 32])
def test_route_partitions_every_source_interval(H):
    """Even split on heads: what rank rs sends to all rd tiles its interval
    exactly once, and every destination ends up with H/Nd heads."""
    for Ns, Nd in itertools.product([1, 2, 4, 8], repeat=2):
        got_at_dst = {rd: [] for rd in range(Nd)}
        for rs in range(Ns):
            cover = []
            for rd in range(Nd):
                so, do, w = orc.route(H, Ns, rs, Nd, rd)
                if w:
                    base_s = rs * (H // Ns)
                    base_d = rd * (H // Nd)
                    assert 0 <= so and so + w <= H // Ns and 0 <= do and do + w <= H // Nd
                    assert base_s + so == base_d + do          # same global heads on both ends
                    cover += list(range(base_s + so, base_s + so + w))
                    got_at_dst[rd] += list(range(base_d + do, base_d + do + w))
            assert cover == list(range(rs * (H // Ns), (rs + 1) * (H // Ns)))
        for rd in range(Nd):
            assert sorted(got_at_dst[rd]) == list(range(rd * (H // Nd), (rd + 1) * (H // Nd)))


def test_route_rejects_uneven_split():
    with pytest.raises(ValueError):
        orc.route(8, 3, 0, 1, 0)
    with pytest.raises(ValueError):
        orc.route(8, 2, 2, 1, 0)


# ------------------------------------------------------------- flattening ---

def test_flatten_token_pages_are_the_slots():
    ctx = [3, 0, 2]
    pages = [7, 1, 4, 9, 0]
    assert orc.flatten(ctx, pages, 1).tolist() == pages


def test_flatten_pages_of_four_with_partial_tail():
    # request 0: 6 tokens in pages 5, 2 (tail holds 2 of 4); request 1: 4 tokens in page 0
    got = orc.flatten([6, 4], [5, 2, 0], 4).tolist()
    assert got == [20, 21, 22, 23, 8, 9, 0, 1, 2, 3]


def test_flatten_rejects_wrong_table_length():
    with pytest.raises(ValueError):
        orc.flatten([5], [1], 4)


# ------------------------------------------------------------ pack/unpack ---

@pytest.mark.parametrize("Hs,off,w", [(8, 0, 8), (8, 4, 4), (4, 1, 2), (2, 1, 1), (3, 0, 2)])
@pytest.mark.parametrize("dtype", [np.uint16, np.uint8, np.uint32])
def test_pack_is_row_gather_with_column_slice(Hs, off, w, dtype):
    rng = SplitMix64(100 + Hs + off)
    L, S, D, T = 3, 37, 6, 23
    src = rand_pool(rng, L, S, Hs, D, dtype)
    sslot = rng.integers(0, S - 1, T).astype(np.int32)          # repeats allowed on the source
    got = orc.pack(src, sslot, off, w)
    want = np.take(src, sslot, axis=2)[:, :, :, off:off + w, :]
    assert got.shape == (L, 2, T, w, D)
    assert np.array_equal(got, want)


def test_pack_identity_case_is_a_prefix_copy():
    rng = SplitMix64(5)
    src = rand_pool(rng, 2, 16, 4, 8)
    got = orc.pack(src, np.arange(11, dtype=np.int32), 0, 4)
    assert got.tobytes() == np.ascontiguousarray(src[:, :, :11]).tobytes()


@pytest.mark.parametrize("Hd,off,w", [(8, 0, 8), (4, 0, 4), (4, 2, 2), (8, 7, 1)])
def test_unpack_is_row_scatter_and_touches_nothing_else(Hd, off, w):
    rng = SplitMix64(200 + Hd + off)
    L, S, D, T = 2, 41, 4, 29
    stream = rand_pool(rng, L, T, w, D)
    dst0 = rand_pool(rng, L, S, Hd, D)
    dslot = rng.permutation(S)[:T].astype(np.int32)
    got = dst0.copy()
    orc.unpack(stream, got, dslot, off)
    want = dst0.copy()
    want[:, :, dslot, off:off + w, :] = stream
    assert np.array_equal(got, want)
    mask = np.ones(dst0.shape, dtype=bool)
    mask[:, :, dslot, off:off + w, :] = False
    assert np.array_equal(got[mask], dst0[mask])                 # sentinel bytes survive
    assert mask.sum() == dst0.size - stream.size


def test_unpack_full_permutation_permutes_rows():
    rng = SplitMix64(9)
    L, S, Hd, D = 2, 12, 2, 4
    stream = rand_pool(rng, L, S, Hd, D)
    perm = rng.permutation(S).astype(np.int32)
    dst = np.zeros((L, 2, S, Hd, D), np.uint16)
    orc.unpack(stream, dst, perm, 0)
    assert np.array_equal(dst[:, :, perm], stream)
    assert sorted(map(bytes, dst.reshape(L * 2 * S, -1))) == sorted(map(bytes, stream.reshape(L * 2 * S, -1)))


def test_unpack_rejects_duplicate_destination_slots():
    stream = np.zeros((1, 2, 2, 1, 2), np.uint16)
    dst = np.zeros((1, 2, 4, 1, 2), np.uint16)
    with pytest.raises(ValueError):
        orc.unpack(stream, dst, np.array([1, 1], np.int32), 0)


def test_stream_bytes_match_paper_size_identity():
    """Sec. 3.2.2 equates 4096 tokens with 0.5 GB and 40960 with 5 GB for a
    16-bit 8B Llama: 128 KiB per token, GB read as GiB."""
    src = np.zeros((M8B.L, 2, 4, M8B.H, M8B.D), np.uint16)
    s = orc.pack(src, np.arange(4, dtype=np.int32), 0, M8B.H)
    per_token = s.nbytes // 4
    assert per_token == 131072 == M8B.token_bytes
    assert 4096 * per_token == 2 ** 29 and 40960 * per_token == 5 * 2 ** 30


# ---------------------------------------------------------------- migrate ---

@pytest.mark.parametrize("tr", [(1, 0, 2, 1), (2, 1, 4, 2), (4, 3, 8, 7), (8, 2, 4, 1), (4, 1, 2, 0), (2, 1, 1, 0), (1, 0, 1, 0)])
def test_migrate_equals_direct_and_closed_form_of_fill(tr):
    Ns, rs, Nd, rd = tr
    H, L, D, S, Sd, T = 8, 2, 8, 64, 52, 40         # the two pools differ in size
    so, do, w = orc.route(H, Ns, rs, Nd, rd)
    Hs, Hd = H // Ns, H // Nd
    rng = SplitMix64(300 + Ns * 10 + Nd)
    src = fill_pool_u16(11, L * 2 * S * Hs * D).reshape(L, 2, S, Hs, D)
    dst0 = fill_pool_u16(12, L * 2 * Sd * Hd * D).reshape(L, 2, Sd, Hd, D)
    sslot = rng.permutation(S)[:T].astype(np.int32)
    dslot = rng.permutation(Sd)[:T].astype(np.int32)
    a, b = dst0.copy(), dst0.copy()
    orc.migrate(src, a, sslot, dslot, so, do, w)
    orc.migrate_direct(src, b, sslot, dslot, so, do, w)
    assert np.array_equal(a, b)
    # closed form: each moved element equals the fill word of its SOURCE coordinate
    for l, c, j, h, x in itertools.product(range(L), range(2), [0, 7, T - 1], range(w), [0, D - 1]):
        lin = ((((l * 2 + c) * S + int(sslot[j])) * Hs + so + h) * D + x)
        word = int(fill_words(11, lin // 4, 1)[0])
        assert int(a[l, c, dslot[j], do + h, x]) == (word >> (16 * (lin % 4))) & 0xFFFF
    # and an untouched element still equals the destination's own fill
    free = sorted(set(range(Sd)) - set(dslot.tolist()))[0]
    lin = (((0 * Sd + free) * Hd + 0) * D + 3)
    assert int(a[0, 0, free, 0, 3]) == (int(fill_words(12, lin // 4, 1)[0]) >> (16 * (lin % 4))) & 0xFFFF


def test_argument_checks_accept_the_last_valid_value_and_reject_the_next():
    """The C loops index without checks, so the Python side's range checks are
    what keeps a bad argument from reading or writing outside a pool: each check
    is tried at its last valid value and one beyond."""
    L, S, H, D = 1, 6, 4, 2
    src = np.arange(L * 2 * S * H * D, dtype=np.uint16).reshape(L, 2, S, H, D)
    last, beyond = np.array([S - 1], np.int32), np.array([S], np.int32)
    assert np.array_equal(orc.pack(src, last, 1, 3)[0, 0, 0], src[0, 0, S - 1, 1:4])       # head slice ends at H
    for bad in [dict(sslot=beyond, src_head_off=0, w=1), dict(sslot=np.array([-1], np.int32), src_head_off=0, w=1),
                dict(sslot=np.array([0, S], np.int32), src_head_off=0, w=1),              # one bad slot among good ones
                dict(sslot=np.array([2, -1], np.int32), src_head_off=0, w=1),
                dict(sslot=last, src_head_off=2, w=3), dict(sslot=last, src_head_off=-1, w=1),
                dict(sslot=last, src_head_off=0, w=0)]:
        with pytest.raises(ValueError):
            orc.pack(src, **bad)
    stream = orc.pack(src, last, 1, 3)
    dst = np.zeros((L, 2, S, H, D), np.uint16)
    orc.unpack(stream, dst, last, 1)                                                        # ends at H: fine
    assert np.array_equal(dst[0, 0, S - 1, 1:4], src[0, 0, S - 1, 1:4]) and not dst[0, 0, S - 1, 0].any()
    for slots, off in [(last, 2), (last, -1), (beyond, 0)]:
        with pytest.raises(ValueError):
            orc.unpack(stream, np.zeros_like(dst), slots, off)
    # the direct form checks each side by itself: a slice that fits one pool but not the other is refused
    narrow = np.zeros((L, 2, S, 2, D), np.uint16)
    orc.migrate_direct(src, narrow, last, last, 2, 0, 2)                                    # both end at their pool's H
    assert np.array_equal(narrow[0, 0, S - 1], src[0, 0, S - 1, 2:4])
    for so, do, w in [(1, 0, 3), (2, 1, 2), (3, 0, 2), (0, 0, 0), (-1, 0, 1), (0, -1, 1)]:
        with pytest.raises(ValueError):
            orc.migrate_direct(src, np.zeros_like(narrow), last, last, so, do, w)
    with pytest.raises(ValueError):
        orc.migrate_direct(src, np.zeros_like(narrow), beyond, last, 2, 0, 2)
    with pytest.raises(ValueError):
        orc.head_interval(8, 0, 0)
    # ranks whose head ranges only touch exchange nothing, and "nothing" is always (0, 0, 0)
    assert orc.route(8, 2, 0, 4, 2) == (0, 0, 0) and orc.route(8, 4, 3, 2, 0) == (0, 0, 0)


@pytest.mark.parametrize("tr", [(2, 1, 4, 2), (4, 1, 2, 0), (2, 1, 4, 3), (1, 0, 1, 0), (4, 0, 2, 0), (8, 5, 2, 1)])
def test_migrated_element_source_against_dictionary_model(tr):
    """``migrated_element_source`` names, for one destination (slot, local head),
    the source (slot, local head) it must hold afterwards.  Expected side: a
    literal dictionary from global coordinates (token, global head) to where
    the source GPU keeps them and where the destination GPU must keep them,
    built from the even head split alone.  Every destination (slot, head) is
    checked, moved and untouched, with non-zero offsets on both sides."""
    Ns, rs, Nd, rd = tr
    H, T, S_src, S_dst = 8, 9, 23, 17
    Hs, Hd = H // Ns, H // Nd
    rng = SplitMix64(4100 + 10 * Ns + Nd + rd)
    sslot = rng.permutation(S_src)[:T].astype(np.int32)
    dslot = rng.permutation(S_dst)[:T].astype(np.int32)
    # where the source rank keeps (token j, global head gh), where the destination rank wants it
    at_src, at_dst = {}, {}
    for j in range(T):
        for gh in range(H):
            if rs * Hs <= gh < (rs + 1) * Hs:
                at_src[(j, gh)] = (int(sslot[j]), gh - rs * Hs)
            if rd * Hd <= gh < (rd + 1) * Hd:
                at_dst[(j, gh)] = (int(dslot[j]), gh - rd * Hd)
    want = {at_dst[k]: at_src[k] for k in at_dst if k in at_src}
    so, do, w = orc.route(H, Ns, rs, Nd, rd)
    assert w > 0 and len(want) == T * w
    if tr == (2, 1, 4, 2):
        assert (so, do) == (0, 0)
    if tr == (2, 1, 4, 3):
        assert so == 2 and do == 0                      # slice starts inside the source's row
    if tr == (4, 1, 2, 0):
        assert so == 0 and do == 2                      # slice lands inside the destination's row
    j_of = {int(s): j for j, s in enumerate(dslot)}
    for slot in range(S_dst):
        for head in range(Hd):
            got = orc.migrated_element_source(j_of, sslot, slot, head, so, do, w)
            assert got == want.get((slot, head)), (tr, slot, head)
    # the same table must describe what migrate() does to a pool of coordinates
    L, D = 1, 1
    src = np.zeros((L, 2, S_src, Hs, D), np.uint16)
    for s in range(S_src):
        for h in range(Hs):
            src[0, :, s, h, 0] = 1 + s * Hs + h
    dst = np.zeros((L, 2, S_dst, Hd, D), np.uint16)
    orc.migrate(src, dst, sslot, dslot, so, do, w)
    for slot in range(S_dst):
        for head in range(Hd):
            srcpos = want.get((slot, head))
            assert int(dst[0, 1, slot, head, 0]) == (0 if srcpos is None else 1 + srcpos[0] * Hs + srcpos[1])


@pytest.mark.parametrize("p", [1, 2, 4])
def test_whole_chain_against_dictionary_model(p):
    """Tiny exhaustive check: the chain route -> flatten -> pack -> unpack must
    place every (request, token, layer, K|V, head) where a literal dictionary
    model of paged KV says it lives."""
    H, L, D = 4, 2, 2
    ctx = [3, 1, 2]
    n_pg = [(n + p - 1) // p for n in ctx]
    tot_pg = sum(n_pg)
    S = (tot_pg + 2) * p
    base = list(range(tot_pg + 2))
    perms = list(itertools.permutations(base, tot_pg)) if tot_pg <= 4 else None
    rng = SplitMix64(77 + p)
    trials = perms[:200] if perms else [tuple(rng.permutation(tot_pg + 2)[:tot_pg]) for _ in range(60)]
    for Ns, rs, Nd, rd in [(1, 0, 2, 1), (2, 0, 4, 1), (4, 2, 2, 1), (2, 1, 1, 0)]:
        Hs, Hd = H // Ns, H // Nd
        so, do, w = orc.route(H, Ns, rs, Nd, rd)
        assert w > 0
        for trial_i, src_pages in enumerate(trials[:: max(1, len(trials) // 25)]):
            dst_pages = tuple(reversed(src_pages)) if trial_i % 2 else tuple(
                (x + 1) % (tot_pg + 2) for x in src_pages)
            # dictionary model: value of (req, tok, l, c, global head, x)
            val = {}
            src = np.zeros((L, 2, S, Hs, D), np.uint16)
            want = np.full((L, 2, S, Hd, D), 0xEEEE, np.uint16)
            k = 1
            pg_at = 0
            for r, n in enumerate(ctx):
                for t in range(n):
                    s_slot = src_pages[pg_at + t // p] * p + t % p
                    d_slot = dst_pages[pg_at + t // p] * p + t % p
                    for l in range(L):
                        for c in range(2):
                            for gh in range(H):
                                for x in range(D):
                                    val[(r, t, l, c, gh, x)] = k
                                    if rs * Hs <= gh < (rs + 1) * Hs:
                                        src[l, c, s_slot, gh - rs * Hs, x] = k
                                        if rd * Hd <= gh < (rd + 1) * Hd:
                                            want[l, c, d_slot, gh - rd * Hd, x] = k
                                    k += 1
                pg_at += n_pg[r]
            got = np.full((L, 2, S, Hd, D), 0xEEEE, np.uint16)
            sslot = orc.flatten(ctx, list(src_pages), p)
            dslot = orc.flatten(ctx, list(dst_pages), p)
            stream = orc.pack(src, sslot, so, w)
            orc.unpack(stream, got, dslot, do)
            assert np.array_equal(got, want), (p, Ns, rs, Nd, rd, src_pages)


def test_chain_on_generated_case_c1():
    """The generated small configuration runs through the oracle and its
    result is independent of how the stream is cut into chunks."""
    for case in make_case("c1", tokens=48)[:3]:
        sh = case.shape
        so, do, w = orc.route(sh.H, case.Ns, case.rs, case.Nd, case.rd)
        L, D = 2, 8                                         # reduced layers/dim for speed
        src = fill_pool_u16(case.seed_src, L * 2 * case.S_src * case.Hs * D).reshape(L, 2, case.S_src, case.Hs, D)
        dst = fill_pool_u16(case.seed_dst, L * 2 * case.S_dst * case.Hd * D).reshape(L, 2, case.S_dst, case.Hd, D)
        sslot = orc.flatten(case.ctx_len, case.src_pages, case.p)
        dslot = orc.flatten(case.ctx_len, case.dst_pages, case.p)
        whole = dst.copy()
        orc.migrate(src, whole, sslot, dslot, so, do, w)
        # chunked: flat stream cut at arbitrary fragment boundaries, then reassembled
        stream = orc.pack(src, sslot, so, w)
        flat = stream.reshape(-1, w * D)
        pieces = [flat[i:i + 7] for i in range(0, flat.shape[0], 7)]
        again = np.concatenate(pieces).reshape(stream.shape)
        chunked = dst.copy()
        orc.unpack(np.ascontiguousarray(again), chunked, dslot, do)
        assert np.array_equal(whole, chunked)
