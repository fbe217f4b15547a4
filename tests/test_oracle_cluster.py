"""Virtual-GPU pins of the oracle: the TP1 -> TP2 -> TP4 example of the
paper's Fig. "KV Conversion" carried on to TP8 and back (Sec. 3.2.2 says the
same process reverses), checked per request against the KV the requests
started with: a value that never passes through the oracle."""
import numpy as np

from oracle import kvmig as orc
from workload import SplitMix64


def _build(G, H, L, D, S, ctx_of_req, rng):
    """TP1 (data parallel): request r lives on GPU r % G with all H heads."""
    truth = {}
    gpus = {}
    for g in range(G):
        gpus[g] = orc.VGpu(pool=np.full((L, 2, S, H, D), 0xDEAD, np.uint16))
    free = {g: list(rng.permutation(S)) for g in range(G)}
    home = {}
    for r, n in ctx_of_req.items():
        g = r % G
        kv = (rng.words(L * 2 * n * H * D) & np.uint64(0xFFFF)).astype(np.uint16).reshape(L, 2, n, H, D)
        truth[r] = kv
        slots = np.array([free[g].pop() for _ in range(n)], np.int32)
        gpus[g].slots[r] = slots
        gpus[g].pool[:, :, slots] = kv
        home[r] = g
    cl = orc.Cluster(L=L, H=H, D=D, S=S, dtype=np.uint16, groups=[[g] for g in range(G)],
                     home=home, ctx=dict(ctx_of_req), gpus=gpus)
    return cl, truth


def _step(cl, new_groups, home_new, rng):
    free = {}

    def alloc(gpu, n):
        if gpu not in free:
            free[gpu] = list(rng.permutation(cl.S))
        return [free[gpu].pop() for _ in range(n)]

    def sentinel(gpu, shape):
        return np.full(shape, 0xBEEF, np.uint16)

    return orc.transition(cl, new_groups, home_new, alloc, sentinel)


def _check(cl, truth):
    # per request: reassembled KV equals what the request started with
    for r, kv in truth.items():
        assert np.array_equal(cl.gather_request(r), kv), r
    # even head split and exactly-once placement
    live = 0
    for g, members in enumerate(cl.groups):
        for gpu in members:
            v = cl.gpus[gpu]
            assert v.pool.shape[3] == cl.H // len(members)
            used = np.concatenate([s for s in v.slots.values()]) if v.slots else np.zeros(0, np.int32)
            assert len(set(used.tolist())) == used.size
            mask = np.ones(cl.S, bool)
            mask[used] = False
            assert (v.pool[:, :, mask] == 0xBEEF).all() or (v.pool[:, :, mask] == 0xDEAD).all()
            live += used.size * cl.L * 2 * v.pool.shape[3] * cl.D
            assert set(v.slots) == {r for r, h in cl.home.items() if h == g}
    return live


def test_tp_round_trip_is_identity_and_conserves_kv():
    G, H, L, D, S = 8, 8, 2, 4, 40
    rng = SplitMix64(2024)
    ctx = {r: int(n) for r, n in enumerate(rng.integers(1, 4, 2 * G))}
    cl, truth = _build(G, H, L, D, S, ctx, rng)
    total = _check(cl, truth)
    first_home = dict(cl.home)

    def merged(groups_of):
        return [sum(([g for g in grp] for grp in chunk), []) for chunk in groups_of]

    plan = []
    # up: pair neighbouring groups; a request follows its GPU
    for size in (2, 4, 8):
        plan.append([list(range(i, i + size)) for i in range(0, G, size)])
    # down again
    for size in (4, 2, 1):
        plan.append([list(range(i, i + size)) for i in range(0, G, size)])
    for new_groups in plan:
        size = len(new_groups[0])
        # a request goes to the new group that contains the GPU it started on
        home_new = {r: first_home[r] // size for r in ctx}
        cl = _step(cl, new_groups, home_new, rng)
        assert _check(cl, truth) == total
    assert all(len(g) == 1 for g in cl.groups)
    for r in ctx:                                         # back on the original GPU, whole
        gpu = cl.groups[cl.home[r]][0]
        assert gpu == first_home[r]
        v = cl.gpus[gpu]
        assert np.array_equal(v.pool[:, :, v.slots[r]], truth[r])


def test_paper_example_four_gpus_eight_heads():
    """TP1 -> TP2 -> TP4 on four GPUs: after each step every GPU of a group
    holds H/N heads of all the group's requests."""
    G, H, L, D, S = 4, 8, 1, 2, 16
    rng = SplitMix64(7)
    ctx = {r: 2 + r for r in range(G)}
    cl, truth = _build(G, H, L, D, S, ctx, rng)
    cl = _step(cl, [[0, 1], [2, 3]], {0: 0, 1: 0, 2: 1, 3: 1}, rng)
    _check(cl, truth)
    # GPU-1 (index 0) now holds heads 0..3 of the requests of GPU-1 and GPU-2
    for r in (0, 1):
        v = cl.gpus[0]
        assert np.array_equal(v.pool[:, :, v.slots[r]], truth[r][:, :, :, 0:4])
        v = cl.gpus[1]
        assert np.array_equal(v.pool[:, :, v.slots[r]], truth[r][:, :, :, 4:8])
    cl = _step(cl, [[0, 1, 2, 3]], {r: 0 for r in range(G)}, rng)
    _check(cl, truth)
    for gpu in range(4):
        v = cl.gpus[gpu]
        for r in range(G):
            assert np.array_equal(v.pool[:, :, v.slots[r]], truth[r][:, :, :, 2 * gpu:2 * gpu + 2])
