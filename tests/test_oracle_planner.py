"""Pins of the goodput planner's oracle: Eq. 1 by hand, the balance rule by its
closed form, the greedy by a hand-worked run and by invariants / brute force."""
import itertools

import pytest

from oracle import planner as op


def test_eq1_hand_values():
    # one prefill instance at TP2 serving 6 req/s, two decode instances at TP1 serving 3 req/s each
    assert op.goodput_efficiency(6.0, 2, 3.0, 1, 1, 2, rps=100.0) == 6.0 / 4.0
    # the tier only sends 3 req/s: Eq. 1 caps the numerator at rps
    assert op.goodput_efficiency(6.0, 2, 3.0, 1, 1, 2, rps=3.0) == 3.0 / 4.0
    # Eq. 1 by hand on an unbalanced block (P*THP = 6 against D*THD = 3): the printed numerator
    # holds the prefill rate only, so the score is 6 / 3 GPUs although the block can serve only 3
    assert op.goodput_efficiency(6.0, 2, 3.0, 1, 1, 1, rps=100.0) == 6.0 / 3.0
    assert op.goodput_efficiency(6.0, 2, 3.0, 1, 1, 1, rps=4.0) == 4.0 / 3.0
    # ... and what such a block adds to its tier is the slower stage's rate (both SLOs must hold)
    allocs, left = op.plan(3, [op.Tier(100.0, [0, 6.0, 0, 0], [3.0, 0, 0, 0])], max_inst=1)
    assert [(a.P, a.D, a.gpus, a.served) for a in allocs] == [(1, 1, 3, 3.0)] and left == 0


def test_balanced_block_is_the_rate_ratio_when_it_is_integral():
    """P*THP = D*THD has the integer solution P:D = THD:THP in lowest terms."""
    assert op.balanced_block(6.0, 3.0) == (1, 2)
    assert op.balanced_block(4.0, 6.0) == (3, 2)
    assert op.balanced_block(5.0, 5.0) == (1, 1)
    assert op.balanced_block(1.0, 8.0) == (8, 1)
    # the instance limit binds: 8:1 is out of reach with four instances a side, 4:1 is the closest
    assert op.balanced_block(1.0, 8.0, 4) == (4, 1) and op.balanced_block(8.0, 1.0, 4) == (1, 4)
    # and when balanced, Eq. 1 without the rps cap equals 1 / (TPi/THP + TPj/THD)
    for thp, tpi, thd, tpj in [(6.0, 2, 3.0, 1), (4.0, 4, 6.0, 2), (5.0, 1, 5.0, 8)]:
        P, D = op.balanced_block(thp, thd)
        ge = op.goodput_efficiency(thp, tpi, thd, tpj, P, D, rps=1e9)
        assert ge == pytest.approx(1.0 / (tpi / thp + tpj / thd), rel=1e-12)


def test_balanced_block_brute_force_property():
    for thp, thd in itertools.product([1.0, 2.5, 3.0, 7.0, 10.0], repeat=2):
        P, D = op.balanced_block(thp, thd, 6)
        gap = abs(P * thp - D * thd) / max(P * thp, D * thd)
        for p, d in itertools.product(range(1, 7), repeat=2):
            g = abs(p * thp - d * thd) / max(p * thp, d * thd)
            assert gap <= g + 1e-15


def test_greedy_hand_worked_run():
    """Two tiers, 8 GPUs, only TP1 and TP2 feasible.
    tier 0: rps 10, THP = [4, 10], THD = [4, 10];  tier 1: rps 2, THP = [2, 0], THD = [2, 0].
    Blocks (all balanced 1:1): t0 TP1/TP1: 4 req/s on 2 GPUs (GE 2), t0 TP2/TP2: 10 on 4 (GE 2.5),
    t0 TP1/TP2 and TP2/TP1: 4 on 3 (GE 1.33); t1 TP1/TP1: 2 on 2 (GE 1).
    Step 1: both tiers fresh; best GE is t0 TP2/TP2 (2.5): serves 10, tier 0 done, 4 GPUs left.
    Step 2: tier 1 TP1/TP1: serves 2 on 2 GPUs, done.  2 GPUs stay free."""
    tiers = [op.Tier(10.0, [4, 10, 0, 0], [4, 10, 0, 0]), op.Tier(2.0, [2, 0, 0, 0], [2, 0, 0, 0])]
    allocs, left = op.plan(8, tiers)
    assert [(a.tier, a.tp_prefill, a.tp_decode, a.P, a.D, a.gpus, a.served) for a in allocs] == \
        [(0, 2, 2, 1, 1, 4, 10.0), (1, 1, 1, 1, 1, 2, 2.0)]
    assert left == 2


def test_weighted_greedy_hand_worked_order():
    """Sec. 3.3.1's weight, GE times the tier's rate over what it is already served, by hand.
    Only TP1 is feasible and every block is one prefill plus one decode instance (2 GPUs).
    Tier A: 100 req/s wanted, 10 per block, GE 5.  Tier B: 12 wanted, 4 per block, GE 2.
    Fresh tiers go first, best GE first: A, then B.  From then on A scores 5 * 100 / served_A and
    B scores 2 * 12 / served_B: with B at 4 served (score 6) A wins at 10, 20, ... 80 served
    (50, 25, 16.7, 12.5, 10, 8.3, 7.1, 6.25) and loses at 90 (5.56 < 6): B gets its second block
    (score drops to 3), A its tenth (done), B its third (done)."""
    tiers = [op.Tier(100.0, [10, 0, 0, 0], [10, 0, 0, 0]), op.Tier(12.0, [4, 0, 0, 0], [4, 0, 0, 0])]
    allocs, left = op.plan(26, tiers)
    assert [a.tier for a in allocs] == [0, 1] + [0] * 8 + [1, 0, 1] and left == 0
    assert all(a.gpus == 2 and (a.P, a.D) == (1, 1) for a in allocs)
    assert [a.served for a in allocs if a.tier == 1] == [4.0, 4.0, 4.0]
    # two blocks fewer: B's second block still comes before A's tenth
    allocs, left = op.plan(22, tiers)
    assert [a.tier for a in allocs] == [0, 1] + [0] * 8 + [1] and left == 0


def test_weighting_keeps_a_low_efficiency_tier_from_starving():
    """Without the rps/served weight the efficient tier would take every GPU."""
    tiers = [op.Tier(100.0, [10, 0, 0, 0], [10, 0, 0, 0]), op.Tier(100.0, [1, 0, 0, 0], [1, 0, 0, 0])]
    allocs, left = op.plan(20, tiers)
    served = [sum(a.served for a in allocs if a.tier == k) for k in (0, 1)]
    assert served[1] > 0 and served[0] > served[1] and left == 0
    # after every step the chosen tier was the one with the highest weighted score
    assert allocs[0].tier == 0 and allocs[1].tier == 1


def test_invariants_on_random_instances():
    from workload import SplitMix64
    rng = SplitMix64(11)
    for trial in range(40):
        n_t = 1 + trial % 4
        tiers = []
        for _ in range(n_t):
            u = rng.uniform(9)
            thp = [2 + 10 * u[0], 5 + 18 * u[1], (8 + 30 * u[2]) * (u[3] > 0.2), (12 + 50 * u[4]) * (u[3] > 0.5)]
            thd = [3 + 10 * u[5], 6 + 16 * u[6], 10 + 30 * u[7], 0.0]
            tiers.append(op.Tier(5 + 60 * u[8], thp, thd))
        G = 4 + 4 * (trial % 9)
        allocs, left = op.plan(G, tiers)
        assert left >= 0 and left + sum(a.gpus for a in allocs) == G
        for k, t in enumerate(tiers):
            s = sum(a.served for a in allocs if a.tier == k)
            assert s <= t.rps * (1 + 1e-12)
        for a in allocs:
            t = tiers[a.tier]
            i, j = op.TP_LEVELS.index(a.tp_prefill), op.TP_LEVELS.index(a.tp_decode)
            assert (a.P, a.D) == op.balanced_block(t.thp[i], t.thd[j])
            assert a.gpus == a.P * a.tp_prefill + a.D * a.tp_decode
            assert a.served <= min(a.P * t.thp[i], a.D * t.thd[j]) * (1 + 1e-12)
        # nothing that still fits and is still wanted was left undone
        for k, t in enumerate(tiers):
            unmet = t.rps - sum(a.served for a in allocs if a.tier == k)
            if unmet > 1e-9:
                for i, j in itertools.product(range(4), repeat=2):
                    if t.thp[i] > 0 and t.thd[j] > 0:
                        P, D = op.balanced_block(t.thp[i], t.thd[j])
                        assert P * op.TP_LEVELS[i] + D * op.TP_LEVELS[j] > left


def test_single_tier_single_config_matches_brute_force():
    """One tier, one feasible configuration: the greedy must serve as much as any
    way of spending the GPUs on whole blocks can."""
    t = op.Tier(37.0, [0, 6, 0, 0], [3, 0, 0, 0])          # prefill TP2 at 6, decode TP1 at 3: block 1:2, 4 GPUs, 6 req/s
    for G in range(0, 30):
        allocs, left = op.plan(G, [t])
        best = min(37.0, 6.0 * (G // 4))
        assert sum(a.served for a in allocs) == pytest.approx(best)
        # levels with no throughput are never used: every block is the 4-GPU one, serves something,
        # and the GPUs that do not make up a block (or are not needed) stay free
        assert all(a.gpus == 4 and a.served > 0 for a in allocs) and left == G - 4 * len(allocs)
        assert len(allocs) == min(G // 4, 7)
