"""Planner instances chosen for what they tell apart (used by the library-vs-oracle tests of Sec. 3.3.1's planner,
through the C ABI and in the sanitizer build): tiers as (rps, THP per TP level, THD per TP level)."""

# Only TP1, blocks of one prefill and one decode instance.  Tier A: 100 req/s wanted, 10 per block; tier B: 12
# wanted, 4 per block.  After the two first (fresh) picks the order depends on the weight alone: A until it is
# served 90 of 100 (5 * 100 / 90 < 2 * 12 / 4), then B, A, B.  A sum or a product in place of the quotient, or
# no weight at all, orders these steps differently.
WEIGHTED = [(100.0, [10.0, 0.0, 0.0, 0.0], [10.0, 0.0, 0.0, 0.0]), (12.0, [4.0, 0.0, 0.0, 0.0], [4.0, 0.0, 0.0, 0.0])]
WEIGHTED_ORDER_26 = [0, 1] + [0] * 8 + [1, 0, 1]

# Rates below one request per second are rates like any other.
FRACTIONAL = [(3.0, [0.5, 0.9, 0.0, 0.0], [0.25, 1.0, 0.0, 0.0]), (0.75, [0.0, 0.3, 0.6, 0.0], [0.1, 0.0, 0.0, 1.0])]

# Three tiers that stay unmet for many steps, so that most picks are between tiers already served.
LONG_RUN = [(500.0, [3.0, 7.0, 16.0, 30.0], [5.0, 9.0, 20.0, 44.0]),
            (220.0, [1.5, 4.0, 7.0, 0.0], [2.0, 3.0, 9.0, 15.0]),
            (90.0, [0.0, 2.0, 5.0, 11.0], [1.0, 2.5, 0.0, 13.0])]

INSTANCES = [(26, WEIGHTED), (22, WEIGHTED), (7, WEIGHTED), (64, FRACTIONAL), (9, FRACTIONAL)] + \
            [(G, LONG_RUN) for G in (5, 40, 96, 128, 512)]

# each refused for one reason: a negative or NaN rate anywhere, first or last tier, first or last TP level
NAN = float("nan")
INVALID_TIERS = [
    [(-1.0, [1.0] * 4, [1.0] * 4), (5.0, [1.0] * 4, [1.0] * 4)],
    [(5.0, [1.0] * 4, [1.0] * 4), (NAN, [1.0] * 4, [1.0] * 4)],
    [(5.0, [-2.0, 1.0, 1.0, 1.0], [1.0] * 4)],
    [(5.0, [1.0] * 4, [1.0, 1.0, 1.0, -0.5])],
    [(5.0, [1.0] * 4, [NAN, 1.0, 1.0, 1.0])],
    [(5.0, [1.0] * 4, [1.0] * 4), (5.0, [1.0, 1.0, 1.0, -1.0], [1.0] * 4)],
]
