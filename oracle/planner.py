"""CPU oracle for the goodput-efficiency planner: TEST INFRASTRUCTURE ONLY.

Sec. 3.3.1 of the paper ("Distributed Serving Configuration"): per control
window the global scheduler (1) enumerates, per SLO tier k, the configurations
(TPi for prefill, TPj for decode) over a small TP set, balances prefill and
decode instances so that P*THP = D*THD, and scores each with the goodput
efficiency of Eq. 1,
      GE = min(P*THP, rps_k) / (P*TPi + D*TPj),
then (2) hands out the GPU pool greedily by the weighted score
      WGE = GE * rps_k / served_rps_k.
THP / THD are the profiled maximum prefill / decode request rates of one
instance at that TP level under the tier's TTFT / TPOT SLO.

The paper leaves the integer details open; this is the reading used (the same
in the library, listed in the design notes):
 R1  An allocation step is one *block* of a configuration: integers P, D >= 1
     with P, D <= max_inst whose stage rates are closest (smallest
     |P*THP - D*THD| / max of the two; ties: fewer instances P+D, then smaller P).
     A block serves min(P*THP, D*THD): both SLOs must hold for goodput.
 R2  Eq. 1 is evaluated as printed, on the block's P and D and with the tier's
     still unmet rate: GE = min(P*THP, unmet_k) / (P*TPi + D*TPj).  Only the
     prefill rate enters the numerator (the paper drops the decode rate once
     the stages are balanced); with integer P, D the balance is not exact, so
     the score of a block can exceed what it serves (R1) by the residual gap.
 R3  WGE weights by rps_k / served_k; a tier that has been given nothing yet
     (served_k = 0) outranks every tier that has, and among such tiers, and
     among equal scores, the order is larger GE, then lower tier index, then
     lower TPi, then lower TPj.
 R4  Each step gives one block to the best configuration whose block fits in
     the GPUs left, until no tier has unmet demand or no block fits.  A TP level
     with THP or THD equal to 0 cannot meet the SLO and is skipped.
Pins: tests/test_oracle_planner.py.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Sequence, Tuple

TP_LEVELS = (1, 2, 4, 8)


@dataclass
class Tier:
    rps: float
    thp: Sequence[float]     # per entry of TP_LEVELS
    thd: Sequence[float]


@dataclass
class Alloc:
    tier: int
    tp_prefill: int
    tp_decode: int
    P: int
    D: int
    gpus: int
    served: float


def balanced_block(thp: float, thd: float, max_inst: int = 8) -> Tuple[int, int]:
    """R1: the (P, D) whose prefill and decode rates are closest."""
    best = None
    for P in range(1, max_inst + 1):
        for D in range(1, max_inst + 1):
            a, b = P * thp, D * thd
            gap = abs(a - b) / max(a, b)
            key = (gap, P + D, P)
            if best is None or key < best[0]:
                best = (key, P, D)
    return best[1], best[2]


def goodput_efficiency(thp: float, tpi: int, thd: float, tpj: int, P: int, D: int, rps: float) -> float:
    """Eq. 1 as printed: the prefill rate of the block, capped by the tier's rate,
    per GPU of the block.  ``thd`` does not enter (it fixed P : D beforehand)."""
    del thd
    return min(P * thp, rps) / (P * tpi + D * tpj)


def plan(n_gpus: int, tiers: List[Tier], max_inst: int = 8) -> Tuple[List[Alloc], int]:
    served = [0.0] * len(tiers)
    left = n_gpus
    out: List[Alloc] = []
    while True:
        best = None
        for k, t in enumerate(tiers):
            unmet = t.rps - served[k]
            if unmet <= 0:
                continue
            for i, tpi in enumerate(TP_LEVELS):
                for j, tpj in enumerate(TP_LEVELS):
                    if t.thp[i] <= 0 or t.thd[j] <= 0:
                        continue
                    P, D = balanced_block(t.thp[i], t.thd[j], max_inst)
                    gpus = P * tpi + D * tpj
                    if gpus > left:
                        continue
                    ge = goodput_efficiency(t.thp[i], tpi, t.thd[j], tpj, P, D, unmet)
                    fresh = served[k] == 0.0
                    wge = ge if fresh else ge * (t.rps / served[k])
                    key = (1 if fresh else 0, wge, ge, -k, -i, -j)
                    if best is None or key > best[0]:
                        best = (key, k, tpi, tpj, P, D, gpus, min(min(P * t.thp[i], D * t.thd[j]), unmet))
        if best is None:
            return out, left
        _, k, tpi, tpj, P, D, gpus, got = best
        out.append(Alloc(k, tpi, tpj, P, D, gpus, got))
        served[k] += got
        left -= gpus
