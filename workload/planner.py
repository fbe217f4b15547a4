"""Seeded synthetic tiers for the goodput planner: request rates and per-TP
prefill / decode capacity tables.  Real tables come from offline profiling of a
model on a GPU type (paper Sec. 3.3.1); those need trained weights, so these are
shaped stand-ins: capacity grows sub-linearly with the TP level, strict tiers
cannot meet their SLO at low TP (entry 0).  Input generation only."""
from __future__ import annotations

from typing import List, Tuple

from .splitmix import SplitMix64

Tier = Tuple[float, List[float], List[float]]


def synthetic_tiers(seed: int, n_tiers: int, rps_scale: float = 40.0) -> List[Tier]:
    rng = SplitMix64(seed)
    tiers: List[Tier] = []
    for k in range(n_tiers):
        u = rng.uniform(8)
        base_p, base_d = 3.0 + 9.0 * u[0], 4.0 + 10.0 * u[1]
        eff_p, eff_d = 0.70 + 0.25 * u[2], 0.55 + 0.30 * u[3]      # scaling efficiency per TP doubling
        strict = int(u[4] * 3)                                      # levels below this cannot meet the SLO
        thp = [0.0 if i < strict else base_p * (2 * eff_p) ** i for i in range(4)]
        thd = [0.0 if i < strict // 2 else base_d * (2 * eff_d) ** i for i in range(4)]
        if u[5] < 0.3:
            thd[3] = 0.0                                            # decode at TP8 not profiled / not worth it
        tiers.append((rps_scale * (0.2 + u[6]), thp, thd))
    return tiers
