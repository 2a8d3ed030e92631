"""Oracle for the subgroup-to-tier allocation of Section 3.3 (Eq. 1) - TEST INFRASTRUCTURE ONLY.

Eq. 1: T_i = ceil(M * B_i / sum_j B_j), with the T_i then corrected so that they sum to M.  The paper leaves the
correction open;
the reading taken (and written in the library's header) is: while there is a surplus, take one subgroup back from the
tier that would finish last, i.e. with the largest T_i / B_i; among equals from the tier with the lower bandwidth,
then the higher index.  Tiers with a capacity keep at most that many subgroups and Eq. 1 is applied again to the rest.
Exact rational arithmetic, plain loops.  Imports nothing from the product package."""
from __future__ import annotations

from fractions import Fraction
from math import ceil
from typing import List, Optional, Sequence


def _eq1(m: int, tiers: List[int], bw: Sequence[Fraction]) -> dict:
    total = sum(bw[i] for i in tiers)
    t = {i: ceil(Fraction(m) * bw[i] / total) for i in tiers}
    while sum(t.values()) > m:
        cand = [i for i in tiers if t[i] > 0]
        # finishing time first, then lower bandwidth, then higher index
        worst = max(cand, key=lambda i: (Fraction(t[i]) / bw[i], -bw[i], i))
        t[worst] -= 1
    return t


def assign_tiers(m: int, bandwidth: Sequence[float], capacity: Optional[Sequence[int]] = None):
    """Counts per tier and the tier of every subgroup id (slower tiers take the lower ids)."""
    n = len(bandwidth)
    bw = [Fraction(b) for b in bandwidth]          # the exact value of each double
    count = [0] * n
    live = list(range(n))
    left = m
    while left > 0:
        if not live:
            raise MemoryError("capacities too small")
        trial = _eq1(left, live, bw)
        over = [i for i in live if capacity is not None and capacity[i] >= 0 and trial[i] > capacity[i]]
        if over:
            for i in over:
                count[i] = capacity[i]
                left -= capacity[i]
                live.remove(i)
        else:
            for i in live:
                count[i] = trial[i]
            left = 0
    order = sorted(range(n), key=lambda i: (bw[i], -i))     # slowest first; among equals the higher index first
    tier_of = [i for i in order for _ in range(count[i])]
    return count, tier_of


def update_bandwidth(bandwidth: Sequence[float], bytes_moved: Sequence[float], seconds: Sequence[float]):
    """Section 3.3: after an iteration B_i becomes the observed average, bytes / time; idle tiers keep theirs."""
    return [bm / s if bm > 0 and s > 0 else b for b, bm, s in zip(bandwidth, bytes_moved, seconds)]
