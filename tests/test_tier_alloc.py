"""Eq. 1 (Section 3.3): the oracle against the paper's stated split, invariants and a brute-force optimum; then the
library's host routine against the oracle, exactly (integers)."""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import tier_alloc as O
from paper_2509_02480_amd import binding as B


def test_paper_two_to_one_split():
    path = os.path.join(os.path.dirname(__file__), "golden", "eq1_tier_split.txt")
    rows = [ln.split() for ln in open(path) if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 2
    for m, b0, b1, t0, t1 in rows:
        count, tier_of = O.assign_tiers(int(m), [float(b0), float(b1)])
        assert count == [int(t0), int(t1)]
        assert tier_of == [1, 0, 0]          # the slower path takes the lowest id


def makespan(count, bw):
    return max(Fraction(c) / Fraction(b) for c, b in zip(count, bw))


def test_oracle_minimises_the_finishing_time_brute_force():
    # Eq. 1 bounds every tier by the ceiling of its proportional share; among all allocations within those bounds
    # that sum to M (found by enumeration) the adjusted result has the smallest finishing time max_i T_i / B_i
    rng = np.random.default_rng(0)
    for _ in range(300):
        n = int(rng.integers(1, 4))
        m = int(rng.integers(0, 13))
        bw = [float(x) for x in rng.integers(1, 9, size=n)]
        count, _ = O.assign_tiers(m, bw)
        assert sum(count) == m and min(count) >= 0
        tot = sum(Fraction(b) for b in bw)
        ceil_share = [-(-Fraction(m) * Fraction(b) // tot) for b in bw]
        assert all(c <= u for c, u in zip(count, ceil_share))
        best = min(makespan(c, bw) for c in itertools.product(*(range(int(u) + 1) for u in ceil_share))
                   if sum(c) == m)
        assert makespan(count, bw) == best, (m, bw, count)


def test_oracle_special_cases():
    assert O.assign_tiers(10, [7.0])[0] == [10]
    assert O.assign_tiers(0, [1.0, 2.0])[0] == [0, 0]
    assert O.assign_tiers(12, [1.0, 1.0, 1.0])[0] == [4, 4, 4]
    assert O.assign_tiers(35, [1.0, 1.0])[0] == [18, 17]
    assert O.assign_tiers(9, [2.0, 1.0])[0] == [6, 3]                       # exact proportions need no adjustment
    # a small fast tier: HBM holds 10 subgroups, the link path takes the rest (the 70 / 30 workload's split)
    count, tier_of = O.assign_tiers(35, [239.0, 4.14], [10, -1])
    assert count == [10, 25] and tier_of == [1] * 25 + [0] * 10
    assert O.assign_tiers(35, [239.0, 4.14])[0] == [35, 0]                  # with room, everything is resident
    assert O.assign_tiers(20, [3.0, 2.0, 1.0], [4, 4, -1])[0] == [4, 4, 12]
    with pytest.raises(MemoryError):
        O.assign_tiers(20, [3.0, 2.0], [4, 4])
    assert O.update_bandwidth([5.3, 3.6], [10e9, 0.0], [2.5, 0.0]) == [4e9, 3.6]


def test_bandwidth_update_follows_the_observations():
    # Section 3.3: the estimate of a path becomes what the last iteration showed; a path that moved nothing, or for
    # no measurable time, keeps its estimate.  A path seen at half its estimate gives up subgroups in the next split.
    bw = [48.0e9, 24.0e9]
    assert O.assign_tiers(30, bw)[0] == [20, 10]
    seen = O.update_bandwidth(bw, [12.0e9, 12.0e9], [0.5, 0.5])
    assert seen == [24.0e9, 24.0e9] and O.assign_tiers(30, seen)[0] == [15, 15]
    assert O.update_bandwidth(bw, [0.0, 6.0e9], [1.0, 0.0]) == bw
    assert O.update_bandwidth([1.0, 2.0, 3.0], [10.0, 0.0, 9.0], [4.0, 5.0, 3.0]) == [2.5, 2.0, 3.0]
    # three paths, observed at the rates of Table 1's two paths and at their sum
    seen = O.update_bandwidth([1.0, 1.0, 1.0], [5.3e9, 3.6e9 * 2, 8.9e9 * 3], [1.0, 2.0, 3.0])
    assert seen == [5.3e9, 3.6e9, 8.9e9]
    assert O.assign_tiers(60, seen)[0] == [18, 12, 30]
    assert B.mlpo_update_bandwidth([1.0, 2.0, 3.0], [10.0, 0.0, 9.0], [4.0, 5.0, 3.0]) == [2.5, 2.0, 3.0]


def test_library_matches_oracle_exactly():
    rng = np.random.default_rng(1)
    for trial in range(400):
        n = int(rng.integers(1, 6))
        m = int(rng.integers(0, 200))
        bw = [float(x) for x in np.round(rng.uniform(0.1, 60.0, size=n), 3)]
        cap = None
        if trial % 3 == 0:
            cap = [int(x) for x in rng.integers(-1, m + 2, size=n)]
            if all(c >= 0 for c in cap) and sum(cap) < m:
                cap[int(rng.integers(0, n))] = -1
        want = O.assign_tiers(m, bw, cap)
        got = B.mlpo_assign_tiers(m, bw, cap)
        assert got[0] == want[0] and got[1] == want[1], (m, bw, cap, got, want)
    assert B.mlpo_update_bandwidth([5.3, 3.6], [10e9, 0.0], [2.5, 0.0]) == O.update_bandwidth([5.3, 3.6], [10e9, 0.0], [2.5, 0.0])


def test_library_takes_the_exact_ceiling_of_shares_next_to_an_integer():
    # Eq. 1's ceiling is of the exact quotient: a share a few 1e-13 above an integer rounds up, one as far below
    # stays.  Cases where an estimate with a tolerance ends with a different allocation, then random ones of the kind.
    cases = [(12, [2.0000000000002, 1.0, 4.0, 1.0], None, [4, 1, 6, 1]),
             (14, [3.0, 1.0, 8.0, 3.9999999999996], None, [3, 0, 8, 3]),
             (40, [9.0, 8.0, 6.0, 1.9999999999994], [10, 25, 33, 14], [10, 16, 11, 3]),
             (26, [3.0, 6.0, 2.9999999999994], [24, 15, 23], [6, 14, 6])]
    for m, bw, cap, want in cases:
        assert O.assign_tiers(m, bw, cap)[0] == want
        assert B.mlpo_assign_tiers(m, bw, cap)[0] == want, (m, bw, cap)
    rng = np.random.default_rng(7)
    for _ in range(3000):
        n = int(rng.integers(2, 6))
        m = int(rng.integers(1, 300))
        bw = [float(x) for x in rng.integers(1, 12, size=n)]
        j = int(rng.integers(0, n))
        bw[j] = float(np.nextafter(bw[j], [0.0, 100.0][int(rng.integers(0, 2))])) if rng.random() < 0.5 else \
            bw[j] * (1.0 + float(rng.integers(-9, 10)) * 1e-13)
        want = O.assign_tiers(m, bw)
        got = B.mlpo_assign_tiers(m, bw)
        assert got[0] == want[0] and got[1] == want[1], (m, bw, got, want)
    # bandwidths of very different size: the exact sum still decides
    for bw in ([1e-30, 3e-30], [1e30, 1.0], [4.14e9, 239e9, 3.7e9]):
        assert B.mlpo_assign_tiers(35, bw)[0] == O.assign_tiers(35, bw)[0]


def test_library_argument_errors():
    for bad in ([0.0, 1.0], [float("nan")], [-1.0, 2.0], [float("inf"), 1.0]):
        with pytest.raises(B.MlpoError) as e:
            B.mlpo_assign_tiers(5, bad)
        assert e.value.code == B.MLPO_EINVAL
    with pytest.raises(B.MlpoError) as e:
        B.mlpo_assign_tiers(20, [3.0, 2.0], [4, 4])
    assert e.value.code == B.MLPO_ENOMEM
    with pytest.raises(B.MlpoError):
        B.mlpo_update_bandwidth([1.0], [-1.0], [1.0])
