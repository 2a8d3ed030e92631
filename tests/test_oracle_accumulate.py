"""Pins for the oracle's gradient accumulation (the half-precision accumulation buffer of Section 3.2 "Delayed
In-place Mixed-Precision Gradient Conversion"): hand-worked bit patterns, the correctly rounded exact sum computed
with rationals (no floating point on the checking side), the stagnation point of a bf16 counter, commutativity, and
the copy semantics of the first micro-batch."""
import os
from bisect import bisect_left
from fractions import Fraction

import numpy as np


def _value(bits):
    """Exact value of a finite bf16 pattern as a rational."""
    e = (bits >> 7) & 0xFF
    mant = bits & 0x7F
    mag = Fraction(mant, 128) * Fraction(2) ** -126 if e == 0 else (1 + Fraction(mant, 128)) * Fraction(2) ** (e - 127)
    return -mag if bits >> 15 else mag


_POS = [_value(b) for b in range(0x7F80)]  # ascending: 0x0000 .. 0x7F7F
_HALF_TOP_ULP = Fraction(2) ** 119


def _round_to_bf16(x):
    """Nearest bf16 pattern of a non-zero rational, ties to the even pattern, overflow to infinity."""
    sign = 0x8000 if x < 0 else 0
    a = abs(x)
    if a >= _POS[-1] + _HALF_TOP_ULP:
        return sign | 0x7F80
    hi = bisect_left(_POS, a)
    if hi == len(_POS):
        return sign | 0x7F7F
    if _POS[hi] == a:
        return sign | hi
    lo = hi - 1
    dl, dh = a - _POS[lo], _POS[hi] - a
    if dl < dh:
        return sign | lo
    if dh < dl:
        return sign | hi
    return sign | (lo if lo % 2 == 0 else hi)


def _exact_accumulate(a, g):
    nan_a, nan_g = (a & 0x7FFF) > 0x7F80, (g & 0x7FFF) > 0x7F80
    inf_a, inf_g = (a & 0x7FFF) == 0x7F80, (g & 0x7FFF) == 0x7F80
    if nan_a or nan_g or (inf_a and inf_g and a != g):
        return 0x7FC0
    if inf_a:
        return a
    if inf_g:
        return g
    x = _value(a) + _value(g)
    if x == 0:
        return 0x8000 if (a == 0x8000 and g == 0x8000) else 0x0000
    return _round_to_bf16(x)


def test_hand_cases(oracle):
    path = os.path.join(os.path.dirname(__file__), "golden", "bf16_accumulate_cases.txt")
    rows = [ln.split("#")[0].split() for ln in open(path) if ln.split("#")[0].strip()]
    assert len(rows) >= 20
    acc = np.array([int(r[0], 16) for r in rows], np.uint16)
    g = np.array([int(r[1], 16) for r in rows], np.uint16)
    want = [int(r[2], 16) for r in rows]
    oracle.grad_accumulate(acc, g, first=False)
    assert [hex(x) for x in acc] == [hex(x) for x in want]
    # the checker used below agrees with the hand-worked rows too
    assert [hex(_exact_accumulate(int(r[0], 16), int(r[1], 16))) for r in rows] == [hex(x) for x in want]


def _patterns():
    rng = np.random.default_rng(20250902)
    special = [0x0000, 0x8000, 0x0001, 0x8001, 0x007F, 0x0080, 0x0081, 0x3F7F, 0x3F80, 0x3F81, 0x3B80, 0x3B7F, 0x3B81,
               0x4380, 0x4381, 0x7F7F, 0xFF7F, 0x7F7E, 0x7B00, 0x7A80, 0x7F80, 0xFF80, 0x7FC0, 0xFFC1, 0x7F81]
    # gradients of one scale (neighbouring exponents: cancellation and ties are common) and of any scale
    near = rng.integers(0x3A00, 0x3D00, 180) | (rng.integers(0, 2, 180) << 15)
    wide = rng.integers(0, 0x10000, 120)
    return np.unique(np.concatenate([np.array(special), near, wide]).astype(np.uint16))


def test_sum_is_the_correctly_rounded_exact_sum(oracle):
    pats = _patterns()
    a, g = np.meshgrid(pats, pats, indexing="ij")
    a0 = a.ravel().copy()
    gg = g.ravel().copy()
    acc = a0.copy()
    oracle.grad_accumulate(acc, gg, first=False)
    assert acc.size > 90_000
    bad = [(hex(int(x)), hex(int(y)), hex(int(z)), hex(_exact_accumulate(int(x), int(y))))
           for x, y, z in zip(a0, gg, acc) if int(z) != _exact_accumulate(int(x), int(y))]
    assert not bad, bad[:5]


def test_commutative_bitwise(oracle):
    rng = np.random.default_rng(7)
    a = rng.integers(0, 0x10000, 200_000).astype(np.uint16)
    g = rng.integers(0, 0x10000, 200_000).astype(np.uint16)
    x, y = a.copy(), g.copy()
    oracle.grad_accumulate(x, g, first=False)
    oracle.grad_accumulate(y, a, first=False)
    assert np.array_equal(x, y)


def test_first_micro_batch_overwrites(oracle):
    g = np.arange(65536, dtype=np.uint32).astype(np.uint16)  # every pattern, NaN payloads included
    acc = np.full(g.size, 0x7FC0, np.uint16)
    oracle.grad_accumulate(acc, g, first=True)
    assert np.array_equal(acc, g)


def test_bf16_counter_stops_at_256(oracle):
    one = np.full(3, 0x3F80, np.uint16)
    acc = np.zeros(3, np.uint16)
    seen = []
    for k in range(300):
        oracle.grad_accumulate(acc, one, first=(k == 0))
        seen.append(float(oracle.bf16_to_f32(acc)[0]))
    assert seen[:256] == [float(k + 1) for k in range(256)]  # exact while 8 bits suffice
    assert set(seen[256:]) == {256.0}  # 256 + 1 ties to even and the buffer no longer moves


def test_micro_batches_of_small_gradients_track_the_fp64_sum(oracle):
    # k micro-batches of gradients of one scale: the buffer stays within k half-ulps of the exact sum
    rng = np.random.default_rng(11)
    n, k = 50_000, 8
    exact = np.zeros(n)
    acc = np.zeros(n, np.uint16)
    for j in range(k):
        g = oracle.f32_to_bf16_rne((rng.standard_normal(n) * 1e-3).astype(np.float32))
        exact += oracle.bf16_to_f32(g).astype(np.float64)
        oracle.grad_accumulate(acc, g, first=(j == 0))
    got = oracle.bf16_to_f32(acc).astype(np.float64)
    # every partial sum is below 8 sigma * k in magnitude; each rounding errs by at most 2^-9 of the partial sum
    bound = (k - 1) * 2.0 ** -9 * np.maximum(np.abs(exact), 8e-3 * 1.0) + 1e-30
    assert np.all(np.abs(got - exact) <= bound)
    assert np.abs(got - exact).max() > 0  # it does round
