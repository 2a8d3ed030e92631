"""Pins for the oracle's two conversions (Section 2 "Mixed Precision Training"): the widening is checked against values
built with ldexp from the bit fields; the rounding against hand-worked cases, an exact nearest/ties-to-even property
evaluated in fp64, and an independent library conversion."""
import os

import numpy as np
import pytest


def _bf16_value_from_fields(bits):
    bits = bits.astype(np.int64)
    sign = np.where(bits >> 15, -1.0, 1.0)
    e = (bits >> 7) & 0xFF
    mant = bits & 0x7F
    normal = np.ldexp(1.0 + mant / 128.0, (e - 127).astype(np.int64))
    denorm = np.ldexp(mant / 128.0, -126)
    val = np.where(e == 0, denorm, normal)
    val = np.where((e == 255) & (mant == 0), np.inf, val)
    val = np.where((e == 255) & (mant != 0), np.nan, val)
    return sign * val


def test_bf16_to_f32_exhaustive(oracle):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    with np.errstate(invalid="ignore"):       # widening a signalling NaN pattern raises the flag, as it should
        got = oracle.bf16_to_f32(bits).astype(np.float64)
    want = _bf16_value_from_fields(bits)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def test_rne_hand_cases(oracle):
    path = os.path.join(os.path.dirname(__file__), "golden", "bf16_rne_cases.txt")
    rows = [ln.split("#")[0].split() for ln in open(path) if ln.split("#")[0].strip()]
    assert len(rows) >= 15
    src = np.array([int(r[0], 16) for r in rows], dtype=np.uint32).view(np.float32)
    want = np.array([int(r[1], 16) for r in rows], dtype=np.uint16)
    got = oracle.f32_to_bf16_rne(src)
    assert [hex(x) for x in got] == [hex(x) for x in want]


def _patterns():
    rng = np.random.default_rng(7)
    upper = np.arange(65536, dtype=np.uint32) << 16
    lows = np.array([0, 1, 0x7FFF, 0x8000, 0x8001, 0xFFFF, 0x4000, 0xC000], dtype=np.uint32)
    edge = (upper[:, None] | lows[None, :]).ravel()
    rnd = rng.integers(0, 1 << 32, size=2_000_000, dtype=np.uint64).astype(np.uint32)
    return np.concatenate([edge, rnd])


def test_rne_is_nearest_ties_even(oracle):
    w = _patterns()
    x = w.view(np.float32)
    finite = np.isfinite(x)
    w, x = w[finite], x[finite]
    got = oracle.f32_to_bf16_rne(x)
    xd = x.astype(np.float64)
    lo = (w >> 16).astype(np.uint16)            # truncation toward zero
    hi = (lo.astype(np.uint32) + 1).astype(np.uint16)  # next bf16 away from zero (may be inf)
    with np.errstate(over="ignore"):
        vlo = _bf16_value_from_fields(lo)
        # the round-up neighbour of the largest finite is treated as 2^128, as IEEE rounding does
        vhi = np.where((hi & 0x7FFF) == 0x7F80, np.sign(xd) * 2.0 ** 128, _bf16_value_from_fields(hi))
    dlo, dhi = np.abs(xd - vlo), np.abs(vhi - xd)
    want = np.where(dlo < dhi, lo, np.where(dhi < dlo, hi, np.where(lo & 1, hi, lo)))
    assert np.array_equal(got, want.astype(np.uint16))


def test_rne_matches_torch_library_conversion(oracle):
    torch = pytest.importorskip("torch")
    w = _patterns()
    x = w.view(np.float32)
    keep = ~np.isnan(x)
    x = np.ascontiguousarray(x[keep])
    got = oracle.f32_to_bf16_rne(x)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, want)


def test_rne_nan_is_canonical_quiet(oracle):
    w = np.array([0x7F800001, 0x7FFFFFFF, 0xFF800001, 0xFFC12345, 0x7F80FFFF], dtype=np.uint32)
    got = oracle.f32_to_bf16_rne(w.view(np.float32))
    assert [hex(v) for v in got] == ["0x7fc0", "0x7fc0", "0xffc0", "0xffc0", "0x7fc0"]


def test_roundtrip_identity_on_bf16_values(oracle):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    f = oracle.bf16_to_f32(bits)
    back = oracle.f32_to_bf16_rne(f)
    nan = np.isnan(f)
    assert np.array_equal(back[~nan], bits[~nan])
