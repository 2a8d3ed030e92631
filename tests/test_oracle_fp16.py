"""Pins for the oracle's FP16 forms (the paper allows FP16 or BF16 for gradients and working parameters, Section 2
"Mixed Precision Training", and writes FP16 in Algorithm 1): the two conversions against values built from the bit
fields, hand-worked cases, an exact nearest / ties-to-even property and two independent library conversions; the
non-finite test; AdamW, the gradient statistics and the accumulation through the same closed forms and brute-force
checks that pin the bf16 forms."""
import os
from bisect import bisect_left
from fractions import Fraction

import numpy as np
import pytest


def _f16_value_from_fields(bits):
    bits = bits.astype(np.int64)
    sign = np.where(bits >> 15, -1.0, 1.0)
    e = (bits >> 10) & 0x1F
    frac = bits & 0x3FF
    normal = np.ldexp(1.0 + frac / 1024.0, (e - 15).astype(np.int64))
    sub = np.ldexp(frac / 1024.0, -14)
    val = np.where(e == 0, sub, normal)
    val = np.where((e == 31) & (frac == 0), np.inf, val)
    val = np.where((e == 31) & (frac != 0), np.nan, val)
    return sign * val


ALL = np.arange(65536, dtype=np.uint32).astype(np.uint16)


def test_f16_to_f32_exhaustive(oracle):
    with np.errstate(invalid="ignore"):
        got = oracle.f16_to_f32(ALL).astype(np.float64)
    want = _f16_value_from_fields(ALL)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def test_rne_hand_cases(oracle):
    path = os.path.join(os.path.dirname(__file__), "golden", "f16_rne_cases.txt")
    rows = [ln.split("#")[0].split() for ln in open(path) if ln.split("#")[0].strip()]
    assert len(rows) >= 25
    src = np.array([int(r[0], 16) for r in rows], dtype=np.uint32).view(np.float32)
    want = [int(r[1], 16) for r in rows]
    assert [hex(x) for x in oracle.f32_to_f16_rne(src)] == [hex(x) for x in want]


def test_rne_round_trip_and_nearest(oracle):
    # every finite fp16 value survives the round trip, and a value strictly between two neighbours goes to the nearer
    finite = ALL[(ALL & 0x7C00) != 0x7C00]
    assert np.array_equal(oracle.f32_to_f16_rne(oracle.f16_to_f32(finite)), finite)
    grid = np.sort(_f16_value_from_fields(ALL[(ALL < 0x7C00)]))          # non-negative finite values, ascending
    rng = np.random.default_rng(3)
    x = np.concatenate([rng.uniform(0, 70000, 200_000), np.exp(rng.uniform(np.log(1e-9), np.log(7e4), 400_000)),
                        rng.uniform(0, 2.0 ** -13, 200_000)]).astype(np.float32)
    got = oracle.f16_to_f32(oracle.f32_to_f16_rne(x)).astype(np.float64)
    x64 = x.astype(np.float64)
    hi = np.searchsorted(grid, x64, side="left").clip(1, grid.size - 1)
    lo = hi - 1
    dl, dh = x64 - grid[lo], grid[hi] - x64
    inside = x64 < 65520.0
    nearer = np.where(dl < dh, grid[lo], grid[hi])
    tie = dl == dh
    exact = x64 == grid[hi]
    ok = np.where(exact, got == x64, np.where(tie, (got == grid[lo]) | (got == grid[hi]), got == nearer))
    assert ok[inside].all()
    assert np.isinf(got[~inside]).all()


def test_rne_against_two_libraries(oracle):
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(4)
    bits = rng.integers(0, 2 ** 32, 2_500_000, dtype=np.uint64).astype(np.uint32)
    x = bits.view(np.float32)
    got = oracle.f32_to_f16_rne(x)
    nan = np.isnan(x)
    with np.errstate(all="ignore"):
        ref_np = x.astype(np.float16).view(np.uint16)
    assert np.array_equal(got[~nan], ref_np[~nan])
    ref_t = torch.from_numpy(x.copy()).to(torch.float16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got[~nan], ref_t[~nan])
    assert np.all((got[nan] & 0x7FFF) == 0x7E00)
    assert np.array_equal(got[nan] >> 15, (bits[nan] >> 31).astype(np.uint16))


def test_every_non_finite_pattern_is_flagged(oracle):
    bad = [s | 0x7C00 | m for s in (0, 0x8000) for m in range(1024)]
    for pat in bad:
        g = np.array([0x3C00, pat, 0x0001], np.uint16)
        assert oracle.grad_stats(g, 1.0, half="fp16")[1] == 1, hex(pat)
    g = np.array([0x7BFF, 0xFBFF, 0x0000, 0x8000, 0x03FF], np.uint16)      # the largest finite values are not
    s, flag = oracle.grad_stats(g, 1.0, half="fp16")
    assert flag == 0 and s == 2 * 65504.0 ** 2 + (1023 * 2.0 ** -24) ** 2


def test_norm_exact_cases(oracle):
    ones = np.full(4 ** 8, 0x3C00, np.uint16)
    s, f = oracle.grad_stats(ones, 1.0, half="fp16")
    assert (s, f) == (float(4 ** 8), 0)
    assert oracle.norm_finish(s, 1.0, 0.0)[0] == np.float32(256.0)
    g = np.array([0x4200, 0x4400], np.uint16)                                # 3 and 4
    assert oracle.norm_finish(oracle.grad_stats(g, 1.0, half="fp16")[0], 1.0, 0.0)[0] == np.float32(5.0)
    # the same bits mean different numbers in the two formats
    assert oracle.grad_stats(g, 1.0, half="bf16")[0] != 25.0
    # unscaling: 2048 and 1024 under scale 1024 are 2 and 1
    g = np.array([0x6800, 0x6400], np.uint16)
    assert oracle.grad_stats(g, 1.0 / 1024.0, half="fp16")[0] == 5.0


def _hp(oracle, **kw):
    return oracle.HParams(**kw)


def test_adamw_step1_closed_form(oracle):
    # from m = v = 0 without decay the first step moves p by -lr * g / (|g| + eps), whatever the gradient's size
    hp = _hp(oracle, lr=1e-3, weight_decay=0.0, eps=1e-8)
    gvals = np.array([1.0, -1.0, 0.5, -2.0 ** -10, 3.0e-5, 65504.0, -6.0e-8, 2.0 ** -24], np.float32)
    g = oracle.f32_to_f16_rne(gvals)
    gf = oracle.f16_to_f32(g).astype(np.float64)
    p0 = np.linspace(-1, 1, g.size).astype(np.float32)
    p, m, v = p0.copy(), np.zeros_like(p0), np.zeros_like(p0)
    p16 = np.zeros(g.size, np.uint16)
    oracle.adamw_f32(p, m, v, g, p16, hp, 1, half="fp16")
    want = p0.astype(np.float64) - 1e-3 * gf / (np.abs(gf) + 1e-8)
    tol = np.spacing(np.maximum(np.abs(p0), np.abs(p)).astype(np.float32)).astype(np.float64) + 1e-6 * np.abs(want - p0)
    assert np.all(np.abs(p.astype(np.float64) - want) <= tol)
    assert np.array_equal(p16, oracle.f32_to_f16_rne(p))                     # the working copy is the rounded new p
    omb1, omb2 = 1.0 - float(np.float32(0.9)), 1.0 - float(np.float32(0.999))     # the betas are fp32 values
    assert np.allclose(m, omb1 * gf, rtol=1e-6, atol=0) and np.allclose(v, omb2 * gf * gf, rtol=1e-6, atol=0)


def test_adamw_matches_fp64_brute_force_and_differs_from_bf16(oracle):
    rng = np.random.default_rng(5)
    n = 64
    hp = _hp(oracle, lr=2e-3, weight_decay=0.01)
    g = oracle.f32_to_f16_rne((rng.standard_normal(n) * 1e-2).astype(np.float32))
    p = (rng.standard_normal(n) * 0.02).astype(np.float32)
    m = np.zeros(n, np.float32)
    v = np.zeros(n, np.float32)
    p64, m64, v64 = p.astype(np.float64), m.astype(np.float64), v.astype(np.float64)
    p16 = np.zeros(n, np.uint16)
    for t in range(1, 9):
        oracle.adamw_f32(p, m, v, g, p16, hp, t, half="fp16")
        oracle.adamw_f64(p64, m64, v64, g, hp, t, half="fp16")
    assert np.allclose(p, p64, rtol=2e-6, atol=1e-9) and np.allclose(v, v64, rtol=2e-6, atol=0)
    assert np.allclose(m, m64, rtol=1e-5, atol=1e-9)
    pb = (rng.standard_normal(n) * 0.02).astype(np.float32)
    q = pb.copy()
    mb, vb = np.zeros(n, np.float32), np.zeros(n, np.float32)
    oracle.adamw_f32(q, mb, vb, g, p16, hp, 1, half="bf16")                  # the same bits read as bf16: other numbers
    assert not np.allclose(mb, 0.1 * oracle.f16_to_f32(g), rtol=1e-3)


def test_power_of_two_loss_scale_is_neutral(oracle):
    rng = np.random.default_rng(6)
    n = 4096
    hp = _hp(oracle)
    small = oracle.f32_to_f16_rne((rng.standard_normal(n) * 1e-2).astype(np.float32))
    scaled = oracle.f32_to_f16_rne(oracle.f16_to_f32(small) * np.float32(256.0))      # exact: no overflow, normals
    assert np.array_equal(oracle.f16_to_f32(scaled), oracle.f16_to_f32(small) * np.float32(256.0))
    normal = (small & 0x7C00) != 0
    outs = []
    for g, inv in ((small, 1.0), (scaled, 1.0 / 256.0)):
        sub = [{"p": np.full(n, 0.5, np.float32), "m": np.zeros(n, np.float32), "v": np.zeros(n, np.float32),
                "g": g.copy(), "p16": np.zeros(n, np.uint16)}]
        assert oracle.step(sub, hp, 0, inv, 0.0, half="fp16")[0]
        outs.append(sub[0])
    for key in ("p", "m", "v", "p16"):
        assert np.array_equal(outs[0][key][normal], outs[1][key][normal]), key


def _value(bits):
    e = (bits >> 10) & 0x1F
    frac = bits & 0x3FF
    mag = Fraction(frac, 1024) * Fraction(2) ** -14 if e == 0 else (1 + Fraction(frac, 1024)) * Fraction(2) ** (e - 15)
    return -mag if bits >> 15 else mag


_POS = [_value(b) for b in range(0x7C00)]


def _round(x):
    sign = 0x8000 if x < 0 else 0
    a = abs(x)
    if a >= 65520:
        return sign | 0x7C00
    hi = bisect_left(_POS, a)
    if hi == len(_POS):
        return sign | 0x7BFF
    if _POS[hi] == a:
        return sign | hi
    lo = hi - 1
    dl, dh = a - _POS[lo], _POS[hi] - a
    if dl != dh:
        return sign | (lo if dl < dh else hi)
    return sign | (lo if lo % 2 == 0 else hi)


def _exact_accumulate(a, g):
    nan_a, nan_g = (a & 0x7FFF) > 0x7C00, (g & 0x7FFF) > 0x7C00
    inf_a, inf_g = (a & 0x7FFF) == 0x7C00, (g & 0x7FFF) == 0x7C00
    if nan_a or nan_g or (inf_a and inf_g and a != g):
        return 0x7E00
    if inf_a:
        return a
    if inf_g:
        return g
    x = _value(a) + _value(g)
    if x == 0:
        return 0x8000 if (a == 0x8000 and g == 0x8000) else 0
    return _round(x)


def test_accumulate_is_the_correctly_rounded_exact_sum(oracle):
    rng = np.random.default_rng(7)
    special = [0x0000, 0x8000, 0x0001, 0x8001, 0x03FF, 0x0400, 0x3C00, 0x3BFF, 0x3C01, 0x1000, 0x1001, 0x6800, 0x6801,
               0x7BFF, 0xFBFF, 0x7800, 0x5C00, 0x7C00, 0xFC00, 0x7E00, 0xFE01]
    near = rng.integers(0x2000, 0x2C00, 150) | (rng.integers(0, 2, 150) << 15)
    wide = rng.integers(0, 0x10000, 100)
    pats = np.unique(np.concatenate([np.array(special), near, wide]).astype(np.uint16))
    a, g = np.meshgrid(pats, pats, indexing="ij")
    a0, g0 = a.ravel().copy(), g.ravel().copy()
    acc = a0.copy()
    oracle.grad_accumulate(acc, g0, False, half="fp16")
    bad = [(hex(int(x)), hex(int(y)), hex(int(z))) for x, y, z in zip(a0, g0, acc)
           if int(z) != _exact_accumulate(int(x), int(y))]
    assert not bad, bad[:5]
    # hand-worked: 2048 + 1 ties to 2048 (11 bits), 1 + 2^-11 ties to 1, overflow, inf - inf
    hand = [(0x6800, 0x3C00, 0x6800), (0x6801, 0x3C00, 0x6802), (0x3C00, 0x1000, 0x3C00), (0x7BFF, 0x7BFF, 0x7C00),
            (0x7C00, 0xFC00, 0x7E00), (0x0001, 0x0001, 0x0002), (0x3C00, 0xBC00, 0x0000)]
    acc = np.array([h[0] for h in hand], np.uint16)
    oracle.grad_accumulate(acc, np.array([h[1] for h in hand], np.uint16), False, half="fp16")
    assert [hex(x) for x in acc] == [hex(h[2]) for h in hand]
    first = ALL.copy()
    oracle.grad_accumulate(first, ALL[::-1].copy(), True, half="fp16")
    assert np.array_equal(first, ALL[::-1])
