"""Pins for the oracle's gradient statistics (non-finite flag, global L2 norm of the unscaled gradients, clip factor)
and for the whole-step driver (skip semantics, independence from subgroup order and partition - Section 3.2
"Cache-Friendly Ordering": the order in which subgroups are processed does not change the result)."""
import numpy as np
import pytest

from paper_2509_02480_amd import workloads as W


def bits_of(x):
    return (np.asarray(x, np.float32).view(np.uint32) >> 16).astype(np.uint16)


@pytest.mark.parametrize("k", [0, 1, 5, 10])
def test_norm_of_ones_is_exact(oracle, k):
    n = 4 ** k
    s, f = oracle.grad_stats(np.full(n, 0x3F80, np.uint16), 1.0)
    assert s == float(n) and f == 0
    norm, coef, gmul = oracle.norm_finish(s, 1.0, 0.0)
    assert norm == np.float32(2 ** k) and coef == 1 and gmul == 1


def test_norm_known_vectors(oracle):
    s, _ = oracle.grad_stats(bits_of([3.0, -4.0]), 1.0)
    assert oracle.norm_finish(s, 1.0, 0.0)[0] == np.float32(5.0)
    s, _ = oracle.grad_stats(bits_of([2.0 ** -j for j in range(1, 20)]), 1.0)
    assert s == sum(4.0 ** -j for j in range(1, 20))           # exact in fp64
    s, f = oracle.grad_stats(np.zeros(100, np.uint16), 1.0)
    assert s == 0 and f == 0 and oracle.norm_finish(s, 1.0, 1.0)[0] == 0
    s, _ = oracle.grad_stats(np.zeros(0, np.uint16), 1.0)
    assert s == 0
    # 1 + 2 + ... pattern: sum of squares of 1..100 = 338350
    s, _ = oracle.grad_stats(bits_of(np.arange(1, 101)), 1.0)
    assert s == 338350.0


def test_norm_is_of_unscaled_gradients(oracle):
    rng = np.random.default_rng(0)
    g = bits_of(rng.standard_normal(10000) * 1e-3)
    gs = bits_of(((g.astype(np.uint32) << 16).view(np.float32)) * np.float32(65536.0))
    s1, _ = oracle.grad_stats(g, 1.0)
    s2, _ = oracle.grad_stats(gs, float(np.float32(1 / 65536.0)))
    assert s1 == s2
    # against fp64 numpy on the decoded values
    gd = (g.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    assert abs(s1 / np.dot(gd, gd) - 1) < 1e-13
    # accumulation across calls (subgroups) continues the same sum
    a, fa = oracle.grad_stats(g[:3000], 1.0)
    b, fb = oracle.grad_stats(g[3000:], 1.0, a, fa)
    assert b == s1


def test_norm_statistics_of_config_1():
    import oracle as orc
    g = np.empty(W.C1.sub_elems, np.uint16)
    W.fill_grads(W.C1, 0, 0, g)
    s, f = orc.grad_stats(g, 1.0)
    assert f == 0
    assert abs(np.sqrt(s) / 1.024 - 1) < 5e-3       # 1e-3 * sqrt(2^20); bf16 truncation lowers it by ~0.2 %


def test_flag_every_nonfinite_pattern(oracle):
    base = bits_of(np.linspace(-1, 1, 64))
    assert oracle.grad_stats(base, 1.0)[1] == 0
    assert oracle.grad_stats(np.array([0x7F7F, 0xFF7F, 0x0001, 0x8000], np.uint16), 1.0)[1] == 0
    for sign in (0, 0x8000):
        for mant in range(128):
            for pos in (0, 31, 63):
                g = base.copy()
                g[pos] = sign | 0x7F80 | mant
                assert oracle.grad_stats(g, 1.0)[1] == 1


def test_clip_coefficient(oracle):
    g = bits_of([3.0, 4.0])
    s, _ = oracle.grad_stats(g, 1.0)
    norm, coef, gmul = oracle.norm_finish(s, 1.0, 1.0)
    assert norm == 5 and abs(float(coef) - 1 / (5 + 1e-6)) < 1e-8 and gmul == coef
    assert abs(float(coef) * 5.0 - 1.0) < 1e-6           # clipped gradients have norm max_norm
    assert oracle.norm_finish(s, 1.0, 5.0)[1] == 1       # not above the bound: untouched
    assert oracle.norm_finish(s, 1.0, 10.0)[1] == 1
    assert oracle.norm_finish(s, 1.0, 0.0)[1] == 1 and oracle.norm_finish(s, 1.0, -1.0)[1] == 1
    n2, c2, g2 = oracle.norm_finish(s, 0.25, 1.0)        # gmul folds the unscale factor in
    assert g2 == np.float32(0.25) * c2


def _small_workload(n_sub=4, sub=3001, **kw):
    return W.Workload("t", n_sub=n_sub, sub_elems=sub, **kw)


def _state_bits(sgs):
    return [s[k].copy() for s in sgs for k in ("p", "m", "v", "p16")]


def test_skip_leaves_everything_untouched_and_step_count(oracle):
    wl = _small_workload()
    hp = oracle.HParams()
    sgs = W.host_subgroups(wl, warm=True)
    ref = W.host_subgroups(wl, warm=True)
    before = _state_bits(sgs)
    sgs[2]["g"][17] = 0x7F80
    applied, norm, flag, gmul = oracle.step(sgs, hp, 0)
    assert not applied and flag == 1
    after = _state_bits(sgs)
    assert all(np.array_equal(a, b) for a, b in zip(before, after))
    # the next (clean) step is the first applied one: same as never having seen the bad gradient
    sgs[2]["g"][17] = ref[2]["g"][17]
    a1 = oracle.step(sgs, hp, 0)
    a2 = oracle.step(ref, hp, 0)
    assert a1[0] and a2[0] and a1[1] == a2[1]
    assert all(np.array_equal(a, b) for a, b in zip(_state_bits(sgs), _state_bits(ref)))
    for bad in (0xFF80, 0x7FC0, 0x7FFF):
        sgs[0]["g"][0] = bad
        assert oracle.step(sgs, hp, 1)[0] is False


def test_order_and_partition_do_not_matter(oracle):
    hp = oracle.HParams()
    wl = _small_workload(n_sub=6, sub=2500, loss_scale=1024.0, max_norm=0.01)
    a = W.host_subgroups(wl, warm=True)
    b = W.host_subgroups(wl, warm=True)
    ra = oracle.step(a, hp, 3, wl.inv_scale, wl.max_norm)
    rb = oracle.step(b, hp, 3, wl.inv_scale, wl.max_norm, order=[5, 3, 1, 0, 2, 4])
    assert ra == rb and ra[0] and ra[3] < np.float32(wl.inv_scale)      # clip active
    assert all(np.array_equal(x, y) for x, y in zip(_state_bits(a), _state_bits(b)))
    # one subgroup holding the concatenation gives the same bits
    c = W.host_subgroups(wl, warm=True)
    one = [{k: np.concatenate([s[k] for s in c]) for k in ("p", "m", "v", "g", "p16")}]
    rc = oracle.step(one, hp, 3, wl.inv_scale, wl.max_norm)
    assert rc == ra
    for k in ("p", "m", "v", "p16"):
        assert np.array_equal(one[0][k], np.concatenate([s[k] for s in a]))


def test_step_equals_its_parts(oracle):
    # the driver is stats -> finish -> per-subgroup update with step = applied + 1
    hp = oracle.HParams()
    wl = _small_workload(n_sub=2, sub=1000, max_norm=0.01)
    a = W.host_subgroups(wl, warm=True)
    b = W.host_subgroups(wl, warm=True)
    applied, norm, flag, gmul = oracle.step(a, hp, 6, 1.0, wl.max_norm)
    s = f = 0
    for sg in b:
        s, f = oracle.grad_stats(sg["g"], 1.0, s, f)
    n2, c2, g2 = oracle.norm_finish(s, 1.0, wl.max_norm)
    for sg in b:
        oracle.adamw_f32(sg["p"], sg["m"], sg["v"], sg["g"], sg["p16"], hp, 7, g2)
    assert (norm, gmul) == (n2, g2)
    assert all(np.array_equal(x, y) for x, y in zip(_state_bits(a), _state_bits(b)))


def test_chunked_stats_match(oracle):
    rng = np.random.default_rng(5)
    g = bits_of(rng.standard_normal((1 << 21) + 777) * 1e-3)
    s1, f1 = oracle.grad_stats(g, 1.0)
    s2, f2 = oracle.grad_stats_chunked(g, 1.0)
    assert abs(s2 / s1 - 1) < 1e-13 and f1 == f2 == 0
    g[-1] = 0xFF80
    assert oracle.grad_stats_chunked(g, 1.0)[1] == 1


def test_a_norm_beyond_fp32_skips_the_step(oracle):
    """Finite gradients whose norm does not fit fp32: the clip factor would be 0 (or infinity would enter the
    moments), so the step is skipped like one with a non-finite gradient.  Worked by hand: the largest finite bf16
    value is (2 - 2^-7) * 2^127 = 3.39e38 = 0.9961 * FLT_MAX; one of them has the norm 3.39e38 (fits), two have
    sqrt(2) * 3.39e38 = 4.79e38 > FLT_MAX = 3.40e38 (does not)."""
    big = np.float32((2.0 - 2.0 ** -7) * 2.0 ** 127)
    assert bits_of([big])[0] == 0x7F7F

    def sub(gbits):
        n = len(gbits)
        return {"p": np.full(n, 0.5, np.float32), "m": np.zeros(n, np.float32), "v": np.zeros(n, np.float32),
                "g": np.asarray(gbits, np.uint16), "p16": np.full(n, 0x1234, np.uint16)}

    one = sub([0x7F7F, 0, 0])
    applied, norm, flag, _ = oracle.step([one], oracle.HParams(), 0, 1.0, 0.0)
    assert applied and flag == 0 and norm == big
    two = sub([0x7F7F, 0, 0x7F7F])
    before = {k: v.copy() for k, v in two.items()}
    applied, norm, flag, _ = oracle.step([two], oracle.HParams(), 0, 1.0, 1.0)
    assert not applied and flag == 1 and np.isinf(norm)
    assert all(np.array_equal(two[k], before[k]) for k in two)         # nothing touched
    # the bit test alone does not see it: neither gradient is non-finite
    assert oracle.grad_stats(two["g"], 1.0)[1] == 0
    # an unscale factor above 1 can take a single finite gradient out of range: 2^127 * 4
    up = sub([0x7F00, 0x3F80])
    applied, norm, flag, _ = oracle.step([up], oracle.HParams(), 0, 4.0, 0.0)
    assert not applied and flag == 1
    # and just inside the range nothing is flagged: 2^126 * 2 = 2^127
    ok = sub([0x7E80, 0])
    applied, norm, flag, _ = oracle.step([ok], oracle.HParams(), 0, 2.0, 0.0)
    assert applied and flag == 0 and norm == np.float32(2.0 ** 127)
