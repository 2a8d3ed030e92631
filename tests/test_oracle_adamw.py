"""Pins for the oracle's AdamW step (Algorithm 1's per-subgroup update; Adam named in Section 3.2 "Cache-Friendly
Ordering").  None of them re-types the oracle's fp32 sequence: they are closed forms, invariants, an all-fp64 brute
force, and PyTorch's own optimizer as an independent third opinion."""
import numpy as np
import pytest


def bf16_bits(x):
    """bf16 patterns of values that are exactly representable (or just truncated): test inputs only."""
    return (np.asarray(x, np.float32).view(np.uint32) >> 16).astype(np.uint16)


def bf16_val(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32)


def fresh(n, rng, p_std=0.02):
    p = (rng.standard_normal(n) * p_std).astype(np.float32)
    return p, np.zeros(n, np.float32), np.zeros(n, np.float32), np.zeros(n, np.uint16)


def test_step1_closed_form(oracle):
    # from m = v = 0, wd = 0, step 1 with bias correction: delta p = -lr * g / (|g| + eps)
    rng = np.random.default_rng(1)
    n = 4096
    hp = oracle.HParams(lr=1e-4, weight_decay=0.0)
    g = bf16_bits(rng.standard_normal(n) * 1e-3)
    # include gradients of eps' own magnitude so the placement of eps matters, and exact zeros
    g[:8] = bf16_bits(np.array([1e-8, -1e-8, 3e-8, -2e-9, 1e-7, 0.0, -0.0, 1e-10], np.float32))
    gd = bf16_val(g).astype(np.float64)
    want_dp = -float(np.float32(1e-4)) * gd / (np.abs(gd) + float(np.float32(1e-8)))
    # (a) p = 0: the new p is the update itself
    p, m, v, p16 = fresh(n, rng)
    p[:] = 0
    oracle.adamw_f32(p, m, v, g, p16, hp, 1)
    assert np.allclose(p, want_dp, rtol=1e-6, atol=1e-30)
    assert abs(p[0] / -5e-5 - 1) < 0.02 and p[5] == 0 and p[6] == 0   # |g| = eps halves the step; g = 0 gives none
    # (b) random p: within an ulp of the larger of old and new p, plus the rounding of the update itself
    p, m, v, p16 = fresh(n, rng)
    p0 = p.astype(np.float64)
    oracle.adamw_f32(p, m, v, g, p16, hp, 1)
    ulp = np.spacing(np.maximum(np.abs(p0), np.abs(p)).astype(np.float32)).astype(np.float64)
    assert np.all(np.abs(p - (p0 + want_dp)) <= ulp + 1e-6 * np.abs(want_dp))
    # |g| >> eps: a step of lr against the sign of g
    big = np.abs(gd) > 1e-5
    assert np.allclose((p - p0)[big], -1e-4 * np.sign(gd[big]), rtol=2e-3, atol=3e-9)


def test_constant_gradient_closed_form(oracle):
    # constant g from m = v = 0: m_t = (1-b1^t) g, v_t = (1-b2^t) g^2, so every Adam term is c = lr g/(|g|+eps) and
    # p_t = decay^t p_0 - c (1 - decay^t)/(1 - decay)
    hp = oracle.HParams(lr=1e-3, weight_decay=0.1)
    lr, wd, b1, b2, eps = (float(np.float32(x)) for x in (1e-3, 0.1, 0.9, 0.999, 1e-8))
    gvals = np.array([0.5, -0.25, 2 ** -10, -3 * 2 ** -12, 1.0, -1.0], np.float32)
    g = bf16_bits(gvals)
    gd = gvals.astype(np.float64)
    p0 = np.array([0.3, -0.2, 0.01, 0.5, -1.0, 0.0], np.float32)
    p, m, v, p16 = p0.copy(), np.zeros(6, np.float32), np.zeros(6, np.float32), np.zeros(6, np.uint16)
    decay = 1 - lr * wd
    c = lr * gd / (np.abs(gd) + eps)
    for t in range(1, 41):
        oracle.adamw_f32(p, m, v, g, p16, hp, t)
        assert np.allclose(m, (1 - b1 ** t) * gd, rtol=2e-6)
        assert np.allclose(v, (1 - b2 ** t) * gd * gd, rtol=2e-5)
        want = decay ** t * p0.astype(np.float64) - c * (1 - decay ** t) / (1 - decay)
        assert np.allclose(p, want, rtol=1e-5, atol=1e-7), t


def test_zero_gradient_invariants(oracle):
    rng = np.random.default_rng(2)
    n = 1000
    p, m, v, p16 = fresh(n, rng)
    g = np.zeros(n, np.uint16)
    p0 = p.copy()
    hp0 = oracle.HParams(weight_decay=0.0)
    for t in range(1, 6):
        oracle.adamw_f32(p, m, v, g, p16, hp0, t)
    assert np.array_equal(p.view(np.uint32), p0.view(np.uint32))
    assert not m.any() and not v.any()
    # with decay: p_t = decay^t p_0 as an iterated fp32 product, state still zero
    hp = oracle.HParams(lr=1e-2, weight_decay=0.5)
    decay = np.float32(1 - float(np.float32(1e-2)) * float(np.float32(0.5)))
    want = p0.copy()
    for t in range(1, 6):
        oracle.adamw_f32(p, m, v, g, p16, hp, t)
        want = want * decay
    assert np.array_equal(p, want)
    assert abs(float(p[3]) / (float(p0[3]) * 0.995 ** 5) - 1) < 1e-6
    assert not m.any() and not v.any()


def test_sign_symmetry_bitwise(oracle):
    rng = np.random.default_rng(3)
    n = 2048
    hp = oracle.HParams()
    p, m, v, p16 = fresh(n, rng)
    m[:] = rng.standard_normal(n) * 3e-4
    v[:] = (rng.standard_normal(n) * 1e-3) ** 2
    g = bf16_bits(rng.standard_normal(n) * 1e-3)
    pn, mn, vn, p16n, gn = -p, -m, v.copy(), p16.copy(), g ^ np.uint16(0x8000)
    for t in range(1, 4):
        oracle.adamw_f32(p, m, v, g, p16, hp, t)
        oracle.adamw_f32(pn, mn, vn, gn, p16n, hp, t)
    assert np.array_equal((-pn).view(np.uint32), p.view(np.uint32))
    assert np.array_equal((-mn).view(np.uint32), m.view(np.uint32))
    assert np.array_equal(vn.view(np.uint32), v.view(np.uint32))
    assert np.array_equal(p16n ^ np.uint16(0x8000), p16)


def test_power_of_two_loss_scale_is_bitwise_neutral(oracle):
    rng = np.random.default_rng(4)
    n = 2048
    hp = oracle.HParams()
    p, m, v, p16 = fresh(n, rng)
    gv = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    g = bf16_bits(gv)
    gs = bf16_bits(bf16_val(g) * np.float32(1024.0))   # exact: exponent shift
    p2, m2, v2, p162 = p.copy(), m.copy(), v.copy(), p16.copy()
    for t in range(1, 4):
        oracle.adamw_f32(p, m, v, g, p16, hp, t, gmul=1.0)
        oracle.adamw_f32(p2, m2, v2, gs, p162, hp, t, gmul=1.0 / 1024.0)
    for a, b in ((p, p2), (m, m2), (v, v2)):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    assert np.array_equal(p16, p162)


def _run_both(oracle, hp, n, steps, seed, gmul=1.0):
    rng = np.random.default_rng(seed)
    p, m, v, p16 = fresh(n, rng)
    pd, md, vd = p.astype(np.float64), m.astype(np.float64), v.astype(np.float64)
    for t in range(1, steps + 1):
        g = bf16_bits(rng.standard_normal(n) * 1e-3)
        oracle.adamw_f32(p, m, v, g, p16, hp, t, gmul)
        oracle.adamw_f64(pd, md, vd, g, hp, t, float(np.float32(gmul)))
    return (p, m, v, p16), (pd, md, vd)


@pytest.mark.parametrize("hp_kw", [dict(), dict(weight_decay=0.0), dict(bias_correction=False),
                                   dict(lr=3e-3, beta1=0.8, beta2=0.95, eps=1e-6, weight_decay=0.1)])
def test_fp32_tracks_fp64_brute_force(oracle, hp_kw):
    hp = oracle.HParams(**hp_kw)
    (p, m, v, _), (pd, md, vd) = _run_both(oracle, hp, 64, 10, 5)
    # v and p: a few fp32 ulp per step; m cancels, so its error is measured against the size of its terms
    assert np.allclose(v, vd, rtol=2e-6, atol=1e-30)
    assert np.allclose(p, pd, rtol=2e-6, atol=1e-9)
    assert np.all(np.abs(m - md) <= 1e-6 * 1e-3)


def test_gmul_scales_the_gradient(oracle):
    # a clip/unscale factor must act on g before both moments: halving g via gmul equals feeding g/2
    rng = np.random.default_rng(6)
    n = 512
    hp = oracle.HParams()
    p, m, v, p16 = fresh(n, rng)
    g = bf16_bits(rng.standard_normal(n) * 1e-3)
    gh = bf16_bits(bf16_val(g) * np.float32(0.5))
    p2, m2, v2, p162 = p.copy(), m.copy(), v.copy(), p16.copy()
    oracle.adamw_f32(p, m, v, g, p16, hp, 1, gmul=0.5)
    oracle.adamw_f32(p2, m2, v2, gh, p162, hp, 1, gmul=1.0)
    assert np.array_equal(p, p2) and np.array_equal(m, m2) and np.array_equal(v, v2)
    assert np.allclose(m, 0.1 * 0.5 * bf16_val(g), rtol=1e-6)
    assert np.allclose(v, 0.001 * (0.5 * bf16_val(g).astype(np.float64)) ** 2, rtol=1e-5)


@pytest.mark.parametrize("hp_kw", [dict(), dict(lr=3e-3, beta1=0.8, beta2=0.95, eps=1e-6, weight_decay=0.1)])
def test_against_torch_adamw(oracle, hp_kw):
    """PyTorch's AdamW (a library routine the oracle does not call) on the same inputs, in fp64 against the fp64 brute
    force (tight) and in fp32 against the fp32 routine (its operation order differs: tolerance, not bits)."""
    torch = pytest.importorskip("torch")
    hp = oracle.HParams(**hp_kw)
    n, steps = 256, 8
    for dtype, tol in ((torch.float64, 1e-12), (torch.float32, 3e-6)):
        rng = np.random.default_rng(11)
        p, m, v, p16 = fresh(n, rng)
        pd, md, vd = p.astype(np.float64), m.astype(np.float64), v.astype(np.float64)
        tp = torch.tensor(p, dtype=dtype, requires_grad=True)
        opt = torch.optim.AdamW([tp], lr=float(np.float32(hp.lr)), betas=(float(np.float32(hp.beta1)),
                                float(np.float32(hp.beta2))), eps=float(np.float32(hp.eps)),
                                weight_decay=float(np.float32(hp.weight_decay)), foreach=False, fused=False)
        for t in range(1, steps + 1):
            g = bf16_bits(rng.standard_normal(n) * 1e-3)
            tp.grad = torch.tensor(bf16_val(g), dtype=dtype)
            opt.step()
            oracle.adamw_f32(p, m, v, g, p16, hp, t)
            oracle.adamw_f64(pd, md, vd, g, hp, t)
        st = opt.state[tp]
        ours = (pd, md, vd) if dtype == torch.float64 else (p, m, v)
        assert np.allclose(ours[0], tp.detach().numpy(), rtol=tol, atol=tol * 1e-3)
        assert np.allclose(ours[1], st["exp_avg"].numpy(), rtol=max(tol, 1e-12), atol=tol * 1e-3)
        assert np.allclose(ours[2], st["exp_avg_sq"].numpy(), rtol=tol, atol=1e-30)


def test_p16_is_rne_of_new_p(oracle):
    # the working copy is the rounding of the *new* master value; checked with torch's conversion
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(8)
    n = 5000
    p, m, v, p16 = fresh(n, rng)
    g = bf16_bits(rng.standard_normal(n) * 1e-3)
    oracle.adamw_f32(p, m, v, g, p16, oracle.HParams(), 1)
    want = torch.from_numpy(p).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(p16, want)


def test_consts_are_rounded_once_from_fp64(oracle):
    hp = oracle.HParams()
    c = oracle.adamw_consts(hp, 3)
    b1, b2, lr, wd = (float(np.float32(x)) for x in (0.9, 0.999, 1e-4, 0.01))
    assert c["omb1"] == np.float32(1 - b1) and c["omb2"] == np.float32(1 - b2)
    assert c["step_size"] == np.float32(lr / (1 - b1 ** 3))
    assert c["sqbc2"] == np.float32(np.sqrt(1 - b2 ** 3))
    assert c["decay"] == np.float32(1 - lr * wd)
    c0 = oracle.adamw_consts(oracle.HParams(bias_correction=False), 3)
    assert c0["step_size"] == np.float32(lr) and c0["sqbc2"] == np.float32(1.0)


def test_chunked_driver_is_bitwise_the_plain_routine(oracle):
    rng = np.random.default_rng(9)
    n = (1 << 21) + 12345
    p, m, v, p16 = fresh(n, rng)
    g = bf16_bits(rng.standard_normal(n) * 1e-3)
    p2, m2, v2, p162 = p.copy(), m.copy(), v.copy(), p16.copy()
    oracle.adamw_f32(p, m, v, g, p16, oracle.HParams(), 2)
    oracle.adamw_f32(p2, m2, v2, g, p162, oracle.HParams(), 2, chunked=True)
    assert np.array_equal(p, p2) and np.array_equal(m, m2) and np.array_equal(v, v2) and np.array_equal(p16, p162)


# ---- the other textbook form: Adam with the decay term added to the gradient (l2_mode) -------------------------------

def test_l2_mode_step1_closed_form_and_what_tells_it_from_adamw(oracle):
    # from m = v = 0 the first step moves p by -lr * g' / (|g'| + eps) with g' = g + wd * p
    rng = np.random.default_rng(21)
    n = 2048
    wd = 0.1
    hp = oracle.HParams(lr=1e-3, weight_decay=wd, l2_mode=True)
    g = bf16_bits(rng.standard_normal(n) * 1e-3)
    g[:4] = 0                                                   # no gradient at all: only the decay term acts
    p, m, v, p16 = fresh(n, rng)
    p0 = p.astype(np.float64)
    gd = bf16_val(g).astype(np.float64) + float(np.float32(wd)) * p0
    oracle.adamw_f32(p, m, v, g, p16, hp, 1)
    want = p0 - float(np.float32(1e-3)) * gd / (np.abs(gd) + float(np.float32(1e-8)))
    ulp = np.spacing(np.maximum(np.abs(p0), np.abs(p)).astype(np.float32)).astype(np.float64)
    assert np.all(np.abs(p - want) <= ulp + 2e-6 * np.abs(want - p0))
    # with g = 0 Adam-with-L2 takes a full step of lr towards zero; AdamW only shrinks p by lr * wd * p
    assert np.allclose((p - p0)[:4], -1e-3 * np.sign(p0[:4]), rtol=1e-3)
    q, m2, v2, q16 = p0.astype(np.float32), np.zeros(n, np.float32), np.zeros(n, np.float32), np.zeros(n, np.uint16)
    oracle.adamw_f32(q, m2, v2, g, q16, oracle.HParams(lr=1e-3, weight_decay=wd), 1)
    assert np.allclose((q - p0)[:4], -1e-3 * wd * p0[:4], rtol=1e-3, atol=0)
    assert not m2[:4].any() and m[:4].all()                     # the decay enters the moments only in l2_mode


def test_l2_mode_without_decay_is_adamw_bitwise(oracle):
    rng = np.random.default_rng(22)
    n = 5000
    outs = []
    for l2 in (False, True):
        r = np.random.default_rng(23)
        p, m, v, p16 = fresh(n, r)
        hp = oracle.HParams(weight_decay=0.0, l2_mode=l2)
        for t in range(1, 5):
            g = bf16_bits(np.random.default_rng(100 + t).standard_normal(n) * 1e-3)
            oracle.adamw_f32(p, m, v, g, p16, hp, t)
        outs.append((p, m, v, p16))
    for a, b in zip(*outs):
        assert np.array_equal(a, b)
    assert rng is not None


@pytest.mark.parametrize("hp_kw", [dict(weight_decay=0.01), dict(lr=3e-3, beta1=0.8, beta2=0.95, eps=1e-6,
                                                               weight_decay=0.1)])
def test_l2_mode_against_torch_adam(oracle, hp_kw):
    """PyTorch's Adam with weight_decay (the decay term added to the gradient) in fp64 against the fp64 brute force
    (tight) and in fp32 against the fp32 routine (operation order differs: tolerance, not bits)."""
    torch = pytest.importorskip("torch")
    hp = oracle.HParams(l2_mode=True, **hp_kw)
    n, steps = 256, 8
    for dtype, tol in ((torch.float64, 1e-12), (torch.float32, 3e-6)):
        rng = np.random.default_rng(12)
        p, m, v, p16 = fresh(n, rng)
        pd, md, vd = p.astype(np.float64), m.astype(np.float64), v.astype(np.float64)
        tp = torch.tensor(p, dtype=dtype, requires_grad=True)
        opt = torch.optim.Adam([tp], lr=float(np.float32(hp.lr)), betas=(float(np.float32(hp.beta1)),
                               float(np.float32(hp.beta2))), eps=float(np.float32(hp.eps)),
                               weight_decay=float(np.float32(hp.weight_decay)), foreach=False, fused=False)
        for t in range(1, steps + 1):
            g = bf16_bits(rng.standard_normal(n) * 1e-3)
            tp.grad = torch.tensor(bf16_val(g), dtype=dtype)
            opt.step()
            oracle.adamw_f32(p, m, v, g, p16, hp, t)
            oracle.adamw_f64(pd, md, vd, g, hp, t)
        st = opt.state[tp]
        ours = (pd, md, vd) if dtype == torch.float64 else (p, m, v)
        assert np.allclose(ours[0], tp.detach().numpy(), rtol=tol, atol=tol * 1e-3)
        assert np.allclose(ours[1], st["exp_avg"].numpy(), rtol=max(tol, 1e-12), atol=tol * 1e-3)
        assert np.allclose(ours[2], st["exp_avg_sq"].numpy(), rtol=tol, atol=1e-30)
