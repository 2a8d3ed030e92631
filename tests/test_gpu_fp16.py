"""GPU parity with FP16 gradients and working parameters (the paper allows FP16 or BF16, Section 2 "Mixed Precision
Training", and writes FP16 in Algorithm 1) against the oracle's FP16 forms: whole steps with a loss scale, a clip and
an injected infinity, both layouts and the element-wise kernel; every finite gradient pattern; the downcast over all
2^32 fp32 patterns; the tiered pipeline; the accumulation.  Same bars as for bf16: flag and half-precision copy
bit-exact, fp32 state max relative error 1e-6 (observed: identical words), norm 1e-5."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2509_02480_amd import binding as B  # noqa: E402

from gpu_util import DeviceSubgroups, Scratch, assert_state_parity, dev, from_dev_u16, gpu_step, hp_pair  # noqa: E402

FP16 = B.HALF_FP16


def f16_bits(x):
    """fp16 bit patterns of an array, rounded by numpy (input preparation only)."""
    with np.errstate(over="ignore"):
        return np.asarray(x, dtype=np.float32).astype(np.float16).view(np.uint16).copy()


def make_host(rng, sizes, sigma, scale):
    host = []
    for n in sizes:
        host.append({"p": (rng.standard_normal(n) * 0.02).astype(np.float32),
                     "m": (rng.standard_normal(n) * 1e-4).astype(np.float32),
                     "v": ((rng.standard_normal(n) * 1e-3) ** 2).astype(np.float32),
                     "g": f16_bits(rng.standard_normal(n) * sigma * scale), "p16": np.zeros(n, np.uint16)})
    return host


@pytest.mark.parametrize("tile,flat,offset", [(0, True, 0), (0, True, 3), (0, False, 0), (B.TILE_DEFAULT, False, 0),
                                               (1024, False, 0)])
def test_steps_with_loss_scale_clip_and_injected_infinity(oracle, tile, flat, offset):
    ohp, ghp = hp_pair(oracle, lr=3e-4, weight_decay=0.01)
    rng = np.random.default_rng(tile + offset)
    sizes = [100_001, 64, 7, 262_144, 33_333]
    scale = 1024.0
    host = make_host(rng, sizes, 1e-3, scale)
    ds = DeviceSubgroups(host, flat=flat, elem_offset=offset, tile=tile, half=FP16)
    scratch = Scratch()
    applied = 0
    for s in range(5):
        if s > 0:
            for k, sg in enumerate(host):
                sg["g"][:] = f16_bits(rng.standard_normal(sg["g"].size) * 1e-3 * scale)
        if s == 2:
            host[3]["g"][12_345] = 0xFC00                                # -inf
        for k, sg in enumerate(host):
            ds.set_grads(k, sg["g"])
        ok_o, norm_o, flag_o, gmul_o = oracle.step(host, ohp, applied, 1.0 / scale, 0.02, half="fp16")
        ok_g, sc = gpu_step(ds, scratch, ghp, applied, 1.0 / scale, 0.02)
        assert ok_g == ok_o == (s != 2) and sc["found_inf"] == flag_o
        if ok_o:
            assert abs(float(sc["norm"]) - float(norm_o)) <= 1e-5 * float(norm_o) and sc["gmul"] == gmul_o
            applied += 1
        for k in range(len(sizes)):
            assert_state_parity(ds.fetch(k), host[k], f"tile={tile} step {s} sg {k}")
    assert applied == 4


def test_every_finite_gradient_pattern(oracle):
    # all 63 488 finite fp16 patterns (subnormals, both zeros, the largest values) against eight different states
    ohp, ghp = hp_pair(oracle)
    pats = np.array([b for b in range(65536) if (b & 0x7C00) != 0x7C00], dtype=np.uint16)
    rng = np.random.default_rng(5)
    reps = 8
    n = pats.size * reps
    base = {"p": (rng.standard_normal(n) * 0.02).astype(np.float32),
            "m": (rng.standard_normal(n) * 3e-4).astype(np.float32),
            "v": ((rng.standard_normal(n) * 1e-3) ** 2).astype(np.float32),
            "g": np.tile(pats, reps), "p16": np.zeros(n, np.uint16)}
    base["m"][:pats.size] = 0
    base["v"][:pats.size] = 0
    for tile in (0, B.TILE_DEFAULT):
        cur = [{k: a.copy() for k, a in base.items()}]
        ds = DeviceSubgroups(cur, tile=tile, half=FP16)
        oracle.adamw_f32(cur[0]["p"], cur[0]["m"], cur[0]["v"], cur[0]["g"], cur[0]["p16"], ohp, 3, 2.0 ** -7,
                         half="fp16")
        rec = torch.tensor([0.0, 1.0, 2.0 ** -7, 0.0], dtype=torch.float32, device=dev())
        B.mlpo_adamw_step(ds.table, ghp, 3, rec, torch.cuda.current_stream())
        got = ds.fetch(0)
        for key in ("p", "m", "v"):
            same = got[key].view(np.uint32) == cur[0][key].view(np.uint32)
            assert np.all(same | (np.isnan(got[key]) & np.isnan(cur[0][key]))), f"tile={tile} {key}"
        assert np.array_equal(got["p16"], cur[0]["p16"])


def test_every_non_finite_pattern_raises_the_flag(oracle):
    scratch = Scratch()
    bad = np.array([s | 0x7C00 | m for s in (0, 0x8000) for m in range(1024)], np.uint16)
    n = 50_000
    g = f16_bits(np.random.default_rng(1).standard_normal(n))
    host = [{"p": np.zeros(n, np.float32), "m": np.zeros(n, np.float32), "v": np.zeros(n, np.float32), "g": g,
             "p16": np.zeros(n, np.uint16)}]
    ds = DeviceSubgroups(host, half=FP16)
    positions = [0, 1, 7, 8, 4097, n - 1]
    for i, pat in enumerate(bad[::37].tolist() + [0x7C00, 0xFC00, 0x7FFF]):
        cur = g.copy()
        cur[positions[i % len(positions)]] = pat
        ds.set_grads(0, cur)
        B.mlpo_grad_unscale_norm(ds.table, 1.0, 0.0, scratch.ws, scratch.ws_bytes, scratch.scalars, None)
        torch.cuda.synchronize()
        assert scratch.read()["found_inf"] == 1, hex(pat)
    cur = g.copy()
    cur[:4] = [0x7BFF, 0xFBFF, 0x0001, 0x8000]                               # the largest finite values are fine
    ds.set_grads(0, cur)
    B.mlpo_grad_unscale_norm(ds.table, 1.0, 0.0, scratch.ws, scratch.ws_bytes, scratch.scalars, None)
    torch.cuda.synchronize()
    sc = scratch.read()
    s, flag = oracle.grad_stats(cur, 1.0, half="fp16")
    assert sc["found_inf"] == flag == 0 and abs(float(sc["norm"]) / np.sqrt(s) - 1) <= 1e-5


def test_downcast_exhaustive_over_all_fp32_patterns(oracle):
    # every fp32 word as a master parameter with lr = 0 (so p' = p); its fp16 copy against the oracle's rounding
    ghp = B.HParams(lr=0.0, weight_decay=0.0)
    chunk = 1 << 28
    d = dev()
    p = torch.empty(chunk, dtype=torch.int32, device=d)
    m = torch.zeros(chunk, dtype=torch.float32, device=d)
    v = torch.zeros(chunk, dtype=torch.float32, device=d)
    g = torch.zeros(chunk, dtype=torch.int16, device=d)
    p16 = torch.empty(chunk, dtype=torch.int16, device=d)
    tab = B.SubgroupTable([B.subgroup(p, m, v, g, p16, n=chunk, half=FP16)])
    ar = torch.arange(chunk, dtype=torch.int64, device=d)
    for c in range(16):
        p.copy_((ar + (c * chunk - ((1 << 32) if c >= 8 else 0))).to(torch.int32))
        B.mlpo_adamw_step(tab, ghp, 1, None, torch.cuda.current_stream())
        torch.cuda.synchronize()
        pw = p.cpu().numpy().view(np.uint32)
        expect_in = (np.arange(chunk, dtype=np.uint64) + c * chunk).astype(np.uint32)
        notnan = (expect_in & 0x7FFFFFFF) <= 0x7F800000
        assert np.array_equal(pw[notnan], expect_in[notnan]), f"chunk {c}: p changed"
        want = oracle.f32_to_f16_rne(pw.view(np.float32))
        got = from_dev_u16(p16)
        assert np.array_equal(got, want), f"chunk {c}"
        print(f"fp16 downcast chunk {c + 1}/16 ok", flush=True)


@pytest.mark.parametrize("mode,tile,chunk", [("staged", 2048, 8192), ("staged", 0, 0), ("direct", 2048, 0)])
def test_pipeline(oracle, mode, tile, chunk):
    ohp, ghp = hp_pair(oracle)
    rng = np.random.default_rng(9)
    sizes = [70_001, 50_000, 70_001, 12_288]
    tiers = [1, 0, 1, 1]
    host = make_host(rng, sizes, 1e-3, 256.0)
    ds = DeviceSubgroups(host, tiers=tiers, flat=False, tile=tile, half=FP16)
    scratch = Scratch()
    streams = (torch.cuda.Stream(), torch.cuda.Stream())
    if mode == "direct":
        cfg = B.direct_cfg(streams[0], streams[1], 16)
    else:
        need = B.mlpo_stream_staging_bytes(ds.table, 2, chunk)
        stg = torch.empty(need, dtype=torch.uint8, device=dev())
        cfg = B.stream_cfg(2, stg, need, None, streams[1], None, chunk)
    for s in range(3):
        if s > 0:
            for k, sg in enumerate(host):
                sg["g"][:] = f16_bits(rng.standard_normal(sg["g"].size) * 1e-3 * 256.0)
                ds.set_grads(k, sg["g"])
        torch.cuda.synchronize()
        ok_o, norm_o, flag_o, gmul_o = oracle.step(host, ohp, s, 1 / 256.0, 0.05, half="fp16")
        B.mlpo_grad_unscale_norm(ds.table, 1 / 256.0, 0.05, scratch.ws, scratch.ws_bytes, scratch.scalars, streams[1])
        assert B.mlpo_stream_update(ds.table, None, ghp, s + 1, scratch.scalars, cfg) and ok_o
        streams[1].synchronize()
        assert scratch.read()["gmul"] == gmul_o
    for k in range(len(sizes)):
        assert_state_parity(ds.fetch(k), host[k], f"{mode} tile={tile} sg {k}")


def test_accumulate_every_pattern_and_statistics(oracle):
    pats = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    addends = [0x0000, 0x8000, 0x0001, 0x1000, 0x9000, 0x3C00, 0xBC00, 0x6800, 0x7BFF, 0xFBFF, 0x7C00, 0xFC00, 0x7E01,
               0x2E66, 0xAE66, 0x0400]
    a = np.tile(pats, len(addends))
    g = np.repeat(np.array(addends, np.uint16), pats.size)
    da = torch.from_numpy(a.view(np.int16)).to(dev())
    dg = torch.from_numpy(g.view(np.int16)).to(dev())
    B.mlpo_grad_accumulate(da, dg, a.size, half=FP16)
    torch.cuda.synchronize()
    want = a.copy()
    oracle.grad_accumulate(want, g, False, half="fp16")
    got = from_dev_u16(da)
    bad = np.nonzero(got != want)[0]
    assert bad.size == 0, [(hex(int(a[i])), hex(int(g[i])), hex(int(got[i])), hex(int(want[i]))) for i in bad[:5]]
    # the last micro-batch with statistics, device and pinned-host pieces
    rng = np.random.default_rng(2)
    scratch = Scratch()
    inv = 1.0 / 512.0
    pieces = []
    for j, n in enumerate([100_003, 9, 65_536]):
        acc = f16_bits(rng.standard_normal(n) * 0.3 * 512)
        g = f16_bits(rng.standard_normal(n) * 0.3 * 512)
        t = torch.empty(n, dtype=torch.int16, pin_memory=True) if j == 1 else torch.empty(n, dtype=torch.int16,
                                                                                          device=dev())
        t.copy_(torch.from_numpy(acc.view(np.int16)))
        pieces.append((acc, g, t, torch.from_numpy(g.view(np.int16)).to(dev())))
    for j, (acc, g, t, dg) in enumerate(pieces):
        B.mlpo_grad_accumulate_norm(t, dg, acc.size, False, 8 if j == 1 else 0, inv, scratch.ws, scratch.ws_bytes,
                                    begin=(j == 0), half=FP16)
    B.mlpo_grad_norm_finish(scratch.ws, scratch.ws_bytes, inv, 0.5, scratch.scalars)
    torch.cuda.synchronize()
    sumsq, flag = 0.0, 0
    for acc, g, t, dg in pieces:
        oracle.grad_accumulate(acc, g, False, half="fp16")
        assert np.array_equal((t.numpy() if not t.is_cuda else t.cpu().numpy()).view(np.uint16), acc)
        sumsq, flag = oracle.grad_stats(acc, inv, sumsq, flag, half="fp16")
    norm_o, coef_o, gmul_o = oracle.norm_finish(sumsq, inv, 0.5)
    sc = scratch.read()
    assert sc["found_inf"] == flag == 0 and sc["gmul"] == gmul_o and sc["clip_coef"] == coef_o
    assert abs(float(sc["norm"]) - float(norm_o)) <= 1e-5 * float(norm_o)
