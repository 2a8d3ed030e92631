"""GPU parity of the HBM-resident path (gradient pass + fused AdamW) against the CPU oracle, through the C ABI.

Bars: non-finite flag and bf16 copy bit-exact, fp32 state max relative error 1e-6 (expected: bit-identical), norm
relative error 1e-5."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2509_02480_amd import binding as B  # noqa: E402
from paper_2509_02480_amd import workloads as W  # noqa: E402

from gpu_util import (DeviceSubgroups, Scratch, assert_state_parity, dev, from_dev_u16, gpu_step, hp_pair,  # noqa: E402
                      to_dev_u16)


@pytest.fixture(scope="module")
def scratch():
    assert torch.cuda.is_available()
    return Scratch()


def run_workload(oracle, scratch, wl, warm, flat=True, elem_offset=0, check_every_step=False, threads=8, tile=0,
                 lead=False):
    ohp, ghp = hp_pair(oracle, **wl.hp.__dict__)
    host = W.host_subgroups(wl, warm=warm, threads=threads)
    ds = DeviceSubgroups(host, flat=flat, elem_offset=elem_offset, tile=tile, lead=lead)
    applied_o = applied_g = 0
    for s in range(wl.steps):
        if s > 0 and wl.fresh_grads:
            for k, sg in enumerate(host):
                W.fill_grads(wl, k, s, sg["g"], threads)
        inj = None
        if wl.injects(s):
            idx = wl.inject_index(s)
            inj = (idx // wl.sub_elems, idx % wl.sub_elems)
            host[inj[0]]["g"][inj[1]] = 0x7F80
        if s > 0 or inj:
            for k, sg in enumerate(host):
                ds.set_grads(k, sg["g"])
        ok_o, norm_o, flag_o, gmul_o = oracle.step(host, ohp, applied_o, wl.inv_scale, wl.max_norm)
        ok_g, sc = gpu_step(ds, scratch, ghp, applied_g, wl.inv_scale, wl.max_norm)
        print(f"[{wl.name}] step {s}: oracle applied={ok_o} norm={norm_o:.6g}  gpu applied={ok_g} "
              f"norm={sc['norm']:.6g} gmul={sc['gmul']:.6g}", flush=True)
        assert sc["found_inf"] == flag_o and ok_g == ok_o
        assert bool(flag_o) == (inj is not None)
        if not flag_o:
            assert abs(float(sc["norm"]) - float(norm_o)) <= 1e-5 * float(norm_o)
            assert abs(float(sc["gmul"]) - float(gmul_o)) <= 1e-5 * float(gmul_o)
        applied_o += int(ok_o)
        applied_g += int(ok_g)
        if check_every_step or s == wl.steps - 1 or inj:
            for k in range(wl.n_sub):
                assert_state_parity(ds.fetch(k), host[k], f"{wl.name} step {s} subgroup {k}")
    return applied_g


TILES = [0, B.TILE_DEFAULT, 1024]   # planar, the default tiled layout, the smallest tile


@pytest.mark.parametrize("tile", TILES)
@pytest.mark.parametrize("warm", [False, True])
def test_config1_three_steps(oracle, scratch, warm, tile):
    assert run_workload(oracle, scratch, W.C1, warm, check_every_step=True, tile=tile) == 3


@pytest.mark.parametrize("tile,lead", [(t, False) for t in TILES] + [(B.TILE_DEFAULT, True), (1024, True)])
def test_config2_shape_small_with_inf_injection(oracle, scratch, tile, lead):
    # config 2's structure at 1/25 of its size: 16 slices of one flat buffer whose length is a multiple of 4 but not
    # of 8 (odd slices start 8-byte- but not 16-byte-aligned in bf16), loss scale 1024, +inf on the fifth step
    wl = W.Workload("C2/25", n_sub=16, sub_elems=312_500, loss_scale=1024.0, steps=10, inject_every=50)
    assert wl.sub_elems % 4 == 0 and wl.sub_elems % 8 != 0
    assert run_workload(oracle, scratch, wl, warm=False, check_every_step=True, tile=tile, lead=lead) == 9


@pytest.mark.parametrize("tile,lead", [(0, False), (B.TILE_DEFAULT, False), (B.TILE_DEFAULT, True)])
def test_config2_full_size(oracle, scratch, tile, lead):
    # the benchmark workload itself in the layouts the benchmark times (the tiled one as the benchmark sets it up:
    # g and p16 cut from flat buffers, every subgroup shifted by its lead), every element compared after the last
    # step and around the skipped step
    assert run_workload(oracle, scratch, W.C2, warm=False, threads=16, tile=tile, lead=lead) == 9


@pytest.mark.parametrize("n", [0, 1, 2, 3, 4, 5, 7, 8, 63, 64, 1023, 1024, 1025, 2047, 2048, 2049, 4095, 4096,
                               4097, 8191, 8192, 8193, 12289, 100_003])
@pytest.mark.parametrize("flat,offset,tile", [(False, 0, 0), (True, 1, 0), (True, 2, 0), (False, 0, 1024),
                                              (False, 0, 4096)])
def test_ragged_sizes_and_alignments(oracle, scratch, n, flat, offset, tile):
    # two subgroups of n and n+1 elements: tails, tile edges, (with an odd element offset) the element-wise kernel,
    # and tiled state whose last layout tile is partly filled
    ohp, ghp = hp_pair(oracle)
    wl = W.Workload("r", n_sub=1, sub_elems=2 * n + 1, max_norm=0.01, seed=n)
    whole = W.host_subgroups(wl, warm=True)[0]
    host = [{k: a[:n].copy() for k, a in whole.items()}, {k: a[n:].copy() for k, a in whole.items()}]
    ds = DeviceSubgroups(host, flat=flat, elem_offset=offset, tile=tile)
    ok_o, norm_o, flag_o, gmul_o = oracle.step(host, ohp, 5, 1.0, wl.max_norm)
    ok_g, sc = gpu_step(ds, scratch, ghp, 5, 1.0, wl.max_norm)
    assert ok_g and ok_o and abs(float(sc["norm"]) / float(norm_o) - 1) <= 1e-5
    for k in range(2):
        assert_state_parity(ds.fetch(k), host[k], f"n={n} flat={flat} off={offset} tile={tile} sg={k}")


@pytest.mark.parametrize("tile", [0, 2048])
def test_many_subgroups_span_several_launches(oracle, scratch, tile):
    # more subgroups than one argument block holds, of uneven sizes including empty ones
    ohp, ghp = hp_pair(oracle)
    rng = np.random.default_rng(0)
    sizes = [int(x) for x in rng.integers(0, 5000, size=230)]
    sizes[3] = 0
    sizes[100] = 0
    wl = W.Workload("many", n_sub=1, sub_elems=sum(sizes), loss_scale=8.0)
    whole = W.host_subgroups(wl, warm=True)[0]
    cuts = np.cumsum([0] + sizes)
    host = [{k: a[cuts[i]:cuts[i + 1]].copy() for k, a in whole.items()} for i in range(len(sizes))]
    ds = DeviceSubgroups(host, flat=True, tile=tile)
    ok_o, norm_o, flag_o, gmul_o = oracle.step(host, ohp, 0, wl.inv_scale, 0.0)
    ok_g, sc = gpu_step(ds, scratch, ghp, 0, wl.inv_scale, 0.0)
    assert ok_g and abs(float(sc["norm"]) / float(norm_o) - 1) <= 1e-5 and sc["gmul"] == gmul_o
    for k in range(len(sizes)):
        assert_state_parity(ds.fetch(k), host[k], f"many sg={k}")


def test_without_scalars_is_unit_gmul_and_never_skips(oracle, scratch):
    ohp, ghp = hp_pair(oracle)
    wl = W.Workload("ns", n_sub=2, sub_elems=10_001)
    host = W.host_subgroups(wl, warm=True)
    ds = DeviceSubgroups(host)
    for sg in host:
        oracle.adamw_f32(sg["p"], sg["m"], sg["v"], sg["g"], sg["p16"], ohp, 3, 1.0)
    B.mlpo_adamw_step(ds.table, ghp, 3, None, torch.cuda.current_stream())
    for k in range(2):
        assert_state_parity(ds.fetch(k), host[k], f"no scalars sg={k}")


@pytest.mark.parametrize("hp_kw", [dict(weight_decay=0.0), dict(bias_correction=False),
                                   dict(lr=3e-3, beta1=0.8, beta2=0.95, eps=1e-6, weight_decay=0.1),
                                   dict(lr=0.0), dict(beta1=0.0, beta2=0.0),
                                   dict(l2_mode=True), dict(l2_mode=True, lr=3e-3, weight_decay=0.1, eps=1e-6),
                                   dict(l2_mode=True, weight_decay=0.0, bias_correction=False)])
def test_hyperparameter_variants(oracle, scratch, hp_kw):
    wl = W.Workload("hp", n_sub=3, sub_elems=50_001, hp=W.AdamW(**hp_kw), steps=4, loss_scale=64.0, max_norm=0.5)
    run_workload(oracle, scratch, wl, warm=True, check_every_step=True)


def test_special_values(oracle, scratch):
    # denormal and huge state, denormal and zero gradients, values whose bf16 rounding overflows or ties
    ohp, ghp = hp_pair(oracle)
    f = np.float32
    specials = np.array([0.0, -0.0, 1e-45, -1e-45, 1e-40, 1.1754944e-38, 3.4028235e38, -3.4028235e38, 3.39e38,
                         1.00390625, 1.01171875, -1.00390625, 65504.0, 1e-20, 0.02, -0.02], f)
    gbits = np.array([0x0000, 0x8000, 0x0001, 0x8001, 0x007F, 0x0080, 0x7F7F, 0xFF7F, 0x3F80, 0xBF80, 0x3A83, 0x1234,
                      0x0040, 0x7F00, 0x3C00, 0x0002], np.uint16)
    P, G = np.meshgrid(specials, gbits, indexing="ij")
    n = P.size
    rng = np.random.default_rng(1)
    host = [{"p": P.ravel().copy(), "m": (rng.standard_normal(n) * 1e-3).astype(f),
             "v": np.abs(rng.standard_normal(n) * 1e-6).astype(f), "g": G.ravel().copy(), "p16": np.zeros(n, np.uint16)}]
    host[0]["m"][::7] = 1e-42
    host[0]["v"][::5] = 1e-44
    host[0]["v"][::11] = 0.0
    host[0]["m"][::11] = 0.0
    ds = DeviceSubgroups(host)
    for sg in host:
        oracle.adamw_f32(sg["p"], sg["m"], sg["v"], sg["g"], sg["p16"], ohp, 2, 1.0)
    B.mlpo_adamw_step(ds.table, ghp, 2, None, torch.cuda.current_stream())
    got = ds.fetch(0)
    for key in ("p", "m", "v"):
        assert np.array_equal(got[key].view(np.uint32), host[0][key].view(np.uint32)), key
    assert np.array_equal(got["p16"], host[0]["p16"])


@pytest.mark.parametrize("tile", [0, 2048])
def test_skip_leaves_every_bit_untouched(oracle, scratch, tile):
    ohp, ghp = hp_pair(oracle)
    wl = W.Workload("skip", n_sub=4, sub_elems=70_003)
    for bad, where in ((0x7F80, (0, 0)), (0xFF80, (3, 70_002)), (0x7FC0, (1, 4097)), (0xFFFF, (2, 12345))):
        host = W.host_subgroups(wl, warm=True)
        host[where[0]]["g"][where[1]] = bad
        for sg in host:
            sg["p16"][:] = 0x1234
        ds = DeviceSubgroups(host, flat=True, elem_offset=1 if bad == 0x7FC0 else 0, tile=tile)
        ok_g, sc = gpu_step(ds, scratch, ghp, 0)
        ok_o, _, flag_o, _ = oracle.step(host, ohp, 0)
        assert not ok_g and not ok_o and sc["found_inf"] == 1 == flag_o
        for k in range(wl.n_sub):
            got = ds.fetch(k)
            for key in ("p", "m", "v"):
                assert np.array_equal(got[key].view(np.uint32), host[k][key].view(np.uint32))
            assert np.array_equal(got["p16"], host[k]["p16"])
        # the next clean step is the first applied one
        host[where[0]]["g"][where[1]] = 0x3A83
        ds.set_grads(where[0], host[where[0]]["g"])
        assert gpu_step(ds, scratch, ghp, 0)[0] and oracle.step(host, ohp, 0)[0]
        for k in range(wl.n_sub):
            assert_state_parity(ds.fetch(k), host[k], f"after skip sg={k}")


def test_norm_exact_cases_and_flags(oracle, scratch):
    st = torch.cuda.current_stream()

    def gpu_norm(bits_list, inv_scale=1.0, max_norm=0.0, offset=0):
        tens = []
        for b in bits_list:
            buf = torch.zeros(b.size + offset, dtype=torch.int16, device=dev())
            buf[offset:].copy_(torch.from_numpy(b.view(np.int16)))
            tens.append(buf[offset:])
        tab = B.SubgroupTable(B.subgroup(0, 0, 0, t, 0, n=t.numel()) for t in tens)
        B.mlpo_grad_unscale_norm(tab, inv_scale, max_norm, scratch.ws, scratch.ws_bytes, scratch.scalars, st)
        torch.cuda.synchronize()
        return scratch.read()

    for k in (0, 3, 6, 10, 12):
        r = gpu_norm([np.full(4 ** k, 0x3F80, np.uint16)])
        assert r["norm"] == np.float32(2 ** k) and r["found_inf"] == 0 and r["gmul"] == 1
    r = gpu_norm([np.array([0x4040, 0xC080], np.uint16)], max_norm=1.0)          # (3, -4)
    assert r["norm"] == 5 and r["clip_coef"] == np.float32(1.0) / (np.float32(5.0) + np.float32(1e-6))
    r = gpu_norm([np.zeros(1000, np.uint16)], inv_scale=0.5, max_norm=1.0)
    assert r["norm"] == 0 and r["gmul"] == np.float32(0.5) and r["found_inf"] == 0
    r = gpu_norm([], inv_scale=0.25)
    assert r["norm"] == 0 and r["gmul"] == np.float32(0.25) and r["found_inf"] == 0
    r = gpu_norm([np.zeros(0, np.uint16), np.zeros(0, np.uint16)])
    assert r["norm"] == 0 and r["found_inf"] == 0
    # more subgroups than one argument block holds: the running sum is carried across launches
    parts = [np.full(1 + (i % 7), 0x3F80, np.uint16) for i in range(300)]
    r = gpu_norm(parts)
    assert r["norm"] == np.float32(np.sqrt(sum(p.size for p in parts)))
    # every non-finite pattern, at the head / body / tail of a slice that starts off a 16-byte boundary
    rng = np.random.default_rng(3)
    base = (rng.standard_normal(20_011).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
    assert gpu_norm([base], offset=3)["found_inf"] == 0
    want, _ = oracle.grad_stats(base, 1.0)
    assert abs(float(gpu_norm([base], offset=3)["norm"]) / np.sqrt(want) - 1) < 1e-6
    pats = [s | 0x7F80 | m for s in (0, 0x8000) for m in range(128)]
    positions = [0, 1, 4, 5, 8191, 8192, 16388, 20_009, 20_010]
    for i, pat in enumerate(pats):
        g = base.copy()
        g[positions[i % len(positions)]] = pat
        assert gpu_norm([g], offset=3)["found_inf"] == 1, hex(pat)
    for pos in positions:
        g = base.copy()
        g[pos] = 0x7F7F                                       # largest finite: not flagged
        assert gpu_norm([g], offset=3)["found_inf"] == 0
    # finite gradients whose norm does not fit fp32 skip the step as well (two of the largest finite value; one
    # value that an unscale factor above 1 takes out of range); just inside the range nothing is flagged
    g = base.copy()
    g[[5, 16388]] = 0x7F7F
    r = gpu_norm([g], offset=3)
    assert r["found_inf"] == 1 and np.isinf(r["norm"])
    r = gpu_norm([np.array([0x7F00, 0x3F80], np.uint16)], inv_scale=4.0)
    assert r["found_inf"] == 1
    r = gpu_norm([np.array([0x7E80, 0], np.uint16)], inv_scale=2.0)
    assert r["found_inf"] == 0 and r["norm"] == np.float32(2.0 ** 127)


def test_norm_is_deterministic(scratch):
    wl = W.Workload("det", n_sub=5, sub_elems=1_000_003)
    g = np.empty(wl.n_total, np.uint16)
    W.fill_grad_bf16(g, 1, 0, 0, 1e-3, threads=8)
    t = to_dev_u16(g)
    tab = B.SubgroupTable(B.subgroup(0, 0, 0, t[k * wl.sub_elems:(k + 1) * wl.sub_elems], 0, n=wl.sub_elems)
                          for k in range(wl.n_sub))
    vals = set()
    for _ in range(5):
        B.mlpo_grad_unscale_norm(tab, 1.0, 0.0, scratch.ws, scratch.ws_bytes, scratch.scalars,
                                 torch.cuda.current_stream())
        torch.cuda.synchronize()
        vals.add(scratch.scalars.cpu().numpy().tobytes())
    assert len(vals) == 1


def test_downcast_exhaustive_over_all_fp32_patterns(oracle, scratch):
    # every fp32 word goes through the kernel as a master parameter with lr = 0 (so p' = p) and its bf16 copy is
    # compared with the oracle's rounding of the fp32 value the kernel wrote
    ghp = B.HParams(lr=0.0, weight_decay=0.0)
    chunk = 1 << 28
    d = dev()
    p = torch.empty(chunk, dtype=torch.int32, device=d)
    m = torch.zeros(chunk, dtype=torch.float32, device=d)
    v = torch.zeros(chunk, dtype=torch.float32, device=d)
    g = torch.zeros(chunk, dtype=torch.int16, device=d)
    p16 = torch.empty(chunk, dtype=torch.int16, device=d)
    tab = B.SubgroupTable([B.subgroup(p, m, v, g, p16, n=chunk)])
    ar = torch.arange(chunk, dtype=torch.int64, device=d)
    for c in range(16):
        # bit pattern c * chunk + i as a two's-complement int32
        p.copy_((ar + (c * chunk - ((1 << 32) if c >= 8 else 0))).to(torch.int32))
        B.mlpo_adamw_step(tab, ghp, 1, None, torch.cuda.current_stream())
        torch.cuda.synchronize()
        pw = p.cpu().numpy().view(np.uint32)
        expect_in = (np.arange(chunk, dtype=np.uint64) + c * chunk).astype(np.uint32)
        notnan = (expect_in & 0x7FFFFFFF) <= 0x7F800000
        assert np.array_equal(pw[notnan], expect_in[notnan]), f"chunk {c}: p changed"
        assert np.all((pw[~notnan] & 0x7FFFFFFF) > 0x7F800000)
        want = oracle.f32_to_bf16_rne(pw.view(np.float32))
        got = from_dev_u16(p16)
        assert np.array_equal(got, want), f"chunk {c}"
        assert not m.any().item() and not v.any().item()
        print(f"downcast chunk {c + 1}/16 ok", flush=True)


def test_kernel_timing_records_every_launch(scratch):
    wl = W.Workload("time", n_sub=2, sub_elems=1 << 20)
    host = W.host_subgroups(wl, warm=True)
    ds = DeviceSubgroups(host, tile=B.TILE_DEFAULT)
    st = torch.cuda.current_stream()
    B.mlpo_kernel_timing(True)
    try:
        for t in range(1, 6):
            B.mlpo_grad_unscale_norm(ds.table, 1.0, 0.0, scratch.ws, scratch.ws_bytes, scratch.scalars, st)
            B.mlpo_adamw_step(ds.table, B.HParams(), t, scratch.scalars, st)
        upd, nrm = B.mlpo_kernel_times(0), B.mlpo_kernel_times(1)
        assert len(upd) == 5 and len(nrm) == 5
        # 2 M elements move 56 MB per update: between a few microseconds and a millisecond on any working device
        assert all(0.002 < x < 1.0 for x in upd) and all(0.001 < x < 1.0 for x in nrm)
        assert B.mlpo_kernel_times(0) == []                       # read-out forgets
    finally:
        B.mlpo_kernel_timing(False)
    B.mlpo_adamw_step(ds.table, B.HParams(), 6, None, st)
    assert B.mlpo_kernel_times(0) == []                           # nothing recorded when off


def test_every_finite_gradient_pattern(oracle, scratch):
    # all 65 280 finite bf16 gradient patterns (every exponent, denormals, both zeros) against eight different states
    ohp, ghp = hp_pair(oracle)
    pats = np.array([b for b in range(65536) if (b & 0x7F80) != 0x7F80], dtype=np.uint16)
    rng = np.random.default_rng(5)
    reps = 8
    n = pats.size * reps
    host = [{"p": (rng.standard_normal(n) * 0.02).astype(np.float32),
             "m": (rng.standard_normal(n) * 3e-4).astype(np.float32),
             "v": ((rng.standard_normal(n) * 1e-3) ** 2).astype(np.float32),
             "g": np.tile(pats, reps), "p16": np.zeros(n, np.uint16)}]
    host[0]["m"][:pats.size] = 0
    host[0]["v"][:pats.size] = 0
    for tile in (0, B.TILE_DEFAULT):
        cur = [{k: a.copy() for k, a in host[0].items()}]
        ds = DeviceSubgroups(cur, tile=tile)
        oracle.adamw_f32(cur[0]["p"], cur[0]["m"], cur[0]["v"], cur[0]["g"], cur[0]["p16"], ohp, 3, 0.5)
        half = torch.tensor([0.0, 1.0, 0.5, 0.0], dtype=torch.float32, device=dev())
        half[3:4].view(torch.int32).zero_()
        B.mlpo_adamw_step(ds.table, ghp, 3, half, torch.cuda.current_stream())      # gmul = 0.5 from a scalar record
        got = ds.fetch(0)
        for key in ("p", "m", "v"):
            same = got[key].view(np.uint32) == cur[0][key].view(np.uint32)
            both_nan = np.isnan(got[key]) & np.isnan(cur[0][key])
            assert np.all(same | both_nan), f"tile={tile} {key}: {(~(same | both_nan)).sum()} words differ"
        assert np.array_equal(got["p16"], cur[0]["p16"])


def test_subgroup_longer_than_32_bit_indices(oracle, scratch):
    # one tiled subgroup of 2^32 + 77 777 elements (69 GB of buffers): windows around the 2^31 and 2^32 element
    # marks and at both ends are checked; inputs are drawn on the device and the windows copied back for the oracle
    free, _ = torch.cuda.mem_get_info()
    n = (1 << 32) + 77_777
    T = B.TILE_DEFAULT
    per = B.mlpo_state_floats(n, T)
    if free < 4 * per + 4 * n + (8 << 30):
        pytest.skip("not enough free device memory for a 2^32-element subgroup")
    d = dev()
    gen = torch.Generator(device=d)
    gen.manual_seed(1234)
    state = torch.empty(per, dtype=torch.float32, device=d)
    chunk = 1 << 28
    for lo in range(0, per, chunk):
        hi = min(per, lo + chunk)
        state[lo:hi].normal_(0.0, 0.02, generator=gen)
    sv = state.view(-1, 3, T)
    sv[:, 1, :].mul_(0.015)            # momentum ~ N(0, 3e-4)
    sv[:, 2, :].mul_(0.05).square_()   # variance ~ N(0, 1e-3)^2
    g = torch.empty(n, dtype=torch.bfloat16, device=d)
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        g[lo:hi].normal_(0.0, 1e-3, generator=gen)
    g = g.view(torch.int16)
    p16 = torch.zeros(n, dtype=torch.int16, device=d)
    table = B.SubgroupTable([B.tiled_subgroup(state, g, p16, n=n, tile_elems=T)])
    W_ = 50_001
    starts = [0, (1 << 31) - 25_000, (1 << 32) - 25_000, n - W_]
    ohp, ghp = hp_pair(oracle)

    def window(lo):
        i = torch.arange(lo, lo + W_, dtype=torch.int64, device=d)
        phys = (i // T) * (3 * T) + i % T
        return {"p": state[phys].cpu().numpy(), "m": state[phys + T].cpu().numpy(), "v": state[phys + 2 * T].cpu().numpy(),
                "g": g[lo:lo + W_].cpu().numpy().view(np.uint16).copy(),
                "p16": p16[lo:lo + W_].cpu().numpy().view(np.uint16).copy()}

    want = [window(lo) for lo in starts]
    # the oracle's own norm over all 2^32 + 77 777 gradients (chunked fp64 sums on the host)
    g_host = g.cpu().numpy().view(np.uint16)
    sumsq, flag = oracle.grad_stats_chunked(g_host, 1.0)
    norm_o, coef_o, gmul_o = oracle.norm_finish(sumsq, 1.0, 1.0)
    del g_host
    assert flag == 0 and coef_o < 1                      # clip is active
    B.mlpo_grad_unscale_norm(table, 1.0, 1.0, scratch.ws, scratch.ws_bytes, scratch.scalars,
                             torch.cuda.current_stream())
    B.mlpo_adamw_step(table, ghp, 4, scratch.scalars, torch.cuda.current_stream())
    torch.cuda.synchronize()
    sc = scratch.read()
    assert sc["found_inf"] == 0
    assert abs(float(sc["norm"]) - float(norm_o)) <= 1e-5 * float(norm_o)
    assert abs(float(norm_o) / (1e-3 * np.sqrt(n)) - 1) < 5e-3       # n draws of N(0, 1e-3), rounded to bf16
    assert sc["gmul"] == gmul_o, "gradient multiplier differs from the oracle's: the state cannot match bit for bit"
    for lo, w in zip(starts, want):
        oracle.adamw_f32(w["p"], w["m"], w["v"], w["g"], w["p16"], ohp, 4, gmul_o)
        got = window(lo)
        for key in ("p", "m", "v"):
            assert np.array_equal(got[key].view(np.uint32), w[key].view(np.uint32)), (lo, key)
        assert np.array_equal(got["p16"], w["p16"]), lo
    del state, g, p16
    torch.cuda.empty_cache()


@pytest.mark.parametrize("n,T", [(0, 1024), (1, 1024), (1023, 1024), (1024, 1024), (5000, 2048), (100_001, 8192),
                                 (3_000_001, 8192), (70_000, 16384)])
def test_state_pack_and_unpack(n, T):
    # layout conversion is data movement: compared bit for bit with the index definition written out in numpy
    from gpu_util import pack_tiled
    rng = np.random.default_rng(n)
    src = [rng.standard_normal(n).astype(np.float32) for _ in range(3)]
    dv = [torch.from_numpy(a).to(dev()) for a in src]
    floats = B.mlpo_state_floats(n, T)
    state = torch.full((max(floats, 1),), 7.0, dtype=torch.float32, device=dev())
    st = torch.cuda.current_stream()
    B.mlpo_state_pack(dv[0], dv[1], dv[2], n, T, state, st)
    torch.cuda.synchronize()
    want = pack_tiled(src[0], src[1], src[2], T)
    assert np.array_equal(state.cpu().numpy()[:floats].view(np.uint32), want.view(np.uint32))
    back = [torch.full((max(n, 1),), -1.0, dtype=torch.float32, device=dev()) for _ in range(3)]
    B.mlpo_state_unpack(state, n, T, back[0], back[1], back[2], st)
    torch.cuda.synchronize()
    for a, bck in zip(src, back):
        assert np.array_equal(bck.cpu().numpy()[:n].view(np.uint32), a.view(np.uint32))
    if n:
        pinned = torch.empty(floats, dtype=torch.float32, pin_memory=True)       # pinned host destination
        B.mlpo_state_pack(dv[0], dv[1], dv[2], n, T, pinned, st)
        torch.cuda.synchronize()
        assert np.array_equal(pinned.numpy().view(np.uint32), want.view(np.uint32))


def test_step_captured_in_a_hip_graph_and_replayed(oracle, scratch):
    """The resident step only enqueues kernels (no allocation, no memset, no host wait), so it can be captured once
    and replayed.  Without bias correction the per-step constants do not depend on the step number, so every replay
    is one more AdamW step on whatever the gradient buffers hold by then.  Replays alternate with eager work (new
    gradients copied in, state read back), one of them with a non-finite gradient; every replay is checked."""
    hp_kw = dict(lr=3e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1, bias_correction=False)
    ohp, ghp = hp_pair(oracle, **hp_kw)
    wl = W.Workload("graph", n_sub=5, sub_elems=150_001, hp=W.AdamW(**hp_kw), loss_scale=32.0, max_norm=0.02, steps=6)
    host = W.host_subgroups(wl, warm=True)
    ds = DeviceSubgroups(host, tile=2048)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        st = torch.cuda.current_stream()
        B.mlpo_grad_unscale_norm(ds.table, wl.inv_scale, wl.max_norm, scratch.ws, scratch.ws_bytes, scratch.scalars, st)
        B.mlpo_adamw_step(ds.table, ghp, 1, scratch.scalars, st)
    torch.cuda.synchronize()
    before = [ds.fetch(k) for k in range(wl.n_sub)]
    for k in range(wl.n_sub):                       # capturing ran nothing
        assert_state_parity(before[k], host[k], f"after capture sg {k}")
    applied = 0
    for s in range(wl.steps):
        inject = s == 3
        for k, sg in enumerate(host):
            W.fill_grads(wl, k, s, sg["g"])
        if inject:
            host[2]["g"][4321] = 0xFF80
        for k, sg in enumerate(host):
            ds.set_grads(k, sg["g"])
        torch.cuda.synchronize()
        ok_o, norm_o, flag_o, gmul_o = oracle.step(host, ohp, applied, wl.inv_scale, wl.max_norm)
        graph.replay()
        torch.cuda.synchronize()
        sc = scratch.read()
        assert sc["found_inf"] == flag_o == int(inject) and ok_o == (not inject)
        if ok_o:
            assert abs(float(sc["norm"]) - float(norm_o)) <= 1e-5 * float(norm_o) and sc["gmul"] == gmul_o
            applied += 1
        for k in range(wl.n_sub):
            assert_state_parity(ds.fetch(k), host[k], f"replay {s} sg {k}")
    assert applied == wl.steps - 1
