"""GPU parity of mlpo_grad_accumulate (the half-precision gradient accumulation buffer of Section 3.2 "Delayed
In-place Mixed-Precision Gradient Conversion") against the oracle: bit-exact on arbitrary bit patterns (non-finite
values included), for device and pinned-host buffers, every alignment phase, persistent and one-tile-per-workgroup
grids; then the whole flow the paper describes: micro-batches accumulated into a host buffer, the update reading it."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2509_02480_amd import binding as B  # noqa: E402
from paper_2509_02480_amd import workloads as W  # noqa: E402

from gpu_util import DeviceSubgroups, Scratch, assert_state_parity, dev, hp_pair  # noqa: E402


def bits(rng, n):
    return rng.integers(0, 0x10000, n, dtype=np.uint32).astype(np.uint16)


def to_dev(a):
    return torch.from_numpy(a.view(np.int16)).to(dev())


def back(t):
    return t.cpu().numpy().view(np.uint16)


@pytest.mark.parametrize("n", [1, 7, 8, 9, 1023, 8191, 8192, 8193, 100_003, (1 << 20) + 5, 3 * 8192 * 4])
@pytest.mark.parametrize("first", [False, True])
def test_matches_oracle_on_any_bits(oracle, n, first):
    rng = np.random.default_rng(n)
    a, g = bits(rng, n), bits(rng, n)
    da, dg = to_dev(a), to_dev(g)
    B.mlpo_grad_accumulate(da, dg, n, first=first)
    torch.cuda.synchronize()
    oracle.grad_accumulate(a, g, first)
    assert np.array_equal(back(da), a)
    assert np.array_equal(back(dg), g)


def test_every_pattern_against_selected_addends(oracle):
    pats = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    addends = [0x0000, 0x8000, 0x0001, 0x3B80, 0xBB80, 0x3F80, 0xBF80, 0x7B00, 0x7F7F, 0xFF7F, 0x7F80, 0xFF80, 0x7FC1,
               0x3A83, 0xBA83, 0x0080]
    a = np.tile(pats, len(addends))
    g = np.repeat(np.array(addends, np.uint16), pats.size)
    da, dg = to_dev(a), to_dev(g)
    B.mlpo_grad_accumulate(da, dg, a.size)
    torch.cuda.synchronize()
    oracle.grad_accumulate(a, g, False)
    got = back(da)
    bad = np.nonzero(got != a)[0]
    assert bad.size == 0, [(hex(int(np.tile(pats, len(addends))[i])), hex(int(g[i])), hex(int(got[i])), hex(int(a[i])))
                           for i in bad[:5]]


@pytest.mark.parametrize("n", [40_000, 10, 63, 64, 65, 130])
@pytest.mark.parametrize("off_a,off_g", [(0, 0), (1, 1), (3, 3), (7, 7), (5, 13), (0, 1), (2, 7), (4, 0), (20, 20),
                                         (33, 33), (63, 63), (40, 8), (17, 49), (8, 40)])
def test_alignment_phases(oracle, off_a, off_g, n):
    # the vector body starts at the first 128-byte line of acc (up to 63 elements further on) when acc and g agree
    # modulo 16 bytes; everything else, and ranges that end before that line, go element by element
    rng = np.random.default_rng(off_a * 64 + off_g + n)
    a, g = bits(rng, n), bits(rng, n)
    guard = 0x1234
    ba = torch.full((n + 64,), guard, dtype=torch.int16, device=dev())
    bg = torch.zeros(n + 64, dtype=torch.int16, device=dev())
    ba[off_a:off_a + n].copy_(to_dev(a))
    bg[off_g:off_g + n].copy_(to_dev(g))
    B.mlpo_grad_accumulate(ba[off_a:], bg[off_g:], n)
    torch.cuda.synchronize()
    oracle.grad_accumulate(a, g, False)
    out = back(ba)
    assert np.array_equal(out[off_a:off_a + n], a)
    assert np.all(out[:off_a] == guard) and np.all(out[off_a + n:] == guard)   # nothing outside the range is touched


@pytest.mark.parametrize("blocks", [0, 1, 7, 64])
def test_pinned_host_buffer_and_persistent_grids(oracle, blocks):
    n = 1_000_003
    rng = np.random.default_rng(blocks)
    acc = torch.empty(n, dtype=torch.int16, pin_memory=True)
    ref = np.zeros(n, np.uint16)
    for j in range(4):
        g = oracle.f32_to_bf16_rne((rng.standard_normal(n) * 1e-3 * 1024).astype(np.float32))
        B.mlpo_grad_accumulate(acc, to_dev(g), n, first=(j == 0), blocks=blocks)
        torch.cuda.synchronize()
        oracle.grad_accumulate(ref, g, j == 0)
    assert np.array_equal(acc.numpy().view(np.uint16), ref)
    assert np.count_nonzero(ref) > n // 2


def test_micro_batches_on_the_host_then_update(oracle):
    """Four micro-batches accumulated into pinned-host buffers, then the gradient pass and a staged update that fetches
    those gradients with the state (the data placement of Section 3.2): state, bf16 copy, norm and flag as the oracle's
    on the oracle's own accumulation."""
    ohp, ghp = hp_pair(oracle)
    wl = W.Workload("accum", n_sub=4, sub_elems=120_007, n_host=3, loss_scale=512.0, max_norm=0.1, steps=2)
    host = W.host_subgroups(wl, warm=True)
    tiers = [B.TIER_HOST_GRADS if wl.tier(k) else B.TIER_HBM for k in range(wl.n_sub)]
    ds = DeviceSubgroups(host, tiers=[1 if t else 0 for t in tiers], flat=False, tile=2048)
    accs, descs = [], []
    for k, e in enumerate(ds.t):
        acc = torch.empty(ds.sizes[k], dtype=torch.int16, pin_memory=True) if tiers[k] else \
            torch.empty(ds.sizes[k], dtype=torch.int16, device=dev())
        accs.append(acc)
        descs.append(B.tiled_subgroup(e["state"], acc, e["p16"], n=ds.sizes[k], tier=tiers[k], tile_elems=2048))
    table = B.SubgroupTable(descs)
    scratch = Scratch()
    cmp_ = torch.cuda.Stream()
    need = B.mlpo_stream_staging_bytes(table, 2, 32_768)
    stg = torch.empty(need, dtype=torch.uint8, device=dev())
    cfg = B.stream_cfg(2, stg, need, None, cmp_, None, 32_768)
    micro = np.empty(wl.sub_elems, np.uint16)
    dmicro = torch.empty(wl.sub_elems, dtype=torch.int16, device=dev())
    for s in range(wl.steps):
        for k, sg in enumerate(host):
            for j in range(4):
                W.fill_grads(wl, k, 10 * s + j, micro)
                oracle.grad_accumulate(sg["g"], micro, j == 0)
                dmicro.copy_(torch.from_numpy(micro.view(np.int16)))
                torch.cuda.synchronize()
                B.mlpo_grad_accumulate(accs[k], dmicro, first=(j == 0), blocks=16 if tiers[k] else 0, stream=cmp_)
                cmp_.synchronize()
        ok_o, norm_o, flag_o, gmul_o = oracle.step(host, ohp, s, wl.inv_scale, wl.max_norm)
        B.mlpo_grad_unscale_norm(table, wl.inv_scale, wl.max_norm, scratch.ws, scratch.ws_bytes, scratch.scalars, cmp_)
        assert B.mlpo_stream_update(table, None, ghp, s + 1, scratch.scalars, cfg) and ok_o
        cmp_.synchronize()
        sc = scratch.read()
        assert abs(float(sc["norm"]) / float(norm_o) - 1) <= 1e-5 and sc["gmul"] == gmul_o
        for k in range(wl.n_sub):
            got = accs[k].numpy() if tiers[k] else accs[k].cpu().numpy()
            assert np.array_equal(got.view(np.uint16), host[k]["g"]), f"accumulated gradients sg={k}"
    for k in range(wl.n_sub):
        assert_state_parity(ds.fetch(k), host[k], f"accumulate then update sg={k}")


def _norm_of(oracle, arrays, inv_scale, max_norm):
    sumsq, flag = 0.0, 0
    for a in arrays:
        sumsq, flag = oracle.grad_stats(a, inv_scale, sumsq, flag)
    return oracle.norm_finish(sumsq, inv_scale, max_norm) + (flag,)


@pytest.mark.parametrize("sizes,first,blocks,max_norm", [
    ([100_003], False, 0, 0.0), ([100_003], True, 0, 0.5), ([8192 * 4 * 3, 5, 70_001], False, 0, 0.01),
    ([1, 9, 17], False, 3, 0.0), ([300_000, 0, 123_457, 1 << 20], False, 16, 0.02), ([0, 0], False, 0, 1.0),
])
def test_last_micro_batch_also_gives_the_norm(oracle, sizes, first, blocks, max_norm):
    """mlpo_grad_accumulate_norm over several pieces + mlpo_grad_norm_finish: the accumulated buffers bit-exact, the
    scalars as the oracle's gradient statistics over the oracle's accumulated buffers."""
    rng = np.random.default_rng(sum(sizes) + blocks)
    inv_scale = 1.0 / 256.0
    scratch = Scratch()
    accs, gs, dev_acc, dev_g = [], [], [], []
    for j, n in enumerate(sizes):
        a = oracle.f32_to_bf16_rne((rng.standard_normal(n) * 0.3).astype(np.float32))
        g = oracle.f32_to_bf16_rne((rng.standard_normal(n) * 0.3).astype(np.float32))
        accs.append(a)
        gs.append(g)
        if j % 2 == 1 and n:      # every other piece keeps its buffer in pinned host memory
            t = torch.empty(n, dtype=torch.int16, pin_memory=True)
            t.copy_(torch.from_numpy(a.view(np.int16)))
        else:
            t = to_dev(a)
        dev_acc.append(t)
        dev_g.append(to_dev(g))
    # poison the workspace: begin must reset whatever an earlier step left there
    scratch.ws.fill_(0xFF)
    torch.cuda.synchronize()
    for j, n in enumerate(sizes):
        B.mlpo_grad_accumulate_norm(dev_acc[j], dev_g[j], n, first, blocks, inv_scale, scratch.ws, scratch.ws_bytes,
                                    begin=(j == 0))
    B.mlpo_grad_norm_finish(scratch.ws, scratch.ws_bytes, inv_scale, max_norm, scratch.scalars)
    torch.cuda.synchronize()
    for a, g in zip(accs, gs):
        oracle.grad_accumulate(a, g, first)
    norm_o, coef_o, gmul_o, flag_o = _norm_of(oracle, accs, inv_scale, max_norm)
    for j, n in enumerate(sizes):
        got = dev_acc[j].numpy() if not dev_acc[j].is_cuda else dev_acc[j].cpu().numpy()
        assert np.array_equal(got.view(np.uint16), accs[j]), f"piece {j}"
    sc = scratch.read()
    assert sc["found_inf"] == flag_o == 0
    assert abs(float(sc["norm"]) - float(norm_o)) <= 1e-5 * float(norm_o)
    assert sc["clip_coef"] == coef_o and sc["gmul"] == gmul_o
    # and the separate gradient pass over the same buffers agrees
    if sum(sizes):
        table = B.SubgroupTable(B.subgroup(0, 0, 0, t, 0, n=n) for t, n in zip(dev_acc, sizes))
        other = Scratch()
        B.mlpo_grad_unscale_norm(table, inv_scale, max_norm, other.ws, other.ws_bytes, other.scalars, None)
        torch.cuda.synchronize()
        o = other.read()
        assert abs(float(o["norm"]) - float(sc["norm"])) <= 2e-7 * float(norm_o) and o["gmul"] == sc["gmul"]


@pytest.mark.parametrize("base,blocks", [(20, 0), (1, 0), (36, 5)])
def test_norm_pieces_cut_from_flat_buffers(oracle, base, blocks):
    """The pieces of a step as consecutive slices of one flat accumulation buffer and one flat gradient buffer, so
    that they begin in the middle of 128-byte lines (the vector body of each call starts at the next line)."""
    sizes = [100_004, 65_556, 7_812, 31]
    rng = np.random.default_rng(base)
    inv_scale, max_norm = 1.0 / 64.0, 0.02
    total = sum(sizes)
    a_all = oracle.f32_to_bf16_rne((rng.standard_normal(total) * 0.3).astype(np.float32))
    g_all = oracle.f32_to_bf16_rne((rng.standard_normal(total) * 0.3).astype(np.float32))
    guard = 0x1234
    flat_a = torch.full((base + total + 64,), guard, dtype=torch.int16, device=dev())
    flat_g = torch.zeros(base + total + 64, dtype=torch.int16, device=dev())
    flat_a[base:base + total].copy_(to_dev(a_all))
    flat_g[base:base + total].copy_(to_dev(g_all))
    scratch = Scratch()
    off, accs = base, []
    for j, n in enumerate(sizes):
        B.mlpo_grad_accumulate_norm(flat_a[off:off + n], flat_g[off:off + n], n, False, blocks, inv_scale, scratch.ws,
                                    scratch.ws_bytes, begin=(j == 0))
        a = a_all[off - base:off - base + n].copy()
        oracle.grad_accumulate(a, g_all[off - base:off - base + n], False)
        accs.append(a)
        off += n
    B.mlpo_grad_norm_finish(scratch.ws, scratch.ws_bytes, inv_scale, max_norm, scratch.scalars)
    torch.cuda.synchronize()
    out = back(flat_a)
    assert np.array_equal(out[base:base + total], np.concatenate(accs))
    assert np.all(out[:base] == guard) and np.all(out[base + total:] == guard)
    norm_o, coef_o, gmul_o, flag_o = _norm_of(oracle, accs, inv_scale, max_norm)
    sc = scratch.read()
    assert sc["found_inf"] == flag_o == 0
    assert abs(float(sc["norm"]) - float(norm_o)) <= 1e-5 * float(norm_o)
    assert sc["clip_coef"] == coef_o and sc["gmul"] == gmul_o


def test_norm_of_exact_sums(oracle):
    # 4^9 ones plus 4^9 ones: every element becomes 2, the norm is exactly 2 * 2^9
    n = 4 ** 9
    scratch = Scratch()
    acc = to_dev(np.full(n, 0x3F80, np.uint16))
    g = to_dev(np.full(n, 0x3F80, np.uint16))
    B.mlpo_grad_accumulate_norm(acc, g, n, False, 0, 1.0, scratch.ws, scratch.ws_bytes, True)
    B.mlpo_grad_norm_finish(scratch.ws, scratch.ws_bytes, 1.0, 0.0, scratch.scalars)
    torch.cuda.synchronize()
    sc = scratch.read()
    assert sc["norm"] == np.float32(1024.0) and sc["found_inf"] == 0 and sc["gmul"] == np.float32(1.0)
    assert np.all(back(acc) == 0x4000)


@pytest.mark.parametrize("where,a_bits,g_bits", [
    (0, 0x7F7F, 0x7F7F),          # the sum overflows to +inf in the first element
    (-1, 0x7F80, 0xFF80),         # inf - inf = NaN in the last element (a scalar tail)
    (12_345, 0x3F80, 0x7FC1),     # a NaN gradient in the vector body
    (3, 0xFF80, 0x3F80),          # the buffer already held -inf, in the unaligned head
])
def test_non_finite_sums_raise_the_flag(oracle, where, a_bits, g_bits):
    n = 50_001
    rng = np.random.default_rng(5)
    a = oracle.f32_to_bf16_rne(rng.standard_normal(n).astype(np.float32))
    g = oracle.f32_to_bf16_rne(rng.standard_normal(n).astype(np.float32))
    a[where], g[where] = a_bits, g_bits
    scratch = Scratch()
    base_a = torch.zeros(n + 8, dtype=torch.int16, device=dev())
    base_g = torch.zeros(n + 8, dtype=torch.int16, device=dev())
    base_a[5:5 + n].copy_(to_dev(a))
    base_g[5:5 + n].copy_(to_dev(g))
    B.mlpo_grad_accumulate_norm(base_a[5:], base_g[5:], n, False, 0, 1.0, scratch.ws, scratch.ws_bytes, True)
    B.mlpo_grad_norm_finish(scratch.ws, scratch.ws_bytes, 1.0, 1.0, scratch.scalars)
    torch.cuda.synchronize()
    oracle.grad_accumulate(a, g, False)
    assert np.array_equal(back(base_a)[5:5 + n], a)
    _, flag = oracle.grad_stats(a, 1.0)
    assert flag == 1 and scratch.read()["found_inf"] == 1


def test_buffer_of_more_than_2_to_32_elements(oracle):
    """Element indices that do not fit 32 bits: 4.3 G gradients accumulated over two micro-batches (one tile per
    workgroup, then a bounded persistent grid), windows at the start, past 2^31 and past 2^32 against the oracle, and
    the statistics of the last micro-batch against the gradient pass over the finished buffer."""
    n = (1 << 32) + 4099
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    if free < 4 * n + (4 << 30):
        pytest.skip(f"needs {4 * n / 1e9:.0f} GB of free device memory")
    win = 50_003
    starts = [0, (1 << 31) + 12_345, n - win]
    inv_scale = 1.0 / 64.0
    host = np.empty(n, np.uint16)
    acc = torch.empty(n, dtype=torch.int16, device=dev())
    g = torch.empty(n, dtype=torch.int16, device=dev())
    want = []
    for mb in range(3):                                   # the buffer's first content, then two micro-batches
        wl = W.Workload("bigacc", n_sub=1, sub_elems=n, loss_scale=64.0, seed=40 + mb)
        W.fill_grads(wl, 0, 0, host, threads=16)
        (acc if mb == 0 else g).copy_(torch.from_numpy(host.view(np.int16)))
        if mb == 0:
            want = [host[s:s + win].copy() for s in starts]
            continue
        for w, s in zip(want, starts):
            oracle.grad_accumulate(w, host[s:s + win].copy(), False)
        scratch = Scratch()
        if mb == 1:
            B.mlpo_grad_accumulate(acc, g, n, False, 0)
        else:
            B.mlpo_grad_accumulate_norm(acc, g, n, False, 300, inv_scale, scratch.ws, scratch.ws_bytes, begin=True)
            B.mlpo_grad_norm_finish(scratch.ws, scratch.ws_bytes, inv_scale, 0.0, scratch.scalars)
        torch.cuda.synchronize()
    for w, s in zip(want, starts):
        assert np.array_equal(back(acc[s:s + win]), w), f"window at {s}"
    sc = scratch.read()
    other = Scratch()
    table = B.SubgroupTable([B.subgroup(0, 0, 0, acc, 0, n=n)])
    B.mlpo_grad_unscale_norm(table, inv_scale, 0.0, other.ws, other.ws_bytes, other.scalars, None)
    torch.cuda.synchronize()
    o = other.read()
    assert sc["found_inf"] == o["found_inf"] == 0
    assert abs(float(sc["norm"]) - float(o["norm"])) <= 2e-7 * float(o["norm"])
    # the norm itself, from the generator's statistics: three sums of N(0, 1e-3 * 64) draws, unscaled by 1 / 64
    expect = 1e-3 * np.sqrt(3.0 * n)
    assert abs(float(sc["norm"]) - expect) <= 0.01 * expect
