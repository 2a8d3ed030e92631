"""GPU parity of the tiered pipeline (mlpo_stream_update): host-tier subgroups fetched into staging slots, updated and
flushed back, HBM-tier subgroups updated in place.  The result must be bit-identical to the oracle (and hence to the
resident path) whatever the number of slots, the chunking and the processing order are - the paper's statement that the
order of independent subgroup updates is inconsequential (Section 3.2 "Cache-Friendly Ordering") and that subgroup
size does not affect results (Section 4.1 "Runtime Configurations")."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2509_02480_amd import binding as B  # noqa: E402
from paper_2509_02480_amd import workloads as W  # noqa: E402

from gpu_util import DeviceSubgroups, Scratch, assert_state_parity, dev, hp_pair  # noqa: E402


@pytest.fixture(scope="module")
def scratch():
    assert torch.cuda.is_available()
    return Scratch()


@pytest.fixture(scope="module")
def streams():
    return torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()


def stream_step(ds, scratch, ghp, steps_applied, wl, streams, n_slots, chunk, order, staging_holder, norm=True,
                direct_blocks=None):
    h2d, cmp_, d2h = streams
    if direct_blocks is not None:
        cfg = B.direct_cfg(h2d, cmp_, direct_blocks)
    else:
        need = B.mlpo_stream_staging_bytes(ds.table, n_slots, chunk)
        if staging_holder.get("bytes", -1) < need:
            staging_holder["t"] = torch.empty(max(need, 256), dtype=torch.uint8, device=dev())
            staging_holder["bytes"] = need
        if staging_holder.get("own_streams"):
            h2d = d2h = None                      # the library's own copy streams
        cfg = B.stream_cfg(n_slots, staging_holder["t"], staging_holder["t"].numel(), h2d, cmp_, d2h, chunk)
    torch.cuda.synchronize()
    scal = None
    if norm:
        B.mlpo_grad_unscale_norm(ds.table, wl.inv_scale, wl.max_norm, scratch.ws, scratch.ws_bytes, scratch.scalars,
                                 cmp_)
        scal = scratch.scalars
    applied = B.mlpo_stream_update(ds.table, order, ghp, steps_applied + 1, scal, cfg)
    cmp_.synchronize()          # documented: the compute stream joins the last flush
    return applied


@pytest.mark.parametrize("n_slots,chunk,order_kind,tile", [
    (1, 0, "asc", 0), (2, 0, "asc", 0), (3, 0, "desc", 0), (4, 0, "perm", 0),
    (3, 4096, "asc", 0), (2, 10_000, "perm", 0), (4, 1 << 20, "desc", 0), (8, 33_332, "asc", 0),
    (1, 0, "asc", 2048), (3, 0, "perm", 8192), (2, 8192, "desc", 2048), (4, 16_384, "perm", 8192),
    (3, 1 << 20, "asc", 1024),
])
def test_mixed_tiers_match_oracle(oracle, scratch, streams, n_slots, chunk, order_kind, tile):
    ohp, ghp = hp_pair(oracle)
    wl = W.Workload("mix", n_sub=7, sub_elems=100_001, n_host=4, loss_scale=256.0, max_norm=0.05, steps=3)
    host = W.host_subgroups(wl, warm=True)
    tiers = [wl.tier(k) for k in range(wl.n_sub)]
    ds = DeviceSubgroups(host, tiers=tiers, flat=False, tile=tile)
    rng = np.random.default_rng(n_slots)
    hold = {"own_streams": n_slots % 2 == 1}      # half of the cases leave the copy streams to the library
    applied = 0
    for s in range(wl.steps):
        order = {"asc": None, "desc": list(range(wl.n_sub))[::-1], "perm": [int(x) for x in rng.permutation(wl.n_sub)]}[
            order_kind]
        if s > 0:
            for k, sg in enumerate(host):
                W.fill_grads(wl, k, s, sg["g"])
                ds.set_grads(k, sg["g"])
        ok_o, norm_o, flag_o, gmul_o = oracle.step(host, ohp, applied, wl.inv_scale, wl.max_norm, order=order)
        ok_g = stream_step(ds, scratch, ghp, applied, wl, streams, n_slots, chunk, order, hold)
        assert ok_g == ok_o is True
        sc = scratch.read()
        assert abs(float(sc["norm"]) / float(norm_o) - 1) <= 1e-5 and sc["gmul"] == gmul_o
        applied += 1
        for k in range(wl.n_sub):
            assert_state_parity(ds.fetch(k), host[k], f"slots={n_slots} chunk={chunk} tile={tile} step={s} sg={k}")


@pytest.mark.parametrize("blocks,order_kind,tile,flat_off", [
    (0, "asc", 0, None), (1, "perm", 0, None), (64, "desc", 8192, None), (300, "perm", 2048, None),
    (4096, "asc", 1024, None), (16, "asc", 0, 1),
])
def test_direct_mode_matches_oracle(oracle, scratch, streams, blocks, order_kind, tile, flat_off):
    # the host tier updated in place over the link by a bounded number of persistent workgroups
    ohp, ghp = hp_pair(oracle)
    wl = W.Workload("dir", n_sub=7, sub_elems=100_001, n_host=4, loss_scale=256.0, max_norm=0.05, steps=3)
    host = W.host_subgroups(wl, warm=True)
    tiers = [wl.tier(k) for k in range(wl.n_sub)]
    if flat_off is not None:
        # host-tier state that is only 4-byte aligned (a view one element into a pinned buffer): element-wise kernel
        ds = DeviceSubgroups(host, tiers=tiers, flat=False)
        keep = []
        descs = []
        for k, e in enumerate(ds.t):
            if tiers[k] == 1:
                for key in ("p", "m", "v"):
                    buf = torch.empty(e[key].numel() + flat_off, dtype=torch.float32, pin_memory=True)
                    buf[flat_off:].copy_(e[key])
                    keep.append(buf)
                    e[key] = buf[flat_off:]
            descs.append(B.subgroup(e["p"], e["m"], e["v"], e["g"], e["p16"], n=ds.sizes[k], tier=tiers[k]))
        ds.table = B.SubgroupTable(descs)
    else:
        ds = DeviceSubgroups(host, tiers=tiers, flat=False, tile=tile)
    rng = np.random.default_rng(blocks)
    applied = 0
    for s in range(wl.steps):
        order = {"asc": None, "desc": list(range(wl.n_sub))[::-1], "perm": [int(x) for x in rng.permutation(wl.n_sub)]}[
            order_kind]
        if s > 0:
            for k, sg in enumerate(host):
                W.fill_grads(wl, k, s, sg["g"])
                ds.set_grads(k, sg["g"])
        ok_o, norm_o, flag_o, gmul_o = oracle.step(host, ohp, applied, wl.inv_scale, wl.max_norm, order=order)
        ok_g = stream_step(ds, scratch, ghp, applied, wl, streams, 0, 0, order, {}, direct_blocks=blocks)
        assert ok_g == ok_o is True
        assert scratch.read()["gmul"] == gmul_o
        applied += 1
        for k in range(wl.n_sub):
            assert_state_parity(ds.fetch(k), host[k], f"direct blocks={blocks} tile={tile} step={s} sg={k}")


def test_direct_skip_leaves_host_state_untouched(oracle, scratch, streams):
    ohp, ghp = hp_pair(oracle)
    wl = W.Workload("dskip", n_sub=3, sub_elems=40_000, n_host=2)
    host = W.host_subgroups(wl, warm=True)
    host[0]["g"][123] = 0x7F80
    ds = DeviceSubgroups(host, tiers=[1, 1, 0], flat=False, tile=2048)
    assert stream_step(ds, scratch, ghp, 0, wl, streams, 0, 0, None, {}, direct_blocks=8) is False
    for k in range(wl.n_sub):
        got = ds.fetch(k)
        for key in ("p", "m", "v"):
            assert np.array_equal(got[key].view(np.uint32), host[k][key].view(np.uint32))


@pytest.mark.parametrize("tile", [0, 4096])
def test_skip_moves_nothing(oracle, scratch, streams, tile):
    ohp, ghp = hp_pair(oracle)
    wl = W.Workload("sskip", n_sub=4, sub_elems=50_000, n_host=2)
    host = W.host_subgroups(wl, warm=True)
    host[3]["g"][77] = 0xFF80
    for sg in host:
        sg["p16"][:] = 0x4321
    ds = DeviceSubgroups(host, tiers=[1, 1, 0, 0], flat=False, tile=tile)
    hold = {}
    assert stream_step(ds, scratch, ghp, 0, wl, streams, 3, 0, None, hold) is False
    assert scratch.read()["found_inf"] == 1
    # staging was never written: fill it with a pattern first and look again
    hold["t"].fill_(0x5A)
    assert stream_step(ds, scratch, ghp, 0, wl, streams, 3, 0, None, hold) is False
    assert bool((hold["t"] == 0x5A).all().item())
    for k in range(wl.n_sub):
        got = ds.fetch(k)
        for key in ("p", "m", "v"):
            assert np.array_equal(got[key].view(np.uint32), host[k][key].view(np.uint32))
        assert np.array_equal(got["p16"], host[k]["p16"])


@pytest.mark.parametrize("tile", [0, 8192])
def test_streamed_equals_resident_bitwise(oracle, scratch, streams, tile):
    # the same inputs once all-resident (planar) and once all-host with an awkward chunk size (planar or tiled):
    # identical bits
    _, ghp = hp_pair(oracle)
    wl = W.Workload("eq", n_sub=3, sub_elems=250_003, n_host=3, steps=2)
    host = W.host_subgroups(wl, warm=True)
    a = DeviceSubgroups(host, tiers=[0, 0, 0], flat=True)
    b = DeviceSubgroups(host, tiers=[1, 1, 1], flat=False, tile=tile)
    hold = {}
    for s in range(wl.steps):
        B.mlpo_adamw_step(a.table, ghp, s + 1, None, torch.cuda.current_stream())
        stream_step(b, scratch, ghp, s, wl, streams, 2, 65_536, [2, 0, 1], hold, norm=False)
    for k in range(wl.n_sub):
        ga, gb = a.fetch(k), b.fetch(k)
        for key in ("p", "m", "v", "p16"):
            assert np.array_equal(ga[key].view(np.uint8), gb[key].view(np.uint8)), (k, key)


def test_same_stream_for_everything(oracle, scratch):
    # the three roles may share one stream (no overlap, same result)
    ohp, ghp = hp_pair(oracle)
    wl = W.Workload("one", n_sub=3, sub_elems=30_000, n_host=2)
    host = W.host_subgroups(wl, warm=True)
    ds = DeviceSubgroups(host, tiers=[1, 1, 0], flat=False)
    s = torch.cuda.Stream()
    hold = {}
    assert stream_step(ds, scratch, ghp, 0, wl, (s, s, s), 2, 8192, None, hold)
    oracle.step(host, ohp, 0)
    for k in range(wl.n_sub):
        assert_state_parity(ds.fetch(k), host[k], f"one-stream sg={k}")


@pytest.mark.parametrize("tile", [0, 8192])
def test_config3_shape_scaled(oracle, scratch, streams, tile):
    # config 3's structure (13 host-tier subgroups, all state in pinned memory, 2-4 slots) at 1/100 of its size
    ohp, ghp = hp_pair(oracle)
    wl = W.Workload("C3/100", n_sub=13, sub_elems=1_000_000, n_host=13, steps=5, fresh_grads=False)
    host = W.host_subgroups(wl, warm=False, threads=8)
    ds = DeviceSubgroups(host, tiers=[1] * 13, flat=False, tile=tile)
    hold = {}
    for s in range(wl.steps):
        oracle.step(host, ohp, s)
        assert stream_step(ds, scratch, ghp, s, wl, streams, 2 + s % 3, 0, None, hold)
    for k in range(wl.n_sub):
        assert_state_parity(ds.fetch(k), host[k], f"C3/100 sg={k}")


@pytest.mark.parametrize("n_slots,tile,blocks", [(1, 0, 0), (2, 2048, 0), (3, 0, 0), (4, 8192, 3), (5, 0, 0),
                                                 (9, 2048, 0), (2, 1024, 200), (3, 4096, 1)])
def test_slot_cache_alternating_order(oracle, scratch, streams, n_slots, tile, blocks):
    """Cache-friendly ordering (Section 3.2): slots keep their subgroups, the order is reversed every step, a slot
    gives up its subgroup only when it is needed for another one.  The subgroups have one shape, so in the tiled
    layout every miss is served by the kernel that exchanges the two over the link (with `blocks` workgroups; the
    last element of each subgroup goes through the element-wise kernel); planar subgroups move by copies.  State
    must equal the oracle's after a final flush, and the transfer counts must be the ones the scheme promises."""
    ohp, ghp = hp_pair(oracle)
    wl = W.Workload("cache", n_sub=7, sub_elems=60_001, n_host=5, loss_scale=16.0, max_norm=0.05, steps=5)
    H = wl.n_host
    host = W.host_subgroups(wl, warm=True)
    tiers = [wl.tier(k) for k in range(wl.n_sub)]
    ds = DeviceSubgroups(host, tiers=tiers, flat=False, tile=tile)
    initial_last = {k: v.copy() for k, v in ds.fetch(H - 1).items()}
    cache = B.SlotCacheC()
    need = B.mlpo_stream_staging_bytes(ds.table, n_slots, 0)
    stg = torch.empty(need, dtype=torch.uint8, device=dev())
    cfg = B.stream_cfg(n_slots, stg, need, None, streams[1], None, 0, cache=cache, direct_blocks=blocks)
    for s in range(wl.steps):
        order = list(range(wl.n_sub)) if s % 2 == 0 else list(range(wl.n_sub))[::-1]
        if s > 0:
            for k, sg in enumerate(host):
                W.fill_grads(wl, k, s, sg["g"])
                ds.set_grads(k, sg["g"])
        ok_o = oracle.step(host, ohp, s, wl.inv_scale, wl.max_norm, order=order)[0]
        B.mlpo_grad_unscale_norm(ds.table, wl.inv_scale, wl.max_norm, scratch.ws, scratch.ws_bytes, scratch.scalars,
                                 streams[1])
        assert B.mlpo_stream_update(ds.table, order, ghp, s + 1, scratch.scalars, cfg) and ok_o
        streams[1].synchronize()
        if s == 0:
            # lazy flush: the subgroup processed last is still only in its slot, its host copy is the old one
            got = ds.fetch(H - 1)
            assert all(np.array_equal(got[key], initial_last[key]) for key in ("p", "m", "v"))
            assert cache.fetches == H and cache.hits == 0
    kept = min(n_slots, H)
    assert cache.hits == (wl.steps - 1) * kept
    assert cache.fetches == H + (wl.steps - 1) * (H - kept)
    B.mlpo_stream_flush(ds.table, cfg)
    streams[1].synchronize()
    assert cache.flushes == cache.fetches          # every stay in a slot ended with exactly one copy back
    B.mlpo_stream_flush(ds.table, cfg)             # nothing left to do
    assert cache.flushes == cache.fetches
    for k in range(wl.n_sub):
        assert_state_parity(ds.fetch(k), host[k], f"cache slots={n_slots} tile={tile} blocks={blocks} sg={k}")


@pytest.mark.parametrize("n_slots,tile,chunk,host_grads", [
    (2, 1024, 4096, False), (3, 1024, 8192, False), (2, 2048, 2048, True), (3, 1024, 4096, True),
    (2, 0, 4096, False), (2, 1024, B.CHUNK_WHOLE, False), (4, 1024, 1024, False),
])
def test_slot_cache_misses_in_pieces(oracle, scratch, streams, n_slots, tile, chunk, host_grads):
    """Subgroups of different lengths share the slots, so the newcomer is now shorter, now longer than the one it
    displaces, now as long: tiled subgroups are exchanged by kernels over the link (their common layout tiles in one
    pass, the rest of the longer one behind it), planar ones move by copies, the newcomer in pieces of `chunk`.
    State equals the oracle's after the final flush, transfer counts are those of whole-subgroup misses."""
    ohp, ghp = hp_pair(oracle)
    sizes = [50_001, 20_000, 50_001, 35_003, 50_001, 8_192, 3]
    wl = W.Workload("cachepieces", n_sub=len(sizes), sub_elems=max(sizes), n_host=len(sizes), loss_scale=8.0,
                    max_norm=0.04, steps=4)
    full = W.host_subgroups(wl, warm=True)
    host = [{key: a[:n].copy() for key, a in sg.items()} for sg, n in zip(full, sizes)]
    tiers = [1] * len(sizes)
    ds = DeviceSubgroups(host, tiers=tiers, flat=False, tile=tile)
    table = _host_grad_table(ds, tiers, tile) if host_grads else ds.table
    cache = B.SlotCacheC()
    need = B.mlpo_stream_staging_bytes(table, n_slots, B.CHUNK_WHOLE)
    stg = torch.empty(need, dtype=torch.uint8, device=dev())
    cfg = B.stream_cfg(n_slots, stg, need, None, streams[1], None, chunk, cache=cache)
    for s in range(wl.steps):
        order = list(range(wl.n_sub)) if s % 2 == 0 else list(range(wl.n_sub))[::-1]
        if s > 0:
            for k, sg in enumerate(host):
                fresh = np.empty(wl.sub_elems, np.uint16)
                W.fill_grads(wl, k, s, fresh)
                sg["g"][:] = fresh[:sizes[k]]
                if host_grads:
                    ds.t[k]["g_used"].copy_(torch.from_numpy(sg["g"].view(np.int16)))
                else:
                    ds.set_grads(k, sg["g"])
        torch.cuda.synchronize()
        ok_o, norm_o, flag_o, gmul_o = oracle.step(host, ohp, s, wl.inv_scale, wl.max_norm, order=order)
        B.mlpo_grad_unscale_norm(table, wl.inv_scale, wl.max_norm, scratch.ws, scratch.ws_bytes, scratch.scalars,
                                 streams[1])
        assert B.mlpo_stream_update(table, order, ghp, s + 1, scratch.scalars, cfg) and ok_o
        streams[1].synchronize()
        assert scratch.read()["gmul"] == gmul_o
    H = len(sizes)
    assert cache.hits == (wl.steps - 1) * n_slots and cache.fetches == H + (wl.steps - 1) * (H - n_slots)
    B.mlpo_stream_flush(table, cfg)
    streams[1].synchronize()
    assert cache.flushes == cache.fetches
    for k in range(wl.n_sub):
        assert_state_parity(ds.fetch(k), host[k], f"cache pieces slots={n_slots} tile={tile} chunk={chunk} sg={k}")


def test_slot_cache_survives_flush_and_skip(oracle, scratch, streams):
    ohp, ghp = hp_pair(oracle)
    wl = W.Workload("cache2", n_sub=4, sub_elems=30_011, n_host=4, steps=4)
    host = W.host_subgroups(wl, warm=True)
    ds = DeviceSubgroups(host, tiers=[1] * 4, flat=False, tile=1024)
    cache = B.SlotCacheC()
    need = B.mlpo_stream_staging_bytes(ds.table, 2, 0)
    stg = torch.empty(need, dtype=torch.uint8, device=dev())
    cfg = B.stream_cfg(2, stg, need, None, streams[1], None, 0, cache=cache)
    applied = 0
    for s in range(wl.steps):
        order = list(range(4)) if s % 2 == 0 else [3, 2, 1, 0]
        if s == 2:
            host[1]["g"][5] = 0x7F80               # a step that must be skipped: nothing moves, the cache is kept
            ds.set_grads(1, host[1]["g"])
        ok_o = oracle.step(host, ohp, applied, order=order)[0]
        B.mlpo_grad_unscale_norm(ds.table, 1.0, 0.0, scratch.ws, scratch.ws_bytes, scratch.scalars, streams[1])
        before = (cache.fetches, cache.flushes, cache.hits)
        ok_g = B.mlpo_stream_update(ds.table, order, ghp, applied + 1, scratch.scalars, cfg)
        streams[1].synchronize()
        assert ok_g == ok_o
        if not ok_g:
            assert (cache.fetches, cache.flushes, cache.hits) == before
            host[1]["g"][5] = 0x3A00
            ds.set_grads(1, host[1]["g"])
        applied += int(ok_g)
        if s == 1:
            B.mlpo_stream_flush(ds.table, cfg)     # a flush in the middle: host tier current, slots still valid
            streams[1].synchronize()
            for k in range(4):
                assert_state_parity(ds.fetch(k), host[k], f"mid-flush sg={k}")
    B.mlpo_stream_flush(ds.table, cfg)
    streams[1].synchronize()
    for k in range(4):
        assert_state_parity(ds.fetch(k), host[k], f"cache2 sg={k}")


def test_direct_mode_with_gradients_on_the_host(oracle, scratch, streams):
    """The paper's placement of the half-precision gradients (a pinned host buffer, converted on the fly during the
    update, Section 3.2): host-tier subgroups whose g is pinned host memory, read over the link by the gradient pass
    and by the direct-mode kernel."""
    ohp, ghp = hp_pair(oracle)
    wl = W.Workload("hostg", n_sub=5, sub_elems=80_003, n_host=3, loss_scale=128.0, max_norm=0.02, steps=3)
    host = W.host_subgroups(wl, warm=True)
    tiers = [wl.tier(k) for k in range(wl.n_sub)]
    ds = DeviceSubgroups(host, tiers=tiers, flat=False, tile=2048)
    pinned_g, descs = [], []
    for k, e in enumerate(ds.t):
        g = e["g"]
        if tiers[k] == 1:
            g = torch.empty(ds.sizes[k], dtype=torch.int16, pin_memory=True)
            g.copy_(e["g"])
            pinned_g.append(g)
        e["g_used"] = g
        descs.append(B.tiled_subgroup(e["state"], g, e["p16"], n=ds.sizes[k], tier=tiers[k], tile_elems=2048))
    table = B.SubgroupTable(descs)
    cfg = B.direct_cfg(streams[0], streams[1], 32)
    for s in range(wl.steps):
        if s > 0:
            for k, sg in enumerate(host):
                W.fill_grads(wl, k, s, sg["g"])
                ds.t[k]["g_used"].copy_(torch.from_numpy(sg["g"].view(np.int16)))
        torch.cuda.synchronize()
        ok_o, norm_o, flag_o, gmul_o = oracle.step(host, ohp, s, wl.inv_scale, wl.max_norm)
        B.mlpo_grad_unscale_norm(table, wl.inv_scale, wl.max_norm, scratch.ws, scratch.ws_bytes, scratch.scalars,
                                 streams[1])
        assert B.mlpo_stream_update(table, None, ghp, s + 1, scratch.scalars, cfg) and ok_o
        streams[1].synchronize()
        sc = scratch.read()
        assert abs(float(sc["norm"]) / float(norm_o) - 1) <= 1e-5 and sc["gmul"] == gmul_o
    for k in range(wl.n_sub):
        assert_state_parity(ds.fetch(k), host[k], f"host-side gradients sg={k}")


def _host_grad_table(ds, tiers, tile):
    """Subgroup table in which the gradients of every host-tier subgroup live in pinned host memory."""
    descs = []
    for k, e in enumerate(ds.t):
        g = e["g"]
        if tiers[k]:
            g = torch.empty(ds.sizes[k], dtype=torch.int16, pin_memory=True)
            g.copy_(e["g"])
        e["g_used"] = g
        tier = B.TIER_HOST_GRADS if tiers[k] else B.TIER_HBM
        if tile:
            descs.append(B.tiled_subgroup(e["state"], g, e["p16"], n=ds.sizes[k], tier=tier, tile_elems=tile))
        else:
            descs.append(B.subgroup(e["p"], e["m"], e["v"], g, e["p16"], n=ds.sizes[k], tier=tier))
    return B.SubgroupTable(descs)


@pytest.mark.parametrize("mode,n_slots,chunk,tile,cached", [
    ("staged", 1, 0, 0, False), ("staged", 2, 0, 2048, False), ("staged", 3, 4096, 0, False),
    ("staged", 2, 16_384, 2048, False), ("staged", 4, 33_332, 0, False), ("staged", 2, 0, 2048, True),
    ("staged", 3, 0, 0, True), ("staged", 5, 0, 8192, True), ("direct", 0, 0, 2048, False), ("direct", 0, 0, 0, False),
])
def test_gradients_fetched_from_the_host_with_the_state(oracle, scratch, streams, mode, n_slots, chunk, tile, cached):
    """Host-tier subgroups whose bf16 gradients sit in pinned host memory too (Section 3.2 "Delayed In-place
    Mixed-Precision Gradient Conversion"): staged mode brings them into the slot with the state, a slot cache fetches
    them anew every step, direct mode reads them in place.  Fresh gradients every step, alternating order."""
    ohp, ghp = hp_pair(oracle)
    wl = W.Workload("hostg2", n_sub=6, sub_elems=70_001, n_host=4, loss_scale=64.0, max_norm=0.03, steps=4)
    host = W.host_subgroups(wl, warm=True)
    tiers = [wl.tier(k) for k in range(wl.n_sub)]
    ds = DeviceSubgroups(host, tiers=tiers, flat=False, tile=tile)
    table = _host_grad_table(ds, tiers, tile)
    cache = B.SlotCacheC() if cached else None
    if mode == "direct":
        cfg, stg = B.direct_cfg(streams[0], streams[1], 24), None
    else:
        need = B.mlpo_stream_staging_bytes(table, n_slots, chunk)
        stg = torch.empty(need, dtype=torch.uint8, device=dev())
        cfg = B.stream_cfg(n_slots, stg, need, None, streams[1], None, chunk, cache=cache)
    for s in range(wl.steps):
        order = list(range(wl.n_sub)) if s % 2 == 0 else list(range(wl.n_sub))[::-1]
        if s > 0:
            for k, sg in enumerate(host):
                W.fill_grads(wl, k, s, sg["g"])
                ds.t[k]["g_used"].copy_(torch.from_numpy(sg["g"].view(np.int16)))
        torch.cuda.synchronize()
        ok_o, norm_o, flag_o, gmul_o = oracle.step(host, ohp, s, wl.inv_scale, wl.max_norm, order=order)
        B.mlpo_grad_unscale_norm(table, wl.inv_scale, wl.max_norm, scratch.ws, scratch.ws_bytes, scratch.scalars,
                                 streams[1])
        assert B.mlpo_stream_update(table, order, ghp, s + 1, scratch.scalars, cfg) and ok_o
        streams[1].synchronize()
        sc = scratch.read()
        assert abs(float(sc["norm"]) / float(norm_o) - 1) <= 1e-5 and sc["gmul"] == gmul_o
    if cached:
        assert cache.hits > 0
        B.mlpo_stream_flush(table, cfg)
        streams[1].synchronize()
    for k in range(wl.n_sub):
        assert_state_parity(ds.fetch(k), host[k], f"{mode} slots={n_slots} chunk={chunk} tile={tile} sg={k}")


@pytest.mark.parametrize("mode,tile", [("direct", 2048), ("staged", 0), ("staged", 1024)])
def test_gradient_pass_keeps_a_device_copy_of_host_gradients(oracle, scratch, streams, mode, tile):
    """Gradients in pinned host memory (Section 3.2 "Delayed In-place Mixed-Precision Gradient Conversion"): the
    gradient pass reads them over the link once and leaves a copy in device memory, the update that follows reads
    the copy (the subgroup is then described as host-tier state with device gradients).  The copy equals the
    gradients bit for bit - odd lengths and odd starting addresses included -, the record equals the plain pass's, and
    the state equals the oracle's."""
    ohp, ghp = hp_pair(oracle)
    sizes = [70_001, 3, 40_000, 8_191, 25_002]
    wl = W.Workload("keep", n_sub=len(sizes), sub_elems=max(sizes), n_host=3, loss_scale=64.0, max_norm=0.03, steps=3)
    full = W.host_subgroups(wl, warm=True)
    host = [{key: a[:n].copy() for key, a in sg.items()} for sg, n in zip(full, sizes)]
    tiers = [wl.tier(k) for k in range(wl.n_sub)]
    ds = DeviceSubgroups(host, tiers=tiers, flat=False, tile=tile)
    # host-side gradients: slices of one pinned buffer that start at odd elements; device copies with the same phase
    pinned = torch.zeros(sum(sizes) + 64, dtype=torch.int16).pin_memory()
    copies = torch.zeros(sum(sizes) + 64, dtype=torch.int16, device=dev())
    lo, grads_src, keep, update_descs = 3, [], [], []
    for k, n in enumerate(sizes):
        if tile:                        # the tiled kernels want 8-byte aligned gradients
            lo = (lo + 3) // 4 * 4
        src = pinned[lo:lo + n] if tiers[k] else ds.t[k]["g"]
        dst = copies[lo:lo + n] if tiers[k] else None
        grads_src.append(src)
        keep.append(dst)
        lo += n + 1
    norm_descs = []
    for k, n in enumerate(sizes):
        e = ds.t[k]
        g_upd = keep[k] if tiers[k] else e["g"]
        if tile:
            norm_descs.append(B.tiled_subgroup(e["state"], grads_src[k], e["p16"], n=n, tier=tiers[k], tile_elems=tile))
            update_descs.append(B.tiled_subgroup(e["state"], g_upd, e["p16"], n=n, tier=tiers[k], tile_elems=tile))
        else:
            norm_descs.append(B.subgroup(e["p"], e["m"], e["v"], grads_src[k], e["p16"], n=n, tier=tiers[k]))
            update_descs.append(B.subgroup(e["p"], e["m"], e["v"], g_upd, e["p16"], n=n, tier=tiers[k]))
    norm_table, update_table = B.SubgroupTable(norm_descs), B.SubgroupTable(update_descs)
    if mode == "direct":
        cfg, stg = B.direct_cfg(streams[0], streams[1], 24), None
    else:
        need = B.mlpo_stream_staging_bytes(update_table, 2, 16_384)
        stg = torch.empty(need, dtype=torch.uint8, device=dev())
        cfg = B.stream_cfg(2, stg, need, None, streams[1], None, 16_384)
    plain = torch.zeros(4, dtype=torch.float32, device=dev())
    for s in range(wl.steps):
        for k, sg in enumerate(host):
            fresh = np.empty(wl.sub_elems, np.uint16)
            W.fill_grads(wl, k, s, fresh)
            sg["g"][:] = fresh[:sizes[k]]
            grads_src[k].copy_(torch.from_numpy(sg["g"].view(np.int16)))
        copies.zero_()
        torch.cuda.synchronize()
        ok_o, norm_o, flag_o, gmul_o = oracle.step(host, ohp, s, wl.inv_scale, wl.max_norm)
        B.mlpo_grad_unscale_norm(norm_table, wl.inv_scale, wl.max_norm, scratch.ws, scratch.ws_bytes, plain, streams[1])
        B.mlpo_grad_unscale_norm_keep(norm_table, keep, wl.inv_scale, wl.max_norm, scratch.ws, scratch.ws_bytes,
                                      scratch.scalars, streams[1])
        streams[1].synchronize()
        assert scratch.scalars.cpu().numpy().tobytes() == plain.cpu().numpy().tobytes()
        for k in range(wl.n_sub):
            if tiers[k]:
                assert torch.equal(keep[k].cpu(), grads_src[k]), f"copy of subgroup {k}"
        # nothing outside the copies was written
        mask = torch.ones_like(copies, dtype=torch.bool)
        for k in range(wl.n_sub):
            if tiers[k]:
                off = (keep[k].data_ptr() - copies.data_ptr()) // 2
                mask[off:off + sizes[k]] = False
        assert not bool(copies[mask].any())
        assert B.mlpo_stream_update(update_table, None, ghp, s + 1, scratch.scalars, cfg) and ok_o
        streams[1].synchronize()
        assert scratch.read()["gmul"] == gmul_o
        for k in range(wl.n_sub):
            assert_state_parity(ds.fetch(k), host[k], f"keep {mode} tile={tile} step {s} sg {k}")
    with pytest.raises(B.MlpoError):        # a copy with another 16-byte phase than its gradients
        B.mlpo_grad_unscale_norm_keep(norm_table, [copies[1:] if tiers[k] else None for k in range(wl.n_sub)],
                                      wl.inv_scale, wl.max_norm, scratch.ws, scratch.ws_bytes, scratch.scalars)


def test_direct_mode_without_host_wait_captured_in_a_hip_graph(oracle, scratch):
    """Plain direct mode with applied = NULL only enqueues (its kernels read the skip flag on the device), so the
    gradient pass and the update of a table with HBM-tier and host-tier subgroups can be captured once and replayed.
    One eager step comes first (it creates the library's events); without bias correction the constants do not depend
    on the step number, so every replay is one more step on whatever the gradient buffers hold.  Replays alternate
    with eager work, one of them with a non-finite gradient, and every replay is checked against the oracle."""
    hp_kw = dict(lr=3e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1, bias_correction=False)
    ohp, ghp = hp_pair(oracle, **hp_kw)
    wl = W.Workload("dgraph", n_sub=5, sub_elems=120_001, n_host=3, hp=W.AdamW(**hp_kw), loss_scale=32.0,
                    max_norm=0.02, steps=6)
    host = W.host_subgroups(wl, warm=True)
    tiers = [wl.tier(k) for k in range(wl.n_sub)]
    ds = DeviceSubgroups(host, tiers=tiers, flat=False, tile=2048)
    side, link = torch.cuda.Stream(), torch.cuda.Stream()
    cfg = B.direct_cfg(link, side, 24)

    def enqueue(st):
        B.mlpo_grad_unscale_norm(ds.table, wl.inv_scale, wl.max_norm, scratch.ws, scratch.ws_bytes, scratch.scalars, st)
        assert B.mlpo_stream_update(ds.table, None, ghp, 1, scratch.scalars, cfg, want_applied=False) is None

    applied = 0
    graph = None
    for s in range(wl.steps):
        inject = s == 3
        for k, sg in enumerate(host):
            W.fill_grads(wl, k, s, sg["g"])
        if inject:
            host[1]["g"][777] = 0x7F80
        for k, sg in enumerate(host):
            ds.set_grads(k, sg["g"])
        torch.cuda.synchronize()
        ok_o, norm_o, flag_o, gmul_o = oracle.step(host, ohp, applied, wl.inv_scale, wl.max_norm)
        if s == 0:
            enqueue(side)                           # eager
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                enqueue(torch.cuda.current_stream())
            torch.cuda.synchronize()
        else:
            graph.replay()
            torch.cuda.synchronize()
        sc = scratch.read()
        assert sc["found_inf"] == flag_o == int(inject) and ok_o == (not inject)
        if ok_o:
            assert abs(float(sc["norm"]) - float(norm_o)) <= 1e-5 * float(norm_o) and sc["gmul"] == gmul_o
            applied += 1
        for k in range(wl.n_sub):
            assert_state_parity(ds.fetch(k), host[k], f"step {s} sg {k}")
    assert applied == wl.steps - 1
