"""Seeded random scenarios for mlpo_stream_update: subgroups of random sizes (empty ones included) spread over every
tier and both layouts in one table, random mode, slots, chunking, slot cache, order and thread counts, a non-finite
gradient now and then, and in direct mode one or two files (on different file systems: two paths) and subgroups that
are flushed to another place - pinned memory, a file, HBM - than they came from (Algorithm 1 assigns the path anew at
every flush).  After every step every bit of state is compared with the oracle's (the paper's statement that
order and partitioning do not change the result, Section 3.2 "Cache-Friendly Ordering", Section 4.1 "Runtime
Configurations")."""
import math
import os

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2509_02480_amd import binding as B  # noqa: E402
from paper_2509_02480_amd import workloads as W  # noqa: E402

from gpu_util import Scratch, assert_state_parity, dev, hp_pair, pack_tiled, unpack_tiled  # noqa: E402

SIZES = [0, 1, 3, 4, 5, 63, 64, 1023, 1024, 1025, 2047, 4096, 8191, 8192, 12_289, 30_001, 50_000, 65_537]


def build(rng, host, tiers, tiles, paths, pick, half):
    """Device / pinned / file homes for every subgroup; file-tier subgroups go to the file that pick() names (files on
    different file systems are different paths, each with workers and bounce buffers of its own).  Returns (subgroup
    descriptors, file extents, bookkeeping per subgroup, fetch(k), descriptors of the files, their lengths)."""
    d = dev()
    descs, files, keep = [], [], []
    fds = [os.open(p, os.O_RDWR | os.O_CREAT, 0o600) for p in paths]
    offs = [0] * len(fds)
    for k, s in enumerate(host):
        n, T, tier = s["p"].size, tiles[k], tiers[k]
        g_home_host = tier == B.TIER_HOST_GRADS
        gsrc = torch.from_numpy(s["g"].view(np.int16))
        if g_home_host:
            g = torch.empty(max(n, 1), dtype=torch.int16, pin_memory=True)[:n]
            g.copy_(gsrc)
        else:
            g = gsrc.to(d) if n else torch.empty(0, dtype=torch.int16, device=d)
        p16 = torch.from_numpy(s["p16"].view(np.int16)).to(d) if n else torch.empty(0, dtype=torch.int16, device=d)
        ent = {"g": g, "p16": p16, "tier": tier, "T": T, "n": n}
        if n == 0:
            descs.append(B.SubgroupC(None, None, None, None, None, 0, tier, T, half, 0))
            files.append(None)
        elif tier == B.TIER_FILE:
            packed = pack_tiled(s["p"], s["m"], s["v"], T)
            w = pick()
            os.pwrite(fds[w], packed.tobytes(), offs[w])
            ent["off"], ent["fd"] = offs[w], fds[w]
            descs.append(B.SubgroupC(None, None, None, g.data_ptr(), p16.data_ptr(), n, tier, T, half, 0))
            files.append((fds[w], offs[w]))
            offs[w] += (packed.nbytes + 4095) // 4096 * 4096
        else:
            on_host = tier in (B.TIER_HOST, B.TIER_HOST_GRADS)
            if T:
                # HBM-tier subgroups may start a few slots into their state buffer
                lead = int(rng.choice([0, 0, 4, 60, 1020])) if tier == B.TIER_HBM else 0
                ent["lead"] = lead
                packed = torch.from_numpy(pack_tiled(s["p"], s["m"], s["v"], T, lead))
                if on_host:
                    st = torch.empty(packed.numel(), dtype=torch.float32, pin_memory=True)
                    st.copy_(packed)
                else:
                    st = packed.to(d)
                ent["state"] = st
                descs.append(B.tiled_subgroup(st, g, p16, n=n, tier=tier, tile_elems=T, half=half, lead=lead))
            else:
                arrs = []
                for key in ("p", "m", "v"):
                    src = torch.from_numpy(s[key])
                    if on_host:
                        t = torch.empty(n, dtype=torch.float32, pin_memory=True)
                        t.copy_(src)
                    else:
                        t = src.to(d)
                    arrs.append(t)
                ent["pmv"] = arrs
                descs.append(B.subgroup(arrs[0], arrs[1], arrs[2], g, p16, n=n, tier=tier, half=half))
            files.append(None)
        keep.append(ent)
    for fd, off in zip(fds, offs):
        os.ftruncate(fd, max(off, 4096))
        os.fsync(fd)
    torch.cuda.synchronize()

    def fetch(k):
        e = keep[k]
        n, T = e["n"], e["T"]
        p16 = e["p16"].cpu().numpy().view(np.uint16).copy()
        if n == 0:
            z = np.zeros(0, np.float32)
            return {"p": z, "m": z, "v": z, "p16": p16}
        if e["tier"] == B.TIER_FILE:
            buf = np.frombuffer(os.pread(e["fd"], B.mlpo_state_floats(n, T) * 4, e["off"]), dtype=np.float32)
            p, m, v = unpack_tiled(buf, n, T)
        elif T:
            p, m, v = unpack_tiled(e["state"].cpu().numpy(), n, T, e.get("lead", 0))
        else:
            p, m, v = (t.cpu().numpy().copy() for t in e["pmv"])
        return {"p": p, "m": m, "v": v, "p16": p16}

    return descs, files, keep, fetch, fds, offs


# MLPO_RANDOM_SEEDS=a:b runs that range of seeds instead (a wider sweep now and then)
_lo, _, _hi = os.environ.get("MLPO_RANDOM_SEEDS", "0:160").partition(":")
# scenarios from wider sweeps that once failed and stay in the default run: 204 = an EMPTY file-tier subgroup, whose
# file entry names no file, beside file-tier subgroups with a single bounce buffer
_SEEDS = list(range(int(_lo), int(_hi)))
if "MLPO_RANDOM_SEEDS" not in os.environ:
    _SEEDS += [204]


@pytest.mark.parametrize("seed", _SEEDS)
def test_random_scenario(oracle, tmp_path, seed):
    rng = np.random.default_rng(1000 + seed)
    direct = bool(rng.integers(0, 2))
    n_sub = int(rng.integers(1, 9))
    sizes = [int(rng.choice(SIZES)) for _ in range(n_sub)]
    tier_pool = [B.TIER_HBM, B.TIER_HOST, B.TIER_HOST_GRADS] + ([B.TIER_FILE] if direct else [])
    tiers = [int(rng.choice(tier_pool)) for _ in range(n_sub)]
    tiles = [int(rng.choice([0, 1024, 2048, 4096])) for _ in range(n_sub)]
    tiles = [t if tiers[k] != B.TIER_FILE else (t or 1024) for k, t in enumerate(tiles)]
    unit = 4
    for t in tiles:
        if t:
            unit = unit * t // math.gcd(unit, t)
    chunk = 0 if rng.integers(0, 3) == 0 else unit * int(rng.integers(1, 6))
    cached = (not direct) and bool(rng.integers(0, 2))     # misses move whole or in pieces of chunk
    # choices added later come from a generator of their own, so that the scenarios of the first one stay what they were
    rng2 = np.random.default_rng(77_000 + seed)
    if cached and rng2.integers(0, 2):
        # the host-tier subgroups get one shape (tiled): a miss is then one kernel that exchanges the slot's occupants
        n_common, t_common = int(rng2.choice(SIZES[1:])), int(rng2.choice([1024, 2048, 4096]))
        if chunk % t_common == 0:
            for k in range(n_sub):
                if tiers[k] in (B.TIER_HOST, B.TIER_HOST_GRADS):
                    sizes[k], tiles[k] = n_common, t_common
    n_slots = int(rng.integers(1, 6))
    hp_kw = dict(lr=float(rng.choice([1e-4, 3e-3])), weight_decay=float(rng.choice([0.0, 0.01])),
                 bias_correction=bool(rng.integers(0, 2)), l2_mode=bool(rng.integers(0, 2)))
    ohp, ghp = hp_pair(oracle, **hp_kw)
    inv_scale = float(rng.choice([1.0, 1 / 64.0]))
    half = int(rng.integers(0, 2))       # the generator's bit patterns read as bf16 or as fp16: finite either way
    half_name = ["bf16", "fp16"][half]
    max_norm = float(rng.choice([0.0, 0.01]))
    # host copies of the state, generated by the seeded generator subgroup by subgroup
    host = []
    for k, n in enumerate(sizes):
        wl = W.Workload("rnd", n_sub=1, sub_elems=max(n, 1), loss_scale=1.0 / inv_scale, seed=seed * 100 + k)
        s = W.host_subgroups(wl, warm=True)[0]
        host.append({key: a[:n].copy() for key, a in s.items()})
    label = (f"seed {seed}: {'direct' if direct else 'staged'} sizes {sizes} tiers {tiers} tiles {tiles} chunk {chunk} "
             f"slots {n_slots} cached {cached} {half_name}")
    print(label, flush=True)
    # a second file on another file system = a second path behind the offloaded tier
    paths = [str(tmp_path / "state.bin")]
    shm = f"/dev/shm/mlpo_rnd_{os.getpid()}_{seed}.bin"
    if direct and rng2.integers(0, 2) and os.path.isdir("/dev/shm") and \
            os.stat("/dev/shm").st_dev != os.stat(str(tmp_path)).st_dev:
        paths.append(shm)
    pick = lambda: int(rng2.integers(0, len(paths)))  # noqa: E731
    descs, files, keep, fetch, fds, file_end = build(rng, host, tiers, tiles, paths, pick, half)
    table = B.SubgroupTable(descs)
    scratch = Scratch()
    streams = (torch.cuda.Stream(), torch.cuda.Stream())
    cache = B.SlotCacheC() if cached else None
    try:
        if direct:
            slots = max(int(rng.integers(1, 4)), len(paths))    # every path needs a bounce buffer of its own
            blocks, threads = int(rng.integers(1, 40)), int(rng.integers(1, 5))
        else:
            need = B.mlpo_stream_staging_bytes(table, n_slots, B.CHUNK_WHOLE if cached else chunk)
            stg = torch.empty(max(need, 256), dtype=torch.uint8, device=dev())
            own = bool(rng.integers(0, 2))
            cfg = B.stream_cfg(n_slots, stg, stg.numel(), None if own else streams[0], streams[1],
                               None if own else streams[0], chunk, cache=cache)
        applied = 0
        for step in range(3):
            order = None if rng.integers(0, 2) else [int(x) for x in rng.permutation(n_sub)]
            for k, s in enumerate(host):
                n = sizes[k]
                if n == 0:
                    continue
                wl = W.Workload("rnd", n_sub=1, sub_elems=n, loss_scale=1.0 / inv_scale, seed=seed * 100 + k)
                W.fill_grads(wl, 0, step, s["g"])
                if step == 1 and seed % 4 == 0 and k == n_sub - 1:
                    s["g"][n // 2] = 0x7C00 if half else 0x7F80
                keep[k]["g"].copy_(torch.from_numpy(s["g"].view(np.int16)))
            moved = {}          # subgroup -> its new home, if this step's update is applied
            if direct:
                targets = [None] * n_sub
                for k, e in enumerate(keep):
                    movable = e["n"] > 0 and e["T"] and not e.get("lead")
                    if not movable or rng.integers(0, 3) != 0:
                        continue
                    floats = B.mlpo_state_floats(e["n"], e["T"])
                    kinds = {B.TIER_HBM: ["host", "file"], B.TIER_HOST_GRADS: ["host"]}.get(e["tier"],
                                                                                           ["host", "file", "hbm"])
                    kind = str(rng.choice(kinds))
                    if kind == "file":
                        w = pick()
                        targets[k] = (fds[w], file_end[w])
                        moved[k] = {"off": file_end[w], "fd": fds[w], "tier": B.TIER_FILE}
                        file_end[w] += (floats * 4 + 4095) // 4096 * 4096
                        os.ftruncate(fds[w], file_end[w])
                    else:
                        st = torch.full((floats,), float("nan"), dtype=torch.float32,
                                        **({"pin_memory": True} if kind == "host" else {"device": dev()}))
                        targets[k] = st
                        tier = B.TIER_HBM if kind == "hbm" else (
                            B.TIER_HOST_GRADS if e["tier"] == B.TIER_HOST_GRADS else B.TIER_HOST)
                        moved[k] = {"state": st, "tier": tier}
                if moved:
                    print(f"  step {step}: " + ", ".join(
                        f"sg {k} tier {keep[k]['tier']} -> {'file' if 'off' in v else 'tier ' + str(v['tier'])}"
                        for k, v in moved.items()), flush=True)
                need = B.mlpo_stream_bounce_bytes(table, slots, chunk, flush_to=targets)
                bounce = torch.empty(max(need, 4096), dtype=torch.uint8, pin_memory=True)
                cfg = B.direct_cfg(streams[0], streams[1], blocks, chunk_elems=chunk, files=files, bounce=bounce,
                                   bounce_bytes=bounce.numel(), file_slots=slots, file_threads=threads,
                                   flush_to=targets if moved else None)
            torch.cuda.synchronize()
            ok_o, norm_o, flag_o, gmul_o = oracle.step(host, ohp, applied, inv_scale, max_norm, order=order,
                                                       half=half_name)
            B.mlpo_grad_unscale_norm(table, inv_scale, max_norm, scratch.ws, scratch.ws_bytes, scratch.scalars,
                                     streams[1])
            ok_g = B.mlpo_stream_update(table, order, ghp, applied + 1, scratch.scalars, cfg)
            streams[1].synchronize()
            assert ok_g == bool(ok_o), label
            sc = scratch.read()
            assert sc["found_inf"] == flag_o, label
            if ok_o:
                applied += 1
                assert sc["gmul"] == gmul_o, label
                for k, new in moved.items():         # a skipped step moves nothing
                    e = keep[k]
                    e.pop("state", None)
                    e.pop("off", None)
                    e.pop("fd", None)
                    e["lead"] = 0
                    e.update(new)
                    if e["tier"] == B.TIER_FILE:
                        descs[k] = B.SubgroupC(None, None, None, e["g"].data_ptr(), e["p16"].data_ptr(), e["n"],
                                               B.TIER_FILE, e["T"], half, 0)
                        files[k] = (e["fd"], e["off"])
                    else:
                        descs[k] = B.tiled_subgroup(e["state"], e["g"], e["p16"], n=e["n"], tier=e["tier"],
                                                    tile_elems=e["T"], half=half)
                        files[k] = None
                if moved:
                    table = B.SubgroupTable(descs)
            if cached:
                B.mlpo_stream_flush(table, cfg)
                streams[1].synchronize()
            torch.cuda.synchronize()
            for k in range(n_sub):
                assert_state_parity(fetch(k), host[k], f"{label} step {step} sg {k}")
    finally:
        torch.cuda.synchronize()
        for fd in fds:
            os.close(fd)
        if len(paths) > 1:
            os.unlink(shm)
