"""GPU parity of the file path of the offloaded tier (mlpo_stream_update in direct mode with MLPO_TIER_FILE
subgroups): state that lives in a file passes through pinned bounce buffers, is updated in place over the link and is
written back, while host-tier and HBM-tier subgroups are updated as usual (Section 3.2 "Unified Multi-level,
Multi-path Asynchronous Offloading using Virtual Tiers", Section 3.4).  The file's contents after every step must be
bit-identical to the oracle's state, whatever the chunking, the number of bounce buffers and the order are."""
import os

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2509_02480_amd import binding as B  # noqa: E402
from paper_2509_02480_amd import workloads as W  # noqa: E402

from gpu_util import Scratch, assert_state_parity, dev, hp_pair, pack_tiled, unpack_tiled  # noqa: E402


class Shard:
    """Subgroups of a workload spread over HBM, pinned host memory and one file (or two: the subgroups listed in
    ``second`` live in ``path2``, which may lie on another file system, i.e. be another path), in the tiled layout."""

    def __init__(self, host, tiers, T, path, direct_io=True, path2=None, second=()):
        self.T, self.tiers, self.n = T, tiers, [s["p"].size for s in host]
        self.keep, descs, self.files = [], [], []
        d = dev()
        flags = os.O_RDWR | os.O_CREAT
        self.direct_io = False
        self.paths = [path] + ([path2] if path2 else [])
        self.fds = []
        for pth in self.paths:
            fd = -1
            if direct_io:
                try:
                    fd = os.open(pth, flags | os.O_DIRECT, 0o600)
                    self.direct_io = True
                except OSError:
                    fd = -1
            if fd < 0:
                fd = os.open(pth, flags, 0o600)
            self.fds.append(fd)
        self.fd, self.path = self.fds[0], path
        self.file_of = {k: (1 if k in second else 0) for k in range(len(host)) if tiers[k] == B.TIER_FILE}
        self.offsets, self.ends = {}, []
        for which, pth in enumerate(self.paths):
            off = 4096          # a header page the library must leave alone
            with open(pth, "r+b") as f:
                f.write(b"\xAB" * 4096)
                for k, s in enumerate(host):
                    if self.file_of.get(k) != which:
                        continue
                    packed = pack_tiled(s["p"], s["m"], s["v"], T)
                    self.offsets[k] = off
                    f.seek(off)
                    f.write(packed.tobytes())
                    off += (packed.nbytes + 4095) // 4096 * 4096
                f.seek(off)
                f.write(b"\xCD" * 4096)          # and a trailer page
                f.flush()
                os.fsync(f.fileno())
            self.ends.append(off)
        self.end = self.ends[0]
        for k, s in enumerate(host):
            n = self.n[k]
            g = torch.from_numpy(s["g"].view(np.int16)).to(d)
            p16 = torch.from_numpy(s["p16"].view(np.int16)).to(d)
            ent = {"g": g, "p16": p16}
            if tiers[k] == B.TIER_FILE:
                descs.append(B.SubgroupC(None, None, None, g.data_ptr(), p16.data_ptr(), n, B.TIER_FILE, T))
                self.files.append((self.fds[self.file_of[k]], self.offsets[k]))
            else:
                packed = torch.from_numpy(pack_tiled(s["p"], s["m"], s["v"], T))
                if tiers[k] == B.TIER_HOST:
                    st = torch.empty(packed.numel(), dtype=torch.float32, pin_memory=True)
                    st.copy_(packed)
                else:
                    st = packed.to(d)
                ent["state"] = st
                descs.append(B.tiled_subgroup(st, g, p16, n=n, tier=tiers[k], tile_elems=T))
                self.files.append(None)
            self.keep.append(ent)
        torch.cuda.synchronize()
        self.table = B.SubgroupTable(descs)

    def set_grads(self, k, bits):
        self.keep[k]["g"].copy_(torch.from_numpy(bits.view(np.int16)))

    def fetch(self, k):
        torch.cuda.synchronize()
        e = self.keep[k]
        if self.tiers[k] == B.TIER_FILE:
            count = B.mlpo_state_floats(self.n[k], self.T)
            buf = np.fromfile(self.paths[self.file_of[k]], dtype=np.float32, count=count, offset=self.offsets[k])
        else:
            buf = e["state"].cpu().numpy()
        p, m, v = unpack_tiled(buf, self.n[k], self.T)
        return {"p": p, "m": m, "v": v, "p16": e["p16"].cpu().numpy().view(np.uint16).copy()}

    def guards_intact(self):
        for pth, end in zip(self.paths, self.ends):
            with open(pth, "rb") as f:
                head = f.read(4096)
                f.seek(end)
                tail = f.read(4096)
            if head != b"\xAB" * 4096 or tail != b"\xCD" * 4096:
                return False
        return True

    def close(self):
        for fd in self.fds:
            os.close(fd)


def make_cfg(shard, streams, chunk, file_slots, blocks=24):
    need = B.mlpo_stream_bounce_bytes(shard.table, file_slots, chunk)
    bounce = torch.empty(max(need, 4096), dtype=torch.uint8, pin_memory=True)
    assert bounce.data_ptr() % 4096 == 0
    cfg = B.direct_cfg(streams[0], streams[1], blocks, chunk_elems=chunk, files=shard.files, bounce=bounce,
                       bounce_bytes=bounce.numel(), file_slots=file_slots, want_file_stats=True)
    cfg._bounce = bounce
    return cfg


F, H, D = B.TIER_FILE, B.TIER_HOST, B.TIER_HBM


@pytest.mark.parametrize("tiers,chunk,file_slots,order_kind,T", [
    ([F, H, F, H, D, F, D], 0, 3, "asc", 2048),
    ([F, H, F, H, D, F, D], 8192, 2, "desc", 2048),
    ([F, H, F, H, D, F, D], 32_768, 1, "perm", 1024),
    ([F, F, F], 16_384, 3, "asc", 8192),
    ([F], 0, 1, "asc", 2048),
    ([H, F, D], 4096, 4, "perm", 4096),
    ([F, H, H, H, H, H], 8192, 2, "asc", 2048),
])
def test_file_tier_matches_oracle(oracle, tmp_path, tiers, chunk, file_slots, order_kind, T):
    ohp, ghp = hp_pair(oracle)
    wl = W.Workload("filetier", n_sub=len(tiers), sub_elems=100_001, n_host=0, loss_scale=256.0, max_norm=0.05, steps=3)
    host = W.host_subgroups(wl, warm=True)
    shard = Shard(host, tiers, T, str(tmp_path / "state.bin"))
    scratch = Scratch()
    streams = (torch.cuda.Stream(), torch.cuda.Stream())
    cfg = make_cfg(shard, streams, chunk, file_slots)
    rng = np.random.default_rng(len(tiers) + chunk)
    file_bytes = sum(B.mlpo_state_floats(wl.sub_elems, T) * 4 for t in tiers if t == F)
    try:
        for s in range(wl.steps):
            order = {"asc": None, "desc": list(range(wl.n_sub))[::-1],
                     "perm": [int(x) for x in rng.permutation(wl.n_sub)]}[order_kind]
            if s > 0:
                for k, sg in enumerate(host):
                    W.fill_grads(wl, k, s, sg["g"])
                    shard.set_grads(k, sg["g"])
            torch.cuda.synchronize()
            ok_o, norm_o, flag_o, gmul_o = oracle.step(host, ohp, s, wl.inv_scale, wl.max_norm, order=order)
            B.mlpo_grad_unscale_norm(shard.table, wl.inv_scale, wl.max_norm, scratch.ws, scratch.ws_bytes,
                                     scratch.scalars, streams[1])
            assert B.mlpo_stream_update(shard.table, order, ghp, s + 1, scratch.scalars, cfg) and ok_o
            streams[1].synchronize()
            sc = scratch.read()
            assert abs(float(sc["norm"]) / float(norm_o) - 1) <= 1e-5 and sc["gmul"] == gmul_o
            assert cfg.stats.bytes_read == cfg.stats.bytes_written == file_bytes
            assert cfg.stats.read_seconds > 0 and cfg.stats.write_seconds > 0 and cfg.stats.wall_seconds > 0
            for k in range(wl.n_sub):
                assert_state_parity(shard.fetch(k), host[k], f"step {s} sg {k} tier {tiers[k]}")
        assert shard.guards_intact()
    finally:
        torch.cuda.synchronize()
        shard.close()


@pytest.mark.parametrize("chunk,file_slots,threads", [(8192, 6, 2), (16_384, 2, 1), (0, 4, 3)])
def test_three_paths_side_by_side(oracle, tmp_path, chunk, file_slots, threads):
    """Three live paths behind the offloaded tier (Section 3.2 "Unified Multi-level, Multi-path Asynchronous
    Offloading using Virtual Tiers"): pinned host memory, a file in /dev/shm (pageable host memory) and a file on the
    disk.  Eq. 1 (Section 3.3) splits the subgroups over the three from guessed bandwidths, each file path has its
    own workers and bounce buffers, the state equals the oracle's after every step, the statistics come back per
    path, and re-estimating Eq. 1 from what was observed gives an allocation that is carried out by flush targets."""
    if not os.path.isdir("/dev/shm") or os.stat("/dev/shm").st_dev == os.stat(str(tmp_path)).st_dev:
        pytest.skip("no second file system for the third path")
    ohp, ghp = hp_pair(oracle)
    T = 2048
    n_sub = 9
    wl = W.Workload("threepaths", n_sub=n_sub, sub_elems=60_001, n_host=0, loss_scale=32.0, max_norm=0.05, steps=3)
    host = W.host_subgroups(wl, warm=True)
    # Eq. 1 over pinned : shm file : disk file with the guess 4 : 3 : 2 -> 4 / 3 / 2 subgroups; the slowest path takes
    # the lowest ids
    counts, tier_of = B.mlpo_assign_tiers(n_sub, [4.0, 3.0, 2.0])
    assert counts == [4, 3, 2] and tier_of == [2, 2, 1, 1, 1, 0, 0, 0, 0]
    tiers = [H if t == 0 else F for t in tier_of]
    on_disk = [k for k in range(n_sub) if tier_of[k] == 2]
    shm = f"/dev/shm/mlpo_three_{os.getpid()}.bin"
    shard = Shard(host, tiers, T, shm, direct_io=True, path2=str(tmp_path / "disk.bin"), second=on_disk)
    scratch = Scratch()
    streams = (torch.cuda.Stream(), torch.cuda.Stream())
    need = B.mlpo_stream_bounce_bytes(shard.table, file_slots, chunk)
    bounce = torch.empty(max(need, 4096), dtype=torch.uint8, pin_memory=True)
    cfg = B.direct_cfg(streams[0], streams[1], 24, chunk_elems=chunk, files=shard.files, bounce=bounce,
                       bounce_bytes=bounce.numel(), file_slots=file_slots, file_threads=threads, want_file_stats=True)
    per = B.mlpo_state_floats(wl.sub_elems, T) * 4
    ids = [os.fstat(fd).st_dev for fd in shard.fds]
    try:
        for s in range(wl.steps):
            order = None if s % 2 == 0 else list(range(n_sub))[::-1]
            if s > 0:
                for k, sg in enumerate(host):
                    W.fill_grads(wl, k, s, sg["g"])
                    shard.set_grads(k, sg["g"])
            torch.cuda.synchronize()
            ok_o, norm_o, flag_o, gmul_o = oracle.step(host, ohp, s, wl.inv_scale, wl.max_norm, order=order)
            B.mlpo_grad_unscale_norm(shard.table, wl.inv_scale, wl.max_norm, scratch.ws, scratch.ws_bytes,
                                     scratch.scalars, streams[1])
            assert B.mlpo_stream_update(shard.table, order, ghp, s + 1, scratch.scalars, cfg) and ok_o
            streams[1].synchronize()
            assert scratch.read()["gmul"] == gmul_o
            used = [p for p in cfg.paths if p.used]
            assert len(used) == 2 and sorted(p.path_id for p in used) == sorted(ids)
            by_id = {p.path_id: p.stats for p in used}
            assert by_id[ids[0]].bytes_read == by_id[ids[0]].bytes_written == 3 * per       # the file in /dev/shm
            assert by_id[ids[1]].bytes_read == by_id[ids[1]].bytes_written == 2 * per       # the file on the disk
            assert cfg.stats.bytes_read == 5 * per and all(p.stats.wall_seconds > 0 for p in used)
            # ascending order meets the disk's subgroups first, descending the others'
            assert used[0].path_id == (ids[1] if order is None else ids[0])
            for k in range(n_sub):
                assert_state_parity(shard.fetch(k), host[k], f"three paths step {s} sg {k}")
        assert shard.guards_intact()
        # Section 3.3: the next split follows what the paths showed.  Observed (made up here, the files are small):
        # the disk at a quarter of its guess -> Eq. 1 takes a subgroup away from it; the move happens inside an
        # ordinary step, by a flush target (disk file -> pinned memory)
        seen = B.mlpo_update_bandwidth([4.0, 3.0, 2.0], [4.0 * per, 3.0 * per, 2.0 * per], [per, per, 4.0 * per])
        assert seen == [4.0, 3.0, 0.5]
        new_counts, _ = B.mlpo_assign_tiers(n_sub, seen)
        assert new_counts == oracle_tiers(n_sub, seen) and new_counts[2] < 2
        mover = on_disk[-1]
        home = torch.zeros(per // 4, dtype=torch.float32).pin_memory()
        targets = [None] * n_sub
        targets[mover] = home
        move = B.direct_cfg(streams[0], streams[1], 24, chunk_elems=chunk, files=shard.files, bounce=bounce,
                            bounce_bytes=bounce.numel(), file_slots=file_slots, file_threads=threads,
                            want_file_stats=True, flush_to=targets)
        for k, sg in enumerate(host):
            W.fill_grads(wl, k, wl.steps, sg["g"])
            shard.set_grads(k, sg["g"])
        torch.cuda.synchronize()
        ok_o, _, _, gmul_o = oracle.step(host, ohp, wl.steps, wl.inv_scale, wl.max_norm)
        B.mlpo_grad_unscale_norm(shard.table, wl.inv_scale, wl.max_norm, scratch.ws, scratch.ws_bytes, scratch.scalars,
                                 streams[1])
        assert B.mlpo_stream_update(shard.table, None, ghp, wl.steps + 1, scratch.scalars, move) and ok_o
        streams[1].synchronize()
        by_id = {p.path_id: p.stats for p in move.paths if p.used}
        assert by_id[ids[1]].bytes_read == 2 * per and by_id[ids[1]].bytes_written == per   # one left the disk
        p_, m_, v_ = unpack_tiled(home.numpy(), wl.sub_elems, T)
        got = {"p": p_, "m": m_, "v": v_, "p16": shard.keep[mover]["p16"].cpu().numpy().view(np.uint16).copy()}
        assert_state_parity(got, host[mover], "the subgroup that moved from the disk to pinned memory")
    finally:
        torch.cuda.synchronize()
        shard.close()
        for pth in shard.paths:
            if os.path.exists(pth):
                os.unlink(pth)


def oracle_tiers(n_sub, bandwidth):
    from oracle import tier_alloc
    return tier_alloc.assign_tiers(n_sub, bandwidth)[0]


def test_too_few_bounce_buffers_for_the_paths(tmp_path):
    if not os.path.isdir("/dev/shm") or os.stat("/dev/shm").st_dev == os.stat(str(tmp_path)).st_dev:
        pytest.skip("no second file system")
    wl = W.Workload("twopaths", n_sub=2, sub_elems=5000, n_host=0)
    host = W.host_subgroups(wl)
    shm = f"/dev/shm/mlpo_two_{os.getpid()}.bin"
    shard = Shard(host, [F, F], 1024, shm, direct_io=False, path2=str(tmp_path / "b.bin"), second=[1])
    streams = (torch.cuda.Stream(), torch.cuda.Stream())
    try:
        cfg = make_cfg(shard, streams, 0, 1)        # one bounce buffer, two paths
        with pytest.raises(B.MlpoError) as e:
            B.mlpo_stream_update(shard.table, None, B.HParams(), 1, None, cfg)
        assert e.value.code == B.MLPO_EINVAL and "paths" in str(e.value)
    finally:
        shard.close()
        os.unlink(shm)


def test_skipped_step_touches_no_file(oracle, tmp_path):
    ohp, ghp = hp_pair(oracle)
    tiers = [F, H, D, F]
    wl = W.Workload("fileskip", n_sub=4, sub_elems=50_003, n_host=0, loss_scale=64.0, steps=1)
    host = W.host_subgroups(wl, warm=True)
    host[3]["g"][777] = 0x7F80
    path = str(tmp_path / "state.bin")
    shard = Shard(host, tiers, 2048, path)
    before = open(path, "rb").read()
    scratch = Scratch()
    streams = (torch.cuda.Stream(), torch.cuda.Stream())
    cfg = make_cfg(shard, streams, 8192, 2)
    try:
        B.mlpo_grad_unscale_norm(shard.table, wl.inv_scale, 0.0, scratch.ws, scratch.ws_bytes, scratch.scalars,
                                 streams[1])
        cfg.stats.bytes_read = 123          # stale figures from an earlier step must not survive a skipped one
        assert B.mlpo_stream_update(shard.table, None, ghp, 1, scratch.scalars, cfg) is False
        streams[1].synchronize()
        assert cfg.stats.bytes_read == 0 and cfg.stats.bytes_written == 0 and cfg.stats.wall_seconds == 0.0
        assert open(path, "rb").read() == before
        ok_o, *_ = oracle.step(host, ohp, 0, wl.inv_scale, 0.0)
        assert not ok_o
        for k in range(4):
            assert_state_parity(shard.fetch(k), host[k], f"skip sg {k}")
    finally:
        shard.close()


def test_write_failure_is_reported(oracle, tmp_path):
    """A descriptor opened read-only: the reads work, the kernel runs, the write back fails - the call must say so
    (and every thread and kernel must still finish)."""
    _, ghp = hp_pair(oracle)
    wl = W.Workload("fileerr", n_sub=2, sub_elems=30_000, n_host=0, steps=1)
    host = W.host_subgroups(wl, warm=True)
    path = str(tmp_path / "state.bin")
    shard = Shard(host, [F, D], 2048, path, direct_io=False)
    ro = os.open(path, os.O_RDONLY)
    streams = (torch.cuda.Stream(), torch.cuda.Stream())
    files = [(ro, shard.offsets[0]), None]
    need = B.mlpo_stream_bounce_bytes(shard.table, 2, 8192)
    bounce = torch.empty(need, dtype=torch.uint8, pin_memory=True)
    cfg = B.direct_cfg(streams[0], streams[1], 8, chunk_elems=8192, files=files, bounce=bounce, bounce_bytes=need,
                       file_slots=2)
    try:
        with pytest.raises(B.MlpoError) as ei:
            B.mlpo_stream_update(shard.table, None, ghp, 1, None, cfg)
        assert ei.value.code == B.MLPO_EIO and "writing" in str(ei.value)
        torch.cuda.synchronize()
    finally:
        os.close(ro)
        shard.close()


@pytest.mark.parametrize("threads,direct_io,where", [(1, True, "tmp"), (3, False, "tmp"), (5, True, "tmp"),
                                                      (16, False, "tmp"), (1, False, "shm"), (4, False, "shm"),
                                                      (7, False, "shm")])
def test_io_threads_and_kinds_of_descriptors(oracle, tmp_path, threads, direct_io, where):
    """1..16 threads per direction, each moving its share of every piece; descriptors with O_DIRECT (served through
    the library's page-aligned blocks), without (plain pread / pwrite), and files in tmpfs (copied through a
    mapping)."""
    ohp, ghp = hp_pair(oracle)
    tiers = [F, H, F]
    wl = W.Workload("fileio", n_sub=3, sub_elems=90_001, n_host=0, steps=2)
    host = W.host_subgroups(wl, warm=True)
    path = str(tmp_path / "state.bin")
    if where == "shm":
        if not os.access("/dev/shm", os.W_OK):
            pytest.skip("no writable /dev/shm")
        path = f"/dev/shm/mlpo_test_state_{os.getpid()}_{threads}.bin"
    shard = Shard(host, tiers, 2048, path, direct_io=direct_io)
    streams = (torch.cuda.Stream(), torch.cuda.Stream())
    need = B.mlpo_stream_bounce_bytes(shard.table, 2, 16_384)
    bounce = torch.empty(need, dtype=torch.uint8, pin_memory=True)
    cfg = B.direct_cfg(streams[0], streams[1], 16, chunk_elems=16_384, files=shard.files, bounce=bounce,
                       bounce_bytes=need, file_slots=2, file_threads=threads, want_file_stats=True)
    try:
        for s in range(wl.steps):
            oracle.step(host, ohp, s)
            assert B.mlpo_stream_update(shard.table, None, ghp, s + 1, None, cfg)
            streams[1].synchronize()
        assert cfg.stats.bytes_read == cfg.stats.bytes_written == 2 * B.mlpo_state_floats(wl.sub_elems, 2048) * 4
        for k in range(3):
            assert_state_parity(shard.fetch(k), host[k], f"threads={threads} direct_io={shard.direct_io} sg {k}")
        assert shard.guards_intact()
    finally:
        torch.cuda.synchronize()
        shard.close()
        if where == "shm" and os.path.exists(path):
            os.unlink(path)


@pytest.mark.parametrize("chunk,file_slots,direct_io", [(0, 1, False), (8192, 3, True), (16_384, 2, False)])
def test_subgroups_change_their_path_at_flush_time(oracle, tmp_path, chunk, file_slots, direct_io):
    """Algorithm 1 assigns the path anew whenever a subgroup is flushed.  Every subgroup has two device buffers, two
    pinned buffers and two file extents to live in; a schedule moves them around - between pinned memory, the file
    and HBM, to another buffer or extent of the same kind, or not at all - while the updates go on.  After every
    step the state is read from wherever it lives now and compared with the oracle's."""
    ohp, ghp = hp_pair(oracle)
    T, n, n_sub = 2048, 90_001, 5
    wl = W.Workload("move", n_sub=n_sub, sub_elems=n, n_host=0, loss_scale=16.0, max_norm=0.1, steps=5)
    host = W.host_subgroups(wl, warm=True)
    floats = B.mlpo_state_floats(n, T)
    ext = (floats * 4 + 4095) // 4096 * 4096
    path = str(tmp_path / "state.bin")
    with open(path, "wb") as f:
        f.truncate(2 * n_sub * ext)
    try:
        fd = os.open(path, os.O_RDWR | (os.O_DIRECT if direct_io else 0))
    except OSError:
        fd = os.open(path, os.O_RDWR)
    plain = os.open(path, os.O_RDWR)          # the test's own reads and writes (no alignment rules)
    d = dev()
    pinned = [[torch.zeros(floats, dtype=torch.float32, pin_memory=True) for _ in range(2)] for _ in range(n_sub)]
    device = [[torch.zeros(floats, dtype=torch.float32, device=d) for _ in range(2)] for _ in range(n_sub)]
    extent = [[(2 * k + j) * ext for j in range(2)] for k in range(n_sub)]
    g = [torch.from_numpy(s["g"].view(np.int16)).to(d) for s in host]
    p16 = [torch.from_numpy(s["p16"].view(np.int16)).to(d) for s in host]
    # where each subgroup lives: (kind, j) with kind "hbm", "host" or "file" and j the buffer / extent of that kind
    home = [("file", 0), ("host", 0), ("host", 1), ("file", 1), ("hbm", 0)]
    for k, (kind, j) in enumerate(home):
        packed = pack_tiled(host[k]["p"], host[k]["m"], host[k]["v"], T)
        if kind == "host":
            pinned[k][j].copy_(torch.from_numpy(packed))
        elif kind == "hbm":
            device[k][j].copy_(torch.from_numpy(packed))
        else:
            os.pwrite(plain, packed.tobytes() + bytes(ext - packed.nbytes), extent[k][j])
    os.fsync(plain)
    schedule = [
        # file->pinned, pinned->file, pinned->pinned', file->file', HBM->pinned
        [("host", 0), ("file", 0), ("host", 0), ("file", 0), ("host", 0)],
        # pinned->HBM, stays, pinned->HBM, stays, stays
        [("hbm", 0), ("file", 0), ("hbm", 0), ("file", 0), ("host", 0)],
        # HBM->file, file->HBM, HBM->file, file->pinned, pinned->file
        [("file", 1), ("hbm", 1), ("file", 0), ("host", 1), ("file", 0)],
        # file->file', stays in HBM, file->file', pinned->pinned', file->HBM
        [("file", 0), ("hbm", 1), ("file", 1), ("host", 0), ("hbm", 0)],
        # file->pinned, HBM->pinned, file->pinned, stays, stays in HBM
        [("host", 1), ("host", 0), ("host", 0), ("host", 0), ("hbm", 0)],
    ]

    def table_and_files():
        descs, files = [], []
        for k, (kind, j) in enumerate(home):
            if kind == "file":
                descs.append(B.SubgroupC(None, None, None, g[k].data_ptr(), p16[k].data_ptr(), n, B.TIER_FILE, T))
                files.append((fd, extent[k][j]))
            else:
                state, tier = (pinned[k][j], B.TIER_HOST) if kind == "host" else (device[k][j], B.TIER_HBM)
                descs.append(B.tiled_subgroup(state, g[k], p16[k], n=n, tier=tier, tile_elems=T))
                files.append(None)
        return B.SubgroupTable(descs), files

    def fetch(k):
        torch.cuda.synchronize()
        kind, j = home[k]
        if kind == "hbm":
            buf = device[k][j].cpu().numpy()
        elif kind == "host":
            buf = pinned[k][j].numpy()
        else:
            buf = np.frombuffer(os.pread(plain, floats * 4, extent[k][j]), dtype=np.float32)
        p, m, v = unpack_tiled(buf, n, T)
        return {"p": p, "m": m, "v": v, "p16": p16[k].cpu().numpy().view(np.uint16).copy()}

    scratch = Scratch()
    streams = (torch.cuda.Stream(), torch.cuda.Stream())
    try:
        for s in range(wl.steps):
            if s > 0:
                for k, sg in enumerate(host):
                    W.fill_grads(wl, k, s, sg["g"])
                    g[k].copy_(torch.from_numpy(sg["g"].view(np.int16)))
            table, files = table_and_files()
            new_home = schedule[s]
            targets = []
            for k in range(n_sub):
                kind, j = new_home[k]
                if new_home[k] == home[k]:
                    targets.append(None)
                elif kind == "file":
                    targets.append((fd, extent[k][j]))
                else:
                    buf = pinned[k][j] if kind == "host" else device[k][j]
                    buf.fill_(float("nan"))          # whatever was there must be overwritten
                    targets.append(buf)
            need = B.mlpo_stream_bounce_bytes(table, file_slots, chunk, flush_to=targets)
            bounce = torch.empty(max(need, 4096), dtype=torch.uint8, pin_memory=True)
            cfg = B.direct_cfg(streams[0], streams[1], 20, chunk_elems=chunk, files=files, bounce=bounce,
                               bounce_bytes=bounce.numel(), file_slots=file_slots, file_threads=2,
                               want_file_stats=True, flush_to=targets)
            torch.cuda.synchronize()
            ok_o, norm_o, flag_o, gmul_o = oracle.step(host, ohp, s, wl.inv_scale, wl.max_norm)
            B.mlpo_grad_unscale_norm(table, wl.inv_scale, wl.max_norm, scratch.ws, scratch.ws_bytes, scratch.scalars,
                                     streams[1])
            assert B.mlpo_stream_update(table, None, ghp, s + 1, scratch.scalars, cfg) and ok_o
            streams[1].synchronize()
            assert scratch.read()["gmul"] == gmul_o
            reads = sum(1 for k in range(n_sub) if home[k][0] == "file")
            writes = sum(1 for k in range(n_sub) if new_home[k][0] == "file")
            assert cfg.stats.bytes_read == reads * floats * 4 and cfg.stats.bytes_written == writes * floats * 4
            home = list(new_home)
            for k in range(n_sub):
                assert_state_parity(fetch(k), host[k], f"step {s} sg {k} now at {home[k]}")
    finally:
        torch.cuda.synchronize()
        os.close(fd)
        os.close(plain)


@pytest.mark.parametrize("n", [3, 4, 7, 5000, 70_001])
def test_hbm_only_table_with_subgroups_on_their_way_out(oracle, tmp_path, n):
    """Nothing is offloaded yet: three HBM-tier subgroups, of which one goes to pinned memory and one to a file in
    this step.  (A table without host- or file-tier subgroups takes a shortcut to the resident kernel; subgroups that
    leave HBM must not take it.)"""
    ohp, ghp = hp_pair(oracle)
    T = 2048
    wl = W.Workload("out", n_sub=3, sub_elems=n, n_host=0, steps=2, seed=n)
    host = W.host_subgroups(wl, warm=True)
    floats = B.mlpo_state_floats(n, T)
    path = str(tmp_path / "state.bin")
    with open(path, "wb") as f:
        f.truncate(floats * 4)
    fd = os.open(path, os.O_RDWR)
    d = dev()
    state = [torch.from_numpy(pack_tiled(s["p"], s["m"], s["v"], T)).to(d) for s in host]
    g = [torch.from_numpy(s["g"].view(np.int16)).to(d) for s in host]
    p16 = [torch.from_numpy(s["p16"].view(np.int16)).to(d) for s in host]
    table = B.SubgroupTable([B.tiled_subgroup(state[k], g[k], p16[k], n=n, tile_elems=T) for k in range(3)])
    pinned = torch.full((floats,), float("nan"), dtype=torch.float32, pin_memory=True)
    targets = [pinned, None, (fd, 0)]
    need = B.mlpo_stream_bounce_bytes(table, 2, 0, flush_to=targets)
    bounce = torch.empty(need, dtype=torch.uint8, pin_memory=True)
    streams = (torch.cuda.Stream(), torch.cuda.Stream())
    cfg = B.direct_cfg(streams[0], streams[1], 8, bounce=bounce, bounce_bytes=need, file_slots=2, flush_to=targets,
                       want_file_stats=True)
    try:
        oracle.step(host, ohp, 0, 1.0, 0.0)
        assert B.mlpo_stream_update(table, None, ghp, 1, None, cfg)
        streams[1].synchronize()
        torch.cuda.synchronize()
        assert cfg.stats.bytes_read == 0 and cfg.stats.bytes_written == floats * 4
        homes = [pinned.numpy(), state[1].cpu().numpy(),
                 np.frombuffer(os.pread(fd, floats * 4, 0), dtype=np.float32)]
        for k in range(3):
            p, m, v = unpack_tiled(homes[k], n, T)
            got = {"p": p, "m": m, "v": v, "p16": p16[k].cpu().numpy().view(np.uint16).copy()}
            assert_state_parity(got, host[k], f"n {n} sg {k}")
    finally:
        torch.cuda.synchronize()
        os.close(fd)
