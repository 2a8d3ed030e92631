"""Subgroups that start `lead` slots into their tiled state buffer (mlpo_subgroup.lead): the shift that lets the
128-byte lines of g and p16 - slices of flat arrays, cut wherever the subgroup boundaries fall - begin at the same
elements as the lines of p, m, v.  Results must not change (elements are independent, Section 3.2 "Cache-Friendly
Ordering"), the padding must stay untouched, and nothing outside the slices may be read into the result or written."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2509_02480_amd import binding as B  # noqa: E402
from paper_2509_02480_amd import workloads as W  # noqa: E402

from gpu_util import Scratch, assert_state_parity, dev, hp_pair, pack_tiled, unpack_tiled  # noqa: E402

GUARD = 512          # elements of guard pattern around the flat half-precision buffers
GUARD_BITS = 0x7FC1  # a NaN pattern: if it were ever read as a gradient the step would be skipped


class FlatShard:
    """Subgroups as consecutive slices of flat g / p16 buffers that start `offset` elements past an aligned address,
    each with its own tiled state buffer and a lead."""

    def __init__(self, host, T, offset, leads, half=0):
        d = dev()
        self.T, self.sizes, self.half = T, [s["p"].size for s in host], half
        total = sum(self.sizes)
        self.g = torch.full((GUARD + offset + total + GUARD,), GUARD_BITS, dtype=torch.int16, device=d)
        self.p16 = torch.full((GUARD + offset + total + GUARD,), GUARD_BITS, dtype=torch.int16, device=d)
        self.begin = GUARD + offset
        self.state, self.leads, descs = [], [], []
        off = self.begin
        for k, s in enumerate(host):
            n = self.sizes[k]
            gk, hk = self.g[off:off + n], self.p16[off:off + n]
            gk.copy_(torch.from_numpy(s["g"].view(np.int16)))
            hk.copy_(torch.from_numpy(s["p16"].view(np.int16)))
            lead = B.line_lead(hk) if leads == "line" else leads[k % len(leads)]
            if leads == "line":
                assert (hk.data_ptr() - 2 * lead) % 128 == 0
            st = torch.from_numpy(pack_tiled(s["p"], s["m"], s["v"], T, lead)).to(d)
            assert st.numel() == B.mlpo_state_floats(n + lead, T)
            self.state.append(st)
            self.leads.append(lead)
            descs.append(B.tiled_subgroup(st, gk, hk, n=n, tile_elems=T, half=half, lead=lead))
            off += n
        self.table = B.SubgroupTable(descs)
        torch.cuda.synchronize()

    def slice_of(self, buf, k):
        off = self.begin + sum(self.sizes[:k])
        return buf[off:off + self.sizes[k]]

    def set_grads(self, k, bits):
        self.slice_of(self.g, k).copy_(torch.from_numpy(bits.view(np.int16)))

    def fetch(self, k):
        torch.cuda.synchronize()
        n, lead = self.sizes[k], self.leads[k]
        buf = self.state[k].cpu().numpy()
        p, m, v = unpack_tiled(buf, n, self.T, lead)
        # the padding in front and behind the subgroup is never written
        b = buf.reshape(-1, 3, self.T)
        for j in range(3):
            a = b[:, j, :].reshape(-1)
            assert not a[:lead].any() and not a[lead + n:].any(), f"sg {k}: padding of array {j} was written"
        return {"p": p, "m": m, "v": v, "p16": self.slice_of(self.p16, k).cpu().numpy().view(np.uint16).copy()}

    def guards_intact(self):
        for buf in (self.g, self.p16):
            h = buf.cpu().numpy().view(np.uint16)
            end = self.begin + sum(self.sizes)
            if not ((h[:self.begin] == GUARD_BITS).all() and (h[end:] == GUARD_BITS).all()):
                return False
        return True


@pytest.mark.parametrize("T,sizes,offset,leads,half", [
    (8192, [100_004, 65_536, 7_812, 40_000], 20, "line", 0),         # what a caller would do: lines made to coincide
    (1024, [100_004, 65_536, 7_812, 40_000], 44, "line", 1),
    (2048, [4, 8, 12, 1020, 1024, 1028, 2044, 2048, 2052], 8, [0, 4, 60, 1020, 512], 0),   # tiny subgroups, any lead
    (4096, [300_000, 8, 123_456], 0, [1020, 1016, 4], 0),
])
def test_lead_leaves_results_unchanged(oracle, T, sizes, offset, leads, half):
    ohp, ghp = hp_pair(oracle)
    half_name = ["bf16", "fp16"][half]
    wls, host = [], []
    for k, n in enumerate(sizes):
        wl = W.Workload("lead", n_sub=1, sub_elems=n, loss_scale=256.0, seed=17 + k)
        wls.append(wl)
        host.append(W.host_subgroups(wl, warm=True)[0])
    assert not any(n % 4 for n in sizes)     # slices of a flat buffer keep the 8-byte alignment of g and p16
    shard = FlatShard(host, T, offset, leads, half)
    scratch = Scratch()
    st = torch.cuda.Stream()
    inv_scale, max_norm = 1.0 / 256.0, 0.05
    for step in range(3):
        if step:
            for k, s in enumerate(host):
                W.fill_grads(wls[k], 0, step, s["g"])
                shard.set_grads(k, s["g"])
        torch.cuda.synchronize()
        ok_o, norm_o, flag_o, gmul_o = oracle.step(host, ohp, step, inv_scale, max_norm, half=half_name)
        B.mlpo_grad_unscale_norm(shard.table, inv_scale, max_norm, scratch.ws, scratch.ws_bytes, scratch.scalars, st)
        B.mlpo_adamw_step(shard.table, ghp, step + 1, scratch.scalars, st)
        st.synchronize()
        sc = scratch.read()
        assert ok_o and sc["found_inf"] == 0 and sc["gmul"] == gmul_o
        for k in range(len(sizes)):
            assert_state_parity(shard.fetch(k), host[k], f"step {step} sg {k} lead {shard.leads[k]}")
    assert shard.guards_intact()


@pytest.mark.parametrize("n,lead,T", [(50_001, 8, 8192), (77_777, 252, 1024), (3, 1020, 2048), (1, 4, 1024),
                                      (1023, 1020, 1024), (4099, 60, 4096)])
def test_lead_with_separate_buffers(oracle, n, lead, T):
    """Sizes that are no multiple of four (a tail for the element-wise kernel), each array in a buffer of its own."""
    ohp, ghp = hp_pair(oracle, weight_decay=0.0, lr=3e-3)
    wl = W.Workload("lead1", n_sub=1, sub_elems=n, seed=5)
    s = W.host_subgroups(wl, warm=True)[0]
    d = dev()
    g = torch.from_numpy(s["g"].view(np.int16)).to(d)
    p16 = torch.from_numpy(s["p16"].view(np.int16)).to(d)
    state = torch.from_numpy(pack_tiled(s["p"], s["m"], s["v"], T, lead)).to(d)
    table = B.SubgroupTable([B.tiled_subgroup(state, g, p16, n=n, tile_elems=T, lead=lead)])
    st = torch.cuda.Stream()
    for step in range(2):
        oracle.step([s], ohp, step, 1.0, 0.0)
        B.mlpo_adamw_step(table, ghp, step + 1, None, st)
        st.synchronize()
        p, m, v = unpack_tiled(state.cpu().numpy(), n, T, lead)
        got = {"p": p, "m": m, "v": v, "p16": p16.cpu().numpy().view(np.uint16).copy()}
        assert_state_parity(got, s, f"n {n} lead {lead} step {step}")


@pytest.mark.parametrize("n,lead,T", [(10_000, 0, 1024), (10_000, 60, 1024), (8192, 4, 8192), (5, 1020, 2048)])
def test_pack_and_unpack_with_lead(n, lead, T):
    rng = np.random.default_rng(n + lead)
    arrs = [rng.standard_normal(n).astype(np.float32) for _ in range(3)]
    d = dev()
    dv = [torch.from_numpy(a).to(d) for a in arrs]
    floats = B.mlpo_state_floats(n + lead, T)
    state = torch.full((floats,), float("nan"), dtype=torch.float32, device=d)
    st = torch.cuda.current_stream()
    B.mlpo_state_pack(dv[0], dv[1], dv[2], n, T, state, st, lead=lead)
    torch.cuda.synchronize()
    want = pack_tiled(arrs[0], arrs[1], arrs[2], T, lead)
    assert np.array_equal(state.cpu().numpy().view(np.uint32), want.view(np.uint32))
    back = [torch.full((n + 8,), 7.0, dtype=torch.float32, device=d) for _ in range(3)]
    B.mlpo_state_unpack(state, n, T, back[0], back[1], back[2], st, lead=lead)
    torch.cuda.synchronize()
    for a, b in zip(arrs, back):
        h = b.cpu().numpy()
        assert np.array_equal(h[:n], a) and (h[n:] == 7.0).all()


@pytest.mark.parametrize("direct", [False, True])
def test_stream_update_with_lead_on_the_resident_subgroups(oracle, direct):
    ohp, ghp = hp_pair(oracle)
    T, sizes, tiers = 2048, [60_000, 30_004, 45_000, 20_000], [0, 1, 0, 1]
    wls = [W.Workload("leadmix", n_sub=1, sub_elems=n, seed=40 + k) for k, n in enumerate(sizes)]
    host = [W.host_subgroups(w, warm=True)[0] for w in wls]
    d = dev()
    total = sum(sizes)
    g_flat = torch.empty(total + 12, dtype=torch.int16, device=d)[12:]
    p16_flat = torch.zeros(total + 12, dtype=torch.int16, device=d)[12:]
    descs, keep, leads, off = [], [], [], 0
    for k, s in enumerate(host):
        n = sizes[k]
        gk, hk = g_flat[off:off + n], p16_flat[off:off + n]
        gk.copy_(torch.from_numpy(s["g"].view(np.int16)))
        hk.copy_(torch.from_numpy(s["p16"].view(np.int16)))
        lead = B.line_lead(hk) if tiers[k] == 0 else 0
        packed = torch.from_numpy(pack_tiled(s["p"], s["m"], s["v"], T, lead))
        if tiers[k]:
            stt = torch.empty(packed.numel(), dtype=torch.float32, pin_memory=True)
            stt.copy_(packed)
        else:
            stt = packed.to(d)
        keep.append(stt)
        leads.append(lead)
        descs.append(B.tiled_subgroup(stt, gk, hk, n=n, tier=tiers[k], tile_elems=T, lead=lead))
        off += n
    assert any(leads)
    table = B.SubgroupTable(descs)
    scratch = Scratch()
    streams = (torch.cuda.Stream(), torch.cuda.Stream())
    if direct:
        cfg = B.direct_cfg(streams[0], streams[1], 12)
    else:
        need = B.mlpo_stream_staging_bytes(table, 2, 0)
        stg = torch.empty(need, dtype=torch.uint8, device=d)
        cfg = B.stream_cfg(2, stg, need, None, streams[1], None, 0)
    for step in range(2):
        oracle.step(host, ohp, step, 1.0, 0.0)
        B.mlpo_grad_unscale_norm(table, 1.0, 0.0, scratch.ws, scratch.ws_bytes, scratch.scalars, streams[1])
        assert B.mlpo_stream_update(table, None, ghp, step + 1, scratch.scalars, cfg)
        streams[1].synchronize()
        torch.cuda.synchronize()
        off = 0
        for k, s in enumerate(host):
            p, m, v = unpack_tiled(keep[k].cpu().numpy(), sizes[k], T, leads[k])
            got = {"p": p, "m": m, "v": v,
                   "p16": p16_flat[off:off + sizes[k]].cpu().numpy().view(np.uint16).copy()}
            assert_state_parity(got, s, f"step {step} sg {k}")
            off += sizes[k]
