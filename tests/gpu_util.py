"""Helpers for the GPU parity tests: device buffers from numpy subgroups, one GPU step through the C ABI, comparison
with the oracle to the stated bars.  torch is used for device / pinned memory and streams only."""
from __future__ import annotations

import numpy as np
import torch

from paper_2509_02480_amd import binding as B

FLT_MIN = float(np.finfo(np.float32).tiny)


def dev():
    return torch.device("cuda:0")


def to_dev_u16(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(a.view(np.int16)).to(dev())


def from_dev_u16(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint16)


_hip = None


def hip_runtime():
    """The HIP runtime library this process already uses (the one torch loaded), for exact-size pinned allocations:
    torch's own pinned allocator rounds every request up to a power of two, which wastes half of the pinnable host
    memory on multi-gigabyte subgroups."""
    global _hip
    if _hip is None:
        import ctypes as C
        torch.cuda.init()
        path = [ln.split()[-1] for ln in open("/proc/self/maps") if "libamdhip64" in ln][0]
        _hip = C.CDLL(path)
        _hip.hipHostMalloc.argtypes = [C.POINTER(C.c_void_p), C.c_size_t, C.c_uint]
        _hip.hipHostFree.argtypes = [C.c_void_p]
    return _hip


class PinnedF32:
    """n floats of page-locked host memory (hipHostMalloc), seen as a numpy array and as a CPU torch tensor."""

    def __init__(self, n):
        import ctypes as C
        self.ptr = C.c_void_p()
        rc = hip_runtime().hipHostMalloc(C.byref(self.ptr), max(4 * n, 4), 0)
        if rc != 0:
            hip_runtime().hipGetLastError()     # else the next call that checks (torch's) reports the refusal again
            raise MemoryError(f"hipHostMalloc of {4 * n / 1e9:.2f} GB failed (code {rc})")
        self.np = np.ctypeslib.as_array((C.c_float * n).from_address(self.ptr.value))
        self.t = torch.from_numpy(self.np)

    def free(self):
        if self.ptr is not None:
            self.np = self.t = None
            hip_runtime().hipHostFree(self.ptr)
            self.ptr = None


class Scratch:
    """Norm workspace and the 16-byte scalar record, allocated once."""

    def __init__(self):
        self.ws_bytes = B.mlpo_norm_workspace_bytes()
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=dev())
        self.scalars = torch.zeros(4, dtype=torch.float32, device=dev())
        assert self.ws.data_ptr() % 256 == 0 and self.scalars.data_ptr() % 16 == 0

    def read(self):
        h = self.scalars.cpu().numpy()
        return {"norm": np.float32(h[0]), "clip_coef": np.float32(h[1]), "gmul": np.float32(h[2]),
                "found_inf": int(h[3:4].view(np.uint32)[0])}


def pack_tiled(p, m, v, T, lead=0):
    """The tiled state buffer of mlpo.h from three planar arrays (data movement only); ``lead`` slots of padding in
    front."""
    n = p.size + lead
    nt = (n + T - 1) // T
    buf = np.zeros((nt, 3, T), np.float32)
    for j, a in enumerate((p, m, v)):
        pad = np.zeros(nt * T, np.float32)
        pad[lead:n] = a
        buf[:, j, :] = pad.reshape(nt, T)
    return buf.reshape(-1)


def unpack_tiled(buf, n, T, lead=0):
    nt = (n + lead + T - 1) // T
    b = np.asarray(buf).reshape(nt, 3, T)
    return tuple(b[:, j, :].reshape(-1)[lead:lead + n].copy() for j in range(3))


class DeviceSubgroups:
    """Device (and pinned-host) copies of a list of numpy subgroups.

    flat=True lays all subgroups out as consecutive slices of five flat buffers (the way a runtime shards one flat
    partition), so slices inherit whatever alignment their offsets give them; flat=False allocates each separately.
    ``tiers[k] == 1`` puts p, m, v of subgroup k in pinned host memory.  ``tile`` > 0 stores the fp32 state of every
    subgroup in the tiled layout (one buffer per subgroup) instead of three planar arrays."""

    def __init__(self, host_sgs, tiers=None, flat=True, elem_offset=0, tile=0, half=0, lead=False):
        self.half = half            # format of g and p16: B.HALF_BF16 or B.HALF_FP16
        # tiled only: g and p16 are slices of two flat buffers and every subgroup starts `lead` slots into its state
        # buffer, chosen so that the lines of its p16 slice and those of p, m, v begin at the same elements
        self.lead = lead
        self.n_sg = len(host_sgs)
        self.tiers = list(tiers) if tiers is not None else [0] * self.n_sg
        self.sizes = [s["p"].size for s in host_sgs]
        self.t = []
        self.tile = tile
        d = dev()
        if tile:
            self._init_tiled(host_sgs, d)
            return
        if flat:
            tot = sum(self.sizes) + elem_offset
            big = {k: torch.empty(tot, dtype=torch.float32, device=d) for k in ("p", "m", "v")}
            big.update({k: torch.empty(tot, dtype=torch.int16, device=d) for k in ("g", "p16")})
            self._keep = big
        off = elem_offset
        for k, s in enumerate(host_sgs):
            n = self.sizes[k]
            ent = {}
            for key in ("p", "m", "v"):
                src = torch.from_numpy(s[key])
                if self.tiers[k] == 1:
                    ent[key] = torch.empty(n, dtype=torch.float32, pin_memory=True)
                    ent[key].copy_(src)
                elif flat:
                    ent[key] = big[key][off:off + n]
                    ent[key].copy_(src)
                else:
                    ent[key] = src.to(d)
            for key in ("g", "p16"):
                src = torch.from_numpy(s[key].view(np.int16))
                if flat:
                    ent[key] = big[key][off:off + n]
                    ent[key].copy_(src)
                else:
                    ent[key] = src.to(d)
            off += n
            self.t.append(ent)
        torch.cuda.synchronize()
        self.table = B.SubgroupTable(
            B.subgroup(e["p"], e["m"], e["v"], e["g"], e["p16"], n=self.sizes[k], tier=self.tiers[k], half=self.half)
            for k, e in enumerate(self.t))

    def _init_tiled(self, host_sgs, d):
        T = self.tile
        descs = []
        self.leads = []
        if self.lead:
            tot = sum(self.sizes)
            self._keep = {k: torch.empty(tot, dtype=torch.int16, device=d) for k in ("g", "p16")}
        off = 0
        for k, s in enumerate(host_sgs):
            n = self.sizes[k]
            ent = {}
            for key in ("g", "p16"):
                src = torch.from_numpy(s[key].view(np.int16))
                if self.lead:
                    ent[key] = self._keep[key][off:off + n]
                    ent[key].copy_(src)
                else:
                    ent[key] = src.to(d)
            off += n
            lead = B.line_lead(ent["p16"]) if self.lead and n and self.tiers[k] == 0 else 0
            self.leads.append(lead)
            packed = torch.from_numpy(pack_tiled(s["p"], s["m"], s["v"], T, lead))
            assert packed.numel() == B.mlpo_state_floats(n + lead, T)
            if self.tiers[k] == 1:
                state = torch.empty(max(packed.numel(), 1), dtype=torch.float32, pin_memory=True)[:packed.numel()]
                state.copy_(packed)
            else:
                state = packed.to(d) if packed.numel() else torch.empty(0, dtype=torch.float32, device=d)
            ent["state"] = state
            self.t.append(ent)
            descs.append(B.tiled_subgroup(state, ent["g"], ent["p16"], n=n, tier=self.tiers[k], tile_elems=T,
                                          half=self.half, lead=lead)
                         if n else B.subgroup(0, 0, 0, 0, 0, n=0, tier=self.tiers[k], tile_elems=T, half=self.half))
        torch.cuda.synchronize()
        self.table = B.SubgroupTable(descs)

    def set_grads(self, k, g_bits: np.ndarray):
        self.t[k]["g"].copy_(torch.from_numpy(g_bits.view(np.int16)))

    def fetch(self, k):
        torch.cuda.synchronize()
        e = self.t[k]
        if self.tile:
            p, m, v = unpack_tiled(e["state"].cpu().numpy(), self.sizes[k], self.tile, self.leads[k])
            return {"p": p, "m": m, "v": v, "p16": from_dev_u16(e["p16"]).copy()}
        return {"p": e["p"].cpu().numpy().copy(), "m": e["m"].cpu().numpy().copy(), "v": e["v"].cpu().numpy().copy(),
                "p16": from_dev_u16(e["p16"]).copy()}


def gpu_step(ds: DeviceSubgroups, scratch: Scratch, hp: B.HParams, steps_applied: int, inv_scale=1.0, max_norm=0.0,
             stream=None, use_scalars=True):
    """norm pass + resident update through the C ABI; returns (applied, scalars dict)."""
    st = stream if stream is not None else torch.cuda.current_stream()
    B.mlpo_grad_unscale_norm(ds.table, inv_scale, max_norm, scratch.ws, scratch.ws_bytes, scratch.scalars, st)
    B.mlpo_adamw_step(ds.table, hp, steps_applied + 1, scratch.scalars if use_scalars else None, st)
    torch.cuda.synchronize()
    sc = scratch.read()
    return sc["found_inf"] == 0, sc


def max_rel_err(a: np.ndarray, b: np.ndarray) -> float:
    """max |a - b| / max(|b|, FLT_MIN), NaN-safe (a NaN on one side only counts as infinite error)."""
    if a.size == 0:
        return 0.0
    a64, b64 = a.astype(np.float64), b.astype(np.float64)
    both_nan = np.isnan(a64) & np.isnan(b64)
    same_inf = np.isinf(a64) & (a64 == b64)
    with np.errstate(invalid="ignore"):
        err = np.abs(a64 - b64) / np.maximum(np.abs(b64), FLT_MIN)
    err = np.where(both_nan | same_inf, 0.0, err)
    err = np.where(np.isnan(err), np.inf, err)
    return float(err.max())


def assert_state_parity(got: dict, want: dict, label="", tol=1e-6):
    """The parity bars: fp32 state within 1e-6 max relative error, bf16 copy bit-exact.  Because both sides
    round every operation identically the fp32 state is expected to be bit-identical; the count of differing words is
    reported in the failure text."""
    for key in ("p", "m", "v"):
        e = max_rel_err(got[key], want[key])
        ndiff = int((got[key].view(np.uint32) != want[key].view(np.uint32)).sum())
        assert e <= tol, f"{label} {key}: max rel err {e:.3e}, {ndiff} words differ"
    bad = np.nonzero(got["p16"] != want["p16"])[0]
    assert bad.size == 0, f"{label} p16: {bad.size} mismatches, first at {bad[:5]}"


def hp_pair(oracle, **kw):
    """The same hyper-parameters for the oracle and for the library."""
    return oracle.HParams(**kw), B.HParams(**kw)
