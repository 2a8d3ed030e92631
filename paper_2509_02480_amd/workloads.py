"""Seeded synthetic inputs and the workload shapes they come in.

Input generation only: this module holds none of the update's arithmetic and loads no native code, so both the GPU
tests and the CPU checker may draw their inputs from it.  A value depends only on (seed, tensor, step, global element
index): any slice of any tensor can be regenerated on its own, which is what lets the multi-gigabyte workloads be
filled and checked one subgroup at a time.

The shapes follow the update phase the paper measures (Section 4.1 "Runtime Configurations": one flat shard per GPU
cut into equal subgroups, 100 M elements each in the paper's runs; fp32 master parameters, momentum and variance plus
half-precision gradients and a half-precision working copy, Section 2 "Sharded Model and Optimizer States Into
Subgroups").  The paper's gradients come from pre-training runs on a text corpus; the update's cost and its arithmetic
do not depend on the values, so normally distributed stand-ins of a realistic magnitude are used instead.
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field, replace
from typing import List, Optional

import numpy as np

CHUNK = 1 << 20  # generation granule: one Philox stream per (seed, tensor, step, chunk)

T_PARAM, T_MOM, T_VAR, T_GRAD = 0, 1, 2, 3


def _rng(seed: int, tensor: int, step: int, chunk: int) -> np.random.Generator:
    key = [seed & 0xFFFFFFFFFFFFFFFF, ((tensor & 0xFFFF) << 48) | (step & 0xFFFFFFFFFFFF)]
    return np.random.Generator(np.random.Philox(key=key, counter=[0, 0, 0, chunk]))


def _normal_chunk(seed: int, tensor: int, step: int, chunk: int, lo: int, hi: int) -> np.ndarray:
    """Standard normals number lo..hi-1 of one chunk's stream (the stream is always drawn from its start)."""
    x = _rng(seed, tensor, step, chunk).standard_normal(hi, dtype=np.float32)
    return x[lo:hi]


def _for_chunks(start: int, count: int, fn, threads: int) -> None:
    pieces = []
    pos = start
    end = start + count
    while pos < end:
        c = pos // CHUNK
        hi = min(end, (c + 1) * CHUNK)
        pieces.append((c, pos - c * CHUNK, hi - c * CHUNK, pos - start))
        pos = hi
    if threads <= 1 or len(pieces) <= 1:
        for pc in pieces:
            fn(*pc)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(lambda pc: fn(*pc), pieces))


def fill_normal_f32(out: np.ndarray, seed: int, tensor: int, step: int, start: int, std: float,
                    threads: int = 1, square: bool = False) -> None:
    """out[i] = std * z(start + i), z standard normal; with ``square`` the value is squared (a non-negative
    stand-in for a variance estimate)."""
    assert out.dtype == np.float32 and out.ndim == 1
    s = np.float32(std)

    def one(c, lo, hi, off):
        x = _normal_chunk(seed, tensor, step, c, lo, hi) * s
        if square:
            x = x * x
        out[off:off + (hi - lo)] = x

    _for_chunks(start, out.size, one, threads)


def fill_grad_bf16(out: np.ndarray, seed: int, step: int, start: int, std: float, loss_scale: float = 1.0,
                   threads: int = 1) -> None:
    """bf16 bit patterns of gradients ~ N(0, std) multiplied by the loss scale.  The bf16 pattern is the upper half of
    the fp32 draw (a draw in bf16 needs no particular rounding: the lower bits are simply not generated)."""
    assert out.dtype == np.uint16 and out.ndim == 1
    s = np.float32(std * loss_scale)

    def one(c, lo, hi, off):
        x = _normal_chunk(seed, T_GRAD, step, c, lo, hi) * s
        out[off:off + (hi - lo)] = (x.view(np.uint32) >> 16).astype(np.uint16)

    _for_chunks(start, out.size, one, threads)


def splitmix64(x: int) -> int:
    x = (x + 0x9E3779B97F4A7C15) & 0xFFFFFFFFFFFFFFFF
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & 0xFFFFFFFFFFFFFFFF
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & 0xFFFFFFFFFFFFFFFF
    return x ^ (x >> 31)


@dataclass(frozen=True)
class AdamW:
    lr: float = 1e-4
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    weight_decay: float = 0.01
    bias_correction: bool = True
    l2_mode: bool = False


@dataclass(frozen=True)
class Workload:
    """One update-phase workload: ``n_sub`` subgroups of ``sub_elems`` elements, the first ``n_host`` of them kept in
    the pinned-host tier (the low subgroup ids are the ones an ascending pass leaves on the slow tier, Section 3.2
    "Cache-Friendly Ordering"), the rest resident in HBM."""
    name: str
    n_sub: int
    sub_elems: int
    n_host: int = 0
    hp: AdamW = field(default_factory=AdamW)
    loss_scale: float = 1.0
    max_norm: float = 0.0          # <= 0: no clipping
    steps: int = 3
    inject_every: int = 0          # > 0: one +inf gradient on steps s with s % inject_every == inject_phase
    inject_phase: int = 4
    fresh_grads: bool = True       # a new gradient draw each step
    p_std: float = 0.02
    g_std: float = 1e-3
    seed: int = 0
    n_slots: int = 3               # staging slots of the streamed pipeline (in-flight bound)

    @property
    def n_total(self) -> int:
        return self.n_sub * self.sub_elems

    @property
    def inv_scale(self) -> float:
        return float(np.float32(1.0 / self.loss_scale))

    def tier(self, k: int) -> int:
        return 1 if k < self.n_host else 0

    def injects(self, step0: int) -> bool:
        return self.inject_every > 0 and step0 % self.inject_every == self.inject_phase

    def inject_index(self, step0: int) -> int:
        return splitmix64(self.seed * 1000003 + step0) % self.n_total

    def scaled_down(self, factor: int) -> "Workload":
        """The same subgroup size and tier fractions with 1/factor as many subgroups (at least one per tier used)."""
        n_sub = max(1, self.n_sub // factor)
        n_host = 0 if self.n_host == 0 else max(1, math.ceil(n_sub * self.n_host / self.n_sub))
        return replace(self, name=f"{self.name}/{factor}", n_sub=n_sub, n_host=min(n_host, n_sub))


def split_tiers(n_sub: int, frac_host: float) -> int:
    """Subgroups given to the host tier: the slow tier takes the ceiling (Eq. 1 rounds up and then adjusts so the
    counts sum to the total; here the fast tier absorbs the adjustment)."""
    return min(n_sub, math.ceil(frac_host * n_sub - 1e-9))


C1 = Workload("C1-1M-resident", n_sub=1, sub_elems=1_048_576, steps=3)
C2 = Workload("C2-125M-resident-16sg", n_sub=16, sub_elems=7_812_500, loss_scale=1024.0, steps=10, inject_every=50)
C3 = Workload("C3-1.3B-streamed", n_sub=13, sub_elems=100_000_000, n_host=13, steps=5)
C4 = Workload("C4-7B-mixed", n_sub=35, sub_elems=200_000_000, n_host=split_tiers(35, 0.5), steps=5)
C5 = Workload("C5-8.75B-mixed-clip", n_sub=35, sub_elems=250_000_000, n_host=split_tiers(35, 0.7),
              loss_scale=65536.0, max_norm=1.0, steps=5)
CONFIGS = {"C1": C1, "C2": C2, "C3": C3, "C4": C4, "C5": C5}


def fill_state(wl: Workload, k: int, p: np.ndarray, m: Optional[np.ndarray], v: Optional[np.ndarray],
               threads: int = 1, warm: bool = False) -> None:
    """Initial state of subgroup k: p ~ N(0, p_std); m = v = 0, or with ``warm`` a mid-training look
    (m ~ N(0, g_std/3), v = N(0, g_std)^2) so that every term of the update is exercised."""
    start = k * wl.sub_elems
    fill_normal_f32(p, wl.seed, T_PARAM, 0, start, wl.p_std, threads)
    if m is not None:
        if warm:
            fill_normal_f32(m, wl.seed, T_MOM, 0, start, wl.g_std / 3, threads)
        else:
            m[:] = 0
    if v is not None:
        if warm:
            fill_normal_f32(v, wl.seed, T_VAR, 0, start, wl.g_std, threads, square=True)
        else:
            v[:] = 0


def fill_grads(wl: Workload, k: int, step0: int, g: np.ndarray, threads: int = 1) -> None:
    """bf16 gradients of subgroup k for 0-based step ``step0`` (without the injected inf; see ``injects``)."""
    fill_grad_bf16(g, wl.seed, step0 if wl.fresh_grads else 0, k * wl.sub_elems, wl.g_std, wl.loss_scale, threads)


def host_subgroups(wl: Workload, warm: bool = False, step0: int = 0, threads: int = 1) -> List[dict]:
    """All subgroups of a (small) workload as numpy arrays: dicts with p, m, v (fp32), g, p16 (uint16 bf16 bits)."""
    out = []
    for k in range(wl.n_sub):
        n = wl.sub_elems
        s = {"p": np.empty(n, np.float32), "m": np.empty(n, np.float32), "v": np.empty(n, np.float32),
             "g": np.empty(n, np.uint16), "p16": np.zeros(n, np.uint16)}
        fill_state(wl, k, s["p"], s["m"], s["v"], threads, warm)
        fill_grads(wl, k, step0, s["g"], threads)
        out.append(s)
    return out
