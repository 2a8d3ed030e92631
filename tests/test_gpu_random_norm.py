"""Seeded random scenarios for the gradient pass (non-finite flag, L2 norm of the unscaled gradients, clip factor):
1 to 130 gradient arrays of random lengths (empty ones included) cut from one flat device buffer at random places -
adjacent slices, gaps, every alignment - and now and then from pinned host memory; both half formats; a non-finite or
a huge finite value here and there; through each of the three entry points (with a workspace, with device copies of
what it reads, with the library's static workspace).  Flag and copies must be exact, the norm within the tolerance
that the sums in fp64 allow, and two runs must agree bit for bit (the pass uses no atomics)."""
import os

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2509_02480_amd import binding as B  # noqa: E402
from paper_2509_02480_amd import workloads as W  # noqa: E402

from gpu_util import Scratch, dev  # noqa: E402

SIZES = [0, 1, 2, 7, 8, 9, 63, 64, 65, 127, 1000, 2047, 2048, 2049, 4096, 10_000, 16_385, 70_001, 262_144, 300_007]

# MLPO_RANDOM_SEEDS=a:b runs that range of seeds instead (a wider sweep now and then)
_lo, _, _hi = os.environ.get("MLPO_RANDOM_SEEDS", "0:120").partition(":")


@pytest.mark.parametrize("seed", range(int(_lo), int(_hi)))
def test_random_gradient_pass(oracle, seed):
    rng = np.random.default_rng(50_000 + seed)
    half = int(rng.integers(0, 2))
    half_name = ["bf16", "fp16"][half]
    many = rng.integers(0, 8) == 0                       # more arrays than one launch takes
    n_arr = int(rng.integers(97, 131)) if many else int(rng.integers(1, 12))
    pool = SIZES[:12] if many else SIZES
    sizes = [int(rng.choice(pool)) for _ in range(n_arr)]
    inv_scale = float(rng.choice([1.0, 1 / 1024.0, 1 / 65536.0, 0.37]))
    max_norm = float(rng.choice([0.0, 1.0, 1e-3]))
    entry = str(rng.choice(["plain", "keep", "static"]))
    # where every array starts in the flat buffer: right behind the previous one (the pass then sums them as one
    # array), or after a gap of any length
    starts, at = [], int(rng.integers(0, 70))
    for n in sizes:
        if rng.integers(0, 2):
            at += int(rng.integers(1, 200))
        starts.append(at)
        at += n
    total = at + 8
    bits = np.empty(total, np.uint16)
    wl = W.Workload("rndnorm", n_sub=1, sub_elems=total, loss_scale=1.0 / inv_scale, seed=seed)
    W.fill_grads(wl, 0, 0, bits)                          # finite in either format
    special = int(rng.integers(0, 4))                     # 0, 1: nothing; 2: a non-finite value; 3: huge finite values
    live = [k for k, n in enumerate(sizes) if n > 0]
    if special == 2 and live:
        k = int(rng.choice(live))
        j = int(rng.choice([0, sizes[k] - 1, int(rng.integers(0, sizes[k]))]))
        pats = [0x7C00, 0xFC00, 0x7E01] if half else [0x7F80, 0xFF80, 0x7FC1]
        bits[starts[k] + j] = int(rng.choice(pats))
    elif special == 3 and live:
        for k in live[:3]:
            bits[starts[k] + int(rng.integers(0, sizes[k]))] = 0x7BFF if half else 0x7F7F
    flat = torch.from_numpy(bits.view(np.int16)).to(dev())
    on_host = [bool(rng.integers(0, 6) == 0) and entry != "static" for _ in sizes]
    hosts, g_of = [], []
    for k, n in enumerate(sizes):
        if on_host[k] and n > 0:
            skew = int(rng.integers(0, 9))                # pinned arrays start at any alignment as well
            t = torch.empty(n + skew, dtype=torch.int16, pin_memory=True)
            t[skew:].copy_(torch.from_numpy(bits[starts[k]:starts[k] + n].view(np.int16)))
            hosts.append(t)
            g_of.append(t.data_ptr() + 2 * skew)
        else:
            g_of.append(flat.data_ptr() + 2 * starts[k])
    descs = [B.SubgroupC(None, None, None, g_of[k] if n else None, None, n, B.TIER_HBM, 0, half, 0)
             for k, n in enumerate(sizes)]
    table = B.SubgroupTable(descs)
    # device copies: one flat buffer laid out like the source (adjacent slices stay adjacent, addresses agree modulo
    # 16 bytes with the device source); an array from pinned memory gets a copy of its own at the same phase
    keep, copies = None, []
    if entry == "keep":
        shadow = torch.zeros(total + 8, dtype=torch.int16, device=dev())
        base = shadow.data_ptr() + ((flat.data_ptr() - shadow.data_ptr()) & 15)
        keep = []
        for k, n in enumerate(sizes):
            if n == 0 or rng.integers(0, 4) == 0:
                keep.append(None)
            elif on_host[k]:
                c = torch.zeros(n + 16, dtype=torch.int16, device=dev())
                a = c.data_ptr() + ((g_of[k] - c.data_ptr()) & 15)
                copies.append((k, c, (a - c.data_ptr()) // 2))
                keep.append(a)
            else:
                copies.append((k, shadow, (base - shadow.data_ptr()) // 2 + starts[k]))
                keep.append(base + 2 * starts[k])
    label = (f"seed {seed}: {half_name} {entry} {n_arr} arrays sizes {sizes[:12]}{'...' if n_arr > 12 else ''} "
             f"inv_scale {inv_scale} max_norm {max_norm} special {special} host {sum(on_host)}")
    print(label, flush=True)

    sumsq, flag = 0.0, 0
    for k, n in enumerate(sizes):
        if n == 0:
            continue
        sumsq, flag = oracle.grad_stats(bits[starts[k]:starts[k] + n].copy(), inv_scale, sumsq, flag, half=half_name)
    norm_o, coef_o, gmul_o = oracle.norm_finish(sumsq, inv_scale, max_norm)
    if not np.isfinite(norm_o):
        flag = 1

    scratch = Scratch()
    stream = torch.cuda.Stream()
    runs = []
    for _ in range(2):
        scratch.scalars.fill_(float("nan"))
        torch.cuda.synchronize()
        if entry == "plain":
            B.mlpo_grad_unscale_norm(table, inv_scale, max_norm, scratch.ws, scratch.ws_bytes, scratch.scalars, stream)
        elif entry == "keep":
            B.mlpo_grad_unscale_norm_keep(table, keep, inv_scale, max_norm, scratch.ws, scratch.ws_bytes,
                                          scratch.scalars, stream)
        else:
            B.mlpo_grad_unscale_norm_static(table, inv_scale, max_norm, scratch.scalars, stream)
        stream.synchronize()
        runs.append(scratch.scalars.cpu().numpy().view(np.uint32).copy())
    assert (runs[0] == runs[1]).all(), label
    sc = scratch.read()
    assert sc["found_inf"] == flag, label
    if not flag:
        assert abs(float(sc["norm"]) - float(norm_o)) <= 1e-6 * float(norm_o), (label, sc["norm"], norm_o)
        assert abs(float(sc["clip_coef"]) - float(coef_o)) <= 2e-6 * float(coef_o), (label, sc["clip_coef"], coef_o)
        assert abs(float(sc["gmul"]) - float(gmul_o)) <= 2e-6 * float(gmul_o), (label, sc["gmul"], gmul_o)
    for k, c, off in copies:
        got = c.cpu().numpy().view(np.uint16)[off:off + sizes[k]]
        assert (got == bits[starts[k]:starts[k] + sizes[k]]).all(), f"{label}: copy of array {k}"
    if entry == "keep":                                   # nothing outside the copies was written
        sh = shadow.cpu().numpy().view(np.uint16)
        mask = np.ones(sh.size, bool)
        for k, c, off in copies:
            if c is shadow:
                mask[off:off + sizes[k]] = False
        assert not sh[mask].any(), f"{label}: the pass wrote outside the copies"
