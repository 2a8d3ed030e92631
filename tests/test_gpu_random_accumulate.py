"""Seeded random scenarios for the gradient accumulation (Section 3.2 "Delayed In-place Mixed-Precision Gradient
Conversion": half-precision gradients of the micro-batches are added up in a half-precision buffer that may live in
host memory): 1 to 5 accumulation buffers of random lengths, cut from one flat buffer in device memory or in pinned
host memory at random places, gradients from another flat buffer at places of their own (so that the two agree or
disagree modulo 16 bytes), 1 to 3 micro-batches, any number of persistent workgroups, both half formats, values that
now and then add up to infinity.  The last micro-batch goes through mlpo_grad_accumulate_norm and the step's scalars
come from mlpo_grad_norm_finish.  Every bit of every buffer must equal the oracle's, outside the buffers nothing may
be written, flag exact, norm within the tolerance that sums in fp64 allow."""
import os

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2509_02480_amd import binding as B  # noqa: E402
from paper_2509_02480_amd import workloads as W  # noqa: E402

from gpu_util import Scratch, dev  # noqa: E402

SIZES = [0, 1, 3, 7, 8, 9, 63, 64, 65, 1000, 2047, 2048, 2049, 8191, 8192, 8193, 30_001, 100_003, 262_144]

# MLPO_RANDOM_SEEDS=a:b runs that range of seeds instead (a wider sweep now and then)
_lo, _, _hi = os.environ.get("MLPO_RANDOM_SEEDS", "0:120").partition(":")


@pytest.mark.parametrize("seed", range(int(_lo), int(_hi)))
def test_random_accumulation(oracle, seed):
    rng = np.random.default_rng(90_000 + seed)
    half = int(rng.integers(0, 2))
    half_name = ["bf16", "fp16"][half]
    n_buf = int(rng.integers(1, 6))
    sizes = [int(rng.choice(SIZES)) for _ in range(n_buf)]
    micro = int(rng.integers(1, 4))
    first0 = bool(rng.integers(0, 2))                 # does the first micro-batch start the sum or add to what is there?
    blocks = int(rng.choice([0, 0, 1, 7, 64, 300]))
    on_host = bool(rng.integers(0, 3) == 0)           # the accumulation buffers in pinned host memory
    inv_scale = float(rng.choice([1.0, 1 / 256.0, 1 / 65536.0]))
    max_norm = float(rng.choice([0.0, 1.0, 1e-3]))
    big = rng.integers(0, 5) == 0                     # values near the format's largest: sums overflow to infinity

    def place(lengths):
        """Start of every array in a flat buffer: behind the previous one, or after a gap of any length."""
        starts, at = [], int(rng.integers(0, 40))
        for n in lengths:
            if rng.integers(0, 2):
                at += int(rng.integers(1, 100))
            starts.append(at)
            at += n
        return starts, at + 8

    a_start, a_total = place(sizes)
    g_start, g_total = place(sizes)
    label = (f"seed {seed}: {half_name} sizes {sizes} micro {micro} first {first0} blocks {blocks} "
             f"{'host' if on_host else 'device'} acc inv_scale {inv_scale} max_norm {max_norm} big {big}")
    print(label, flush=True)

    def draw(total, tag):
        bits = np.empty(total, np.uint16)
        wl = W.Workload("rndacc", n_sub=1, sub_elems=total, loss_scale=64.0, seed=seed * 10 + tag)
        W.fill_grads(wl, 0, 0, bits)                  # finite in either format
        if big:
            idx = rng.integers(0, total, size=max(total // 50, 1))
            bits[idx] = (0x7BF0 if half else 0x7F70) | (bits[idx] & 0x8000)
        return bits

    acc_bits = draw(a_total, 0)
    acc_before = acc_bits.copy()
    if on_host:
        acc_flat = torch.empty(a_total, dtype=torch.int16, pin_memory=True)
        acc_flat.copy_(torch.from_numpy(acc_bits.view(np.int16)))
    else:
        acc_flat = torch.from_numpy(acc_bits.view(np.int16)).to(dev())
    scratch = Scratch()
    scratch.ws.fill_(0xFF)                            # whatever an earlier step left there
    stream = torch.cuda.Stream()
    want = [acc_bits[a_start[k]:a_start[k] + n].copy() for k, n in enumerate(sizes)]
    keep = []
    for mb in range(micro):
        g_bits = draw(g_total, 1 + mb)
        g_flat = torch.from_numpy(g_bits.view(np.int16)).to(dev())
        keep.append(g_flat)
        first = first0 and mb == 0
        last = mb == micro - 1
        for k, n in enumerate(sizes):
            a_ptr = acc_flat.data_ptr() + 2 * a_start[k]
            g_ptr = g_flat.data_ptr() + 2 * g_start[k]
            if last:
                B.mlpo_grad_accumulate_norm(a_ptr, g_ptr, n, first, blocks, inv_scale, scratch.ws, scratch.ws_bytes,
                                            begin=(k == 0), stream=stream, half=half)
            elif n:
                B.mlpo_grad_accumulate(a_ptr, g_ptr, n, first, blocks, stream=stream, half=half)
            if n:
                oracle.grad_accumulate(want[k], g_bits[g_start[k]:g_start[k] + n].copy(), first, half=half_name)
    B.mlpo_grad_norm_finish(scratch.ws, scratch.ws_bytes, inv_scale, max_norm, scratch.scalars, stream)
    stream.synchronize()
    torch.cuda.synchronize()

    got = (acc_flat if on_host else acc_flat.cpu()).numpy().view(np.uint16)
    mask = np.ones(a_total, bool)
    for k, n in enumerate(sizes):
        assert np.array_equal(got[a_start[k]:a_start[k] + n], want[k]), f"{label}: buffer {k}"
        mask[a_start[k]:a_start[k] + n] = False
    assert np.array_equal(got[mask], acc_before[mask]), f"{label}: written outside the buffers"

    sumsq, flag = 0.0, 0
    for k, n in enumerate(sizes):
        if n:
            sumsq, flag = oracle.grad_stats(want[k], inv_scale, sumsq, flag, half=half_name)
    norm_o, coef_o, gmul_o = oracle.norm_finish(sumsq, inv_scale, max_norm)
    if not np.isfinite(norm_o):
        flag = 1
    sc = scratch.read()
    assert sc["found_inf"] == flag, label
    if not flag:
        assert abs(float(sc["norm"]) - float(norm_o)) <= 1e-6 * float(norm_o), (label, sc["norm"], norm_o)
        assert abs(float(sc["gmul"]) - float(gmul_o)) <= 2e-6 * float(gmul_o), (label, sc["gmul"], gmul_o)
