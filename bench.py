#!/usr/bin/env python3
"""Benchmark of the update-phase hot path on one MI355X.

A step is one pass of the whole resident hot path over the 125 M-parameter workload (16 subgroups of 7 812 500
elements, loss scale 1024, one +inf gradient every 50th step): the gradient pass (non-finite check + L2 norm + clip
factor) followed by the fused AdamW update of every subgroup, all state resident in HBM before the clock starts.  The
JSON line also carries the roofline of the dominant kernel (measured with events around each of its launches), the
CPU oracle timed on the host cores, and - as additional information - the tiered pipeline on the 1.3 B-parameter
host-tier workload (effective PCIe GB/s per direction).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
PCIE_NOMINAL_GBS = 64.0      # PCIe 5.0 x16 per direction, nominal
BYTES_PER_PARAM_STEP = 28    # read p, m, v (12) + g (2); write p, m, v (12) + bf16 p (2)
BYTES_PER_PARAM_NORM = 2     # read g
WHOLE = (1 << 64) - 1        # chunk_elems: whole subgroups per transfer (0 = the library chooses the piece size)


def recorded_traffic(layout):
    """HBM bytes per launch of the update kernel as counted by the profiler (the "recorded:" lines of
    profiles/adamw_update_C2-125M_hbm_traffic.md), or None if the kernel source has changed since the counters were
    taken."""
    import hashlib
    try:
        rec = {}
        for ln in open(os.path.join(ROOT, "profiles", "adamw_update_C2-125M_hbm_traffic.md")):
            if ln.strip().startswith("recorded:"):
                key, _, val = ln.strip()[len("recorded:"):].rpartition("=")
                rec[key.strip()] = val.strip()
        src = open(os.path.join(ROOT, "paper_2509_02480_amd", "csrc", "adamw.hip"), "rb").read()
        if hashlib.sha256(src).hexdigest() != rec["adamw_hip_sha256"]:
            return None
        return int(rec[layout])
    except (OSError, KeyError, ValueError):
        return None


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def resident_setup(args, torch, B, W, np, wl, tile):
    """Device buffers of the resident workload (seeded synthetic state and gradients) and its subgroup table."""
    d = torch.device("cuda:0")
    N, M = wl.n_total, wl.sub_elems
    g_flat = torch.empty(N, dtype=torch.int16, device=d)
    p16_flat = torch.zeros(N, dtype=torch.int16, device=d)
    if tile:
        # every subgroup starts `lead` slots into its tiled buffer, so that the 128-byte lines of its slices of the
        # flat g / p16 arrays begin at the same elements as the lines of p, m, v
        leads = [B.line_lead(p16_flat[k * M:(k + 1) * M]) if args.lead else 0 for k in range(wl.n_sub)]
        floats = [B.mlpo_state_floats(M + lead, tile) for lead in leads]
        starts = [sum(floats[:k]) for k in range(wl.n_sub)]
        state = torch.zeros(sum(floats), dtype=torch.float32, device=d)
        p_dev = torch.zeros(M, dtype=torch.float32, device=d)
        zeros = torch.zeros(M, dtype=torch.float32, device=d)
    else:
        flat = {k: torch.zeros(N, dtype=torch.float32, device=d) for k in ("p", "m", "v")}
    hp_ = np.empty(M, np.float32)
    hg_ = np.empty(M, np.uint16)
    sgs = []
    for k in range(wl.n_sub):
        W.fill_state(wl, k, hp_, None, None, threads=args.threads)   # m = v = 0
        W.fill_grads(wl, k, 0, hg_, threads=args.threads)
        gk, hk = g_flat[k * M:(k + 1) * M], p16_flat[k * M:(k + 1) * M]
        gk.copy_(torch.from_numpy(hg_.view(np.int16)))
        if tile:
            sk = state[starts[k]:starts[k] + floats[k]]
            p_dev.copy_(torch.from_numpy(hp_))
            B.mlpo_state_pack(p_dev, zeros, zeros, M, tile, sk, lead=leads[k])    # p into its slots, m = v = 0
            sgs.append(B.tiled_subgroup(sk, gk, hk, n=M, tile_elems=tile, half=args.half_format, lead=leads[k]))
        else:
            flat["p"][k * M:(k + 1) * M].copy_(torch.from_numpy(hp_))
            sgs.append(B.subgroup(*(flat[key][k * M:(k + 1) * M] for key in ("p", "m", "v")), gk, hk, n=M,
                                  half=args.half_format))
    return {"table": B.SubgroupTable(sgs), "g_flat": g_flat, "p16_flat": p16_flat,
            "params": state if tile else flat["p"], "keep": (state, p_dev, zeros) if tile else flat,
            "leads": leads if tile else None}


def resident_timed_steps(args, torch, B, wl, buf, scal, ws):
    """args.warmup untimed and args.steps timed whole steps (gradient pass + update) on one stream, with the
    workload's injection schedule - the figure `value` comes from, nothing but the library's launches inside the
    clock - and then the same args.steps steps once more with every launch of the two streaming kernels carrying its
    own begin / end timestamps (HIP events attached to the dispatch on this stream), which is where the per-kernel
    durations of `roofline` come from.  Returns (elapsed ms of the timed steps, applied timed steps)."""
    d = torch.device("cuda:0")
    table, g_flat = buf["table"], buf["g_flat"]
    inf_bits = torch.tensor([0x7F80], dtype=torch.int16, device=d)
    saved = torch.zeros(1, dtype=torch.int16, device=d)
    hp = B.HParams(**wl.hp.__dict__)
    stream = torch.cuda.Stream()
    torch.cuda.synchronize()
    total = args.warmup + args.steps
    t_begin, t_end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    applied = 0
    applied_timed = 0
    with torch.cuda.stream(stream):
        for s in range(total + args.steps):
            timed = args.warmup <= s < total
            if s == args.warmup:
                stream.synchronize()
                torch.cuda.synchronize()
                t_begin.record(stream)
            if s == total:
                t_end.record(stream)
                stream.synchronize()
                torch.cuda.synchronize()
                B.mlpo_kernel_timing(True)
            # the instrumented pass repeats the schedule of the timed one
            inject = wl.injects(s if s < total else s - args.steps)
            if inject:
                idx = wl.inject_index(s)
                saved.copy_(g_flat[idx:idx + 1])
                g_flat[idx:idx + 1].copy_(inf_bits)
            B.mlpo_grad_unscale_norm(table, wl.inv_scale, wl.max_norm, ws, ws.numel(), scal, stream)
            B.mlpo_adamw_step(table, hp, applied + 1, scal, stream)
            if inject:
                g_flat[idx:idx + 1].copy_(saved)
            else:
                applied += 1            # the host mirrors the injection schedule: no read-back of the flag
                applied_timed += int(timed)
    stream.synchronize()
    torch.cuda.synchronize()
    return t_begin.elapsed_time(t_end), applied_timed


def resident_bench(args, torch, B, W, np, tile):
    """Times args.steps whole steps on the resident workload with the fp32 state in the given layout
    (tile = 0: three planar arrays; tile = T: the library's tiled layout)."""
    wl = W.CONFIGS[args.workload]
    assert wl.n_host == 0, "the resident benchmark needs an all-HBM workload"
    d = torch.device("cuda:0")
    N = wl.n_total
    layout = f"tiled T={tile}" if tile else "planar"
    t0 = time.time()
    buf = resident_setup(args, torch, B, W, np, wl, tile)
    ws = torch.empty(B.mlpo_norm_workspace_bytes(), dtype=torch.uint8, device=d)
    scal = torch.zeros(4, dtype=torch.float32, device=d)
    torch.cuda.synchronize()
    log(f"[bench] {wl.name} layout={layout}: {N} params resident, setup {time.time() - t0:.1f}s")
    elapsed_ms, applied_timed = resident_timed_steps(args, torch, B, wl, buf, scal, ws)
    total = args.warmup + args.steps
    flag = int(scal.cpu().numpy()[3:4].view(np.uint32)[0])
    assert flag == (1 if wl.injects(total - 1) else 0)
    assert bool(torch.isfinite(buf["params"]).all().item()), "state went non-finite"

    upd_ms = B.mlpo_kernel_times(0)
    nrm_ms = B.mlpo_kernel_times(1)
    B.mlpo_kernel_timing(False)
    assert len(upd_ms) == args.steps and len(nrm_ms) == args.steps, (len(upd_ms), len(nrm_ms))
    inj_timed = [wl.injects(s) for s in range(args.warmup, total)]
    k_ms = [upd_ms[i] for i in range(args.steps) if not inj_timed[i]]   # a skipped step's launch exits at once
    if not k_ms:        # every timed step was one with an injected inf (a run of very few steps)
        raise SystemExit("bench.py: no timed step applied an update; use more --steps")
    k_avg = sum(k_ms) / len(k_ms)
    n_avg = sum(nrm_ms) / len(nrm_ms)
    achieved = BYTES_PER_PARAM_STEP * N / (k_avg * 1e-3) / 1e9
    out = {
        "layout": layout,
        "lead": buf["leads"],
        "value": round(applied_timed * N / (elapsed_ms * 1e-3) / 1e9, 3),
        "ms_per_step": round(elapsed_ms / args.steps, 5),
        "applied_steps": applied_timed,
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": recorded_traffic(layout) if wl.name == W.C2.name else None,
                     "kernel": "adamw_v4_kernel", "avg_launch_ms": round(k_avg, 5),
                     "min_launch_ms": round(min(k_ms), 5), "launches_timed": len(k_ms),
                     "bytes_per_launch": BYTES_PER_PARAM_STEP * N},
        "norm_pass": {"kernel": "grad_stats_kernel", "avg_launch_ms": round(n_avg, 5),
                      "achieved_GBs": round(BYTES_PER_PARAM_NORM * N / (n_avg * 1e-3) / 1e9, 1)},
        "step_hbm_frac": round((BYTES_PER_PARAM_STEP + BYTES_PER_PARAM_NORM) * N * applied_timed
                               / (elapsed_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
    }
    del buf
    torch.cuda.empty_cache()
    return out


def resident_result(args, wl, primary, others):
    res = {
        "metric": "AdamW update throughput, HBM-resident (Gparams/s)",
        "value": primary["value"],
        "unit": "Gparams/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": primary["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": wl.name, "params": wl.n_total, "subgroups": wl.n_sub, "subgroup_elems": wl.sub_elems,
                   "loss_scale": wl.loss_scale, "inf_every": wl.inject_every,
                   "applied_steps": primary["applied_steps"], "state_layout": primary["layout"],
                   "state_lead_elems": primary["lead"],
                   "state": f"fp32 p/m/v + {args.half} grads + {args.half} params, all in HBM",
                   "timed_region": "warmup + steps with nothing but the library's launches inside the clock (value, "
                                   "ms_per_step); the same steps are then run once more with an event pair on every "
                                   "launch of the two streaming kernels (roofline, norm_pass)"},
        "roofline": primary["roofline"],
        "norm_pass": primary["norm_pass"],
        "step_hbm_frac": primary["step_hbm_frac"],
    }
    if others:
        res["other_layouts"] = others
    return res


_ys = None


def ys_lib():
    """The benchmark's own yardstick kernels (bench_yardsticks.hip -> libbench_yardsticks.so, built by
    __graft_entry__.build()); not part of the update library."""
    global _ys
    if _ys is None:
        import ctypes as C
        path = os.path.join(ROOT, "libbench_yardsticks.so")
        if not os.path.exists(path):
            raise RuntimeError(f"{path} is missing: run __graft_entry__.build() first")
        L = C.CDLL(path)
        L.ys_last_error.restype = C.c_char_p
        L.ys_sweep.argtypes = [C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p]
        L.ys_sweep_timed.argtypes = [C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p, C.POINTER(C.c_float)]
        L.ys_update_pattern.argtypes = [C.c_void_p] * 5 + [C.c_uint64, C.c_int32, C.c_void_p]
        L.ys_link.argtypes = [C.c_void_p] * 4 + [C.c_size_t, C.c_int32, C.POINTER(C.c_double)]
        _ys = L
    return _ys


def ys_check(rc):
    if rc != 0:
        raise RuntimeError("yardstick: " + ys_lib().ys_last_error().decode())


def timed_launches(torch, st, launch, reps=30, warm=3):
    """Average duration in seconds of `reps` back-to-back launches on stream st (events around the whole run)."""
    with torch.cuda.stream(st):
        for _ in range(warm):
            launch()
        t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0.record(st)
        for _ in range(reps):
            launch()
        t1.record(st)
    st.synchronize()
    return t0.elapsed_time(t1) * 1e-3 / reps


def yardsticks(torch, wl, tile, update_GBs, planar_GBs, norm_GBs):
    """What the memory system delivers for the update's access patterns without its arithmetic: read-only, write-only
    and in-place sweeps over a buffer of the size of the workload's fp32 state; a read-only sweep of the size of its
    gradients (what bounds the gradient pass: a 36 us kernel pays for its ramp and tail); and the update's own address
    streams (three 16-byte loads and stores plus the two 8-byte streams per four elements) in both state layouts."""
    L = ys_lib()
    d = torch.device("cuda:0")
    st = torch.cuda.Stream()
    sp = st.cuda_stream
    N = wl.n_total
    nbytes = 12 * N // 16 * 16
    buf = torch.ones(nbytes // 4, dtype=torch.float32, device=d)
    out = {"buffer_bytes": nbytes, "launches": 30}
    rates = {}
    for name, kind, factor in (("read", 0, 1), ("write", 1, 1), ("update_in_place", 2, 2)):
        dt = timed_launches(torch, st, lambda: ys_check(L.ys_sweep(kind, buf.data_ptr(), nbytes, sp)))
        rates[name] = factor * nbytes / dt / 1e9
        out[name + "_GBs"] = round(rates[name], 1)
    # The gradient pass is one short kernel (tens of microseconds), timed by its own begin and end: its yardstick is
    # one read sweep of the same size timed the same way, with other work between the launches as in the step.
    # Back-to-back launches of the sweep overlap each other's ramp and tail and look faster than any single one is.
    import ctypes as C
    gbytes = 2 * N // 16 * 16
    dt = timed_launches(torch, st, lambda: ys_check(L.ys_sweep(0, buf.data_ptr(), gbytes, sp)), reps=100)
    out["read_gradient_sized_back_to_back_GBs"] = round(gbytes / dt / 1e9, 1)
    one, ms = [], C.c_float(0.0)
    for i in range(40):
        ys_check(L.ys_sweep(2, buf.data_ptr() + (400 << 20), 400 << 20, sp))     # other traffic in between
        ys_check(L.ys_sweep_timed(0, buf.data_ptr(), gbytes, sp, C.byref(ms)))
        if i >= 5:
            one.append(ms.value * 1e-3)
    dt1 = sum(one) / len(one)
    out["read_gradient_sized_GBs"] = round(gbytes / dt1 / 1e9, 1)
    out["read_gradient_sized_us"] = round(dt1 * 1e6, 2)
    out["read_gradient_sized_bytes"] = gbytes
    out["norm_pass_GBs"] = norm_GBs
    out["norm_pass_vs_read_yardstick"] = round(norm_GBs / (gbytes / dt1 / 1e9), 4)
    # the update's address streams, nothing else: planar (three arrays N floats apart) and tiled
    n4 = N // 4 * 4
    g16 = torch.zeros(n4, dtype=torch.int16, device=d)
    h16 = torch.zeros(n4, dtype=torch.int16, device=d)
    p_, m_, v_ = (buf[i * N:(i + 1) * N] for i in range(3))
    dt = timed_launches(torch, st, lambda: ys_check(L.ys_update_pattern(p_.data_ptr(), m_.data_ptr(), v_.data_ptr(),
                                                                         g16.data_ptr(), h16.data_ptr(), n4, 0, sp)))
    out["update_pattern_planar_GBs"] = round(28 * n4 / dt / 1e9, 1)
    nt = n4 // tile * tile          # whole layout tiles of the same buffer
    dt = timed_launches(torch, st, lambda: ys_check(L.ys_update_pattern(buf.data_ptr(), None, None, g16.data_ptr(),
                                                                         h16.data_ptr(), nt, tile, sp)))
    out["update_pattern_tiled_GBs"] = round(28 * nt / dt / 1e9, 1)
    # the update moves 14 bytes in and 14 out per parameter: its time at the two one-way rates
    mix = 28.0 / (14.0 / rates["read"] + 14.0 / rates["write"])
    out["half_read_half_write_at_these_rates_GBs"] = round(mix, 1)
    out["update_kernel_GBs"] = update_GBs
    out["update_kernel_vs_in_place_yardstick"] = round(update_GBs / rates["update_in_place"], 4)
    out["update_kernel_vs_its_pattern_tiled"] = round(update_GBs / out["update_pattern_tiled_GBs"], 4)
    if planar_GBs:
        out["update_kernel_planar_GBs"] = planar_GBs
        out["update_kernel_vs_its_pattern_planar"] = round(planar_GBs / out["update_pattern_planar_GBs"], 4)
    del buf, g16, h16
    torch.cuda.empty_cache()
    log(f"[bench] yardsticks {out}")
    return out


def calibration_copies(torch):
    """Plain kernels of known traffic, run only so that a counter-collecting profiler run of this script has a
    reference to scale its HBM byte counters with: a 1 GiB device-to-device copy (reads 1 GiB, writes 1 GiB) and a
    1 GiB in-place scale (same)."""
    d = torch.device("cuda:0")
    n = (1 << 30) // 4
    x = torch.ones(n, dtype=torch.float32, device=d)
    y = torch.empty_like(x)
    for _ in range(3):
        y.copy_(x)
        x.mul_(1.0)
    torch.cuda.synchronize()
    del x, y
    torch.cuda.empty_cache()


def cpu_baseline(args, W, np):
    """The oracle as it stands, all host threads, on the first subgroups of the same workload."""
    import oracle
    wl = W.CONFIGS[args.workload]
    n_sg = min(wl.n_sub, args.cpu_subgroups)
    M = wl.sub_elems
    host = []
    for k in range(n_sg):
        s = {"p": np.empty(M, np.float32), "m": np.zeros(M, np.float32), "v": np.zeros(M, np.float32),
             "g": np.empty(M, np.uint16), "p16": np.zeros(M, np.uint16)}
        W.fill_state(wl, k, s["p"], None, None, threads=args.threads)
        W.fill_grads(wl, k, 0, s["g"], threads=args.threads)
        host.append(s)
    ohp = oracle.HParams(**wl.hp.__dict__)

    def one_step(t):
        sumsq, flag = 0.0, 0
        for s in host:
            a, b = oracle.grad_stats_chunked(s["g"], wl.inv_scale)
            sumsq += a
            flag |= b
        _, _, gmul = oracle.norm_finish(sumsq, wl.inv_scale, wl.max_norm)
        for s in host:
            oracle.adamw_f32(s["p"], s["m"], s["v"], s["g"], s["p16"], ohp, t, gmul, chunked=True)

    one_step(1)  # page in
    t0 = time.perf_counter()
    one_step(2)
    dt1 = time.perf_counter() - t0
    reps = max(2, min(200, int(args.cpu_seconds / max(dt1, 1e-3))))
    t0 = time.perf_counter()
    for r in range(reps):
        one_step(3 + r)
    dt = time.perf_counter() - t0
    n = n_sg * M
    # the same oracle routines on one thread (plain, unchunked calls) over the same sample, one step
    t0 = time.perf_counter()
    sumsq, flag = 0.0, 0
    for s in host:
        sumsq, flag = oracle.grad_stats(s["g"], wl.inv_scale, sumsq, flag)
    _, _, gmul = oracle.norm_finish(sumsq, wl.inv_scale, wl.max_norm)
    for s in host:
        oracle.adamw_f32(s["p"], s["m"], s["v"], s["g"], s["p16"], ohp, 3 + reps, gmul)
    dt_single = time.perf_counter() - t0
    # the oracle's parallel driver runs one thread per core the process may use (its OpenMP default)
    cores = min(oracle.threads(), len(os.sched_getaffinity(0)))
    return {"value": round(reps * n / dt / 1e9, 4), "unit": "Gparams/s", "cores": cores, "kind": "oracle",
            "omp_max_threads": oracle.threads(), "sched_getaffinity": len(os.sched_getaffinity(0)),
            "sample": f"first {n_sg} of {wl.n_sub} subgroups ({n} params) x {reps} steps (norm pass + update), "
                      f"{dt:.1f} s wall",
            "single_thread": {"value": round(n / dt_single / 1e9, 4), "unit": "Gparams/s", "cores": 1,
                              "sample": f"the same {n} params x 1 step, {dt_single:.1f} s wall"}}


class StreamedBench:
    """The host-tier workload: state of the host-tier subgroups in pinned memory (tiled layout), gradients and bf16
    parameters on the device; one timed run per variant of ``--stream-variants``."""

    def __init__(self, args, torch, B, W, np):
        self.args, self.torch, self.B, self.np = args, torch, B, np
        self.wl = wl = W.CONFIGS[args.streamed]
        self.d = d = torch.device("cuda:0")
        self.M = M = wl.sub_elems
        self.T = T = args.tile
        t0 = time.time()
        per = B.mlpo_state_floats(M, T)
        self.g_flat = torch.empty(wl.n_total, dtype=torch.int16, device=d)
        self.p16_flat = torch.zeros(wl.n_total, dtype=torch.int16, device=d)
        self.keep, sgs, self.pinned = [], [], []
        tmp = np.zeros(per // 3, np.float32)
        hg = np.empty(M, np.uint16)
        for k in range(wl.n_sub):
            # fp32 state in the tiled layout: one buffer per subgroup, pinned host memory or HBM by tier; m = v = 0
            W.fill_state(wl, k, tmp[:M], None, None, threads=args.threads)
            if wl.tier(k) == 1:
                buf = PinnedF32(torch, np, per)         # exact size: torch's pinned allocator rounds up to 2^k
                self.pinned.append(buf)
                buf.np[:] = 0
                st = torch.from_numpy(buf.np)
                st.numpy().reshape(-1, 3, T)[:, 0, :] = tmp.reshape(-1, T)
            else:
                st = torch.zeros(per, dtype=torch.float32, device=d)
                st.view(-1, 3, T)[:, 0, :].copy_(torch.from_numpy(tmp).view(-1, T))
            W.fill_grads(wl, k, 0, hg, threads=args.threads)
            self.grads(k).copy_(torch.from_numpy(hg.view(np.int16)))
            self.keep.append(st)
            sgs.append(B.tiled_subgroup(st, self.grads(k), self.p16(k), n=M, tier=wl.tier(k), tile_elems=T))
        self.table = B.SubgroupTable(sgs)
        self.ws_bytes = B.mlpo_norm_workspace_bytes()
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=d)
        self.scal = torch.zeros(4, dtype=torch.float32, device=d)
        self.hp = B.HParams(**wl.hp.__dict__)
        self.h2d, self.cmp, self.d2h = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
        self.applied = 0
        self.host_g_table = self.host_g_all = self.micro = None
        self.n_host_params = wl.n_host * M
        torch.cuda.synchronize()
        log(f"[bench] {wl.name}: {wl.n_host} host-tier + {wl.n_sub - wl.n_host} HBM subgroups of {M}, "
            f"setup {time.time() - t0:.1f}s")

    def release(self):
        """Gives the pinned memory back (the large workloads need all the machine will pin)."""
        self.torch.cuda.synchronize()
        self.table = self.host_g_table = self.host_g_all = None
        self.keep = []
        for b in self.pinned:
            b.free()
        self.pinned = []

    def grads(self, k):
        return self.g_flat[k * self.M:(k + 1) * self.M]

    def p16(self, k):
        return self.p16_flat[k * self.M:(k + 1) * self.M]

    def memcpy_reference(self):
        """Plain pinned copies (hipMemcpyAsync) of one 400 MB subgroup array: each direction alone, then both
        directions at once on two streams - the rate the link gives a pipeline that fetches and flushes at the same
        time, which is what the update phase does.  GB/s per direction: (h2d alone, d2h alone, both at once)."""
        import ctypes as C
        torch, M, wl = self.torch, self.M, self.wl
        dst_dev = torch.empty(M, dtype=torch.float32, device=self.d)
        src_dev = torch.zeros(M, dtype=torch.float32, device=self.d)
        host_k = [k for k in range(wl.n_sub) if wl.tier(k) == 1]
        hsrc = self.keep[host_k[0]][:M]
        hdst = torch.empty(M, dtype=torch.float32, pin_memory=True)
        sec = (C.c_double * 3)()
        torch.cuda.synchronize()
        ys_check(ys_lib().ys_link(hsrc.data_ptr(), dst_dev.data_ptr(), src_dev.data_ptr(), hdst.data_ptr(), 4 * M, 4,
                                  sec))
        return tuple(round(4 * M / t / 1e9, 2) for t in sec)

    def table_with_host_gradients(self):
        """The same subgroups with the gradients of the host-tier ones in pinned host memory too."""
        if self.host_g_table is None:
            torch, B, wl = self.torch, self.B, self.wl
            self.host_g_all, sgs = [], []
            for k in range(wl.n_sub):
                gk = self.grads(k)
                if wl.tier(k) == 1:
                    gk = torch.empty(self.M, dtype=torch.int16, pin_memory=True)
                    gk.copy_(self.grads(k))
                self.host_g_all.append(gk)
                sgs.append(B.tiled_subgroup(self.keep[k], gk, self.p16(k), n=self.M,
                                            tier=B.TIER_HOST_GRADS if wl.tier(k) else B.TIER_HBM, tile_elems=self.T))
            self.host_g_table = B.SubgroupTable(sgs)
            torch.cuda.synchronize()
        return self.host_g_table

    def configure(self, kind, arg):
        """(subgroup table, stream configuration, staging buffer, slot cache) of one variant.  kind is a number of
        staging slots (staged mode, arg = chunk_elems), "d" / "dg" / "dga" (direct mode, arg = workgroups, with the
        gradients on the device / on the host / on the host with the statistics left by the last accumulation), "sg"
        (staged mode with 3 slots and the gradients on the host, arg = chunk_elems) or "c" (staged mode with slots
        that keep their subgroups, arg = slots)."""
        torch, B = self.torch, self.B
        table = self.table_with_host_gradients() if kind in ("dg", "dga", "sg") else self.table
        if kind in ("dgk", "sgk"):
            self.table_with_host_gradients()        # the pass reads these; the update reads their device copies
        if kind in ("d", "dg", "dga", "dgk"):
            return table, B.direct_cfg(self.h2d, self.cmp, arg), None, None
        n_slots, chunk = {"sg": (3, arg), "sgk": (3, arg), "c": (arg, 0)}.get(kind, (kind, arg))
        cache = B.SlotCacheC() if kind == "c" else None
        # with a slot cache the slots hold whole subgroups; chunk_elems then only sizes the pieces of a miss
        need = B.mlpo_stream_staging_bytes(table, n_slots, WHOLE if cache is not None else chunk)
        stg = torch.empty(need, dtype=torch.uint8, device=self.d)
        # no copy streams given: the library's own
        return table, B.stream_cfg(n_slots, stg, need, None, self.cmp, None, chunk, cache=cache,
                                   direct_blocks=self.args.cache_blocks if cache is not None else 0), stg, cache

    def last_micro_batch(self):
        """The last micro-batch of the backward pass (outside the update phase, untimed) accumulates into the host
        buffers and leaves the gradient statistics behind; zeros keep the gradients as they are."""
        torch, B, wl = self.torch, self.B, self.wl
        if self.micro is None:
            self.micro = torch.zeros(self.M, dtype=torch.int16, device=self.d)
        for k in range(wl.n_sub):
            B.mlpo_grad_accumulate_norm(self.host_g_all[k], self.micro, self.M, False, 64 if wl.tier(k) else 0,
                                        wl.inv_scale, self.ws, self.ws_bytes, begin=(k == 0), stream=self.cmp)
        torch.cuda.synchronize()

    def step(self, kind, table, cfg, order):
        """One update phase: gradient statistics, then the pipeline; returns the wall time."""
        torch, B, wl = self.torch, self.B, self.wl
        torch.cuda.synchronize()
        if kind == "dga":
            self.last_micro_batch()
        t = time.perf_counter()
        if kind == "dga":
            B.mlpo_grad_norm_finish(self.ws, self.ws_bytes, wl.inv_scale, wl.max_norm, self.scal, self.cmp)
        elif kind in ("dgk", "sgk"):
            # gradients in pinned host memory: the pass reads them over the link and leaves copies at their device
            # homes, which is where `table` (host-tier state, device gradients) has the update read them
            keep = [self.grads(k) if wl.tier(k) else None for k in range(wl.n_sub)]
            B.mlpo_grad_unscale_norm_keep(self.host_g_table, keep, wl.inv_scale, wl.max_norm, self.ws, self.ws_bytes,
                                          self.scal, self.cmp)
        else:
            B.mlpo_grad_unscale_norm(table, wl.inv_scale, wl.max_norm, self.ws, self.ws_bytes, self.scal, self.cmp)
        ok = B.mlpo_stream_update(table, order, self.hp, self.applied + 1, self.scal, cfg)
        self.cmp.synchronize()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t
        assert ok
        self.applied += 1
        return dt

    def effective_io(self, kind, arg, n_steps, fetch_ms, flush_ms, kern_ms):
        """The paper's effective I/O throughput (Section 4.3): bytes read + written over read time + write time,
        averaged over the transfer units; in direct mode reading and writing both last as long as the kernel that
        does them."""
        M, wl = self.M, self.wl
        if kind in ("d", "dg", "dga", "dgk"):
            eff = [2 * 12 * self.n_host_params / (2 * k * 1e-3) / 1e9 for k in kern_ms if k > 1.0]
        elif kind == "c":
            eff = []                # transfers are not paired one to one when flushes are lazy
        else:
            c = M if arg == WHOLE else (arg or (M if M <= (1 << 25) else 1 << 24))
            both = 26 if kind == "sg" else 24     # bytes per element fetched + flushed
            units = [both * min(c, M - o) for _ in range(wl.n_host * n_steps) for o in range(0, M, c)]
            assert len(units) == len(fetch_ms) == len(flush_ms), (len(units), len(fetch_ms), len(flush_ms))
            eff = [u / ((a + b) * 1e-3) / 1e9 for u, a, b in zip(units, fetch_ms, flush_ms)]
        return round(sum(eff) / len(eff), 2) if eff else None

    def describe(self, kind, arg):
        return {
            "d": {"mode": "direct", "direct_blocks": arg},
            "dg": {"mode": "direct, gradients on the host too (16 B/param in, 12 out)", "direct_blocks": arg},
            "dga": {"mode": "direct, gradients on the host too, statistics from the last accumulation "
                            "(14 B/param in, 12 out)", "direct_blocks": arg},
            "sg": {"mode": "staged, gradients on the host too (16 B/param in, 12 out)", "n_slots": 3,
                   "chunk_elems": arg},
            "dgk": {"mode": "direct, gradients on the host too, the gradient pass keeps a device copy for the update "
                            "(14 B/param in, 12 out)", "direct_blocks": arg},
            "sgk": {"mode": "staged, gradients on the host too, the gradient pass keeps a device copy for the update "
                            "(14 B/param in, 12 out)", "n_slots": 3, "chunk_elems": arg},
            "c": {"mode": "staged+slot-cache, alternating order, a miss = one kernel that exchanges the slot's occupants "
                          "over the link", "n_slots": arg, "exchange_workgroups": self.args.cache_blocks or 80},
        }.get(kind, {"mode": "staged", "n_slots": kind,
                     "chunk_elems": "whole subgroups" if arg == WHOLE else (arg or "library's choice (2^24)")})

    def run_variant(self, kind, arg, memcpy_peak):
        B, wl, args = self.B, self.wl, self.args
        table, cfg, stg, cache = self.configure(kind, arg)
        times, fetches_before = [], 0
        for s in range(args.stream_warmup + wl.steps):
            if s == args.stream_warmup:
                self.torch.cuda.synchronize()
                B.mlpo_kernel_timing(True)
                fetches_before = cache.fetches if cache is not None else 0
            # with a slot cache the processing order alternates (Section 3.2 "Cache-Friendly Ordering")
            order = list(range(wl.n_sub))[::-1] if (cache is not None and s % 2 == 1) else None
            dt = self.step(kind, table, cfg, order)
            if s >= args.stream_warmup:
                times.append(dt)
        fetch_ms, flush_ms, kern_ms = B.mlpo_kernel_times(2), B.mlpo_kernel_times(3), B.mlpo_kernel_times(0)
        B.mlpo_kernel_times(1)
        B.mlpo_kernel_times(4)
        B.mlpo_kernel_timing(False)
        mean = sum(times) / len(times)
        gbs = 12 * self.n_host_params / mean / 1e9
        rec = {**self.describe(kind, arg), "steps": len(times), "ms_per_step": round(mean * 1e3, 2),
               "min_ms": round(min(times) * 1e3, 2), "Gparams_s": round(wl.n_total / mean / 1e9, 3)}
        if cache is not None:
            B.mlpo_stream_flush(self.table, cfg)
            self.cmp.synchronize()
            # fewer subgroups cross the link: the useful figure is the step time; the link rate is what was moved
            moved = (cache.fetches - fetches_before) / wl.steps
            rec.update({"subgroup_transfers_per_step_per_dir": round(moved, 2), "of": wl.n_host,
                        "link_GBs_per_dir": round(gbs * moved / wl.n_host, 2),
                        "traffic_vs_uncached": round(moved / wl.n_host, 3)})
        else:
            rec.update({"pcie_GBs_per_dir": round(gbs, 2), "frac_nominal": round(gbs / PCIE_NOMINAL_GBS, 4),
                        "frac_of_one_way_memcpy": round(gbs / memcpy_peak, 4),
                        "frac_of_bidir_memcpy": round(gbs / self.memcpy_bidir, 4),
                        "effective_io_GBs_paper_formula": self.effective_io(kind, arg, len(times), fetch_ms, flush_ms,
                                                                            kern_ms)})
            # host-side gradients cross the link with the state, and once more for a gradient pass
            inbound = {"dg": 16, "sg": 16, "dga": 14, "dgk": 14, "sgk": 14}.get(kind)
            if inbound:
                rec.update({"pcie_in_GBs": round(inbound * self.n_host_params / mean / 1e9, 2),
                            "pcie_out_GBs": round(12 * self.n_host_params / mean / 1e9, 2)})
        log(f"[bench] streamed {rec}")
        return rec


def promote_bench(sb, host_GBs):
    """Re-balancing between HBM and the offloaded tier (Eq. 1 with capacities, Section 3.3; Algorithm 1 assigns the
    path anew at every flush): HBM has room for ``--hbm-capacity`` more subgroups, one ordinary update step stores
    their new state there instead of sending it back over the link, the following steps run with the new split, and
    a last step sends them back to pinned memory."""
    torch, B, wl, args = sb.torch, sb.B, sb.wl, sb.args
    host_ids = [k for k in range(wl.n_sub) if wl.tier(k) == 1]
    state_bytes = B.mlpo_state_floats(sb.M, sb.T) * 4
    # Eq. 1 in subgroups per second: the HBM "path" at the resident kernel's rate, the link at the measured one
    bw = [HBM_PEAK_GBS * 0.78 * 1e9 / (28 * sb.M), host_GBs * 1e9 / state_bytes]
    counts, _ = B.mlpo_assign_tiers(len(host_ids), bw, [min(args.hbm_capacity, len(host_ids)), len(host_ids)])
    movers = host_ids[:counts[0]]
    res = {"eq1_bandwidth_subgroups_per_s": [round(x, 1) for x in bw], "hbm_capacity": args.hbm_capacity,
           "eq1_split_hbm_pinned": list(counts)}
    if not movers:
        return res
    homes = {k: torch.empty(state_bytes // 4, dtype=torch.float32, device=sb.d) for k in movers}

    def cfg_for(targets):
        return B.direct_cfg(sb.h2d, sb.cmp, 64, chunk_elems=args.multipath_chunk,
                            flush_to=[targets.get(k) for k in range(wl.n_sub)] if targets else None)

    res["promote_step_ms"] = round(sb.step("d", sb.table, cfg_for(homes), None) * 1e3, 2)
    sgs = [B.tiled_subgroup(homes[k] if k in homes else sb.keep[k], sb.grads(k), sb.p16(k), n=sb.M,
                            tier=B.TIER_HBM if k in homes else wl.tier(k), tile_elems=sb.T) for k in range(wl.n_sub)]
    table = B.SubgroupTable(sgs)
    cfg = cfg_for(None)
    times = [sb.step("d", table, cfg, None) for _ in range(args.stream_warmup + wl.steps)][args.stream_warmup:]
    mean = sum(times) / len(times)
    n_left = len(host_ids) - len(movers)
    res.update({"steps": len(times), "ms_per_step_after": round(mean * 1e3, 2), "min_ms": round(min(times) * 1e3, 2),
                "Gparams_s": round(wl.n_total / mean / 1e9, 3),
                "pcie_GBs_per_dir": round(n_left * state_bytes / mean / 1e9, 2)})
    back = {k: sb.keep[k] for k in movers}
    res["demote_step_ms"] = round(sb.step("d", table, cfg_for(back), None) * 1e3, 2)
    log(f"[bench] promote {res}")
    return res


def streamed_bench(args, torch, B, W, np, link_fresh=None):
    sb = StreamedBench(args, torch, B, W, np)
    wl = sb.wl
    out = {"workload": wl.name, "state_layout": f"tiled T={sb.T}", "host_tier_params": sb.n_host_params,
           "bytes_per_direction_per_step": 12 * sb.n_host_params, "pcie_nominal_GBs": PCIE_NOMINAL_GBS, "runs": []}
    out["memcpy_h2d_GBs"], out["memcpy_d2h_GBs"], out["memcpy_bidir_GBs_per_dir"] = sb.memcpy_reference()
    memcpy_peak = min(out["memcpy_h2d_GBs"], out["memcpy_d2h_GBs"])
    # the both-ways yardstick the runs are compared with: the better of this process's and the fresh process's
    sb.memcpy_bidir = max(out["memcpy_bidir_GBs_per_dir"], (link_fresh or {}).get("bidir_GBs_per_dir", 0.0))
    for kind, arg in args.stream_variants:
        out["runs"].append(sb.run_variant(kind, arg, memcpy_peak))
    # the cached runs move less data, so their "GB/s" is not a link rate: the best link rate is among the others
    best = max((r for r in out["runs"] if "pcie_GBs_per_dir" in r), key=lambda r: r["pcie_GBs_per_dir"])
    out["best"] = best
    if args.hbm_capacity > 0:
        out["hbm_rebalance"] = promote_bench(sb, best["pcie_GBs_per_dir"])
    if args.multipath != "none":
        ctx = dict(wl=wl, keep=sb.keep, g_flat=sb.g_flat, p16_flat=sb.p16_flat, T=sb.T, M=sb.M, ws=sb.ws,
                   ws_bytes=sb.ws_bytes, scal=sb.scal, hp=sb.hp, streams=(sb.h2d, sb.cmp), applied=sb.applied,
                   host_GBs=best["pcie_GBs_per_dir"])
        out["multipath"] = []
        for kind in args.multipath.split(","):
            try:
                out["multipath"].append(multipath_bench(args, torch, B, np, ctx, kind))
            except (OSError, MemoryError, RuntimeError) as e:   # no room for the file, no /dev/shm, an I/O error
                out["multipath"].append({"kind": kind, "error": f"{type(e).__name__}: {e}"})
                log(f"[bench] multipath {kind} failed: {e}")
        if args.three_paths:
            two = {r["kind"]: r.get("file_path_GBs_per_dir") for r in out["multipath"] if "kind" in r}
            try:
                out["three_paths"] = three_path_bench(args, torch, B, np, ctx, two)
            except (OSError, MemoryError, RuntimeError, AssertionError) as e:
                out["three_paths"] = {"error": f"{type(e).__name__}: {e}"}
                log(f"[bench] three paths failed: {e}")
    g_flat, p16_flat = sb.g_flat, sb.p16_flat
    sb.release()
    out["grad_accumulate"] = accumulate_bench(torch, B, g_flat, p16_flat, wl)
    del sb, g_flat, p16_flat
    torch.cuda.empty_cache()
    if hasattr(torch._C, "_host_emptyCache"):
        torch._C._host_emptyCache()         # pinned blocks torch still caches would count against the large workloads
    return out


def multipath_bench(args, torch, B, np, ctx, kind):
    """Two paths behind the offloaded tier (Section 3.2 "Unified Multi-level, Multi-path Asynchronous Offloading using
    Virtual Tiers"): pinned host memory, limited to ``--pinned-capacity`` subgroups as if no more could be pinned, and
    a file for the rest - on the machine's disk (kind "disk", O_DIRECT) or in tmpfs (kind "shm": pageable host
    memory moved by CPU threads).  Eq. 1 (Section 3.3) splits the subgroups, the observed bandwidths re-estimate it."""
    import os
    import tempfile
    wl, keep, T, M = ctx["wl"], ctx["keep"], ctx["T"], ctx["M"]
    g_flat, p16_flat, cmp_ = ctx["g_flat"], ctx["p16_flat"], ctx["streams"][1]
    offloaded = [k for k in range(wl.n_sub) if wl.tier(k) == 1]
    state_bytes = B.mlpo_state_floats(M, T) * 4
    # Eq. 1 over the two paths, in subgroups per second; the file path's bandwidth is a guess until it has been seen
    bw = [ctx["host_GBs"] * 1e9 / (state_bytes), args.file_GBs_guess * 1e9 / state_bytes]
    cap = [min(args.pinned_capacity, len(offloaded)), len(offloaded)]
    counts, _ = B.mlpo_assign_tiers(len(offloaded), bw, cap)
    n_file = counts[1]
    file_ids = offloaded[len(offloaded) - n_file:]
    root = "/dev/shm" if kind == "shm" else (args.file_dir or tempfile.gettempdir())
    path = os.path.join(root, f"mlpo_bench_state_{os.getpid()}.bin")
    res = {"kind": kind, "file": path, "offloaded_subgroups": len(offloaded), "pinned_capacity": cap[0],
           "eq1_bandwidth_guess_GBs": [round(ctx["host_GBs"], 2), args.file_GBs_guess],
           "eq1_split_pinned_file": list(counts), "chunk_elems": args.multipath_chunk,
           "file_slots": args.file_slots, "file_threads": args.file_threads}
    fd = plain_fd = -1
    try:
        with open(path, "wb") as f:
            for k in file_ids:
                f.write(keep[k].numpy().tobytes())
            f.flush()
            os.fsync(f.fileno())
        try:
            fd = os.open(path, os.O_RDWR | (os.O_DIRECT if kind == "disk" else 0))
        except OSError:         # a file system without direct I/O
            fd = os.open(path, os.O_RDWR)
            res["direct_io"] = False
        plain_fd = os.open(path, os.O_RDWR)      # for growing the file (no alignment rules)
        leg_t0 = time.perf_counter()
        sgs, files = [], []
        for k in range(wl.n_sub):
            gk, pk = g_flat[k * M:(k + 1) * M], p16_flat[k * M:(k + 1) * M]
            if k in file_ids:
                sgs.append(B.SubgroupC(None, None, None, gk.data_ptr(), pk.data_ptr(), M, B.TIER_FILE, T))
                files.append((fd, file_ids.index(k) * state_bytes))
            else:
                sgs.append(B.tiled_subgroup(keep[k], gk, pk, n=M, tier=wl.tier(k), tile_elems=T))
                files.append(None)
        table = B.SubgroupTable(sgs)
        need = B.mlpo_stream_bounce_bytes(table, args.file_slots, args.multipath_chunk)
        bounce = torch.empty(need, dtype=torch.uint8, pin_memory=True)
        cfg = B.direct_cfg(ctx["streams"][0], cmp_, 64, chunk_elems=args.multipath_chunk, files=files, bounce=bounce,
                           bounce_bytes=need, file_slots=args.file_slots, file_threads=args.file_threads,
                           want_file_stats=True)
        applied = ctx["applied"]

        def timed_steps(cfg, limit_s, count):
            """Up to `count` timed steps after the warm-up ones; stops early once `limit_s` seconds have gone by."""
            nonlocal applied
            times, rd, wr, wall = [], [], [], []
            leg_start = time.perf_counter()
            for s in range(args.stream_warmup + count):
                if times and time.perf_counter() - leg_start > limit_s:
                    break       # a slow disk must not stretch the run: one timed step is enough to report
                torch.cuda.synchronize()
                t = time.perf_counter()
                B.mlpo_grad_unscale_norm(table, wl.inv_scale, wl.max_norm, ctx["ws"], ctx["ws_bytes"], ctx["scal"],
                                         cmp_)
                assert B.mlpo_stream_update(table, None, ctx["hp"], applied + 1, ctx["scal"], cfg)
                cmp_.synchronize()
                torch.cuda.synchronize()
                dt = time.perf_counter() - t
                applied += 1
                if s >= args.stream_warmup:
                    times.append(dt)
                    st = cfg.stats
                    rd.append(st.bytes_read / st.read_seconds * max(args.file_threads, 1) if st.read_seconds else 0.0)
                    wr.append(st.bytes_written / st.write_seconds * max(args.file_threads, 1)
                              if st.write_seconds else 0.0)
                    wall.append(st.wall_seconds)
            return times, rd, wr, wall

        times, rd, wr, wall = timed_steps(cfg, args.multipath_seconds, wl.steps)
        mean = sum(times) / len(times)
        n_pinned = len(offloaded) - n_file
        file_wall = sum(wall) / len(wall)
        res.update({
            "steps": len(times), "ms_per_step": round(mean * 1e3, 2), "min_ms": round(min(times) * 1e3, 2),
            "Gparams_s": round(wl.n_total / mean / 1e9, 3),
            "file_path_wall_ms": round(file_wall * 1e3, 2),
            "file_read_GBs_while_reading": round(sum(rd) / len(rd) / 1e9, 2),
            "file_write_GBs_while_writing": round(sum(wr) / len(wr) / 1e9, 2),
            "file_path_GBs_per_dir": round(n_file * state_bytes / file_wall / 1e9, 2) if n_file else None,
            "link_GBs_per_dir": round(len(offloaded) * state_bytes / mean / 1e9, 2),
            "pinned_only_would_take_ms": round(n_pinned * state_bytes / (ctx["host_GBs"] * 1e9) * 1e3, 2)})
        if n_file:
            # Section 3.3: the next iteration's split uses the bandwidths observed in this one
            # (only the file path was timed on its own; the host path keeps its estimate, as a path that moved
            # nothing does)
            new_bw = B.mlpo_update_bandwidth(bw, [0.0, float(n_file)], [0.0, file_wall])
            res["eq1_bandwidth_observed_GBs"] = [round(x * state_bytes / 1e9, 2) for x in new_bw]
            res["eq1_split_after_update"] = list(B.mlpo_assign_tiers(len(offloaded), new_bw, cap)[0])
            res["eq1_split_after_update_without_capacity"] = list(B.mlpo_assign_tiers(len(offloaded), new_bw)[0])
            # Algorithm 1 assigns the path anew when it flushes a subgroup: the subgroups that the new split puts on
            # the other path move there as part of one ordinary update step (their new state is stored at the new
            # home instead of the old one), and the steps after it run with the new split.
            new_file = res["eq1_split_after_update"][1]
            if new_file != n_file and time.perf_counter() - leg_t0 < 2 * args.multipath_seconds:
                targets = [None] * wl.n_sub
                if new_file > n_file:       # pinned -> file: the last pinned subgroups, to new extents at the end
                    movers = offloaded[len(offloaded) - new_file:len(offloaded) - n_file]
                    zeros = bytes(1 << 24)
                    for j, k in enumerate(movers):
                        off = (n_file + j) * state_bytes
                        for o in range(0, state_bytes, len(zeros)):   # real pages, not a hole
                            os.pwrite(plain_fd, zeros[:min(len(zeros), state_bytes - o)], off + o)
                        targets[k] = (fd, off)
                    os.fsync(plain_fd)
                else:                       # file -> pinned: the first file-tier subgroups, to their pinned buffers
                    movers = file_ids[:n_file - new_file]
                    for k in movers:
                        targets[k] = keep[k]
                need2 = B.mlpo_stream_bounce_bytes(table, args.file_slots, args.multipath_chunk, flush_to=targets)
                if need2 > need:
                    bounce = torch.empty(need2, dtype=torch.uint8, pin_memory=True)
                move_cfg = B.direct_cfg(ctx["streams"][0], cmp_, 64, chunk_elems=args.multipath_chunk, files=files,
                                        bounce=bounce, bounce_bytes=bounce.numel(), file_slots=args.file_slots,
                                        file_threads=args.file_threads, want_file_stats=True, flush_to=targets)
                torch.cuda.synchronize()
                t = time.perf_counter()
                B.mlpo_grad_unscale_norm(table, wl.inv_scale, wl.max_norm, ctx["ws"], ctx["ws_bytes"], ctx["scal"],
                                         cmp_)
                assert B.mlpo_stream_update(table, None, ctx["hp"], applied + 1, ctx["scal"], move_cfg)
                cmp_.synchronize()
                torch.cuda.synchronize()
                move_ms = (time.perf_counter() - t) * 1e3
                applied += 1
                for k in movers:
                    gk, pk = g_flat[k * M:(k + 1) * M], p16_flat[k * M:(k + 1) * M]
                    if new_file > n_file:
                        sgs[k] = B.SubgroupC(None, None, None, gk.data_ptr(), pk.data_ptr(), M, B.TIER_FILE, T)
                        files[k] = targets[k]
                    else:
                        sgs[k] = B.tiled_subgroup(keep[k], gk, pk, n=M, tier=wl.tier(k), tile_elems=T)
                        files[k] = None
                table = B.SubgroupTable(sgs)
                cfg = B.direct_cfg(ctx["streams"][0], cmp_, 64, chunk_elems=args.multipath_chunk, files=files,
                                   bounce=bounce, bounce_bytes=bounce.numel(), file_slots=args.file_slots,
                                   file_threads=args.file_threads, want_file_stats=True)
                t2, _, _, wall2 = timed_steps(cfg, args.multipath_seconds / 2, wl.steps)
                mean2 = sum(t2) / len(t2)
                res["after_rebalance"] = {
                    "split_pinned_file": [len(offloaded) - new_file, new_file], "subgroups_moved": len(movers),
                    "direction": "pinned->file" if new_file > n_file else "file->pinned",
                    "move_step_ms": round(move_ms, 2), "steps": len(t2), "ms_per_step": round(mean2 * 1e3, 2),
                    "min_ms": round(min(t2) * 1e3, 2),
                    "file_path_GBs_per_dir": round(new_file * state_bytes / (sum(wall2) / len(wall2)) / 1e9, 2)
                    if new_file and sum(wall2) > 0 else None,
                    "link_GBs_per_dir": round(len(offloaded) * state_bytes / mean2 / 1e9, 2)}
        ctx["applied"] = applied
    finally:
        torch.cuda.synchronize()
        for d in (fd, plain_fd):
            if d >= 0:
                os.close(d)
        if os.path.exists(path):
            os.unlink(path)
    log(f"[bench] multipath {res}")
    return res


_hip = None


def hip_runtime(torch):
    """The HIP runtime this process already uses (the one torch loaded), for pinned allocations of exact size:
    torch's pinned allocator rounds requests up to a power of two, which would waste a third of what can be pinned."""
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
    """n floats of page-locked host memory as a numpy array; MemoryError if the machine will not pin that much."""

    def __init__(self, torch, np, n):
        import ctypes as C
        self.hip = hip_runtime(torch)
        self.ptr = C.c_void_p()
        if self.hip.hipHostMalloc(C.byref(self.ptr), 4 * n, 0) != 0 or not self.ptr.value:
            self.ptr = None
            self.hip.hipGetLastError()      # the runtime would report the refusal again at the next call that checks
            raise MemoryError(f"cannot pin {4 * n / 1e9:.2f} GB")
        self.np = np.ctypeslib.as_array((C.c_float * n).from_address(self.ptr.value))

    def data_ptr(self):
        return self.ptr.value

    def free(self):
        if self.ptr is not None:
            self.np = None
            self.hip.hipHostFree(self.ptr)
            self.ptr = None


def large_config_leg(args, torch, B, W, np, name, modes, bidir_GBs):
    """One of the two large mixed-tier workloads WHOLE (the 7 B- and the 8.75 B-parameter one): HBM-tier subgroups resident,
    offloaded subgroups in pinned host memory, and - where the machine will not pin all of them - the rest in a file
    in /dev/shm (pageable host memory behind the second path).  Gradient pass + mlpo_stream_update per step, one
    warm-up step and the workload's step count timed, per mode in `modes`."""
    wl = W.CONFIGS[name]
    d = torch.device("cuda:0")
    M, T = wl.sub_elems, args.tile
    per = B.mlpo_state_floats(M, T)
    t_setup = time.time()
    pinned, keep, fd, path = [], [], -1, None
    rec = {"workload": wl.name, "params": wl.n_total, "subgroups": wl.n_sub, "subgroup_elems": M,
           "loss_scale": wl.loss_scale, "max_norm": wl.max_norm, "runs": []}
    try:
        g_flat = torch.empty(wl.n_total, dtype=torch.int16, device=d)
        p16_flat = torch.zeros(wl.n_total, dtype=torch.int16, device=d)
        tmp = np.zeros(per // 3, np.float32)
        hg = np.empty(M, np.uint16)
        homes, file_ids = {}, []
        for k in range(wl.n_sub):
            if wl.tier(k) == 1 and not file_ids:
                try:
                    homes[k] = PinnedF32(torch, np, per)
                    pinned.append(homes[k])
                    continue
                except MemoryError:
                    pass
            if wl.tier(k) == 1:
                file_ids.append(k)          # no more can be pinned: this one and the later ones live in the file
        if file_ids:
            if pinned:                      # leave room for the bounce buffers
                file_ids.insert(0, max(homes))
                homes.pop(max(homes))
                pinned.pop().free()
            path = f"/dev/shm/mlpo_bench_{name}_{os.getpid()}.bin"
            fd = os.open(path, os.O_RDWR | os.O_CREAT | os.O_TRUNC, 0o600)
        tiled = np.zeros(per, np.float32) if file_ids else None
        sgs, files = [], []
        for k in range(wl.n_sub):
            W.fill_state(wl, k, tmp[:M], None, None, threads=args.threads)      # m = v = 0
            W.fill_grads(wl, k, 0, hg, threads=args.threads)
            gk, pk = g_flat[k * M:(k + 1) * M], p16_flat[k * M:(k + 1) * M]
            gk.copy_(torch.from_numpy(hg.view(np.int16)))
            if k in file_ids:
                tiled.reshape(-1, 3, T)[:, 0, :] = tmp.reshape(-1, T)
                off = file_ids.index(k) * per * 4
                mv = memoryview(tiled).cast("B")    # real pages, no holes; one write call moves at most 2 GiB
                done = 0
                while done < len(mv):
                    done += os.pwrite(fd, mv[done:done + (1 << 30)], off + done)
                sgs.append(B.SubgroupC(None, None, None, gk.data_ptr(), pk.data_ptr(), M, B.TIER_FILE, T))
                files.append((fd, off))
                continue
            files.append(None)
            if k in homes:
                homes[k].np[:] = 0
                homes[k].np.reshape(-1, 3, T)[:, 0, :] = tmp.reshape(-1, T)
                sgs.append(B.tiled_subgroup(homes[k].data_ptr(), gk, pk, n=M, tier=B.TIER_HOST, tile_elems=T))
            else:
                st = torch.zeros(per, dtype=torch.float32, device=d)
                st.view(-1, 3, T)[:, 0, :].copy_(torch.from_numpy(tmp).view(-1, T))
                keep.append(st)
                sgs.append(B.tiled_subgroup(st, gk, pk, n=M, tier=B.TIER_HBM, tile_elems=T))
        del tiled
        table = B.SubgroupTable(sgs)
        n_off = wl.n_host
        rec.update({"hbm_subgroups": wl.n_sub - n_off, "pinned_subgroups": len(homes), "file_subgroups": len(file_ids),
                    "file": path, "offloaded_params": n_off * M, "bytes_per_direction_per_step": 12 * n_off * M,
                    "setup_s": round(time.time() - t_setup, 1)})
        ws_bytes = B.mlpo_norm_workspace_bytes()
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device=d)
        scal = torch.zeros(4, dtype=torch.float32, device=d)
        hp = B.HParams(**wl.hp.__dict__)
        h2d, cmp_ = torch.cuda.Stream(), torch.cuda.Stream()
        applied = 0
        for mode in modes:
            stg = bounce = None
            chunk = 1 << 24
            if file_ids or mode == "direct":
                if file_ids:
                    need = B.mlpo_stream_bounce_bytes(table, args.file_slots, chunk)
                    bounce = PinnedF32(torch, np, need // 4)
                    pinned.append(bounce)
                    cfg = B.direct_cfg(h2d, cmp_, 64, chunk_elems=chunk, files=files, bounce=bounce.data_ptr(),
                                       bounce_bytes=need, file_slots=args.file_slots, file_threads=8,
                                       want_file_stats=True)
                else:
                    cfg = B.direct_cfg(h2d, cmp_, 64)
                what = {"mode": "direct" + (", two paths (pinned + file in /dev/shm)" if file_ids else ""),
                        "direct_blocks": 64}
            else:
                need = B.mlpo_stream_staging_bytes(table, 4, chunk)
                stg = torch.empty(need, dtype=torch.uint8, device=d)
                cfg = B.stream_cfg(4, stg, need, None, cmp_, None, chunk)
                what = {"mode": "staged", "n_slots": 4, "chunk_elems": chunk}
            times, file_wall = [], []
            for s_ in range(1 + wl.steps):
                torch.cuda.synchronize()
                t = time.perf_counter()
                B.mlpo_grad_unscale_norm(table, wl.inv_scale, wl.max_norm, ws, ws_bytes, scal, cmp_)
                ok = B.mlpo_stream_update(table, None, hp, applied + 1, scal, cfg)
                cmp_.synchronize()
                torch.cuda.synchronize()
                dt = time.perf_counter() - t
                assert ok, "a step of finite gradients was skipped"
                applied += 1
                if s_ >= 1:
                    times.append(dt)
                    if file_ids:
                        file_wall.append(cfg.stats.wall_seconds)
            mean = sum(times) / len(times)
            gbs = 12 * n_off * M / mean / 1e9
            sc = scal.cpu().numpy()
            run = {**what, "steps": len(times), "ms_per_step": round(mean * 1e3, 2),
                   "min_ms": round(min(times) * 1e3, 2), "Gparams_s": round(wl.n_total / mean / 1e9, 3),
                   "pcie_GBs_per_dir": round(gbs, 2), "frac_nominal": round(gbs / PCIE_NOMINAL_GBS, 4),
                   "frac_of_bidir_memcpy": round(gbs / bidir_GBs, 4) if bidir_GBs else None,
                   "grad_norm": float(sc[0]), "clip_coef": float(sc[1])}
            if file_wall:       # the file path's own pace: its bytes over the time from its first read to its last write
                fw = sum(file_wall) / len(file_wall)
                run.update({"file_path_wall_ms": round(fw * 1e3, 1),
                            "file_path_GBs_per_dir": round(12 * len(file_ids) * M / fw / 1e9, 2)})
            rec["runs"].append(run)
            log(f"[bench] {wl.name} {run}")
            del stg, cfg
            if bounce is not None:
                pinned.remove(bounce)
                bounce.free()
    except (MemoryError, OSError, RuntimeError) as e:
        rec["error"] = f"{type(e).__name__}: {e}"
        log(f"[bench] {name} leg failed: {e}")
    finally:
        torch.cuda.synchronize()
        for b_ in pinned:
            b_.free()
        if fd >= 0:
            os.close(fd)
        if path and os.path.exists(path):
            os.unlink(path)
        keep.clear()
        g_flat = p16_flat = None
        torch.cuda.empty_cache()
    return rec


def three_path_bench(args, torch, B, np, ctx, two_path):
    """Three live paths behind the offloaded tier (Section 3.2 "Unified Multi-level, Multi-path Asynchronous
    Offloading using Virtual Tiers"): pinned host memory (limited to ``--pinned-capacity-3`` subgroups), a file in
    /dev/shm and a file on the disk, each file path with its own workers and bounce buffers.  Eq. 1 (Section 3.3)
    splits the subgroups from guessed bandwidths; the step is compared with what the slowest path needs on its own
    (bytes over the bandwidth that path showed in the two-path runs)."""
    import tempfile
    wl, keep, T, M = ctx["wl"], ctx["keep"], ctx["T"], ctx["M"]
    g_flat, p16_flat, cmp_ = ctx["g_flat"], ctx["p16_flat"], ctx["streams"][1]
    offloaded = [k for k in range(wl.n_sub) if wl.tier(k) == 1]
    state_bytes = B.mlpo_state_floats(M, T) * 4
    guess = [ctx["host_GBs"]] + [float(x) for x in args.three_path_guess.split(",")]      # pinned, shm, disk
    bw = [g * 1e9 / state_bytes for g in guess]
    cap = [min(args.pinned_capacity_3, len(offloaded)), len(offloaded), len(offloaded)]
    counts, tier_of = B.mlpo_assign_tiers(len(offloaded), bw, cap)
    # the slowest path takes the lowest ids (Section 3.2 "Cache-Friendly Ordering")
    where = {k: tier_of[j] for j, k in enumerate(offloaded)}
    paths = [f"/dev/shm/mlpo_bench3_{os.getpid()}.bin",
             os.path.join(args.file_dir or tempfile.gettempdir(), f"mlpo_bench3_{os.getpid()}.bin")]
    res = {"paths": ["pinned host memory", paths[0], paths[1]], "eq1_bandwidth_guess_GBs": [round(g, 2) for g in guess],
           "pinned_capacity": cap[0], "eq1_split_pinned_shm_disk": list(counts), "chunk_elems": args.multipath_chunk,
           "file_slots": 6, "file_threads_per_path": args.file_threads}
    fds = []
    try:
        slot_of, sgs, files = {}, [], []
        for which, path in enumerate(paths):
            mine = [k for k in offloaded if where[k] == which + 1]
            with open(path, "wb") as f:
                for j, k in enumerate(mine):
                    slot_of[k] = j
                    f.write(keep[k].numpy().tobytes())
                f.flush()
                os.fsync(f.fileno())
            try:
                fds.append(os.open(path, os.O_RDWR | (os.O_DIRECT if which == 1 else 0)))
            except OSError:
                fds.append(os.open(path, os.O_RDWR))
        for k in range(wl.n_sub):
            gk, pk = g_flat[k * M:(k + 1) * M], p16_flat[k * M:(k + 1) * M]
            if where.get(k, 0) > 0:
                sgs.append(B.SubgroupC(None, None, None, gk.data_ptr(), pk.data_ptr(), M, B.TIER_FILE, T))
                files.append((fds[where[k] - 1], slot_of[k] * state_bytes))
            else:
                sgs.append(B.tiled_subgroup(keep[k], gk, pk, n=M, tier=wl.tier(k), tile_elems=T))
                files.append(None)
        table = B.SubgroupTable(sgs)
        need = B.mlpo_stream_bounce_bytes(table, 6, args.multipath_chunk)
        bounce = torch.empty(need, dtype=torch.uint8, pin_memory=True)
        cfg = B.direct_cfg(ctx["streams"][0], cmp_, 64, chunk_elems=args.multipath_chunk, files=files, bounce=bounce,
                           bounce_bytes=need, file_slots=6, file_threads=args.file_threads, want_file_stats=True)
        ids = [os.fstat(fd).st_dev for fd in fds]
        applied, times, per_path = ctx["applied"], [], {i: [] for i in ids}
        t_leg = time.perf_counter()
        for s in range(1 + wl.steps):
            if times and time.perf_counter() - t_leg > args.multipath_seconds:
                break
            torch.cuda.synchronize()
            t = time.perf_counter()
            B.mlpo_grad_unscale_norm(table, wl.inv_scale, wl.max_norm, ctx["ws"], ctx["ws_bytes"], ctx["scal"], cmp_)
            assert B.mlpo_stream_update(table, None, ctx["hp"], applied + 1, ctx["scal"], cfg)
            cmp_.synchronize()
            torch.cuda.synchronize()
            dt = time.perf_counter() - t
            applied += 1
            if s >= 1:
                times.append(dt)
                for p in cfg.paths:
                    if p.used and p.stats.wall_seconds > 0:
                        per_path[p.path_id].append(p.stats.bytes_read / p.stats.wall_seconds / 1e9)
        ctx["applied"] = applied
        mean = sum(times) / len(times)
        seen = [ctx["host_GBs"]] + [sum(per_path[i]) / len(per_path[i]) if per_path[i] else g
                                    for i, g in zip(ids, guess[1:])]
        # what each path needs alone for its share, at the bandwidth it showed when it was the only file path
        alone = [ctx["host_GBs"], two_path.get("shm") or seen[1], two_path.get("disk") or seen[2]]
        need_ms = [c * state_bytes / (b * 1e9) * 1e3 for c, b in zip(counts, alone)]
        res.update({"steps": len(times), "ms_per_step": round(mean * 1e3, 2), "min_ms": round(min(times) * 1e3, 2),
                    "Gparams_s": round(wl.n_total / mean / 1e9, 3),
                    "link_GBs_per_dir": round(len(offloaded) * state_bytes / mean / 1e9, 2),
                    "path_GBs_per_dir_observed": [round(x, 2) for x in seen],
                    "path_GBs_per_dir_alone": [round(x, 2) for x in alone],
                    "each_path_alone_would_take_ms": [round(x, 1) for x in need_ms],
                    "step_over_slowest_path_alone": round(mean * 1e3 / max(need_ms), 3)})
        new_bw = B.mlpo_update_bandwidth(bw, [float(c) for c in counts],
                                         [c / (g * 1e9 / state_bytes) if c else 0.0 for c, g in zip(counts, seen)])
        res["eq1_split_after_update"] = list(B.mlpo_assign_tiers(len(offloaded), new_bw, cap)[0])
    finally:
        torch.cuda.synchronize()
        for fd in fds:
            os.close(fd)
        for path in paths:
            if os.path.exists(path):
                os.unlink(path)
    log(f"[bench] three paths {res}")
    return res


def accumulate_bench(torch, B, acc_dev, g_dev, wl):
    """mlpo_grad_accumulate at the shard's size: the accumulation buffer in HBM (6 bytes of HBM traffic per element)
    and in pinned host memory (2 bytes per element over the link in each direction), 4 micro-batches each."""
    n = acc_dev.numel()
    M = wl.sub_elems
    res = {"elements": n, "micro_batches": 4}
    B.mlpo_kernel_timing(True)
    for j in range(5):          # the first call (first=True: a copy, 4 bytes per element) doubles as warm-up
        B.mlpo_grad_accumulate(acc_dev, g_dev, n, first=(j == 0))
    torch.cuda.synchronize()
    ms = B.mlpo_kernel_times(4)[1:]
    avg = sum(ms) / len(ms)
    res["hbm"] = {"avg_launch_ms": round(avg, 4), "achieved_GBs": round(6 * n / avg / 1e6, 1),
                  "frac_hbm_peak": round(6 * n / avg / 1e6 / HBM_PEAK_GBS, 4), "bytes_per_element": 6}
    host = torch.empty(wl.n_host * M, dtype=torch.int16, pin_memory=True)
    nh = host.numel()
    best = None
    for blocks in (32, 64, 128):
        for j in range(5):
            B.mlpo_grad_accumulate(host, g_dev[:nh], nh, first=(j == 0), blocks=blocks)
        torch.cuda.synchronize()
        ms = B.mlpo_kernel_times(4)[1:]
        avg = sum(ms) / len(ms)
        rec = {"blocks": blocks, "elements": nh, "avg_launch_ms": round(avg, 3),
               "pcie_GBs_per_dir": round(2 * nh / avg / 1e6, 2),
               "frac_nominal": round(2 * nh / avg / 1e6 / PCIE_NOMINAL_GBS, 4)}
        res.setdefault("pinned_host", []).append(rec)
        if best is None or rec["pcie_GBs_per_dir"] > best["pcie_GBs_per_dir"]:
            best = rec
    ws_bytes = B.mlpo_norm_workspace_bytes()
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=acc_dev.device)
    for label, buf, nn, blocks in (("hbm_with_statistics", acc_dev, n, 0), ("pinned_host_with_statistics", host, nh, 64)):
        for j in range(4):
            B.mlpo_grad_accumulate_norm(buf, g_dev[:nn], nn, False, blocks, 1.0, ws, ws_bytes, True)
        torch.cuda.synchronize()
        ms = B.mlpo_kernel_times(4)[1:]
        avg = sum(ms) / len(ms)
        res[label] = {"avg_launch_ms": round(avg, 3), "blocks": blocks}
        if blocks:
            res[label]["pcie_GBs_per_dir"] = round(2 * nn / avg / 1e6, 2)
        else:
            res[label]["achieved_GBs"] = round(6 * nn / avg / 1e6, 1)
    B.mlpo_kernel_timing(False)
    res["pinned_host_best"] = best
    log(f"[bench] grad_accumulate {res}")
    return res


def parse_variants(text):
    res = []
    for part in text.split(","):
        a, _, b = part.partition(":")
        res.append((a if a in ("d", "c", "dg", "sg", "dga", "dgk", "sgk") else int(a), WHOLE if b == "w" else int(b or 0)))
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="C2")
    ap.add_argument("--layout", default="both", choices=["tiled", "planar", "both"],
                    help="fp32 state layout(s) to time; the first is the headline figure")
    ap.add_argument("--tile", type=int, default=8192, help="tile_elems of the tiled layout")
    ap.add_argument("--no-lead", dest="lead", action="store_false",
                    help="tiled layout: start every subgroup at the beginning of its state buffer instead of "
                         "shifting it until the lines of its g / p16 slices coincide with those of p, m, v")
    ap.add_argument("--half", default="bf16", choices=["bf16", "fp16"],
                    help="format of gradients and working parameters in the resident run (the workloads are bf16; "
                         "fp16 reads the same generated bit patterns as fp16 values, for timing)")
    ap.add_argument("--streamed", default="C3", help="host-tier workload for the pipeline figures, or 'none'")
    ap.add_argument("--stream-variants", default="2:0,3:w,3:0,4:0,d:64,d:128,dg:64,dga:64,dgk:64,sg:0,sgk:0,c:4,c:8",
                    help="comma list of n_slots:chunk_elems (staged mode; chunk 0 = the library's choice, w = whole subgroups), d:blocks (direct mode), dg:blocks (direct "
                         "mode, gradients in pinned host memory too), dga:blocks (the same with the gradient statistics "
                         "left by the last accumulation instead of a gradient pass), dgk:blocks / sgk:chunk_elems (gradients in pinned host memory, "
                         "the gradient pass keeps a device copy that the update reads), sg:chunk_elems (staged mode with 3 slots, "
                         "gradients in pinned host memory too) or c:n_slots (staged mode with slots that keep their "
                         "subgroups and alternating order)")
    ap.add_argument("--cache-blocks", type=int, default=0,
                    help="c: variants: workgroups of the kernel that exchanges a slot's occupants (0 = the library's "
                         "default)")
    ap.add_argument("--stream-warmup", type=int, default=2)
    ap.add_argument("--large", default="C4,C5",
                    help="comma list of the large mixed-tier workloads to run whole after the streamed one, or 'none'")
    ap.add_argument("--multipath", default="disk,shm",
                    help="comma list of file kinds for the two-path run on the streamed workload: disk (a file in "
                         "--file-dir, O_DIRECT), shm (a file in /dev/shm), or 'none'")
    ap.add_argument("--pinned-capacity", type=int, default=10,
                    help="subgroups the pinned-host path may hold in the two-path run (the rest go to the file)")
    ap.add_argument("--no-link-yardstick", dest="link_yardstick", action="store_false",
                    help="do not start the pinned-copy yardstick in a process of its own before the run")
    ap.add_argument("--no-three-paths", dest="three_paths", action="store_false",
                    help="skip the run with three live paths (pinned memory, a file in /dev/shm, a file on the disk)")
    ap.add_argument("--pinned-capacity-3", type=int, default=8,
                    help="subgroups the pinned-host path may hold in the three-path run")
    ap.add_argument("--three-path-guess", default="20,6",
                    help="initial bandwidth estimates (GB/s) of the /dev/shm path and of the disk path in the three-path run")
    ap.add_argument("--hbm-capacity", type=int, default=4,
                    help="streamed workload: subgroups that HBM has room for in the re-balancing run (0 = skip it)")
    ap.add_argument("--file-GBs-guess", type=float, default=3.0, help="initial bandwidth estimate of the file path")
    ap.add_argument("--file-dir", default="", help="directory for the file path's file (default: the temp dir)")
    ap.add_argument("--file-slots", type=int, default=3)
    ap.add_argument("--file-threads", type=int, default=4)
    ap.add_argument("--multipath-chunk", type=int, default=1 << 24)
    ap.add_argument("--multipath-seconds", type=float, default=20.0,
                    help="a two-path run stops taking further steps after this long (at least one is timed)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-yardsticks", action="store_true", help="skip the bare read / write / in-place sweeps")
    ap.add_argument("--cpu-subgroups", type=int, default=9)
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--threads", type=int, default=16)
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run 1 GiB copy kernels (reference traffic for profiler byte counters)")
    args = ap.parse_args()
    args.stream_variants = parse_variants(args.stream_variants)
    args.half_format = {"bf16": 0, "fp16": 1}[args.half]
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    # Plain pinned copies in a process of their own, before this one touches the GPU: two streams in a fresh process
    # with the system's HIP runtime (the copies of ys_link inside this process share the device with torch's runtime
    # and its streams, and have been seen to take turns there instead of overlapping).
    link_fresh = None
    # (not under a profiler: its preloaded library may have initialised the GPU in this process already, and a
    # process that has must not start another program)
    under_profiler = any("rocprof" in os.environ.get(k, "") for k in ("LD_PRELOAD", "ROCP_TOOL_LIBRARIES",
                                                                     "ROCPROFILER_LIBRARY_CTOR", "HSA_TOOLS_LIB"))
    if args.streamed != "none" and args.link_yardstick and not under_profiler:
        import subprocess
        exe = os.path.join(ROOT, "bench_link_yardstick")
        # three runs, the best one counts: the first process on a machine that has just been handed out has been seen
        # to copy at half the rate of every later one
        for _ in range(3):
            try:
                one = json.loads(subprocess.run([exe, "400"], capture_output=True, text=True, timeout=120,
                                                check=True).stdout.strip().splitlines()[-1])
            except (OSError, subprocess.SubprocessError, ValueError, IndexError) as e:
                one = {"error": f"{type(e).__name__}: {e}"}
            if link_fresh is None or one.get("bidir_GBs_per_dir", 0.0) > link_fresh.get("bidir_GBs_per_dir", 0.0):
                link_fresh = one
        log(f"[bench] link yardstick in a fresh process: {link_fresh}")
    import numpy as np
    import torch

    from paper_2509_02480_amd import binding as B
    from paper_2509_02480_amd import workloads as W
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    B.lib()  # fails loudly if the HIP library is not built
    layouts = {"tiled": [args.tile], "planar": [0], "both": [args.tile, 0]}[args.layout]
    runs = [resident_bench(args, torch, B, W, np, t) for t in layouts]
    res = resident_result(args, W.CONFIGS[args.workload], runs[0], runs[1:])
    if args.calib_copy:
        calibration_copies(torch)
    if not args.no_yardsticks:
        planar = [r for r in runs if r["layout"] == "planar"]
        res["yardsticks"] = yardsticks(torch, W.CONFIGS[args.workload], args.tile, res["roofline"]["achieved"],
                                       planar[0]["roofline"]["achieved"] if planar else None,
                                       res["norm_pass"]["achieved_GBs"])
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(args, W, np)
    else:
        res["cpu_baseline"] = None
    if args.streamed != "none":
        res["streamed"] = st = streamed_bench(args, torch, B, W, np, link_fresh)
        st["memcpy_fresh_process"] = link_fresh
        bidir = max(st["memcpy_bidir_GBs_per_dir"], (link_fresh or {}).get("bidir_GBs_per_dir", 0.0))
        best = st["best"]
        # the second half of the metric: effective GB/s per direction over the host link, against the nominal rate of
        # PCIe 5.0 x16 and, as yardsticks, what plain pinned copies reach on this machine
        res["roofline_streamed"] = {
            "bound": "pcie", "achieved": best["pcie_GBs_per_dir"], "peak": PCIE_NOMINAL_GBS, "unit": "GB/s per direction",
            "frac": best["frac_nominal"], "workload": st["workload"], "mode": best["mode"],
            "ms_per_step": best["ms_per_step"], "bytes_per_direction_per_step": st["bytes_per_direction_per_step"],
            "yardstick_memcpy_bidir_GBs_per_dir": bidir,
            "yardstick_memcpy_bidir_in_this_process_GBs_per_dir": st["memcpy_bidir_GBs_per_dir"],
            "yardstick_memcpy_one_way_GBs": [st["memcpy_h2d_GBs"], st["memcpy_d2h_GBs"]],
            "frac_of_bidir_memcpy": round(best["pcie_GBs_per_dir"] / bidir, 4)}
        torch.cuda.empty_cache()
        large = []
        for name in [x for x in args.large.split(",") if x and x != "none"]:
            modes = ["staged", "direct"] if name == "C4" else ["direct"]
            large.append(large_config_leg(args, torch, B, W, np, name, modes, bidir))
        if large:
            res["streamed_large"] = large
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
